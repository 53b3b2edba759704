"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves both the CPU oracle's tests and the GPU path's tests and
benchmark, and for that reason holds none of the method's arithmetic: no
rounding, no precision rule, no tile product.  It only produces dense FP64
matrices, explicit precision maps where a workload prescribes them, and the
parameters (threshold, allowed precisions, alpha, beta) of each workload.

Every value is a pure function of (seed, matrix id, row, column) through a
counter-based generator, so any row panel can be produced on its own and the
oracle and the GPU library always see identical bits.

Workloads (paper Section 5.1/5.2 runs random FP64/FP32 maps at tile 1024/2048;
the covariance matrices mimic the geostatistics applications the paper cites
in its introduction; no public dataset is involved):
  tiny        1024^3, tile 256, N(0,1) with tile (I,J) scaled 10^(-2|I-J|), banded explicit map
  random8k    8192^3, tile 512, U[-1,1], iid random maps FP64 .25 / FP32 .25 / FP16 .5, C FP64/FP32
  cov16k      16384^3, tile 1024, A = B = exp(-dist/0.1), Morton-ordered points, rule 1e-8
  rect32k     32768 x 32768 x 4096, tile 1024, N(0,1) with tile (I,J) scaled 2^(-4|I-J|), rule 1e-4 incl. FP8
  cov64k      65536^3, tile 2048, A = B = exp(-dist/0.05), rule 1e-6
  paperNN     the paper's own experiment (Section 5.2, Figure 3 maps, Figure 4 runs): 32768^3,
              tile 2048, U[-1,1], NN % of the tiles of A, B and C in FP64 and the rest in FP32,
              chosen at random; product precision = the C tile's (policy C_TILE); NN = 100, 80,
              50, 20, 0
"""
import numpy as np

MASTER_SEED = 250814848

FP64, FP32, FP16, FP8 = 0, 1, 2, 3
_U64 = np.uint64
_MATRIX_ID = {"A": 1, "B": 2, "C": 3, "mapA": 11, "mapB": 12, "mapC": 13, "points": 21, "sample": 31}


def _mix(z):
    """splitmix64 output function on uint64 arrays (wrap-around arithmetic)."""
    z = z + _U64(0x9E3779B97F4A7C15)
    z = (z ^ (z >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> _U64(27))) * _U64(0x94D049BB133111EB)
    return z ^ (z >> _U64(31))


def _hash(seed, matrix_id, stream, rows, cols):
    """64-bit hash of (seed, matrix, stream, row, col); rows/cols broadcast."""
    with np.errstate(over="ignore"):
        key = _mix(_mix(np.array([seed], dtype=_U64)) ^ _U64(matrix_id * 0x100 + stream))
        r = np.asarray(rows, dtype=_U64)
        c = np.asarray(cols, dtype=_U64)
        return _mix(_mix(key + r * _U64(0xD1342543DE82EF95)) + c * _U64(0xA0761D6478BD642F))


def uniform01(seed, matrix_id, stream, rows, cols):
    """Uniform in [0,1) with 53 random bits."""
    return (_hash(seed, matrix_id, stream, rows, cols) >> _U64(11)).astype(np.float64) * 2.0 ** -53


def normal01(seed, matrix_id, rows, cols):
    """Standard normal by Box-Muller on two counter streams."""
    u1 = ((_hash(seed, matrix_id, 0, rows, cols) >> _U64(11)).astype(np.float64) + 1.0) * 2.0 ** -53
    u2 = uniform01(seed, matrix_id, 1, rows, cols)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def morton_points(seed, n):
    """n points uniform in the unit square, sorted by the 32-bit Morton code of their
    coordinates quantised to 16 bits per axis (x in the even bits), stable on ties."""
    idx = np.arange(n)
    x = uniform01(seed, _MATRIX_ID["points"], 0, idx, 0)
    y = uniform01(seed, _MATRIX_ID["points"], 1, idx, 0)

    def spread(v):
        v = v.astype(np.uint32)
        v = (v | (v << 8)) & np.uint32(0x00FF00FF)
        v = (v | (v << 4)) & np.uint32(0x0F0F0F0F)
        v = (v | (v << 2)) & np.uint32(0x33333333)
        v = (v | (v << 1)) & np.uint32(0x55555555)
        return v

    qx = np.minimum((x * 65536.0).astype(np.int64), 65535)
    qy = np.minimum((y * 65536.0).astype(np.int64), 65535)
    code = spread(qx) | (spread(qy) << 1)
    order = np.argsort(code, kind="stable")
    return np.stack([x[order], y[order]], axis=1)


class Workload:
    """One GEMM-MP problem: shapes, scalars, how maps are obtained, and dense panels."""

    def __init__(self, name, M, N, K, nb, alpha, beta, seed=MASTER_SEED):
        self.name, self.M, self.N, self.K, self.nb = name, M, N, K, nb
        self.alpha, self.beta, self.seed = float(alpha), float(beta), seed
        self.rule = None          # dict(eps=..., allowed=bitmask) -> maps of A, B from the norm rule
        self.mapA = self.mapB = self.mapC = None
        self.a_equals_b = False
        self.policy = 0           # product-precision policy the workload is meant to run under

    @property
    def MT(self):
        return self.M // self.nb

    @property
    def NT(self):
        return self.N // self.nb

    @property
    def KT(self):
        return self.K // self.nb

    def shape(self, which):
        return {"A": (self.M, self.K), "B": (self.K, self.N), "C": (self.M, self.N)}[which]

    def panel(self, which, r0, r1):            # overridden
        raise NotImplementedError

    def dense(self, which, out=None, panel_rows=2048):
        rows, cols = self.shape(which)
        if out is None:
            out = np.empty((rows, cols), dtype=np.float64)
        for r0 in range(0, rows, panel_rows):
            r1 = min(rows, r0 + panel_rows)
            out[r0:r1] = self.panel(which, r0, r1)
        return out

    def sample_tiles(self, count=64):
        """Seeded sample of distinct C tiles (all of them when there are no more than count)."""
        total = self.MT * self.NT
        if total <= count:
            return [(t // self.NT, t % self.NT) for t in range(total)]
        keys = _hash(self.seed, _MATRIX_ID["sample"], 0, np.arange(total), 0)
        chosen = np.sort(np.argsort(keys, kind="stable")[:count])
        return [(int(t) // self.NT, int(t) % self.NT) for t in chosen]


class _TileScaled(Workload):
    """Entries N(0,1) or U[-1,1]; tile (I,J) of each matrix scaled by base^(-rate*|I-J|),
    each matrix using its own tile indices."""

    def __init__(self, *a, dist="normal", base=1.0, rate=0.0, **kw):
        super().__init__(*a, **kw)
        self.dist, self.base, self.rate = dist, base, rate

    def panel(self, which, r0, r1):
        rows, cols = self.shape(which)
        r = np.arange(r0, r1)[:, None]
        c = np.arange(cols)[None, :]
        mid = _MATRIX_ID[which]
        if self.dist == "normal":
            x = normal01(self.seed, mid, r, c)
        else:
            x = 2.0 * uniform01(self.seed, mid, 0, r, c) - 1.0
        if self.rate != 0.0:
            d = np.abs(r // self.nb - c // self.nb).astype(np.float64)
            x = x * np.power(self.base, -self.rate * d)
        return x


class _Covariance(Workload):
    """A = B = exp(-|x_i - x_j| / ell) on Morton-ordered points; C0 unused (beta = 0)."""

    def __init__(self, name, n, nb, ell, eps, allowed, seed=MASTER_SEED):
        super().__init__(name, n, n, n, nb, 1.0, 0.0, seed=seed)
        self.ell = ell
        self.rule = dict(eps=eps, allowed=allowed)
        self.mapC = np.zeros((self.MT, self.NT), dtype=np.uint16)
        self.a_equals_b = True
        self._pts = None

    def panel(self, which, r0, r1):
        if which == "C":
            return np.zeros((r1 - r0, self.N), dtype=np.float64)
        if self._pts is None:
            self._pts = morton_points(self.seed, self.M)
        p = self._pts
        dx = p[r0:r1, 0][:, None] - p[:, 0][None, :]
        dy = p[r0:r1, 1][:, None] - p[:, 1][None, :]
        d = np.sqrt(dx * dx + dy * dy)
        d *= -1.0 / self.ell
        return np.exp(d, out=d)


def _iid_map(seed, which, rows, cols, probs):
    """Tile precisions drawn independently with the given probabilities (code order)."""
    u = uniform01(seed, _MATRIX_ID[which], 0, np.arange(rows)[:, None], np.arange(cols)[None, :])
    edges = np.cumsum(probs)
    return np.minimum(np.searchsorted(edges, u, side="right"), len(probs) - 1).astype(np.uint16)


def tiny(M=1024, N=1024, K=1024, nb=256, seed=MASTER_SEED):
    w = _TileScaled("tiny", M, N, K, nb, 1.0, 0.0, seed=seed, dist="normal", base=10.0, rate=2.0)

    def band(rows, cols):
        d = np.abs(np.arange(rows)[:, None] - np.arange(cols)[None, :])
        return np.where(d == 0, FP64, np.where(d == 1, FP32, FP16)).astype(np.uint16)

    w.mapA, w.mapB = band(w.MT, w.KT), band(w.KT, w.NT)
    w.mapC = np.zeros((w.MT, w.NT), dtype=np.uint16)
    return w


def random_maps(M=8192, N=8192, K=8192, nb=512, probs=(0.25, 0.25, 0.5), c_probs=(0.5, 0.5),
                alpha=1.5, beta=0.5, seed=MASTER_SEED, name="random8k"):
    w = _TileScaled(name, M, N, K, nb, alpha, beta, seed=seed, dist="uniform")
    w.mapA = _iid_map(seed, "mapA", w.MT, w.KT, probs)
    w.mapB = _iid_map(seed, "mapB", w.KT, w.NT, probs)
    w.mapC = _iid_map(seed, "mapC", w.MT, w.NT, c_probs)
    return w


def _exact_ratio_map(seed, which, rows, cols, pct_double):
    """round(pct/100 * tiles) tiles FP64, the rest FP32; which ones is decided by ranking a hash
    of the tile index, so the ratio is exact and the pattern random."""
    total = rows * cols
    keys = _hash(seed, _MATRIX_ID[which], 1, np.arange(total), 0)
    n64 = int(round(pct_double / 100.0 * total))
    m = np.full(total, FP32, dtype=np.uint16)
    m[np.argsort(keys, kind="stable")[:n64]] = FP64
    return m.reshape(rows, cols)


def paper_ratio(pct_double, n=32768, nb=2048, seed=MASTER_SEED, name=None):
    """The paper's 'aD:bS' runs (Section 5.1 notation): a % of the tiles of each of A, B and C are
    FP64 and b % FP32, placed at random; every task runs at its C tile's precision."""
    w = _TileScaled(name or "paper%d" % pct_double, n, n, n, nb, 1.0, 1.0, seed=seed, dist="uniform")
    w.mapA = _exact_ratio_map(seed, "mapA", w.MT, w.KT, pct_double)
    w.mapB = _exact_ratio_map(seed, "mapB", w.KT, w.NT, pct_double)
    w.mapC = _exact_ratio_map(seed, "mapC", w.MT, w.NT, pct_double)
    w.policy = 1
    return w


def covariance(n=16384, nb=1024, ell=0.1, eps=1e-8, allowed=0b0111, seed=MASTER_SEED, name="cov16k"):
    return _Covariance(name, n, nb, ell, eps, allowed, seed=seed)


def decay_rect(M=32768, N=32768, K=4096, nb=1024, eps=1e-4, allowed=0b1111, seed=MASTER_SEED,
               name="rect32k"):
    w = _TileScaled(name, M, N, K, nb, 1.0, 0.0, seed=seed, dist="normal", base=2.0, rate=4.0)
    w.rule = dict(eps=eps, allowed=allowed)
    w.mapC = np.full((w.MT, w.NT), FP32, dtype=np.uint16)
    return w


def one_format(p, n=16384, nb=1024, seed=MASTER_SEED):
    """Every tile of A and B in one storage format (precision code p), C tiles FP32 (FP64 for
    p = FP64), U[-1,1] entries: one product precision throughout, for per-format rates.  Not one
    of the paper's workloads (its maps are FP64 / FP32 mixtures, Section 5.2)."""
    names = {0: "fp64", 1: "fp32", 2: "fp16", 3: "fp8", 4: "bf16", 5: "mxfp8", 6: "mxfp4", 7: "mxfp6"}
    w = _TileScaled("format-" + names[p], n, n, n, nb, 1.0, 0.0, seed=seed, dist="uniform")
    w.mapA = np.full((w.MT, w.KT), p, dtype=np.uint16)
    w.mapB = np.full((w.KT, w.NT), p, dtype=np.uint16)
    w.mapC = np.full((w.MT, w.NT), FP64 if p == FP64 else FP32, dtype=np.uint16)
    return w


CONFIGS = {
    "tiny": tiny,
    "random8k": random_maps,
    "cov16k": covariance,
    "rect32k": decay_rect,
    "cov64k": lambda: covariance(n=65536, nb=2048, ell=0.05, eps=1e-6, name="cov64k"),
    "paper100": lambda: paper_ratio(100),
    "paper80": lambda: paper_ratio(80),
    "paper50": lambda: paper_ratio(50),
    "paper20": lambda: paper_ratio(20),
    "paper0": lambda: paper_ratio(0),
    "format-fp64": lambda: one_format(0), "format-fp32": lambda: one_format(1), "format-fp16": lambda: one_format(2),
    "format-fp8": lambda: one_format(3), "format-bf16": lambda: one_format(4), "format-mxfp8": lambda: one_format(5),
    "format-mxfp4": lambda: one_format(6), "format-mxfp6": lambda: one_format(7),
}
