"""The checker that stands between the CPU oracle and a result computed elsewhere: the oracle's
view of a workload (maps, stored operands, exponents) and the tolerances a C computed in another
summation order must meet, per C tile and per element.

TEST INFRASTRUCTURE ONLY, like the rest of oracle/: imported by tests/, by the smoke check and by
the benchmark's cpu_baseline leg.  It does not import the GPU package; torch, where a GPU is
present, only multiplies the magnitudes |A||B| that the bounds are made of.
"""
import numpy as np

from . import gemm_mp_oracle as orc

FP64, FP32, FP16, FP8, BF16, MXFP8, MXFP4, MXFP6 = 0, 1, 2, 3, 4, 5, 6, 7
U = {FP64: 2.0 ** -53, FP32: 2.0 ** -24, FP16: 2.0 ** -11, FP8: 2.0 ** -4, BF16: 2.0 ** -8, MXFP8: 2.0 ** -4, MXFP4: 2.0 ** -2, MXFP6: 2.0 ** -4}


class OracleSide:
    """Maps, stored operands and exponents as the oracle defines them."""

    def __init__(self, w, A, B, C0=None):
        self.w = w
        nb = w.nb
        if w.rule is not None:
            sa, ma = orc.tile_scan(A, nb)
            self.mapA = orc.precision_rule(sa, w.rule["eps"], w.rule["allowed"])
            if w.a_equals_b:
                sb, mb, self.mapB = sa, ma, self.mapA
            else:
                sb, mb = orc.tile_scan(B, nb)
                self.mapB = orc.precision_rule(sb, w.rule["eps"], w.rule["allowed"])
            self.sumsq = {"A": sa, "B": sb}
        else:
            self.mapA, self.mapB = w.mapA, w.mapB
            _, ma = orc.tile_scan(A, nb)
            _, mb = orc.tile_scan(B, nb)
        self.mapC = w.mapC
        self.maxabs = {"A": ma, "B": mb}
        self.Ay, self.eA = orc.store_tiles(A, nb, self.mapA, ma)
        if w.a_equals_b:
            self.By, self.eB = self.Ay, self.eA
        else:
            self.By, self.eB = orc.store_tiles(B, nb, self.mapB, mb, mx_axis=1)     # blocks of MXFP8 tiles: down B's columns
        self.Cy = None
        if C0 is not None and w.beta != 0.0:
            Cy, eC = orc.store_tiles(C0, nb, self.mapC)
            self.Cy = orc.stored_values(Cy, nb, eC)       # what the stored C stands for (e = 0 for FP64 / FP32 tiles)

    def gemm(self, jobs, policy=orc.POLICY_OPERAND, alpha=None, beta=None):
        w = self.w
        alpha = w.alpha if alpha is None else alpha
        beta = w.beta if beta is None else beta
        return orc.gemm_jobs(w.nb, self.Ay, self.mapA, self.eA, self.By, self.mapB, self.eB,
                             self.Cy if beta != 0.0 else None, self.mapC, alpha, beta, jobs, policy=policy)


def finish_low_c_tiles(side, C):
    """C tiles stored in FP16 / FP8: the oracle's jobs return their FP32 form; storing whole tiles
    rounds them.  Returns (values the stored C stands for, exponents).  C must hold whole tiles."""
    Y, eC = orc.store_tiles(np.ascontiguousarray(C), side.w.nb, side.mapC)
    return orc.stored_values(Y, side.w.nb, eC), eC


# exponent offset of the scaled maximum and smallest step of the scaled format
LOW_FORMAT = {FP16: (14, 2.0 ** -24), FP8: (7, 2.0 ** -9)}


def job_tolerances(side, jobs, policy, alpha):
    """Per job: (spec tolerance, tight tolerance, all_fp64) multiplying
    sum_L |Ahat(I,L)[rows]|_F |Bhat(L,J)[cols]|_F, norms of the stored operands' values."""
    w = side.w
    nb, KT, K = w.nb, w.KT, w.K
    out = []
    for (I, J, r0, r1, c0, c1) in np.asarray(jobs).reshape(-1, 6):
        pC = int(side.mapC[I, J])
        norm = 0.0
        u_tile, all64 = 0.0, pC == FP64
        for L in range(KT):
            q = orc.product_precision(side.mapA[I, L], side.mapB[L, J], pC, policy)
            u_tile = max(u_tile, U[q])
            all64 &= q == FP64
            a = side.Ay[I * nb + r0:I * nb + r1, L * nb:(L + 1) * nb]
            b = side.By[L * nb:(L + 1) * nb, J * nb + c0:J * nb + c1]
            norm += np.linalg.norm(a) * 2.0 ** float(side.eA[I, L]) * np.linalg.norm(b) * 2.0 ** float(side.eB[L, J])
        u_acc = U[FP64] if all64 else U[FP32]
        # Gradual underflow: a rounded FP32 operation errs by up to (x op y) u plus half the smallest
        # subnormal.  The relative bounds above carry no such term; where a C tile's entries lie in
        # the FP32 subnormal range (products of tiles with tiny scales) two correct evaluations
        # differ by a few units of 2^-149 per entry: one per fold and epilogue operation plus one
        # per 32 terms of a reduction carried out at true magnitude.  Frobenius norm over the block.
        eta = 0.0 if pC == FP64 else (K / 32.0 + KT + 3.0) * 2.0 ** -149 * np.sqrt(float((r1 - r0) * (c1 - c0)))
        if pC >= FP16:
            u_tile = max(u_tile, U[pC])          # the tile's own storage rounding
        out.append(dict(norm=abs(alpha) * norm, tol=4.0 * K * u_tile, tight=2.0 * K * u_acc, all64=all64, eta=eta, pC=pC))
    return out


def _matmul(a, b):
    """|A| |B| in FP64: on the GPU where there is one (checker arithmetic only), else numpy."""
    try:
        import torch
        if torch.cuda.is_available():
            return (torch.from_numpy(np.ascontiguousarray(a)).cuda() @ torch.from_numpy(np.ascontiguousarray(b)).cuda()).cpu().numpy()
    except ImportError:
        pass
    return a @ b


def element_bounds(side, job, policy, alpha, beta):
    """Componentwise bound on the difference of two correct evaluations of one job, both working
    on the same stored operands (the receiver-side conversions are deterministic and identical) but
    adding in different orders.  A term that passes through at most n rounded additions carries a
    relative error of at most gamma_n, so two evaluations differ by at most twice that:
        sum_L c_L |alpha| (|A_IL||B_LJ|)_ij      the tile products, with
              c_L = 2 K u_T    where the product joins one chain over the whole reduction: every
                               product of an FP32 tile, FP64 products of an FP64 tile
              c_L = 2 nb 2^-24 for a product of an FP64 tile formed in its own FP32 accumulator
      + 2 (KT + 3) u_T (|alpha| (|A||B|)_ij + |beta| |C_ij|)   folds and epilogue in T
      + the absolute term of gradual underflow for FP32 tiles.
    Returns (bound, |alpha| |A||B|), arrays of the job's shape."""
    w = side.w
    nb, KT, K = w.nb, w.KT, w.K
    I, J, r0, r1, c0, c1 = (int(x) for x in job)
    pC = int(side.mapC[I, J])
    uT = U[FP64] if pC == FP64 else U[FP32]
    rows, cols = slice(I * nb + r0, I * nb + r1), slice(J * nb + c0, J * nb + c1)
    P = np.zeros((r1 - r0, c1 - c0))
    bound = np.zeros_like(P)

    def coeff(l):
        q = orc.product_precision(side.mapA[I, l], side.mapB[l, J], pC, policy)
        return 2.0 * K * uT if (pC != FP64 or q == FP64) else 2.0 * nb * U[FP32]

    # consecutive reduction tiles with the same coefficient go through one multiplication
    L = 0
    while L < KT:
        L1 = L + 1
        while L1 < KT and coeff(L1) == coeff(L):
            L1 += 1
        a = np.abs(side.Ay[rows, L * nb:L1 * nb]) * np.repeat(2.0 ** side.eA[I, L:L1].astype(np.float64), nb)[None, :]
        b = np.abs(side.By[L * nb:L1 * nb, cols]) * np.repeat(2.0 ** side.eB[L:L1, J].astype(np.float64), nb)[:, None]
        PL = abs(alpha) * _matmul(a, b)
        P += PL
        bound += coeff(L) * PL
        L = L1
    base = P.copy()
    if beta != 0.0 and side.Cy is not None:
        base += abs(beta) * np.abs(side.Cy[rows, cols])
    bound += 2.0 * (KT + 3) * uT * base
    if pC != FP64:
        bound += (K / 32.0 + KT + 3.0) * 2.0 ** -149
    return bound, P


# The per-tile bound 2 K u_acc sum_L |A_IL|_F |B_LJ|_F is a worst case over all rounding patterns;
# what the kernels' orders of summation actually leave is far below it (largest ratio seen over
# all tests: 0.12).  The assertion keeps a factor four over that, not the whole worst case.
TIGHT_FRACTION = 0.5


def compare_jobs(side, jobs, policy, alpha, beta, C_gpu, C_orc, elementwise=True):
    """Assert the per-tile bounds (the stated tolerance 4 K u_tile and the accumulate-precision
    form) and, per element, element_bounds; returns the worst ratios for reporting."""
    w = side.w
    nb = w.nb
    worst = dict(star=0.0, tight=0.0, rel64=0.0, elem=0.0)
    tols = job_tolerances(side, jobs, policy, alpha)
    for job, t in zip(np.asarray(jobs).reshape(-1, 6), tols):
        I, J, r0, r1, c0, c1 = (int(x) for x in job)
        blk = (slice(I * nb + r0, I * nb + r1), slice(J * nb + c0, J * nb + c1))
        g, o = C_gpu[blk], C_orc[blk]
        assert np.all(np.isfinite(g)), "non-finite GPU result in tile (%d,%d)" % (I, J)
        err = np.linalg.norm(g - o)
        base = t["norm"]
        if beta != 0.0 and side.Cy is not None:
            base = base + abs(beta) * np.linalg.norm(side.Cy[blk])
        if t["all64"]:
            rel = err / max(np.linalg.norm(o), 1e-300)
            worst["rel64"] = max(worst["rel64"], rel)
            assert rel <= 1e-12, "all-FP64 tile (%d,%d): rel Frobenius error %.3e" % (I, J, rel)
        if base == 0.0:
            assert err <= t["eta"]
            continue
        tight = TIGHT_FRACTION * t["tight"] * base + t["eta"]
        low_rel, low_abs = 0.0, 0.0
        if t["pC"] >= FP16 and np.any(o != 0.0):
            # storage rounding of the finished tile, on both sides: relative u_p per entry in the
            # format's normal range, a full smallest step below it, both doubled because the two
            # sides' exponents may differ by one when their maxima straddle a power of two
            low_rel = 2.0 * U[t["pC"]]
            tight += low_rel * np.linalg.norm(o)
            if t["pC"] in LOW_FORMAT:               # BF16 has no tile scale and FP32's range; block-scaled tiles scale per block
                E, step = LOW_FORMAT[t["pC"]]
                e_hi = np.floor(np.log2(np.abs(o).max())) - E + 1
                low_abs = step * 2.0 ** e_hi
                tight += np.sqrt(float(o.size)) * low_abs
        worst["star"] = max(worst["star"], err / (t["tol"] * base))
        worst["tight"] = max(worst["tight"], err / tight)
        assert err <= t["tol"] * base, "tile (%d,%d): err %.3e > 4*K*u_tile bound %.3e" % (I, J, err, t["tol"] * base)
        assert err <= tight, "tile (%d,%d): err %.3e > accumulate-precision bound %.3e" % (I, J, err, tight)
        if not elementwise:
            continue
        eb, _ = element_bounds(side, job, policy, alpha, beta)
        if t["pC"] in (MXFP8, MXFP4, MXFP6):
            # a block of 32 along the row is rounded relative to its own largest entry (and
            # saturates just below the next power of two): a quarter of that entry covers both
            ob = np.abs(o)
            if c0 % 32 == 0 and (c1 - c0) % 32 == 0:
                top = np.repeat(ob.reshape(ob.shape[0], -1, 32).max(axis=2), 32, axis=1)
            else:
                top = np.broadcast_to(ob.max(axis=1, keepdims=True), ob.shape)
            eb = eb + 2.0 * max(U[t["pC"]], 0.125) * 2.0 * top
        elif t["pC"] >= FP16:
            eb = eb + low_rel * np.abs(o) + low_abs
        d = np.abs(g - o)
        bad = d > eb
        ratio = float((d / np.maximum(eb, 1e-300)).max())
        worst["elem"] = max(worst["elem"], ratio)
        if bad.any():
            r, c = np.unravel_index(int(np.argmax(d / np.maximum(eb, 1e-300))), d.shape)
            raise AssertionError("tile (%d,%d) element (%d,%d): |gpu - oracle| = %.3e > componentwise bound %.3e (%d elements of the job over their bound)"
                                 % (I, J, r0 + r, c0 + c, d[r, c], eb[r, c], int(bad.sum())))
    return worst


def planted_mistake_is_caught(side, jobs, policy, alpha, beta, C_gpu, C_orc):
    """Self-check of the comparison, on host copies only: one entry of the result replaced by its
    neighbour's value (a misplaced element) must fail compare_jobs.  The entry is the one of the
    first job whose neighbour differs from it by the largest multiple of its bound."""
    w = side.w
    nb = w.nb
    job = np.asarray(jobs).reshape(-1, 6)[0]
    I, J, r0, r1, c0, c1 = (int(x) for x in job)
    blk = (slice(I * nb + r0, I * nb + r1), slice(J * nb + c0, J * nb + c1))
    o = C_orc[blk]
    shifted = np.roll(o, 1, axis=1)
    eb, _ = element_bounds(side, job, policy, alpha, beta)
    score = np.abs(shifted - o) / np.maximum(eb, 1e-300)
    r, c = np.unravel_index(int(np.argmax(score)), o.shape)
    if score[r, c] <= 16.0:
        return False                                # a block of (nearly) equal entries: nothing to tell apart
    at = (I * nb + r0 + r, J * nb + c0 + c)
    keep = C_gpu[at]
    C_gpu[at] = C_gpu[I * nb + r0 + r, J * nb + c0 + (c - 1) % (c1 - c0)]      # spoiled in place, restored below
    try:
        compare_jobs(side, job, policy, alpha, beta, C_gpu, C_orc)
    except AssertionError:
        return True
    finally:
        C_gpu[at] = keep
    raise AssertionError("a misplaced element in tile (%d,%d) passed the comparison" % (I, J))


def packed_codes_expected(side, which, I, J):
    """Bit patterns the oracle assigns to one tile, in the packed layout (B tiles transposed)."""
    w = side.w
    nb = w.nb
    Y = {"A": side.Ay, "B": side.By, "C": side.Cy}[which]
    pmap = {"A": side.mapA, "B": side.mapB, "C": side.mapC}[which]
    tile = Y[I * nb:(I + 1) * nb, J * nb:(J + 1) * nb]
    if which == "B":
        tile = tile.T
    tile = np.ascontiguousarray(tile)
    p = int(pmap[I, J])
    if p == FP64:
        return tile.view(np.uint8).ravel()
    if p == FP32:
        return tile.astype(np.float32).view(np.uint8).ravel()
    if p == FP16:
        return orc.round_fp16(tile)[1].view(np.uint8).ravel()
    if p == BF16:
        return orc.round_bf16(tile)[1].view(np.uint8).ravel()
    return orc.round_fp8(tile)[1].ravel()
