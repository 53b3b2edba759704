"""Pins of the oracle's tile GEMM (paper Section 4, Algorithm 1) against things that do
not come from the oracle: exact rational fused multiply-adds, exact integer products,
the standard error bound, numpy's matmul, and invariance under the visit order.
"""
import itertools
from fractions import Fraction

import numpy as np
import pytest

from oracle import gemm_mp_oracle as orc
from tests.exact import fma32, fma64

FP64, FP32, FP16, FP8, BF16, MXFP8, MXFP4, MXFP6 = 0, 1, 2, 3, 4, 5, 6, 7
U = {FP64: 2.0 ** -53, FP32: 2.0 ** -24, FP16: 2.0 ** -11, FP8: 2.0 ** -4, BF16: 2.0 ** -8}


def _store(X, nb, pmap):
    return orc.store_tiles(np.ascontiguousarray(X), nb, pmap)


def _run(nb, A, mA, B, mB, C0, mC, alpha, beta, policy=orc.POLICY_OPERAND, jobs=None):
    Ay, eA = _store(A, nb, mA)
    By, eB = _store(B, nb, mB)
    Cy = None if C0 is None else _store(C0, nb, mC)[0]
    MT, NT = mC.shape
    if jobs is None:
        jobs = orc.whole_tile_jobs(nb, [(i, j) for i in range(MT) for j in range(NT)])
    return orc.gemm_jobs(nb, Ay, mA, eA, By, mB, eB, Cy, mC, alpha, beta, jobs, policy=policy)


def _maps(shape, value):
    return np.full(shape, value, dtype=np.uint16)


@pytest.mark.parametrize("nb", [2, 4, 8])
def test_all_fp64_map_equals_exact_fma_triple_loop_bit_for_bit(nb):
    rng = np.random.default_rng(10 + nb)
    M, N, K = 8, 8, 16
    A, B, C0 = rng.standard_normal((M, K)), rng.standard_normal((K, N)), rng.standard_normal((M, N))
    alpha, beta = 1.5, -0.25
    got = _run(nb, A, _maps((M // nb, K // nb), FP64), B, _maps((K // nb, N // nb), FP64),
               C0, _maps((M // nb, N // nb), FP64), alpha, beta)
    for i in range(M):
        for j in range(N):
            s = 0.0
            for k in range(K):
                s = fma64(A[i, k], B[k, j], s)
            assert got[i, j] == alpha * s + beta * C0[i, j]


@pytest.mark.parametrize("nb", [2, 4])
def test_all_fp32_map_equals_exact_fmaf_triple_loop_bit_for_bit(nb):
    rng = np.random.default_rng(20 + nb)
    M, N, K = 4, 8, 8
    A, B, C0 = rng.standard_normal((M, K)), rng.standard_normal((K, N)), rng.standard_normal((M, N))
    alpha, beta = 0.75, 2.0
    got = _run(nb, A, _maps((M // nb, K // nb), FP32), B, _maps((K // nb, N // nb), FP32),
               C0, _maps((M // nb, N // nb), FP32), alpha, beta)
    A32, B32, C32 = A.astype(np.float32), B.astype(np.float32), C0.astype(np.float32)
    a32, b32 = np.float32(alpha), np.float32(beta)
    for i in range(M):
        for j in range(N):
            s = np.float32(0)
            for k in range(K):
                s = fma32(A32[i, k], B32[k, j], s)
            want = np.float32(np.float32(a32 * s) + np.float32(b32 * C32[i, j]))
            assert got[i, j] == float(want)


@pytest.mark.parametrize("policy", [orc.POLICY_OPERAND, orc.POLICY_C_TILE])
def test_small_integer_inputs_give_the_exact_integer_product_for_every_map(policy):
    """Entries in {-3..3}: every storage format holds them exactly (with its tile scale) and
    all partial sums are small integers, so any index, transpose or scale mistake shows."""
    rng = np.random.default_rng(30)
    nb, MT, NT, KT = 8, 3, 4, 4
    M, N, K = MT * nb, NT * nb, KT * nb
    for trial in range(6):
        A = rng.integers(-3, 4, (M, K)).astype(np.float64)
        B = rng.integers(-3, 4, (K, N)).astype(np.float64)
        C0 = rng.integers(-5, 6, (M, N)).astype(np.float64)
        A[0:nb, 0:nb] = 0.0                                    # an all-zero tile (scale exponent 0)
        mA = rng.integers(0, 4, (MT, KT)).astype(np.uint16)
        mB = rng.integers(0, 4, (KT, NT)).astype(np.uint16)
        mC = rng.integers(0, 2, (MT, NT)).astype(np.uint16)
        got = _run(nb, A, mA, B, mB, C0, mC, 2.0, -3.0, policy=policy)
        want = 2 * (A.astype(np.int64) @ B.astype(np.int64)) - 3 * C0.astype(np.int64)
        assert np.array_equal(got, want.astype(np.float64))


def test_product_precision_table():
    """q = pC under the paper-literal reading; under the default reading the better-stored
    operand's precision, capped by what C keeps (FP64 C: no cap; FP32 C: FP32)."""
    rank = {FP64: 3, FP32: 2, FP16: 1, FP8: 0}
    by_rank = {v: k for k, v in rank.items()}
    for pA, pB, pC in itertools.product(range(4), range(4), range(2)):
        assert orc.product_precision(pA, pB, pC, orc.POLICY_C_TILE) == pC
        want = by_rank[min(rank[pC], max(rank[pA], rank[pB]))]
        assert orc.product_precision(pA, pB, pC, orc.POLICY_OPERAND) == want
    # the only FP64/FP32 case where the two readings differ
    assert orc.product_precision(FP32, FP32, FP64, orc.POLICY_OPERAND) == FP32
    assert orc.product_precision(FP32, FP32, FP64, orc.POLICY_C_TILE) == FP64


def test_product_counts_of_the_banded_tiny_map_and_of_iid_maps():
    import workloads as W
    w = W.tiny()
    counts = [0, 0, 0, 0]
    for I, J, L in itertools.product(range(4), range(4), range(4)):
        counts[orc.product_precision(w.mapA[I, L], w.mapB[L, J], w.mapC[I, J])] += 1
    assert counts == [28, 26, 10, 0]              # closed form for |I-L|, |L-J| bands, FP64 C
    w = W.random_maps()
    c = np.zeros(4)
    for I, J, L in itertools.product(range(w.MT), range(w.NT), range(w.KT)):
        c[orc.product_precision(w.mapA[I, L], w.mapB[L, J], w.mapC[I, J])] += 1
    frac = c / c.sum()
    # expectation: FP64 (7/16)/2, FP32 (7/16)/2 + 5/16, FP16 1/4
    assert abs(frac[0] - 0.21875) < 0.04 and abs(frac[1] - 0.53125) < 0.04 and abs(frac[2] - 0.25) < 0.04
    assert frac[3] == 0


def _mixed_problem(seed, nb=16, MT=3, NT=3, KT=4, with_fp8=True, pc_codes=(FP64, FP32)):
    rng = np.random.default_rng(seed)
    M, N, K = MT * nb, NT * nb, KT * nb
    A, B, C0 = rng.standard_normal((M, K)), rng.standard_normal((K, N)), rng.standard_normal((M, N))
    hi = 4 if with_fp8 else 3
    mA = rng.integers(0, hi, (MT, KT)).astype(np.uint16)
    mB = rng.integers(0, hi, (KT, NT)).astype(np.uint16)
    mC = rng.choice(pc_codes, (MT, NT)).astype(np.uint16)
    return nb, A, mA, B, mB, C0, mC


@pytest.mark.parametrize("policy", [orc.POLICY_OPERAND, orc.POLICY_C_TILE])
def test_error_stays_within_the_standard_bound_and_is_not_suspiciously_small(policy):
    """|C - exact(alpha*Ahat*Bhat + beta*Chat)| <= sum_L nb*u_q*|a||b| + (K+3)*u_T*(|a||b| + |c|)
    elementwise; and where a product ran below FP64 the error is not at FP64 level either."""
    nb, A, mA, B, mB, C0, mC = _mixed_problem(40)
    alpha, beta = 1.25, 0.5
    Ay, eA = _store(A, nb, mA)
    By, eB = _store(B, nb, mB)
    Cy, _ = _store(C0, nb, mC)
    Ah = Ay * np.kron(2.0 ** eA, np.ones((nb, nb)))
    Bh = By * np.kron(2.0 ** eB, np.ones((nb, nb)))
    MT, NT = mC.shape
    KT = mA.shape[1]
    jobs = orc.whole_tile_jobs(nb, [(i, j) for i in range(MT) for j in range(NT)])
    got = orc.gemm_jobs(nb, Ay, mA, eA, By, mB, eB, Cy, mC, alpha, beta, jobs, policy=policy)
    exact = alpha * (Ah.astype(np.longdouble) @ Bh.astype(np.longdouble)) + beta * Cy
    err = np.abs(got - exact).astype(np.float64)
    absprod = np.zeros_like(got)
    bound = np.zeros_like(got)
    lowq = np.zeros(mC.shape, dtype=bool)
    for I in range(MT):
        for J in range(NT):
            T = mC[I, J]
            blk = (slice(I * nb, (I + 1) * nb), slice(J * nb, (J + 1) * nb))
            for L in range(KT):
                q = orc.product_precision(mA[I, L], mB[L, J], mC[I, J], policy)
                lowq[I, J] |= q != FP64
                p = np.abs(Ah[I * nb:(I + 1) * nb, L * nb:(L + 1) * nb]) @ np.abs(Bh[L * nb:(L + 1) * nb, J * nb:(J + 1) * nb])
                # storage-to-q down-cast (FP64 -> FP32) adds 2u per product term
                bound[blk] += abs(alpha) * (nb + 2) * max(U[q], U[FP32] if q != FP64 else 0) * p
                absprod[blk] += p
            bound[blk] += (KT * nb + 3) * U[T] * (abs(alpha) * absprod[blk] + abs(beta) * np.abs(Cy[blk]))
    assert np.all(err <= bound)
    for I in range(MT):
        for J in range(NT):
            blk = (slice(I * nb, (I + 1) * nb), slice(J * nb, (J + 1) * nb))
            if lowq[I, J]:
                assert np.linalg.norm(err[blk]) > 2.0 ** -30 * np.linalg.norm(absprod[blk])


@pytest.mark.parametrize("p,dtype,tol", [(FP64, np.float64, 1e-14), (FP32, np.float32, 1e-5), (FP16, np.float16, 2e-3)])
def test_uniform_map_single_reduction_tile_matches_numpy_matmul_in_that_dtype(p, dtype, tol):
    rng = np.random.default_rng(50 + p)
    nb = 32
    A, B = rng.uniform(-1, 1, (nb, nb)), rng.uniform(-1, 1, (nb, nb))
    mC = _maps((1, 1), FP64 if p == FP64 else FP32)
    got = _run(nb, A, _maps((1, 1), p), B, _maps((1, 1), p), None, mC, 1.0, 0.0)
    with np.errstate(over="ignore"):
        want = (A.astype(dtype).astype(np.float32 if p == FP16 else dtype) @
                B.astype(dtype).astype(np.float32 if p == FP16 else dtype)).astype(np.float64)
    # FP16 tiles carry a power-of-two scale, so their stored values are at least as accurate
    # as an unscaled half cast; compare at the level of the half unit roundoff.
    assert np.linalg.norm(got - want) <= tol * np.linalg.norm(np.abs(A) @ np.abs(B))


def test_visit_order_listing_loop_nest_equals_tile_owner_loop_nest_bit_for_bit():
    """Algorithm 1 prints the reduction tile index outermost; the oracle's default walks one C
    tile at a time.  With the per-tile reduction order kept ascending both give the same bits,
    for every map, as does any permutation or splitting of the jobs."""
    for seed in (60, 61):
        nb, A, mA, B, mB, C0, mC = _mixed_problem(seed)
        alpha, beta = -0.5, 1.5
        Ay, eA = _store(A, nb, mA)
        By, eB = _store(B, nb, mB)
        Cy, _ = _store(C0, nb, mC)
        MT, NT = mC.shape
        KT = mA.shape[1]
        tiles = [(i, j) for i in range(MT) for j in range(NT)]
        jobs = orc.whole_tile_jobs(nb, tiles)
        ref = orc.gemm_jobs(nb, Ay, mA, eA, By, mB, eB, Cy, mC, alpha, beta, jobs)
        # (a) listing order: for l, for i, for j, each task one call that carries the running sums
        state = {t: np.zeros(nb * nb) for t in tiles}
        out = np.full_like(ref, np.nan)
        for L in range(KT):
            for (i, j) in tiles:
                orc.gemm_jobs(nb, Ay, mA, eA, By, mB, eB, Cy, mC, alpha, beta,
                              orc.whole_tile_jobs(nb, [(i, j)]), out=out, L_range=(L, L + 1),
                              state=state[(i, j)], resume=L > 0, finish=L == KT - 1)
        assert np.array_equal(out, ref)
        # (b) permuted jobs, and tiles cut into ragged sub-rectangles
        rng = np.random.default_rng(seed)
        perm = rng.permutation(len(tiles))
        out = orc.gemm_jobs(nb, Ay, mA, eA, By, mB, eB, Cy, mC, alpha, beta, jobs[perm])
        assert np.array_equal(out, ref)
        pieces = []
        for (i, j) in tiles:
            r, c = int(rng.integers(1, nb)), int(rng.integers(1, nb))
            pieces += [[i, j, 0, r, 0, c], [i, j, r, nb, 0, c], [i, j, 0, r, c, nb], [i, j, r, nb, c, nb]]
        out = orc.gemm_jobs(nb, Ay, mA, eA, By, mB, eB, Cy, mC, alpha, beta, np.array(pieces, dtype=np.int32))
        assert np.array_equal(out, ref)


def test_beta_zero_never_reads_c_and_alpha_zero_skips_products():
    nb, A, mA, B, mB, C0, mC = _mixed_problem(70)
    poisoned = np.full_like(C0, np.nan)
    Ay, eA = _store(A, nb, mA)
    By, eB = _store(B, nb, mB)
    MT, NT = mC.shape
    jobs = orc.whole_tile_jobs(nb, [(i, j) for i in range(MT) for j in range(NT)])
    got = orc.gemm_jobs(nb, Ay, mA, eA, By, mB, eB, poisoned, mC, 1.0, 0.0, jobs)
    assert np.all(np.isfinite(got))
    Cy, _ = _store(C0, nb, mC)
    Ay[0, 0] = np.inf                       # would poison every product of row 0 if it were formed
    got = orc.gemm_jobs(nb, Ay, mA, eA, By, mB, eB, Cy, mC, 0.0, 0.5, jobs)
    want = np.empty_like(Cy)
    for I in range(MT):
        for J in range(NT):
            blk = (slice(I * nb, (I + 1) * nb), slice(J * nb, (J + 1) * nb))
            if mC[I, J] == FP64:
                want[blk] = 0.5 * Cy[blk]
            else:
                want[blk] = (np.float32(0.5) * Cy[blk].astype(np.float32)).astype(np.float64)
    assert np.array_equal(got, want)


def test_low_precision_products_are_scaled_back_by_the_tile_exponents():
    """FP16 x FP16 product of tiles holding tiny and huge numbers: without the per-tile
    exponents the stored tiles would flush to zero / overflow."""
    rng = np.random.default_rng(80)
    nb = 16
    A = rng.standard_normal((nb, nb)) * 1e-9
    B = rng.standard_normal((nb, nb)) * 1e7
    m16 = _maps((1, 1), FP16)
    for pC in (FP64, FP32):
        got = _run(nb, A, m16, B, m16, None, _maps((1, 1), pC), 1.0, 0.0)
        ref = A @ B
        assert np.linalg.norm(got - ref) <= 4 * 2.0 ** -11 * np.linalg.norm(np.abs(A) @ np.abs(B))
        assert np.linalg.norm(got) > 0.5 * np.linalg.norm(ref)


def test_stored_tiles_match_library_casts_and_scale_window():
    rng = np.random.default_rng(90)
    nb = 8
    X = rng.standard_normal((2 * nb, 4 * nb)) * np.kron(10.0 ** rng.integers(-12, 6, (2, 4)), np.ones((nb, nb)))
    X[0:nb, 0:nb] = 0.0
    pmap = np.array([[FP16, FP64, FP32, FP16], [FP8, FP16, FP8, FP32]], dtype=np.uint16)
    pmap[0, 0] = FP16
    Y, e = orc.store_tiles(X, nb, pmap)
    for I in range(2):
        for J in range(4):
            blk = (slice(I * nb, (I + 1) * nb), slice(J * nb, (J + 1) * nb))
            p = pmap[I, J]
            if p == FP64:
                assert e[I, J] == 0 and np.array_equal(Y[blk], X[blk])
            elif p == FP32:
                assert e[I, J] == 0 and np.array_equal(Y[blk], X[blk].astype(np.float32).astype(np.float64))
            else:
                m = np.abs(X[blk]).max()
                if m == 0:
                    assert e[I, J] == 0 and not Y[blk].any()
                    continue
                top = 15 if p == FP16 else 8
                assert 2.0 ** (top - 1) <= m * 2.0 ** -float(e[I, J]) < 2.0 ** top
                scaled = X[blk] * 2.0 ** -float(e[I, J])
                if p == FP16:
                    assert np.array_equal(Y[blk], scaled.astype(np.float16).astype(np.float64))
                else:
                    torch = pytest.importorskip("torch")
                    # scaled magnitudes stay below 256, far from e4m3's saturation; torch may go
                    # through FP32, which for these seeded values lands on no e4m3 midpoint
                    t = torch.from_numpy(scaled).to(torch.float8_e4m3fn).to(torch.float64).numpy()
                    assert np.array_equal(Y[blk], t)


def test_a_ragged_problem_is_its_zero_padded_extension():
    """Sizes that are no multiples of the tile size: the oracle works on the zero-padded
    matrices.  Pinned against what does not depend on tiling at all: the exact integer product of
    the unpadded matrices, numpy's sums of squares and maxima of the partial tiles, and zeros
    (exactly) in the padding of C."""
    rng = np.random.default_rng(17)
    nb, M, N, K = 8, 19, 13, 21
    A = rng.integers(-3, 4, (M, K)).astype(np.float64)
    B = rng.integers(-3, 4, (K, N)).astype(np.float64)
    C0 = rng.integers(-5, 6, (M, N)).astype(np.float64)
    Ap, Bp, Cp = orc.pad_to_tiles(A, nb), orc.pad_to_tiles(B, nb), orc.pad_to_tiles(C0, nb)
    assert Ap.shape == (24, 24) and Bp.shape == (24, 16) and Cp.shape == (24, 16)
    assert np.array_equal(Ap[:M, :K], A) and not Ap[M:].any() and not Ap[:, K:].any()
    MT, NT, KT = 3, 2, 3
    mA = rng.integers(0, 4, (MT, KT)).astype(np.uint16)
    mB = rng.integers(0, 4, (KT, NT)).astype(np.uint16)
    mC = rng.integers(0, 2, (MT, NT)).astype(np.uint16)
    for policy in (orc.POLICY_OPERAND, orc.POLICY_C_TILE):
        C = _run(nb, Ap, mA, Bp, mB, Cp, mC, 2.0, -3.0, policy=policy)
        want = 2 * (A.astype(np.int64) @ B.astype(np.int64)) - 3 * C0.astype(np.int64)
        assert np.array_equal(C[:M, :N], want.astype(np.float64))
        assert not C[M:].any() and not C[:, N:].any()
    X = rng.standard_normal((M, K))
    s, m = orc.tile_scan(orc.pad_to_tiles(X, nb), nb)
    for I in range(MT):
        for L in range(KT):
            t = X[I * nb:(I + 1) * nb, L * nb:(L + 1) * nb]
            assert m[I, L] == np.abs(t).max()
            assert abs(s[I, L] - np.sum(t * t)) <= 1e-14 * np.sum(t * t)


@pytest.mark.parametrize("policy", [orc.POLICY_OPERAND, orc.POLICY_C_TILE])
def test_c_tiles_stored_in_fp16_or_fp8_hold_small_integer_results_exactly(policy):
    """C tiles in FP16 / FP8 (a reading, the paper's tiles are FP64 / FP32): accumulated as an
    FP32 tile, then stored with the tile's own scale.  With the largest entry of a tile scaled
    into [2^14,2^15) an FP16 tile holds every integer up to 2047 and an FP8 tile (largest entry
    in [2^7,2^8), four significant bits) every integer up to 15 exactly, so on such results the
    whole path, old C tile included, must return the exact integer matrix; and before the
    storage step a job's result must not depend on whether the tile is FP32, FP16 or FP8."""
    rng = np.random.default_rng(77)
    nb, MT, NT, KT = 8, 3, 3, 2
    M, N, K = MT * nb, NT * nb, KT * nb
    for trial in range(6):
        A = np.zeros((M, K))
        B = np.zeros((K, N))
        # one nonzero per row of A and per column of B inside each reduction tile keeps |C| small
        for r in range(M):
            for L in range(KT):
                A[r, L * nb + rng.integers(nb)] = rng.integers(-2, 3)
        for c in range(N):
            for L in range(KT):
                B[L * nb + rng.integers(nb), c] = rng.integers(-1, 2)
        C0 = rng.integers(-3, 4, (M, N)).astype(np.float64)
        mA = rng.integers(0, 4, (MT, KT)).astype(np.uint16)
        mB = rng.integers(0, 4, (KT, NT)).astype(np.uint16)
        mC = rng.integers(0, 4, (MT, NT)).astype(np.uint16)
        mC[0, 0], mC[1, 1] = FP16, FP8
        want = (A.astype(np.int64) @ B.astype(np.int64)) + 2 * C0.astype(np.int64)
        assert np.abs(want).max() <= 15
        Ay, eA = _store(A, nb, mA)
        By, eB = _store(B, nb, mB)
        Cy, eC = _store(C0, nb, mC)
        Cv = orc.stored_values(Cy, nb, eC)
        assert np.array_equal(Cv, C0)
        jobs = orc.whole_tile_jobs(nb, [(i, j) for i in range(MT) for j in range(NT)])
        pre = orc.gemm_jobs(nb, Ay, mA, eA, By, mB, eB, Cv, mC, 1.0, 2.0, jobs, policy=policy)
        as32 = np.where(mC >= FP16, FP32, mC).astype(np.uint16)
        assert np.array_equal(pre, orc.gemm_jobs(nb, Ay, mA, eA, By, mB, eB, Cv, as32, 1.0, 2.0, jobs, policy=policy))
        Y, e = _store(pre, nb, mC)
        got = orc.stored_values(Y, nb, e)
        assert np.array_equal(got, want.astype(np.float64))
        # the stored numbers lie in the scale window of their format
        for I in range(MT):
            for J in range(NT):
                m = np.abs(Y[I * nb:(I + 1) * nb, J * nb:(J + 1) * nb]).max()
                if mC[I, J] == FP16 and m:
                    assert 2.0 ** 14 <= m < 2.0 ** 15
                if mC[I, J] == FP8 and m:
                    assert 2.0 ** 7 <= m < 2.0 ** 8


def test_c_tiles_stored_in_fp16_or_fp8_round_once_within_their_unit_roundoff():
    """General data: the stored tile differs from the FP32 form of the same job by at most
    u_p relative per entry in the normal range (FP16 2^-11, FP8 2^-4), and the FP32 form is that
    of an FP32 tile, which the pins above tie to exact arithmetic."""
    rng = np.random.default_rng(78)
    nb, MT, NT, KT = 8, 2, 2, 3
    A = rng.standard_normal((MT * nb, KT * nb))
    B = rng.standard_normal((KT * nb, NT * nb))
    mA = rng.integers(0, 4, (MT, KT)).astype(np.uint16)
    mB = rng.integers(0, 4, (KT, NT)).astype(np.uint16)
    mC = np.array([[FP16, FP8], [FP8, FP16]], dtype=np.uint16)
    pre = _run(nb, A, mA, B, mB, None, mC, 1.5, 0.0)
    assert np.array_equal(pre, pre.astype(np.float32).astype(np.float64))        # FP32 numbers
    Y, e = _store(pre, nb, mC)
    got = orc.stored_values(Y, nb, e)
    for I in range(MT):
        for J in range(NT):
            blk = (slice(I * nb, (I + 1) * nb), slice(J * nb, (J + 1) * nb))
            p = int(mC[I, J])
            big = np.abs(pre[blk]) >= np.abs(pre[blk]).max() * 2.0 ** -8      # well inside the normal range
            rel = np.abs(got[blk] - pre[blk])[big] / np.abs(pre[blk])[big]
            assert rel.max() <= U[p]
            assert rel.max() > U[p] / 16                                       # and it did round


def test_c_tiles_stored_in_block_scaled_formats_are_fp32_tiles_quantised_along_their_rows():
    """A block-scaled C tile is an FP32 tile until it is stored: the job returns bit for bit what
    the same job returns for an FP32 tile, and storing it quantises each block of 32 along a row
    by that block's own maximum: element error at most half a step of the block's top binade
    (2^-4 / 2^-2 / 2^-4 of the block maximum's power of two for e4m3 / e2m1 / e2m3), except above the
    element format's largest number (1.75 / 1.5 / 1.875 times that power of two), where it saturates."""
    rng = np.random.default_rng(79)
    nb, MT, NT, KT = 32, 2, 2, 2
    A = rng.standard_normal((MT * nb, KT * nb))
    B = rng.standard_normal((KT * nb, NT * nb))
    mA = rng.integers(0, 4, (MT, KT)).astype(np.uint16)
    mB = rng.integers(0, 4, (KT, NT)).astype(np.uint16)
    mC = np.array([[MXFP8, MXFP4], [MXFP6, MXFP8]], dtype=np.uint16)
    pre = _run(nb, A, mA, B, mB, None, mC, 1.5, 0.0)
    assert np.array_equal(pre, _run(nb, A, mA, B, mB, None, np.full((MT, NT), FP32, dtype=np.uint16), 1.5, 0.0))
    Y, e = _store(pre, nb, mC)
    assert not e.any()
    got = orc.stored_values(Y, nb, e)
    seen_beyond = False
    for I in range(MT):
        for J in range(NT):
            half_step, largest = {MXFP8: (2.0 ** -4, 1.75), MXFP4: (2.0 ** -2, 1.5), MXFP6: (2.0 ** -4, 1.875)}[int(mC[I, J])]
            for r in range(nb):
                row = pre[I * nb + r, J * nb:(J + 1) * nb]             # one block: nb = 32
                top = 2.0 ** np.floor(np.log2(np.abs(row).max()))
                out = got[I * nb + r, J * nb:(J + 1) * nb]
                beyond = np.abs(row) > largest * top                   # above the format's largest number: saturates
                assert np.array_equal(out[beyond], np.sign(row[beyond]) * largest * top)
                assert np.abs(out - row)[~beyond].max() <= half_step * top
                assert out[np.abs(row).argmax()] != 0.0
                seen_beyond |= bool(beyond.any())
    assert seen_beyond


def test_product_precision_with_bf16_is_the_smallest_format_holding_both_operands():
    """BF16 and FP16 hold different numbers, so the formats form a lattice, written out here as
    sets of (fraction bits, least exponent, greatest exponent) of what each can hold once a tile
    scale is allowed for FP16 / FP8: a format holds another's numbers if it has at least its
    fraction bits and, unless one of them is scaled per tile, its exponent range."""
    frac = {FP64: 52, FP32: 23, FP16: 10, BF16: 7, FP8: 3}
    wide = {FP64: 3, FP32: 2, BF16: 2, FP16: 1, FP8: 0}              # exponent range classes
    def holds(big, small):
        if frac[big] < frac[small]:
            return False
        return wide[big] >= wide[small] or small == FP8             # an FP8 tile keeps its scale under FP16 / BF16
    fmts = [FP64, FP32, FP16, BF16, FP8]
    for pA, pB in itertools.product(fmts, fmts):
        cands = [f for f in fmts if holds(f, pA) and holds(f, pB)]
        want = max(cands, key=lambda f: -frac[f])                    # the one with the fewest fraction bits
        assert orc.product_precision(pA, pB, FP64, orc.POLICY_OPERAND) == want, (pA, pB)
        capped = FP32 if want == FP64 else want
        for pC in (FP32, FP16, FP8, BF16):
            assert orc.product_precision(pA, pB, pC, orc.POLICY_OPERAND) == capped
            assert orc.product_precision(pA, pB, pC, orc.POLICY_C_TILE) == FP32
    assert orc.product_precision(FP16, BF16, FP64) == FP32 and orc.product_precision(BF16, FP8, FP32) == BF16


def test_bf16_tiles_small_integers_are_exact_and_general_data_within_bound():
    """Integers up to 255 fit BF16 exactly, so a problem of small integers with BF16 tiles
    anywhere (C included: stored BF16 after FP32 accumulation) must give the exact product; on
    general data an all-BF16 product agrees with an FP64 product of the BF16-rounded operands
    (rounded with torch's cast) to FP32 accumulation accuracy."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(41)
    nb, MT, NT, KT = 8, 3, 3, 3
    M, N, K = MT * nb, NT * nb, KT * nb
    for trial in range(6):
        A = rng.integers(-3, 4, (M, K)).astype(np.float64)
        B = rng.integers(-3, 4, (K, N)).astype(np.float64)
        C0 = rng.integers(-5, 6, (M, N)).astype(np.float64)
        mA = rng.integers(0, 5, (MT, KT)).astype(np.uint16)
        mB = rng.integers(0, 5, (KT, NT)).astype(np.uint16)
        mC = rng.choice([FP64, FP32, BF16], (MT, NT)).astype(np.uint16)
        mA[0, 0], mB[0, 0], mC[0, 0] = BF16, BF16, BF16
        pre = _run(nb, A, mA, B, mB, C0, mC, 1.0, 1.0)
        Y, e = _store(pre, nb, mC)
        got = orc.stored_values(Y, nb, e)
        want = (A.astype(np.int64) @ B.astype(np.int64)) + C0.astype(np.int64)
        assert np.abs(want).max() < 256
        assert np.array_equal(got, want.astype(np.float64))
        assert not e.any()                                           # no BF16 / FP32 / FP64 tile has a scale
    A = rng.standard_normal((M, K)) * np.exp(rng.uniform(-20, 20, (M, K)))
    B = rng.standard_normal((K, N))
    full = lambda shape: np.full(shape, BF16, dtype=np.uint16)
    got = _run(nb, A, full((MT, KT)), B, full((KT, NT)), None, np.full((MT, NT), FP64, dtype=np.uint16), 1.0, 0.0)
    cast = lambda X: torch.from_numpy(X.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    Ab, Bb = cast(A), cast(B)                       # FP32 first is harmless here only if no tie changes: compare loosely
    ref = Ab @ Bb
    bound = 2 * K * 2.0 ** -24 * (np.abs(Ab) @ np.abs(Bb)) + 2.0 ** -8 * 1e-3 * (np.abs(Ab) @ np.abs(Bb))
    assert np.all(np.abs(got - ref) <= bound)
    assert np.abs(got - A @ B).max() > 0                              # and it did round the operands


def test_mxfp8_tiles_follow_the_reduction_index_and_give_exact_integer_products():
    """MXFP8 tiles: the blocks of 32 run along the reduction index (rows of A, columns of B), so
    storing B with blocks down its columns equals storing its transpose with blocks along rows;
    MXFP8 with MXFP8 is an MXFP8 product, with anything else FP32 (FP64 if the other is FP64 and C
    allows); small integers come through exactly whatever the maps."""
    rng = np.random.default_rng(43)
    nb, MT, NT, KT = 32, 2, 2, 3
    M, N, K = MT * nb, NT * nb, KT * nb
    X = rng.standard_normal((K, N)) * np.exp(rng.uniform(-5, 5, (K, N)))
    mx = np.full((KT, NT), MXFP8, dtype=np.uint16)
    Yb, eb = orc.store_tiles(X, nb, mx, mx_axis=1)
    Yt, et = orc.store_tiles(np.ascontiguousarray(X.T), nb, np.ascontiguousarray(mx.T), mx_axis=0)
    assert np.array_equal(Yb, Yt.T) and not eb.any()
    Ya, _ = orc.store_tiles(X, nb, mx, mx_axis=0)
    assert not np.array_equal(Ya, Yb)                     # the orientation matters
    rel = np.abs(Yb - X) / np.abs(X)
    assert rel[np.abs(X) > np.abs(X).max() * 2.0 ** -60].max() <= 1.0 and np.median(rel) < 2.0 ** -4
    for pA, pB, pC, want in ((MXFP8, MXFP8, FP32, MXFP8), (MXFP8, MXFP8, FP64, MXFP8), (MXFP8, FP8, FP32, FP32), (MXFP8, FP16, FP64, FP32),
                             (FP64, MXFP8, FP64, FP64), (FP64, MXFP8, FP32, FP32), (BF16, MXFP8, FP32, FP32),
                             (MXFP4, MXFP4, FP32, MXFP4), (MXFP4, MXFP8, FP32, FP32), (MXFP4, FP64, FP64, FP64), (FP8, MXFP4, FP64, FP32),
                             (MXFP6, MXFP6, FP32, MXFP6), (MXFP6, MXFP6, FP64, MXFP6), (MXFP6, MXFP4, FP32, FP32), (MXFP8, MXFP6, FP64, FP32),
                             (MXFP6, FP64, FP64, FP64), (MXFP6, FP64, FP32, FP32), (FP16, MXFP6, FP64, FP32)):
        assert orc.product_precision(pA, pB, pC, orc.POLICY_OPERAND) == want
    for trial in range(5):
        A = rng.integers(-3, 4, (M, K)).astype(np.float64)
        B = rng.integers(-3, 4, (K, N)).astype(np.float64)
        C0 = rng.integers(-5, 6, (M, N)).astype(np.float64)
        mA = rng.choice([FP64, FP32, FP16, FP8, BF16, MXFP8, MXFP4, MXFP6], (MT, KT)).astype(np.uint16)
        mB = rng.choice([FP64, FP32, FP16, FP8, BF16, MXFP8, MXFP4, MXFP6], (KT, NT)).astype(np.uint16)
        if trial == 0:
            mA[:], mB[:] = MXFP8, MXFP8
        if trial == 1:
            mA[:], mB[:] = MXFP4, MXFP4
        if trial == 2:
            mA[:], mB[:] = MXFP6, MXFP6
        mC = rng.integers(0, 2, (MT, NT)).astype(np.uint16)
        Ay, eA = orc.store_tiles(A, nb, mA, mx_axis=0)
        By, eB = orc.store_tiles(B, nb, mB, mx_axis=1)
        Cy, _ = orc.store_tiles(C0, nb, mC)
        jobs = orc.whole_tile_jobs(nb, [(i, j) for i in range(MT) for j in range(NT)])
        got = orc.gemm_jobs(nb, Ay, mA, eA, By, mB, eB, Cy, mC, 2.0, -1.0, jobs)
        want = 2 * (A.astype(np.int64) @ B.astype(np.int64)) - C0.astype(np.int64)
        assert np.array_equal(got, want.astype(np.float64))
