"""Pins of three parts of the oracle that a looser test cannot see: the one lossy receiver-side
conversion (FP64 operands under an FP32 product, Section 4), the FP32 side accumulator and its
fold into an FP64 C tile (with and without tile scales), alpha and beta that FP32 cannot hold,
and BF16's place in the norm rule.  Every expected value comes from exact rational arithmetic
(tests/exact.py), numpy's casts or a formula written out here; nothing comes from oracle/.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import gemm_mp_oracle as orc
from tests.exact import fma32

FP64, FP32, FP16, FP8, BF16 = 0, 1, 2, 3, 4


def _maps(shape, value):
    return np.full(shape, value, dtype=np.uint16)


def _run(nb, A, mA, B, mB, C0, mC, alpha, beta, policy=orc.POLICY_OPERAND):
    Ay, eA = orc.store_tiles(np.ascontiguousarray(A), nb, mA)
    By, eB = orc.store_tiles(np.ascontiguousarray(B), nb, mB)
    Cy = None if C0 is None else orc.store_tiles(np.ascontiguousarray(C0), nb, mC)[0]
    MT, NT = mC.shape
    jobs = orc.whole_tile_jobs(nb, [(i, j) for i in range(MT) for j in range(NT)])
    return orc.gemm_jobs(nb, Ay, mA, eA, By, mB, eB, Cy, mC, alpha, beta, jobs, policy=policy)


def _around_fp32_midpoints(rng, shape):
    """FP64 numbers that sit on the midpoint of two neighbouring FP32 numbers, or one FP64 unit
    in the last place to either side of it: round-to-nearest-even, truncation and rounding away
    from zero all give different FP32 numbers on a third of them."""
    x = rng.standard_normal(shape).astype(np.float32)
    up = np.nextafter(x, np.float32(np.inf))
    mid = (x.astype(np.float64) + up.astype(np.float64)) / 2          # exact in FP64
    pick = rng.integers(0, 3, shape)
    out = np.where(pick == 0, mid, np.where(pick == 1, np.nextafter(mid, np.inf), np.nextafter(mid, -np.inf)))
    assert np.all((out > x) & (out < up))
    return out


@pytest.mark.parametrize("nb", [2, 4])
@pytest.mark.parametrize("policy", [orc.POLICY_OPERAND, orc.POLICY_C_TILE])
def test_fp64_operands_under_an_fp32_product_are_rounded_to_nearest_even(nb, policy):
    """A and B stored FP64, C tiles FP32: every product is an FP32 product (either policy) whose
    operands are down-cast on the receiving side.  Expected: numpy's FP64 -> FP32 cast (round to
    nearest even), then one FP32 chain of exact fused multiply-adds over the whole reduction."""
    rng = np.random.default_rng(100 + nb)
    M, N, K = 4, 4, 8
    A, B = _around_fp32_midpoints(rng, (M, K)), _around_fp32_midpoints(rng, (K, N))
    C0 = rng.standard_normal((M, N))
    alpha, beta = 0.1, -1.0 / 3.0
    got = _run(nb, A, _maps((M // nb, K // nb), FP64), B, _maps((K // nb, N // nb), FP64),
               C0, _maps((M // nb, N // nb), FP32), alpha, beta, policy=policy)
    A32, B32, C32 = A.astype(np.float32), B.astype(np.float32), C0.astype(np.float32)
    # the cast is not a truncation on these inputs
    assert np.any(A32.astype(np.float64) > A) and np.any(A32.astype(np.float64) < A)
    a32, b32 = np.float32(alpha), np.float32(beta)
    for i in range(M):
        for j in range(N):
            s = np.float32(0)
            for k in range(K):
                s = fma32(A32[i, k], B32[k, j], s)
            want = np.float32(np.float32(a32 * s) + np.float32(b32 * C32[i, j]))
            assert got[i, j] == float(want), (i, j)


def test_fp64_operand_beside_an_fp32_one_under_an_fp32_product():
    """The same with only A stored FP64 (B is FP32 already): one side is down-cast, the other is
    taken as it is."""
    rng = np.random.default_rng(105)
    nb, M, N, K = 2, 4, 4, 4
    A, B = _around_fp32_midpoints(rng, (M, K)), _around_fp32_midpoints(rng, (K, N))
    got = _run(nb, A, _maps((2, 2), FP64), B, _maps((2, 2), FP32), None, _maps((2, 2), FP32), 1.0, 0.0)
    A32, B32 = A.astype(np.float32), B.astype(np.float32)
    for i in range(M):
        for j in range(N):
            s = np.float32(0)
            for k in range(K):
                s = fma32(A32[i, k], B32[k, j], s)
            assert got[i, j] == float(s)


@pytest.mark.parametrize("nb", [2, 4])
def test_alpha_and_beta_are_rounded_to_the_accumulate_type_before_use(nb):
    """alpha = 0.1, beta = -1/3 are no FP32 numbers: on an FP32 tile they are rounded to FP32
    first and the epilogue is two rounded FP32 products and one rounded FP32 sum."""
    rng = np.random.default_rng(110 + nb)
    M, N, K = 4, 4, 8
    A, B, C0 = rng.standard_normal((M, K)), rng.standard_normal((K, N)), rng.standard_normal((M, N))
    for alpha, beta in ((0.1, -1.0 / 3.0), (1e-3, 0.7), (-2.0 / 3.0, 0.0)):
        got = _run(nb, A, _maps((M // nb, K // nb), FP32), B, _maps((K // nb, N // nb), FP32),
                   C0, _maps((M // nb, N // nb), FP32), alpha, beta)
        A32, B32, C32 = A.astype(np.float32), B.astype(np.float32), C0.astype(np.float32)
        a32, b32 = np.float32(alpha), np.float32(beta)
        assert float(a32) != alpha
        differs = False
        for i in range(M):
            for j in range(N):
                s = np.float32(0)
                for k in range(K):
                    s = fma32(A32[i, k], B32[k, j], s)
                want = np.float32(a32 * s)
                if beta != 0.0:
                    want = np.float32(want + np.float32(b32 * C32[i, j]))
                assert got[i, j] == float(want)
                # what "alpha times s in double, rounded once" would give
                other = alpha * float(s) + (beta * float(C32[i, j]) if beta != 0.0 else 0.0)
                differs |= float(np.float32(other)) != float(want)
        assert differs                                  # the inputs tell the two readings apart


def _tile_exponent(T, top):
    m = np.abs(T).max()
    return 0 if m == 0 else int(np.floor(np.log2(m))) - top


@pytest.mark.parametrize("pa,pb", [(FP32, FP32), (FP16, FP16), (FP32, FP16)])
def test_products_below_fp64_of_an_fp64_tile_go_through_an_fp32_accumulator_and_one_fold(pa, pb):
    """C tile FP64, operands stored below FP64: each tile product is an FP32 chain started from
    zero (FP16 x FP16 on the scaled numbers, whose products are exact in FP32), and the finished
    product joins the FP64 running sum with one FP64 addition, times 2^(eA+eB) where the operands
    stayed scaled.  Expected values by exact rational fused multiply-adds and numpy's casts."""
    rng = np.random.default_rng(120 + pa * 8 + pb)
    nb, KT = 4, 3
    M = N = nb
    K = KT * nb
    A = rng.standard_normal((M, K)) * 2.0 ** rng.integers(-20, 20)
    B = rng.standard_normal((K, N)) * 2.0 ** rng.integers(-20, 20)
    got = _run(nb, A, _maps((1, KT), pa), B, _maps((KT, 1), pb), None, _maps((1, 1), FP64), 1.0, 0.0)
    q = FP16 if (pa == FP16 and pb == FP16) else FP32

    def stored(T, p):
        if p == FP32:
            return T.astype(np.float32), 0
        e = _tile_exponent(T, 14)
        return (T * 2.0 ** -e).astype(np.float16).astype(np.float32), e     # numpy rounds FP64 -> FP16 once

    for i in range(M):
        for j in range(N):
            s = 0.0
            for L in range(KT):
                a, ea = stored(A[:, L * nb:(L + 1) * nb], pa)
                b, eb = stored(B[L * nb:(L + 1) * nb, :], pb)
                if q == FP32:                           # operands take their scale on conversion (exact)
                    a, b, esum = np.ldexp(a, ea).astype(np.float32), np.ldexp(b, eb).astype(np.float32), 0
                else:
                    esum = ea + eb
                t = np.float32(0)
                for k in range(nb):
                    t = fma32(a[i, k], b[k, j], t)
                s = s + float(np.ldexp(np.float64(t), esum))
            assert got[i, j] == s, (i, j)
    # and that is not what one FP64 chain over the same stored numbers gives
    ref = sum(Fraction(float(x)) * Fraction(float(y)) for x, y in zip(A[0].astype(np.float32), B[:, 0].astype(np.float32)))
    assert pa != FP32 or pb != FP32 or got[0, 0] != float(ref)


# ---- BF16 in the norm rule ---------------------------------------------------------------------

U = {FP64: 2.0 ** -53, FP32: 2.0 ** -24, FP16: 2.0 ** -11, BF16: 2.0 ** -8, FP8: 2.0 ** -4}


def _rule_by_formula(sumsq, eps, allowed):
    """The rule as a formula: the allowed format with the largest unit roundoff u such that
    |T| sqrt(n) / |X| <= eps / u, else the allowed one with the smallest u.  Square roots and
    numpy norms here, squares in a fixed order there: the callers keep clear of the thresholds."""
    n = sumsq.size
    normX = np.sqrt(sumsq.sum())
    out = np.empty(sumsq.shape, dtype=np.uint16)
    fmts = sorted((p for p in U if allowed >> p & 1), key=lambda p: -U[p])
    for idx, st in np.ndenumerate(sumsq):
        ratio = np.sqrt(st) * np.sqrt(n) / normX
        out[idx] = next((p for p in fmts if ratio <= eps / U[p]), fmts[-1])
    return out


def test_rule_places_bf16_between_fp8_and_fp16_at_unit_roundoff_two_to_the_minus_eight():
    n, eps = 16, 1e-3
    s = np.ones(n)
    # ratio^2 of tile 0 is 16 s0 / (15 + s0); limits (eps/u)^2: FP8 2.56e-4, BF16 0.065536, FP16 4.194
    limit = lambda u: (eps / u) ** 2
    ratio2 = lambda s0: 16 * s0 / (15 + s0)
    assert limit(2.0 ** -4) < ratio2(0.055) < limit(2.0 ** -8) < ratio2(0.07) < limit(2.0 ** -11)
    s[0] = 0.055                                    # just below the BF16 limit
    got = orc.precision_rule(s, eps, 0x1F)
    assert got[0] == BF16 and np.all(got[1:] == FP16)
    s[0] = 0.07                                     # just above it
    assert orc.precision_rule(s, eps, 0x1F)[0] == FP16
    s[0] = 0.0002                                   # below the FP8 limit (ratio^2 = 2.13e-4)
    assert ratio2(0.0002) < limit(2.0 ** -4)
    assert orc.precision_rule(s, eps, 0x1F)[0] == FP8
    # a unit roundoff of 2^-7 would put the limit at 0.0164 and send 0.055 to FP16
    assert ratio2(0.055) > (eps * 2.0 ** 7) ** 2
    # BF16 not allowed: a tile between the FP8 and the FP16 limit is an FP16 tile
    s[0] = 0.055
    assert orc.precision_rule(s, eps, 0x0F)[0] == FP16
    # FP16 not allowed: the tiles above the BF16 limit go up to FP32, those below stay BF16
    got = orc.precision_rule(s, eps, 0x1B)
    assert got[0] == BF16 and np.all(got[1:] == FP32)


def test_rule_ranks_by_unit_roundoff_not_by_code():
    rng = np.random.default_rng(7)
    s = rng.uniform(0.5, 2.0, (3, 5))
    s[2, 1] = 0.0
    # (mask, highest = smallest u, lowest = largest u)
    for mask, hi, lo in ((0b10100, FP16, BF16), (0b11000, BF16, FP8), (0b10001, FP64, BF16), (0b10010, FP32, BF16),
                         (0b11111, FP64, FP8), (0b10000, BF16, BF16)):
        m = orc.precision_rule(s, 0.0, mask)
        assert m[2, 1] == lo                        # a zero tile passes every test
        m[2, 1] = hi
        assert np.all(m == hi)                      # eps = 0: nothing else passes anything
        assert np.all(orc.precision_rule(s, 1e30, mask) == lo)


@pytest.mark.parametrize("step,eps", [(2.0, 1e-3), (4.0, 1e-3), (1.5, 2e-4)])
def test_rule_on_geometrically_decaying_tiles_equals_the_formula_with_all_five_formats(step, eps):
    """Tile t has |T|^2 = step^(-2t): the ratios walk down through every limit, a few tiles per
    format.  The map must equal the formula's wherever a tile is not within 1e-9 of a limit."""
    n = 40
    s = step ** (-2.0 * np.arange(n))
    want = _rule_by_formula(s, eps, 0x1F)
    ratio = np.sqrt(s * n / s.sum())
    for u in U.values():
        assert np.all(np.abs(ratio / (eps / u) - 1) > 1e-9)
    got = orc.precision_rule(s, eps, 0x1F)
    assert np.array_equal(got, want)
    assert set(np.unique(got)) >= {FP32, FP16, BF16, FP8}
    # the formats appear in the order of their unit roundoffs as the tiles shrink
    order = [int(p) for k, p in enumerate(got) if k == 0 or got[k] != got[k - 1]]
    assert order == sorted(order, key=lambda p: U[p])
