"""Pins of the oracle's tile scan and norm-based precision rule: exact rational sums,
the stated summation order re-enacted with exact fused multiply-adds, the rule's
invariants, its closed form on the decaying-tile workload, and its limiting cases.
"""
from fractions import Fraction

import numpy as np
import pytest

import workloads as W
from oracle import gemm_mp_oracle as orc
from tests.exact import fma64

FP64, FP32, FP16, FP8 = 0, 1, 2, 3
U = {FP64: 2.0 ** -53, FP32: 2.0 ** -24, FP16: 2.0 ** -11, FP8: 2.0 ** -4}


@pytest.mark.parametrize("nb", [4, 5, 6, 8])
def test_scan_follows_the_stated_order_bit_for_bit(nb):
    """Column-wise running fma over the rows, then neighbour pairs level by level
    (an odd element is carried up): re-enacted here with exact rational fmas."""
    rng = np.random.default_rng(nb)
    X = rng.standard_normal((2 * nb, 3 * nb)) * 10.0 ** rng.integers(-3, 4, (2 * nb, 3 * nb))
    sumsq, maxabs = orc.tile_scan(X, nb)
    for I in range(2):
        for J in range(3):
            T = X[I * nb:(I + 1) * nb, J * nb:(J + 1) * nb]
            level = []
            for c in range(nb):
                s = 0.0
                for r in range(nb):
                    s = fma64(T[r, c], T[r, c], s)
                level.append(s)
            while len(level) > 1:
                nxt = [level[2 * i] + level[2 * i + 1] for i in range(len(level) // 2)]
                if len(level) % 2:
                    nxt.append(level[-1])
                level = nxt
            assert sumsq[I, J] == level[0]
            assert maxabs[I, J] == np.abs(T).max()


def test_scan_is_exact_on_integers_and_close_to_the_exact_sum_otherwise():
    rng = np.random.default_rng(1)
    nb = 16
    Xi = rng.integers(-9, 10, (2 * nb, 2 * nb)).astype(np.float64)
    s, _ = orc.tile_scan(Xi, nb)
    for I in range(2):
        for J in range(2):
            assert s[I, J] == float((Xi[I * nb:(I + 1) * nb, J * nb:(J + 1) * nb].astype(np.int64) ** 2).sum())
    X = rng.standard_normal((nb, nb))
    s, _ = orc.tile_scan(X, nb)
    exact = sum(Fraction(float(v)) ** 2 for v in X.ravel())
    assert abs(Fraction(float(s[0, 0])) - exact) <= (nb + 8) * Fraction(2) ** -53 * exact


def _rule_maps(w, which):
    X = w.dense(which)
    sumsq, maxabs = orc.tile_scan(X, w.nb)
    return X, sumsq, maxabs, orc.precision_rule(sumsq, w.rule["eps"], w.rule["allowed"])


@pytest.mark.parametrize("make", [
    lambda: W.covariance(n=1024, nb=64, ell=0.1, eps=1e-8),
    lambda: W.covariance(n=1024, nb=64, ell=0.05, eps=1e-6),
    lambda: W.decay_rect(M=1024, N=1024, K=256, nb=64, eps=1e-4),
])
def test_rule_keeps_its_error_budget(make):
    """sum_T u_p(T)^2 |T|_F^2 <= eps^2 |X|_F^2 by construction, and the stored matrix is
    within eps of the original in the Frobenius norm."""
    w = make()
    for which in ("A", "B"):
        X, sumsq, maxabs, pmap = _rule_maps(w, which)
        eps = w.rule["eps"]
        u2 = np.vectorize(lambda p: U[p] ** 2)(pmap)
        highest = min(p for p in range(4) if w.rule["allowed"] >> p & 1)
        forced = pmap == highest                     # tiles that passed no test keep the best format
        budget = (u2 * sumsq)[~forced].sum()
        assert budget <= eps ** 2 * sumsq.sum() * (1 + 1e-12)
        Y, e = orc.store_tiles(X, w.nb, pmap, maxabs)
        Xhat = Y * np.kron(2.0 ** e.astype(np.float64), np.ones((w.nb, w.nb)))
        slack = U[highest] * np.sqrt(sumsq[forced].sum())
        assert np.linalg.norm(X - Xhat) <= eps * np.linalg.norm(X) + slack
        assert len(np.unique(pmap)) >= 2             # the workload really is mixed


def test_rule_closed_form_on_decaying_tiles():
    """Tiles scaled 2^(-4d), d = |I-J|: E|T|^2 = nb^2 2^(-8d).  With eps = 1e-4 the ratio
    |T| sqrt(#tiles) / |X| falls below eps/u16 = 0.2048 from d = 2 and below eps/u8 = 1.6e-3
    from d = 3; eps > u32 rules FP64 out: d <= 1 FP32, d = 2 FP16, d >= 3 FP8."""
    w = W.decay_rect(M=2048, N=2048, K=256, nb=64, eps=1e-4)
    for which in ("A", "B"):
        _, _, _, pmap = _rule_maps(w, which)
        I, J = np.indices(pmap.shape)
        d = np.abs(I - J)
        want = np.where(d <= 1, FP32, np.where(d == 2, FP16, FP8))
        assert np.array_equal(pmap, want)


def test_rule_limits_and_allowed_mask():
    rng = np.random.default_rng(5)
    sumsq = rng.uniform(0.5, 2.0, (4, 6))
    sumsq[1, 2] = 0.0
    for mask, hi, lo in ((0b1111, FP64, FP8), (0b0111, FP64, FP16), (0b0110, FP32, FP16), (0b0010, FP32, FP32)):
        m0 = orc.precision_rule(sumsq, 0.0, mask)
        assert m0[1, 2] == lo                        # a zero tile passes every test
        m0[1, 2] = hi
        assert np.all(m0 == hi)                      # eps = 0: nothing else passes
        big = np.sqrt(sumsq.size) * 2.0 ** 60
        assert np.all(orc.precision_rule(sumsq, big, mask) == lo)
    # |T| <= |X| always, so eps/u_lowest >= sqrt(#tiles) sends every tile to the lowest format
    eps = np.sqrt(sumsq.size) * U[FP16]
    assert np.all(orc.precision_rule(sumsq, eps, 0b0111) == FP16)
    # thresholds sit where the formula puts them: one tile just below / above the FP32 limit
    n = 16
    s = np.ones(n)
    eps = 1e-3
    limit = (eps / U[FP16]) ** 2 / n * n                # (|T|^2 n / |X|^2) <= (eps/u)^2
    s[0] = 4.0                                           # ratio^2 = 4*16/19 = 3.37 < (2.048)^2 = 4.19
    assert orc.precision_rule(s, eps, 0b0111)[0] == FP16
    s[0] = 6.0                                           # 6*16/21 = 4.57 > 4.19
    assert orc.precision_rule(s, eps, 0b0111)[0] == FP32
    assert limit > 0


def test_scale_exponent_window():
    for p, top in ((FP16, 15), (FP8, 8)):
        for m in (1.0, 0.75, 1e-30, 3e20, 2.0 ** -1060, np.nextafter(1.0, 0)):
            e = orc.scale_exponent(m, p)
            assert 2.0 ** (top - 1) <= np.ldexp(m, -e) < 2.0 ** top
        assert orc.scale_exponent(0.0, p) == 0
        assert orc.scale_exponent(np.inf, p) == 0
        assert orc.scale_exponent(np.nan, p) == 0
    assert orc.scale_exponent(123.0, FP64) == 0 and orc.scale_exponent(123.0, FP32) == 0
