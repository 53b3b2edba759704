"""The comparison that the GPU parity tests rest on, tried on the CPU: a second correct
evaluation in another order of summation (numpy's matrix product on the stored operands) must
pass it, and the same result with one misplaced element, one wrong 16 x 16 fragment or one
dropped reduction tile must not."""
import numpy as np
import pytest

import workloads as W
from oracle import gemm_mp_oracle as orc
from oracle.checker import FP32, FP64, OracleSide, compare_jobs, element_bounds, planted_mistake_is_caught


def _other_order(side, policy, alpha, beta):
    """C by numpy's blocked products: FP64 tiles from the FP64 product of the stored values, FP32
    tiles from the FP32 product of the operands rounded to FP32 (the receiver-side down-cast),
    epilogue in the tile's type.  Valid for FP64 / FP32 maps under the C-tile policy."""
    w = side.w
    nb = w.nb
    C = np.empty((w.M, w.N))
    for I in range(w.MT):
        for J in range(w.NT):
            rows, cols = slice(I * nb, (I + 1) * nb), slice(J * nb, (J + 1) * nb)
            if side.mapC[I, J] == FP64:
                s = side.Ay[rows] @ side.By[:, cols]
                C[rows, cols] = alpha * s + beta * side.Cy[rows, cols]
            else:
                s = side.Ay[rows].astype(np.float32) @ side.By[:, cols].astype(np.float32)
                v = np.float32(alpha) * s + np.float32(beta) * side.Cy[rows, cols].astype(np.float32)
                C[rows, cols] = v.astype(np.float64)
    return C


@pytest.fixture(scope="module")
def problem():
    w = W.paper_ratio(50, n=512, nb=128)
    A, B, C0 = w.dense("A"), w.dense("B"), w.dense("C")
    side = OracleSide(w, A, B, C0)
    jobs = orc.whole_tile_jobs(w.nb, [(i, j) for i in range(w.MT) for j in range(w.NT)])
    C_orc = side.gemm(jobs, policy=w.policy)
    C_other = _other_order(side, w.policy, w.alpha, w.beta)
    return w, side, jobs, C_orc, C_other


def test_a_second_correct_evaluation_passes_and_sits_well_inside_the_bounds(problem):
    w, side, jobs, C_orc, C_other = problem
    assert not np.array_equal(C_orc, C_other)              # it really is another order
    worst = compare_jobs(side, jobs, w.policy, w.alpha, w.beta, C_other, C_orc)
    assert 0 < worst["tight"] < 1 and 0 < worst["elem"] < 1 and worst["rel64"] < 1e-13


def test_a_misplaced_element_fails(problem):
    w, side, jobs, C_orc, C_other = problem
    for k in range(len(jobs)):
        assert planted_mistake_is_caught(side, jobs[k:], w.policy, w.alpha, w.beta, C_other.copy(), C_orc)


def test_a_wrong_fragment_and_a_dropped_reduction_tile_fail(problem):
    w, side, jobs, C_orc, C_other = problem
    nb = w.nb
    for (I, J) in ((0, 0), (1, 2), (3, 3)):
        job = np.array([[I, J, 0, nb, 0, nb]], dtype=np.int32)
        bad = C_other.copy()
        r, c = I * nb + 32, J * nb + 48
        bad[r:r + 16, c:c + 16] = bad[r:r + 16, c:c + 16].T.copy()      # a 16 x 16 fragment written transposed
        with pytest.raises(AssertionError):
            compare_jobs(side, job, w.policy, w.alpha, w.beta, bad, C_orc)
        bad = C_other.copy()
        rows, cols = slice(I * nb, (I + 1) * nb), slice(J * nb, (J + 1) * nb)
        bad[rows, cols] -= w.alpha * (side.Ay[rows, nb:2 * nb] @ side.By[nb:2 * nb, cols])     # reduction tile 1 left out
        with pytest.raises(AssertionError):
            compare_jobs(side, job, w.policy, w.alpha, w.beta, bad, C_orc)


def test_element_bounds_scale_with_the_products_precisions():
    """An FP64 tile with FP64 products is held to 2^-53-level bounds, an FP32 tile to 2^-24."""
    w = W.paper_ratio(50, n=512, nb=128)
    side = OracleSide(w, w.dense("A"), w.dense("B"), w.dense("C"))
    seen = set()
    for I in range(w.MT):
        for J in range(w.NT):
            b, P = element_bounds(side, [I, J, 0, 8, 0, 8], w.policy, w.alpha, w.beta)
            ratio = (b / P).max()
            pC = int(side.mapC[I, J])
            seen.add(pC)
            if pC == FP64:
                assert ratio < 4 * w.K * 2.0 ** -53
            else:
                assert 2 * w.K * 2.0 ** -24 <= ratio < 4 * w.K * 2.0 ** -24
    assert seen == {FP64, FP32}
