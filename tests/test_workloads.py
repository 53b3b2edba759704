"""The seeded input generators: deterministic, panel-wise reproducible, right shapes and laws."""
import numpy as np

import workloads as W


def test_panels_reproduce_the_dense_matrix_and_runs_repeat():
    for w in (W.tiny(M=512, N=256, K=768, nb=128), W.random_maps(M=256, N=512, K=256, nb=64),
              W.covariance(n=512, nb=64), W.decay_rect(M=512, N=512, K=128, nb=64)):
        for which in ("A", "B", "C"):
            full = w.dense(which)
            assert full.shape == w.shape(which) and full.dtype == np.float64
            assert np.array_equal(w.panel(which, 37, 101), full[37:101])
            assert np.array_equal(w.dense(which, panel_rows=96), full)


def test_value_laws():
    w = W.random_maps(M=512, N=512, K=512, nb=64)
    A = w.dense("A")
    assert -1.0 <= A.min() < -0.99 and 0.99 < A.max() < 1.0 and abs(A.mean()) < 0.01
    assert not np.array_equal(A, w.dense("B")[:512, :512])
    t = W.tiny(M=512, N=512, K=512, nb=128)
    A = t.dense("A")
    assert abs(A[:128, :128].std() - 1.0) < 0.02
    assert abs(A[:128, 256:384].std() / 1e-4 - 1.0) < 0.05
    assert abs(A[384:, :128].std() / 1e-6 - 1.0) < 0.05
    r = W.decay_rect(M=512, N=512, K=128, nb=64)
    A, B = r.dense("A"), r.dense("B")
    assert abs(A[128:192, 0:64].std() / 2.0 ** -8 - 1.0) < 0.05      # A tile (2,0)
    assert abs(B[0:64, 192:256].std() / 2.0 ** -12 - 1.0) < 0.05     # B tile (0,3)


def test_maps_and_samples():
    t = W.tiny()
    assert t.mapA.tolist() == [[0, 1, 2, 2], [1, 0, 1, 2], [2, 1, 0, 1], [2, 2, 1, 0]]
    assert t.mapC.tolist() == [[0] * 4] * 4
    w = W.random_maps()
    for m, probs in ((w.mapA, (.25, .25, .5)), (w.mapB, (.25, .25, .5)), (w.mapC, (.5, .5))):
        assert m.dtype == np.uint16 and m.shape == (16, 16)
        freq = np.bincount(m.ravel(), minlength=len(probs)) / m.size
        assert np.all(np.abs(freq - probs) < 0.1) and m.max() < len(probs)
    r = W.decay_rect()
    assert (r.MT, r.NT, r.KT) == (32, 32, 4) and np.all(r.mapC == W.FP32)
    s = r.sample_tiles(64)
    assert len(s) == len(set(s)) == 64 and s == r.sample_tiles(64)
    assert W.tiny().sample_tiles(64) == [(i, j) for i in range(4) for j in range(4)]


def test_morton_points_are_sorted_and_cluster_neighbours():
    p = W.morton_points(W.MASTER_SEED, 4096)
    assert p.shape == (4096, 2) and p.min() >= 0 and p.max() < 1
    c = W.covariance(n=1024, nb=128)
    A = c.dense("A")
    assert np.allclose(np.diag(A), 1.0) and np.array_equal(A, A.T) and np.array_equal(A, c.dense("B"))
    norms = np.array([[np.linalg.norm(A[i * 128:(i + 1) * 128, j * 128:(j + 1) * 128]) for j in range(8)]
                      for i in range(8)])
    assert np.all(np.diag(norms) > 5 * norms[0, 7])       # off-diagonal tiles decay


def _paper_settings():
    """The ratios and the tile size the paper states (tests/golden/paper_ratio_settings.txt)."""
    import os
    rows, tile = [], None
    for line in open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_ratio_settings.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "tile":
            tile = int(f[1])
        else:
            rows.append(tuple(int(x) for x in f))
    return rows, tile


def test_paper_ratio_maps_have_the_exact_ratio_and_a_random_pattern():
    """The paper's aD:bS runs: a % of the tiles of A, B and C FP64, the rest FP32 (Section 5.1)."""
    rows, tile = _paper_settings()
    assert all(a + b == 100 for a, b, _ in rows) and [a for a, _, _ in rows] == [100, 80, 50, 20, 0]
    assert W.paper_ratio(50).nb == tile and W.paper_ratio(50).M == 16 * tile
    for pct, _, _ in rows:
        w = W.paper_ratio(pct, n=4096, nb=256)
        for m in (w.mapA, w.mapB, w.mapC):
            assert m.shape == (16, 16) and m.dtype == np.uint16
            assert set(np.unique(m)) <= {W.FP64, W.FP32}
            assert int((m == W.FP64).sum()) == round(pct / 100 * 256)
        assert w.policy == 1 and w.alpha == 1.0 and w.beta == 1.0
    w = W.paper_ratio(50, n=4096, nb=256)
    assert not np.array_equal(w.mapA, w.mapB) and not np.array_equal(w.mapA, w.mapC)
    # not a structured pattern: every tile row and column holds both precisions
    assert all(0 < int((w.mapA[i] == W.FP64).sum()) < 16 for i in range(16))
    x = w.panel("A", 0, 8)
    assert x.shape == (8, 4096) and np.all(np.abs(x) <= 1.0)
