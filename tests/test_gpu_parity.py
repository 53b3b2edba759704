"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Integer work (scan order, maps, exponents, packed codes) is compared bit for
bit; C per tile within 4*K*u_tile (and 1e-12 relative for all-FP64 tiles), normalised by
sum_L |A_IL|_F |B_LJ|_F, plus a tighter accumulate-precision bound that makes real bugs visible.
"""
import numpy as np
import pytest

import workloads as W
from oracle import gemm_mp_oracle as orc
from oracle.checker import planted_mistake_is_caught
from tests.harness import (BF16, FP8, FP16, FP32, FP64, MXFP4, MXFP6, MXFP8, OracleSide, compare_jobs, finish_low_c_tiles, gpu_problem,
                           packed_codes_expected)

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _dense(w):
    A = w.dense("A")
    B = A if w.a_equals_b else w.dense("B")
    C0 = w.dense("C") if w.beta != 0.0 else None
    return A, B, C0


def _all_jobs(w):
    return orc.whole_tile_jobs(w.nb, [(i, j) for i in range(w.MT) for j in range(w.NT)])


def _check_storage(d, side, which, tiles):
    """Packed bytes and exponents of the given tiles equal the oracle's codes bit for bit."""
    exps = {"A": side.eA, "B": side.eB}[which]
    for (I, J) in tiles:
        got, prec = d.tile_bytes(which, I, J)
        want = packed_codes_expected(side, which, I, J)
        assert prec == int({"A": side.mapA, "B": side.mapB}[which][I, J])
        assert np.array_equal(got, want), "packed tile %s(%d,%d) differs" % (which, I, J)
        assert d.ctx.tile_info(which, I, J)[2] == int(exps[I, J])


def _run_and_compare(w, policy=0, jobs=None, check_storage_tiles=4, alpha=None, beta=None):
    import torch
    _say("workload", w.name, (w.M, w.N, w.K, w.nb), "policy", policy)
    A, B, C0 = _dense(w)
    side = OracleSide(w, A, B, C0)
    d, dev = gpu_problem(w, A, B, C0, policy=policy)
    assert np.array_equal(d.maps["A"], side.mapA) and np.array_equal(d.maps["B"], side.mapB)
    rng = np.random.default_rng(7)
    for which, (rt, ct) in (("A", (w.MT, w.KT)), ("B", (w.KT, w.NT))):
        picks = {(int(rng.integers(rt)), int(rng.integers(ct))) for _ in range(check_storage_tiles)}
        _check_storage(d, side, which, sorted(picks))
    alpha = w.alpha if alpha is None else alpha
    beta = w.beta if beta is None else beta
    d.run(alpha, beta)
    C_gpu = d.unpack_tiles("C").cpu().numpy()
    torch.cuda.synchronize()
    if jobs is None:
        jobs = _all_jobs(w)
    C_orc = side.gemm(jobs, policy=policy, alpha=alpha, beta=beta)
    worst = compare_jobs(side, jobs, policy, alpha, beta, C_gpu, C_orc)
    _say("  worst error / bound:", worst)
    # the comparison must be able to fail: a misplaced element of the result (host copy) is caught
    caught = planted_mistake_is_caught(side, jobs, policy, alpha, beta, C_gpu, C_orc)
    _say("  planted misplaced element caught:", caught)
    return d, side, C_gpu, C_orc


# ------------------------------------------------------------------------------------------
def test_scan_and_rule_match_the_oracle_bit_for_bit():
    import torch
    for w in (W.covariance(n=1024, nb=128, ell=0.1, eps=1e-8), W.covariance(n=1536, nb=256, ell=0.05, eps=1e-6),
              W.decay_rect(M=2048, N=1024, K=256, nb=128, eps=1e-4), W.decay_rect(M=768, N=768, K=384, nb=384, eps=1e-3)):
        _say("scan", w.name, w.M, w.K, w.nb)
        from paper_2508_14848_amd.device import DeviceGemmMP
        d = DeviceGemmMP(w.M, w.N, w.K, w.nb)
        for which in ("A", "B"):
            X = w.dense(which)
            dX = torch.from_numpy(X).cuda()
            sumsq, maxabs = d.tile_scan(which, dX)
            s0, m0 = orc.tile_scan(X, w.nb)
            assert np.array_equal(sumsq, s0) and np.array_equal(maxabs, m0)
            got = d.compute_precision_map(which, dX, w.rule["eps"], w.rule["allowed"])
            assert np.array_equal(got, orc.precision_rule(s0, w.rule["eps"], w.rule["allowed"]))
        # a padded leading dimension gives the same numbers
        X = w.dense("A")
        pad = torch.zeros((w.M, w.K + 6), dtype=torch.float64, device="cuda")
        pad[:, :w.K] = torch.from_numpy(X).cuda()
        s1, m1 = d.tile_scan("A", pad)
        s0, m0 = orc.tile_scan(X, w.nb)
        assert np.array_equal(s1, s0) and np.array_equal(m1, m0)


def test_pack_is_bit_exact_on_hard_values_and_unpack_round_trips():
    """Every tile precision on values chosen to sit on rounding boundaries: FP16/FP8 midpoints
    (after the tile scale), subnormal results, overflow of FP32, zeros of both signs, NaN/inf."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP
    nb = 128
    rng = np.random.default_rng(11)
    for which in ("A", "B"):
        M, K = 2 * nb, 4 * nb
        shape = (M, K) if which == "A" else (K, M)
        X = rng.standard_normal(shape) * np.exp(rng.uniform(-12, 3, shape))
        # midpoints and near-midpoints of the 11-bit and 4-bit grids, relative to a tile max of 1.75*2^k
        base = 1.75 * 2.0 ** rng.integers(-2, 8)
        mids16 = (1.0 + (rng.integers(0, 1024, 3000) + 0.5) / 1024.0) * 2.0 ** rng.integers(-26, 1, 3000)
        mids8 = (1.0 + (rng.integers(0, 8, 3000) + 0.5) / 8.0) * 2.0 ** rng.integers(-18, 1, 3000)
        hard = np.concatenate([mids16, np.nextafter(mids16, 0), np.nextafter(mids16, 9), mids8,
                               np.nextafter(mids8, 0), np.nextafter(mids8, 9)]) * base
        hard = np.concatenate([hard, -hard, [0.0, -0.0, 1e-320, -1e-310, 3.5e38, 1e39, -1e300, 2.0 ** -149, 2.0 ** -150 * 1.0000001]])
        flat = X.ravel()
        pos = rng.choice(flat.size, hard.size, replace=False)
        flat[pos] = hard
        X.ravel()[rng.choice(flat.size, 40, replace=False)] = base * 1.0001      # keeps tile maxima near base
        tiles = (shape[0] // nb, shape[1] // nb)
        pmap = (np.arange(tiles[0] * tiles[1]).reshape(tiles) % 4).astype(np.uint16)
        Xs = X.copy()
        Xs[0:nb, 0:nb] = 0.0                                                   # an all-zero low-precision tile
        pmap[0, 0] = FP16
        Xn = Xs.copy()
        for I0 in range(tiles[0]):                                             # NaN / inf inside tiles of each format
            sub = Xn[I0 * nb:(I0 + 1) * nb, nb:2 * nb]
            sub.flat[3::97] = np.nan
            if I0 == 0:
                sub.flat[5::101] = np.inf
                sub.flat[7::103] = -np.inf
        for name, data in (("finite", Xs), ("nonfinite", Xn)):
            _say("pack", which, name)
            w = W.Workload("pack", M, M, K, nb, 1.0, 0.0)
            d = DeviceGemmMP(M, M, K, nb)
            d.set_precision_map(which, pmap)
            dX = torch.from_numpy(data).cuda()
            d.pack_tiles(which, dX)
            _, maxabs = orc.tile_scan(data, nb)
            Y, e = orc.store_tiles(data, nb, pmap, maxabs)
            assert np.array_equal(d.exponents(which), e)

            class S:
                pass
            side = S()
            side.w, side.Ay, side.By, side.Cy = w, Y, Y, None
            side.mapA = side.mapB = side.mapC = pmap
            for I in range(tiles[0]):
                for J in range(tiles[1]):
                    got, prec = d.tile_bytes(which, I, J)
                    want = packed_codes_expected(side, which, I, J)
                    if name == "nonfinite" and prec in (FP16, FP64, FP32):
                        # NaN payloads are not compared; positions and everything else are
                        width = {FP64: 8, FP32: 4, FP16: 2}[prec]
                        dt = {8: np.float64, 4: np.float32, 2: np.float16}[width]
                        g, x = got.view(dt), want.view(dt)
                        assert np.array_equal(np.isnan(g), np.isnan(x))
                        assert np.array_equal(got.reshape(-1, width)[~np.isnan(g)], want.reshape(-1, width)[~np.isnan(x)])
                    else:
                        assert np.array_equal(got, want), (which, name, I, J, prec)
            back = d.unpack_tiles(which).cpu().numpy()
            want = Y * np.kron(2.0 ** e.astype(np.float64), np.ones((nb, nb)))
            assert np.array_equal(np.isnan(back), np.isnan(want))
            ok = ~np.isnan(want)
            assert np.array_equal(back[ok], want[ok])


def test_fp64_tiles_without_an_fp64_product_take_the_instance_without_the_fp64_loop():
    """FP64 C tiles whose operands are all stored in FP32 / FP16 (what the norm rule makes of a
    covariance matrix) run on an instance of their own: per-product accumulator in the pinned
    registers, first chunk of the next product handed over in registers, block-wise fold.  Small
    integers must come out exactly through every transition between FP32 products (with and
    without an FP16 operand) and runs of FP16 ring products, old C included; one FP64 tile among
    the operands sends the same problem back to the general instance, with the same result."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(171)
    for (nb, MT, NT, KT) in ((128, 2, 2, 6), (256, 1, 2, 7), (512, 1, 1, 4)):
        M, N, K = MT * nb, NT * nb, KT * nb
        for trial in range(3):
            A = rng.integers(-3, 4, (M, K)).astype(np.float64)
            B = rng.integers(-3, 4, (K, N)).astype(np.float64)
            C0 = rng.integers(-5, 6, (M, N)).astype(np.float64)
            mA = rng.choice([FP32, FP16], (MT, KT), p=[0.6, 0.4]).astype(np.uint16)
            mB = rng.choice([FP32, FP16], (KT, NT), p=[0.6, 0.4]).astype(np.uint16)
            if trial == 1:
                mA[:, KT // 2:] = FP16                     # a run of ring products at the end of some reductions
                mB[KT // 2:, :] = FP16
            mC = np.full((MT, NT), FP64, dtype=np.uint16)
            if NT > 1:
                mC[0, 1] = FP32
            _say("FP64 tiles without FP64 products:", (nb, MT, NT, KT), "trial", trial)
            want = (2 * (A.astype(np.int64) @ B.astype(np.int64)) - 3 * C0.astype(np.int64)).astype(np.float64)
            results = []
            for with_fp64_operand in (False, True):
                mA2 = mA.copy()
                if with_fp64_operand:
                    mA2[0, 0] = FP64
                d = DeviceGemmMP(M, N, K, nb)
                for which, m, X in (("A", mA2, A), ("B", mB, B), ("C", mC, C0)):
                    d.set_precision_map(which, m)
                    d.pack_tiles(which, torch.from_numpy(X).cuda())
                assert d.ctx.get_stats()["owner_instance"][0] == (0 if with_fp64_operand else 3)
                d.run(2.0, -3.0)
                results.append(d.unpack_tiles("C").cpu().numpy())
                assert np.array_equal(results[-1], want), (nb, trial, with_fp64_operand)
    torch.cuda.synchronize()


def test_small_integer_inputs_are_exact_for_every_precision_combination():
    """Entries in {-3..3}: every format holds them exactly and every partial sum is a small
    integer, so the GPU result must equal the integer product bit for bit, whatever the maps.
    Several tile sizes and reduction lengths, so that every kind of product-to-product
    transition inside an owner workgroup occurs many times."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(21)
    for (nb, MT, NT, KT) in ((128, 2, 3, 4), (256, 2, 2, 9), (384, 1, 2, 5)):
        M, N, K = MT * nb, NT * nb, KT * nb
        for policy in (0, 1):
            for trial in range(3):
                A = rng.integers(-3, 4, (M, K)).astype(np.float64)
                B = rng.integers(-3, 4, (K, N)).astype(np.float64)
                C0 = rng.integers(-5, 6, (M, N)).astype(np.float64)
                mA = rng.integers(0, 4, (MT, KT)).astype(np.uint16)
                mB = rng.integers(0, 4, (KT, NT)).astype(np.uint16)
                mC = rng.integers(0, 2, (MT, NT)).astype(np.uint16)
                if trial == 0:
                    A[0:nb, 0:nb] = 0.0
                    mA[0, 0] = FP8
                _say("integers", (nb, MT, NT, KT), "policy", policy, "trial", trial)
                d = DeviceGemmMP(M, N, K, nb, policy=policy)
                for which, m, X in (("A", mA, A), ("B", mB, B), ("C", mC, C0)):
                    d.set_precision_map(which, m)
                    d.pack_tiles(which, torch.from_numpy(X).cuda())
                d.run(2.0, -3.0)
                got = d.unpack_tiles("C").cpu().numpy()
                want = 2 * (A.astype(np.int64) @ B.astype(np.int64)) - 3 * C0.astype(np.int64)
                assert np.array_equal(got, want.astype(np.float64))


def test_runs_of_unconverted_low_precision_products_are_exact():
    """Long and short runs of FP8 / FP16 products whose operands need no conversion (the path
    that streams operands straight into LDS), entered from and left to every other kind of
    product, at one, two, three and four chunks per product; small integers, so exact."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(5)
    pattern = np.array([3, 3, 3, 2, 2, 1, 3, 3, 0, 2, 3, 2, 2, 2], dtype=np.uint16)
    for nb in (128, 256, 384, 512):
        MT, NT, KT = 2, 2, len(pattern)
        M, N, K = MT * nb, NT * nb, KT * nb
        A = rng.integers(-3, 4, (M, K)).astype(np.float64)
        B = rng.integers(-3, 4, (K, N)).astype(np.float64)
        mA = np.tile(pattern, (MT, 1))
        mB = np.tile(pattern[:, None], (1, NT))
        mA[1] = np.roll(pattern, 3)                 # second tile row: runs broken by mixed products
        mC = np.array([[FP32, FP64], [FP32, FP32]], dtype=np.uint16)
        _say("runs", nb)
        d = DeviceGemmMP(M, N, K, nb)
        for which, m, X in (("A", mA, A), ("B", mB, B)):
            d.set_precision_map(which, m)
            d.pack_tiles(which, torch.from_numpy(X).cuda())
        d.set_precision_map("C", mC)
        d.run(1.0, 0.0)
        got = d.unpack_tiles("C").cpu().numpy()
        want = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float64)
        assert np.array_equal(got, want)
        assert d.ctx.get_stats()["products"][FP8] >= 10


def test_fp32_tiles_made_of_fp8_products_only():
    """FP32 C tiles whose every product multiplies two FP8 tiles run in 256 x 256 regions with the
    tile scales applied inside the matrix core.  Small integers first (exact, general alpha and
    beta, several regions per tile, FP64 and mixed C tiles beside them), then scaled tiles of
    very different magnitudes against the oracle."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(33)
    for (nb, MT, NT, KT) in ((256, 2, 3, 5), (512, 2, 2, 3), (768, 1, 2, 2)):
        M, N, K = MT * nb, NT * nb, KT * nb
        A = rng.integers(-3, 4, (M, K)).astype(np.float64)
        B = rng.integers(-3, 4, (K, N)).astype(np.float64)
        C0 = rng.integers(-5, 6, (M, N)).astype(np.float64)
        mA = np.full((MT, KT), FP8, dtype=np.uint16)
        mB = np.full((KT, NT), FP8, dtype=np.uint16)
        mC = np.full((MT, NT), FP32, dtype=np.uint16)
        mC[0, 0] = FP64                              # an FP64 tile: the ordinary kernel
        mB[KT - 1, NT - 1] = FP16                    # last tile column: one FP16 operand, so not FP8 only
        _say("fp8-only tiles", (nb, MT, NT, KT))
        d = DeviceGemmMP(M, N, K, nb)
        for which, m, X in (("A", mA, A), ("B", mB, B), ("C", mC, C0)):
            d.set_precision_map(which, m)
            d.pack_tiles(which, torch.from_numpy(X).cuda())
        big = MT * NT - 1 - MT                       # tiles that qualify
        st = d.ctx.get_stats()
        assert st["work_items"] == (MT * NT - big) * (nb // 128) ** 2 + big * (nb // 256) ** 2
        d.run(2.0, -3.0)
        got = d.unpack_tiles("C").cpu().numpy()
        want = 2 * (A.astype(np.int64) @ B.astype(np.int64)) - 3 * C0.astype(np.int64)
        assert np.array_equal(got, want.astype(np.float64))
        d.pack_tiles("C", torch.from_numpy(C0).cuda())
        d.run(0.0, 1.0)                              # alpha == 0: no product is formed
        assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), C0)
    w = W.tiny(M=512, N=768, K=1024, nb=256)
    w.mapA = np.full((w.MT, w.KT), FP8, dtype=np.uint16)
    w.mapB = np.full((w.KT, w.NT), FP8, dtype=np.uint16)
    w.mapC = np.full((w.MT, w.NT), FP32, dtype=np.uint16)
    _run_and_compare(w)
    w.alpha, w.beta = -0.75, 1.25
    _run_and_compare(w)


def test_extreme_tile_exponents_are_exact():
    """Tiles of small integers times 2^k with k from -140 to +120, paired so that every product
    of a C tile carries 2^-20: exact in every format, whatever route the conversion takes (the
    fused convert-and-scale instructions, the generic conversion for exponents outside their
    range, the block scales of the FP8-only kernel, which split what one E8M0 cannot hold)."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(77)
    ks = np.array([-140, -128, -120, -104, -60, 0, 60, 100], dtype=np.int64)
    for nb, maps in ((256, "fp8"), (256, "mixed"), (128, "mixed")):
        MT, NT, KT = 2, 2, len(ks)
        M, N, K = MT * nb, NT * nb, KT * nb
        Ai = rng.integers(-3, 4, (M, K)).astype(np.float64)
        Bi = rng.integers(-3, 4, (K, N)).astype(np.float64)
        A, B = Ai.copy(), Bi.copy()
        for L, k in enumerate(ks):
            A[:, L * nb:(L + 1) * nb] *= 2.0 ** float(k)
            B[L * nb:(L + 1) * nb, :] *= 2.0 ** float(-20 - k)
        if maps == "fp8":
            mA = np.full((MT, KT), FP8, dtype=np.uint16)
            mB = np.full((KT, NT), FP8, dtype=np.uint16)
            mC = np.array([[FP32, FP32], [FP32, FP64]], dtype=np.uint16)
        else:
            mA = rng.integers(2, 4, (MT, KT)).astype(np.uint16)          # FP16 / FP8
            mB = rng.integers(1, 4, (KT, NT)).astype(np.uint16)          # FP32 / FP16 / FP8
            mB[ks < -100, :] = np.where(mB[ks < -100, :] == FP32, FP16, mB[ks < -100, :])   # 2^(-20-k) * 3 fits FP32 anyway
            mC = np.array([[FP32, FP64], [FP64, FP32]], dtype=np.uint16)
        _say("extreme exponents", nb, maps)
        for policy in (0, 1):
            d = DeviceGemmMP(M, N, K, nb, policy=policy)
            for which, m, X in (("A", mA, A), ("B", mB, B)):
                d.set_precision_map(which, m)
                d.pack_tiles(which, torch.from_numpy(X).cuda())
            d.set_precision_map("C", mC)
            d.run(1.0, 0.0)
            got = d.unpack_tiles("C").cpu().numpy()
            want = (Ai.astype(np.int64) @ Bi.astype(np.int64)).astype(np.float64) * 2.0 ** -20
            assert np.array_equal(got, want)


def _even_ld(X):
    """The array as a device tensor whose rows have an even length (what the library asks)."""
    import torch
    rows, cols = X.shape
    buf = torch.zeros((rows, cols + (cols & 1)), dtype=torch.float64, device="cuda")
    buf[:, :cols] = torch.from_numpy(X).cuda()
    return buf[:, :cols]


def test_sizes_that_are_no_multiples_of_the_tile_size():
    """M, N, K off the tile grid: scan, rule and pack agree bit for bit with the oracle on the
    zero-padded matrices, the product of small integers is exact for random maps, and general
    data stays within the per-tile bounds; nothing outside the M x N entries of C is written."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(123)
    for (M, N, K, nb) in ((300, 520, 777, 128), (1000, 257, 513, 256), (129, 127, 1, 128)):
        MT, NT, KT = -(-M // nb), -(-N // nb), -(-K // nb)
        _say("ragged", (M, N, K, nb))
        # integers: exact
        A = rng.integers(-3, 4, (M, K)).astype(np.float64)
        B = rng.integers(-3, 4, (K, N)).astype(np.float64)
        C0 = rng.integers(-5, 6, (M, N)).astype(np.float64)
        mA = rng.integers(0, 4, (MT, KT)).astype(np.uint16)
        mB = rng.integers(0, 4, (KT, NT)).astype(np.uint16)
        mC = rng.integers(0, 2, (MT, NT)).astype(np.uint16)
        for policy in (0, 1):
            d = DeviceGemmMP(M, N, K, nb, policy=policy)
            for which, m, X in (("A", mA, A), ("B", mB, B), ("C", mC, C0)):
                d.set_precision_map(which, m)
                d.pack_tiles(which, _even_ld(X))
            d.run(2.0, -3.0)
            out = torch.full((M + 3, N + 4 + (N & 1)), -7.0, dtype=torch.float64, device="cuda")
            d.unpack_tiles("C", out=out[:M, :N])
            got = out.cpu().numpy()
            want = 2 * (A.astype(np.int64) @ B.astype(np.int64)) - 3 * C0.astype(np.int64)
            assert np.array_equal(got[:M, :N], want.astype(np.float64))
            assert np.all(got[M:] == -7.0) and np.all(got[:, N:] == -7.0)
        # general data: scan, rule, pack and product against the oracle on the padded matrices
        X = {"A": rng.standard_normal((M, K)) * np.exp(rng.uniform(-8, 8, (M, 1))),
             "B": rng.standard_normal((K, N)) * np.exp(rng.uniform(-8, 8, (1, N)))}
        d = DeviceGemmMP(M, N, K, nb)
        maps, stored, exps = {}, {}, {}
        for which in ("A", "B"):
            dX = _even_ld(X[which])
            Xp = orc.pad_to_tiles(X[which], nb)
            s0, m0 = orc.tile_scan(Xp, nb)
            s1, m1 = d.tile_scan(which, dX)
            assert np.array_equal(s0, s1) and np.array_equal(m0, m1)
            maps[which] = d.compute_precision_map(which, dX, 1e-6, 0b1111)
            assert np.array_equal(maps[which], orc.precision_rule(s0, 1e-6, 0b1111))
            d.pack_tiles(which, dX)
            stored[which], exps[which] = orc.store_tiles(Xp, nb, maps[which], m0)
            rows, cols = X[which].shape
            value = np.ldexp(stored[which], np.kron(exps[which], np.ones((nb, nb), dtype=np.int32)))   # y * 2^e per tile
            assert np.array_equal(d.unpack_tiles(which).cpu().numpy(), value[:rows, :cols])
        d.set_precision_map("C", mC)
        d.run(1.0, 0.0)
        C_gpu = np.zeros((MT * nb, NT * nb))
        C_gpu[:M, :N] = d.unpack_tiles("C").cpu().numpy()
        w = W.Workload("ragged", MT * nb, NT * nb, KT * nb, nb, 1.0, 0.0)
        w.mapA, w.mapB, w.mapC = maps["A"], maps["B"], mC
        side = OracleSide(w, orc.pad_to_tiles(X["A"], nb), orc.pad_to_tiles(X["B"], nb), None)
        jobs = _all_jobs(w)
        compare_jobs(side, jobs, 0, 1.0, 0.0, C_gpu, side.gemm(jobs, alpha=1.0, beta=0.0))


def test_transposed_operands():
    """A and / or B given as the buffer of their transpose: scan, rule, stored values and the
    product are bit for bit those of the same matrices given directly (sizes off the tile grid
    included), and the unpacked buffer is the transpose again."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(9)
    for (M, N, K, nb) in ((384, 256, 512, 128), (300, 200, 457, 128)):
        A = rng.standard_normal((M, K)) * np.exp(rng.uniform(-6, 6, (M, 1)))
        B = rng.standard_normal((K, N)) * np.exp(rng.uniform(-6, 6, (1, N)))
        mC = rng.integers(0, 2, (-(-M // nb), -(-N // nb))).astype(np.uint16)
        results = []
        for (tA, tB) in ((0, 0), (1, 0), (0, 1), (1, 1)):
            _say("transposed", (M, N, K, nb), tA, tB)
            d = DeviceGemmMP(M, N, K, nb)
            d.set_transposed("A", tA)
            d.set_transposed("B", tB)
            scans, maps, back = {}, {}, {}
            for which, X, t in (("A", A, tA), ("B", B, tB)):
                dX = _even_ld(np.ascontiguousarray(X.T) if t else X)
                scans[which] = d.tile_scan(which, dX)
                maps[which] = d.compute_precision_map(which, dX, 1e-5, 0b1111)
                d.pack_tiles(which, dX)
                u = d.unpack_tiles(which).cpu().numpy()
                back[which] = u.T if t else u
            d.set_precision_map("C", mC)
            d.run(1.25, 0.0)
            results.append((scans, maps, back, d.unpack_tiles("C").cpu().numpy()))
        s0, m0, b0, c0 = results[0]
        for (s1, m1, b1, c1) in results[1:]:
            for which in ("A", "B"):
                assert np.array_equal(s0[which][0], s1[which][0]) and np.array_equal(s0[which][1], s1[which][1])
                assert np.array_equal(m0[which], m1[which]) and np.array_equal(b0[which], b1[which])
            assert np.array_equal(c0, c1)
        sA, mA = orc.tile_scan(orc.pad_to_tiles(A, nb), nb)
        assert np.array_equal(s0["A"][0], sA) and np.array_equal(s0["A"][1], mA)


def test_random_small_integer_problems_are_exact():
    """Three hundred seeded problems of small integers: tile sizes 128..512, one to three tiles a
    side and up to six along the reduction, sizes on and off the tile grid, four styles of maps
    (anything; FP16 / FP8 only on FP32 C tiles; all FP8 with exceptions; FP64 / FP32 only), both
    policies, operands given directly or transposed, receiver- or sender-side conversion, integer
    alpha and beta.  Every format holds the data exactly, so C must equal alpha*A*B + beta*C0
    bit for bit whichever kernels, chunk loops and hand-overs a problem happens to exercise."""
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(20250814)
    for case in range(300):
        nb = int(rng.choice([128, 256, 384, 512]))
        MT, NT, KT = int(rng.integers(1, 4)), int(rng.integers(1, 4)), int(rng.integers(1, 7))
        ragged = rng.random() < 0.3
        M = MT * nb - (int(rng.integers(1, nb)) if ragged else 0)
        N = NT * nb - (int(rng.integers(1, nb)) if ragged else 0)
        K = KT * nb - (int(rng.integers(1, nb)) if ragged else 0)
        policy, style = int(rng.integers(0, 2)), int(rng.integers(0, 4))
        if style == 0:
            mA, mB, mC = rng.integers(0, 4, (MT, KT)), rng.integers(0, 4, (KT, NT)), rng.integers(0, 2, (MT, NT))
        elif style == 1:
            mA, mB, mC = rng.integers(2, 4, (MT, KT)), rng.integers(2, 4, (KT, NT)), np.ones((MT, NT), dtype=np.int64)
        elif style == 2:
            mA, mB, mC = np.full((MT, KT), FP8), np.full((KT, NT), FP8), rng.integers(0, 2, (MT, NT))
            if rng.random() < 0.5:
                mA[rng.integers(MT), rng.integers(KT)] = rng.integers(0, 3)
        else:
            mA, mB, mC = rng.integers(0, 2, (MT, KT)), rng.integers(0, 2, (KT, NT)), rng.integers(0, 2, (MT, NT))
        alpha, beta = float(rng.integers(-2, 3)), float(rng.integers(-2, 3))
        A = rng.integers(-3, 4, (M, K)).astype(np.float64)
        B = rng.integers(-3, 4, (K, N)).astype(np.float64)
        C0 = rng.integers(-5, 6, (M, N)).astype(np.float64)
        tA, tB, sender = int(rng.integers(0, 2)), int(rng.integers(0, 2)), rng.random() < 0.3
        what = dict(case=case, nb=nb, M=M, N=N, K=K, policy=policy, style=style, alpha=alpha, beta=beta, tA=tA, tB=tB,
                    sender=bool(sender))
        if case % 50 == 0:
            _say("random integers", what)
        d = DeviceGemmMP(M, N, K, nb, policy=policy)
        d.set_transposed("A", tA)
        d.set_transposed("B", tB)
        for which, m, X, t in (("A", mA, A, tA), ("B", mB, B, tB), ("C", mC, C0, 0)):
            d.set_precision_map(which, m.astype(np.uint16))
            d.pack_tiles(which, _even_ld(np.ascontiguousarray(X.T) if t else X))
        if sender:
            d.convert_tiles()
        d.run(alpha, beta)
        got = d.unpack_tiles("C").cpu().numpy()
        want = alpha * (A @ B) + beta * C0               # exact in FP64: small integers
        assert np.array_equal(got, want), what


def test_c_tiles_stored_in_fp16_and_fp8_hold_small_integer_results_exactly():
    """C tiles in FP16 / FP8 are accumulated in FP32 staging copies and stored with a scale taken
    from the finished tile.  Results that are integers up to 15 fit every format, so C, the
    stored codes' values and the exponents must equal the oracle's exactly, old C included."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(91)
    for nb, MT, NT, KT, cut in ((128, 3, 2, 3, (0, 0, 0)), (256, 2, 3, 2, (0, 0, 0)), (512, 2, 2, 1, (0, 0, 0)),
                                (128, 2, 3, 2, (37, 101, 64))):
        M, N, K = MT * nb, NT * nb, KT * nb
        _say("low C tiles, integers:", (M, N, K, nb), "cut", cut)
        A = np.zeros((M, K))
        B = np.zeros((K, N))
        cols = rng.integers(0, nb, (M, KT)) + nb * np.arange(KT)
        A[np.arange(M)[:, None], cols] = rng.integers(-2, 3, (M, KT))
        rows = rng.integers(0, nb, (KT, N)) + nb * np.arange(KT)[:, None]
        B[rows, np.arange(N)[None, :]] = rng.integers(-1, 2, (KT, N))
        C0 = rng.integers(-3, 4, (M, N)).astype(np.float64)
        M, N, K = M - cut[0], N - cut[1], K - cut[2]           # sizes off the tile grid: edge tiles zero-padded
        A, B, C0 = A[:M, :K], B[:K, :N], C0[:M, :N]
        mA = rng.integers(0, 4, (MT, KT)).astype(np.uint16)
        mB = rng.integers(0, 4, (KT, NT)).astype(np.uint16)
        mC = rng.integers(0, 4, (MT, NT)).astype(np.uint16)
        mC[0, 0], mC[MT - 1, NT - 1] = FP16, FP8
        if nb == 512:
            mA[:], mB[:], mC[0, 1] = FP8, FP8, FP8             # a tile of FP8 products only: large regions
        want = (A.astype(np.int64) @ B.astype(np.int64)) + 2 * C0.astype(np.int64)
        assert np.abs(want).max() <= 15
        for policy in (0, 1):
            d = DeviceGemmMP(M, N, K, nb, policy=policy)
            for k, m in (("A", mA), ("B", mB), ("C", mC)):
                d.set_precision_map(k, m)
            d.pack_tiles("A", _even_ld(A))
            d.pack_tiles("B", _even_ld(B))
            d.pack_tiles("C", _even_ld(C0))
            assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), C0)
            d.run(1.0, 2.0)
            got = d.unpack_tiles("C").cpu().numpy()
            assert np.array_equal(got, want.astype(np.float64))
            _, eC = orc.store_tiles(orc.pad_to_tiles(want.astype(np.float64), nb), nb, mC)
            for I in range(MT):
                for J in range(NT):
                    assert d.ctx.tile_info("C", I, J)[2] == int(eC[I, J])
            # a second run on the result: C <- 0*A*B + 1*C leaves it as it is; then C <- -C
            d.run(0.0, 1.0)
            assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), want.astype(np.float64))
            d.run(0.0, -1.0)
            assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), -want.astype(np.float64))
            d.run(0.0, 0.0)
            assert not d.unpack_tiles("C").any()
            torch.cuda.synchronize()


def test_c_tiles_stored_in_fp16_and_fp8_match_the_oracle_on_general_data():
    """Random data, every map code on A, B and C, alpha and beta at work: per tile within the
    stated tolerance of the oracle's stored result, and the exponents agree wherever the two
    sides' largest magnitudes share a binade."""
    import torch
    w = W.tiny()
    rng = np.random.default_rng(92)
    w.mapC = rng.integers(0, 4, w.mapC.shape).astype(np.uint16)
    w.mapC[0, :4] = (FP64, FP32, FP16, FP8)
    w.alpha, w.beta = 0.75, -1.25
    for policy in (0, 1):
        _say("low C tiles, general data, policy", policy)
        A, B, C0 = _dense(w)
        side = OracleSide(w, A, B, C0)
        d, dev = gpu_problem(w, A, B, C0, policy=policy)
        d.run(w.alpha, w.beta)
        C_gpu = d.unpack_tiles("C").cpu().numpy()
        torch.cuda.synchronize()
        jobs = _all_jobs(w)
        pre = side.gemm(jobs, policy=policy)
        C_orc, eC = finish_low_c_tiles(side, pre)
        worst = compare_jobs(side, jobs, policy, w.alpha, w.beta, C_gpu, C_orc)
        _say("  worst error / bound:", worst)
        low = 0
        for I in range(w.MT):
            for J in range(w.NT):
                if w.mapC[I, J] < FP16:
                    continue
                low += 1
                blk = (slice(I * w.nb, (I + 1) * w.nb), slice(J * w.nb, (J + 1) * w.nb))
                if np.floor(np.log2(np.abs(C_gpu[blk]).max())) == np.floor(np.log2(np.abs(pre[blk]).max())):
                    assert d.ctx.tile_info("C", I, J)[2] == int(eC[I, J])
                # what the GPU stored is a number of the format at its exponent
                e = d.ctx.tile_info("C", I, J)[2]
                scaled = np.ldexp(C_gpu[blk], -e)
                rounded = (orc.round_fp16 if w.mapC[I, J] == FP16 else orc.round_fp8)(scaled)[0]
                assert np.array_equal(scaled, rounded)
        assert low >= 4


def test_c_tiles_stored_in_block_scaled_formats():
    """C tiles in MXFP8 / MXFP4 / MXFP6: accumulated in FP32 staging copies like the other narrow C tiles,
    then stored block by block along the rows of the tile.  Small integers (|x| <= 3 fits both
    element formats at every block maximum) must come back exactly, old C included; general data
    must match the oracle's stored result per tile, and what the GPU stored must be a fixed point
    of the oracle's block quantisation."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(97)
    for nb, MT, NT, KT, cut in ((128, 2, 3, 2, (0, 0, 0)), (512, 2, 2, 2, (0, 0, 0)), (128, 3, 2, 2, (37, 101, 64))):
        M, N, K = MT * nb, NT * nb, KT * nb
        _say("block-scaled C tiles, integers:", (M, N, K, nb), "cut", cut)
        A = np.zeros((M, K))
        B = np.zeros((K, N))
        A[np.arange(M), rng.integers(0, K, M)] = rng.integers(-1, 2, M)          # one entry per row: A @ B in {-1, 0, 1}
        B[:] = rng.integers(-1, 2, (K, N))
        C0 = rng.integers(-1, 2, (M, N)).astype(np.float64)
        M, N, K = M - cut[0], N - cut[1], K - cut[2]
        A, B, C0 = A[:M, :K], B[:K, :N], C0[:M, :N]
        mA = rng.integers(0, 8, (MT, KT)).astype(np.uint16)
        mB = rng.integers(0, 8, (KT, NT)).astype(np.uint16)
        mC = rng.integers(0, 8, (MT, NT)).astype(np.uint16)
        mC[0, 0], mC[MT - 1, NT - 1], mC[0, 1] = MXFP8, MXFP4, MXFP6
        if nb == 512:
            mA[0, :], mB[:, 0], mA[1, :], mB[:, 1] = MXFP8, MXFP8, MXFP4, MXFP4   # C(0,0), C(1,1) on the block-scaled kernel
        want = (A.astype(np.int64) @ B.astype(np.int64)) + 2 * C0.astype(np.int64)
        assert np.abs(want).max() <= 3
        d = DeviceGemmMP(M, N, K, nb)
        for k, m in (("A", mA), ("B", mB), ("C", mC)):
            d.set_precision_map(k, m)
        d.pack_tiles("A", _even_ld(A))
        d.pack_tiles("B", _even_ld(B))
        d.pack_tiles("C", _even_ld(C0))
        assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), C0)
        d.convert_tiles()
        d.run(1.0, 2.0)
        assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), want.astype(np.float64))
        d.run(0.0, 1.0)
        assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), want.astype(np.float64))
        d.run(0.0, -1.0)
        assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), -want.astype(np.float64))
        torch.cuda.synchronize()

    w = W.tiny()
    w.mapC = rng.integers(0, 8, w.mapC.shape).astype(np.uint16)
    w.mapC[0, :4] = (MXFP8, MXFP4, MXFP6, MXFP8)
    w.alpha, w.beta = 0.75, -1.25
    _say("block-scaled C tiles, general data")
    A, B, C0 = _dense(w)
    side = OracleSide(w, A, B, C0)
    d, dev = gpu_problem(w, A, B, C0)
    d.run(w.alpha, w.beta)
    C_gpu = d.unpack_tiles("C").cpu().numpy()
    torch.cuda.synchronize()
    jobs = _all_jobs(w)
    C_orc, _ = finish_low_c_tiles(side, side.gemm(jobs))
    worst = compare_jobs(side, jobs, 0, w.alpha, w.beta, C_gpu, C_orc)
    _say("  worst error / bound:", worst)
    again, _ = finish_low_c_tiles(side, C_gpu)
    for I in range(w.MT):
        for J in range(w.NT):
            if w.mapC[I, J] in (MXFP8, MXFP4, MXFP6):
                blk = (slice(I * w.nb, (I + 1) * w.nb), slice(J * w.nb, (J + 1) * w.nb))
                assert np.array_equal(again[blk], C_gpu[blk])
                assert d.ctx.tile_info("C", I, J)[2] == 0


def test_c_map_from_the_norm_rule_with_all_formats_and_sender_side_conversion():
    """C's own map made by the norm rule over all four formats from the old C (whose tiles decay
    away from the diagonal, so the rule picks every format), A and B likewise, operands converted
    once on the sender side, beta at work: the map and the packed old C must be the oracle's bit
    for bit, the result within tolerance, and equal to the receiver-side result bit for bit."""
    import torch
    w = W.tiny()
    w.alpha, w.beta = 1.0, 0.5
    w.rule = dict(eps=1e-4, allowed=orc.ALL_PRECISIONS_MASK)
    A, B, C0 = _dense(w)
    sc, mc = orc.tile_scan(C0, w.nb)
    w.mapC = orc.precision_rule(sc, w.rule["eps"], w.rule["allowed"])
    assert len(set(w.mapC.ravel().tolist())) >= 3, w.mapC
    side = OracleSide(w, A, B, C0)
    results = []
    for sender in (False, True):
        d, dev = gpu_problem(w, A, B, None)
        assert np.array_equal(d.maps["A"], side.mapA) and np.array_equal(d.maps["B"], side.mapB)
        got_map = d.compute_precision_map("C", torch.from_numpy(C0).cuda(), w.rule["eps"], w.rule["allowed"])
        assert np.array_equal(got_map, w.mapC)
        d.pack_tiles("C", torch.from_numpy(C0).cuda())
        assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), side.Cy)
        if sender:
            assert d.convert_tiles() > 0
        d.run(w.alpha, w.beta)
        results.append(d.unpack_tiles("C").cpu().numpy())
        torch.cuda.synchronize()
    assert np.array_equal(results[0], results[1])
    jobs = _all_jobs(w)
    C_orc, _ = finish_low_c_tiles(side, side.gemm(jobs))
    worst = compare_jobs(side, jobs, 0, w.alpha, w.beta, results[0], C_orc)
    _say("  worst error / bound:", worst)


def test_bf16_tiles_pack_bit_for_bit_and_the_rule_ranks_them_between_fp16_and_fp8():
    """BF16 storage: packed codes equal the oracle's single rounding from FP64 (values spread over
    FP32's whole range, ties, subnormals, overflow to infinity), A row-major and B transposed;
    unpack returns the stored values; the norm rule over all five formats gives the oracle's map."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(55)
    nb, T = 128, 2
    n = nb * T
    X = rng.standard_normal((n, n)) * np.exp(rng.uniform(-80, 80, (n, n)))
    X[0, :8] = [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -40, 3.4e38, -3.4e38, 1e-40, 2.0 ** -134, 0.0]
    d = DeviceGemmMP(n, n, n, nb)
    pm = np.full((T, T), BF16, dtype=np.uint16)
    dX = torch.from_numpy(X).cuda()
    Y, bits = orc.round_bf16(X)
    for which in ("A", "B"):
        d.set_precision_map(which, pm)
        d.pack_tiles(which, dX)
        for I in range(T):
            for J in range(T):
                got, prec = d.tile_bytes(which, I, J)
                tile = bits[I * nb:(I + 1) * nb, J * nb:(J + 1) * nb]
                want = np.ascontiguousarray(tile.T if which == "B" else tile).view(np.uint8).ravel()
                assert prec == BF16 and np.array_equal(got, want)
                assert d.ctx.tile_info(which, I, J)[2] == 0
        U = d.unpack_tiles(which).cpu().numpy()
        assert np.array_equal(U, Y)
    # the rule: decaying tiles, every format allowed
    w = W.tiny()
    A = w.dense("A")
    sa, _ = orc.tile_scan(A, w.nb)
    for eps in (1e-2, 1e-4, 1e-6):
        want = orc.precision_rule(sa, eps, orc.ALL_FORMATS_MASK)
        d2 = DeviceGemmMP(w.M, w.N, w.K, w.nb)
        got = d2.compute_precision_map("A", torch.from_numpy(A).cuda(), eps, orc.ALL_FORMATS_MASK)
        assert np.array_equal(got, want)
    assert BF16 in set(orc.precision_rule(sa, 1e-4, orc.ALL_FORMATS_MASK).ravel().tolist())
    torch.cuda.synchronize()


def test_bf16_tiles_small_integer_problems_are_exact():
    """Maps over all five formats on A and B, C tiles FP64 / FP32 / BF16 / FP16 / FP8, both policies.
    BF16 tiles under an FP32 / FP64 product need the sender-side copies (the call order error says
    so); every result must be the exact integer matrix: BF16 products on the BF16 matrix
    instruction, with an FP8 operand converted in the ring (receiver side) or taken as a BF16 copy
    (sender side), BF16 tiles widened to FP32 / FP64 copies, a BF16 C tile rounded from its FP32
    staging copy."""
    import torch
    from paper_2508_14848_amd import gemm_mp as G
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(56)
    for case in range(24):
        nb = int(rng.choice([128, 256]))
        MT, NT, KT = int(rng.integers(1, 4)), int(rng.integers(1, 4)), int(rng.integers(1, 5))
        M, N, K = MT * nb, NT * nb, KT * nb
        A = np.zeros((M, K))
        B = np.zeros((K, N))
        cols = rng.integers(0, nb, (M, KT)) + nb * np.arange(KT)
        A[np.arange(M)[:, None], cols] = rng.integers(-2, 3, (M, KT))
        rows = rng.integers(0, nb, (KT, N)) + nb * np.arange(KT)[:, None]
        B[rows, np.arange(N)[None, :]] = rng.integers(-1, 2, (KT, N))
        C0 = rng.integers(-3, 4, (M, N)).astype(np.float64)
        style = case % 3
        if style == 0:                                   # anything
            mA, mB = rng.integers(0, 5, (MT, KT)), rng.integers(0, 5, (KT, NT))
        elif style == 1:                                 # BF16 and FP8 only: BF16 and FP8 products
            mA, mB = rng.choice([BF16, FP8], (MT, KT)), rng.choice([BF16, FP8], (KT, NT))
        else:                                            # all BF16: no copies needed
            mA, mB = np.full((MT, KT), BF16), np.full((KT, NT), BF16)
        mC = rng.integers(0, 5, (MT, NT))
        policy = case % 2
        what = dict(case=case, nb=nb, MT=MT, NT=NT, KT=KT, style=style, policy=policy)
        if case % 6 == 0:
            _say("BF16 integers", what)
        want = 2 * (A.astype(np.int64) @ B.astype(np.int64)) - C0.astype(np.int64)
        assert np.abs(want).max() <= 15
        d = DeviceGemmMP(M, N, K, nb, policy=policy)
        for which, m, X in (("A", mA, A), ("B", mB, B), ("C", mC, C0)):
            d.set_precision_map(which, m.astype(np.uint16))
            d.pack_tiles(which, torch.from_numpy(X).cuda())
        need = d.ctx.conversion_bytes()
        if style == 2 and policy == 0:
            assert need == 0
        if need:
            # receiver-side first (BF16 tiles under FP32 / FP64 products are widened by the consumer),
            # then the same from sender-side copies: both strategies must agree
            d.run(2.0, -1.0)
            assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), want.astype(np.float64)), what
            d.pack_tiles("C", torch.from_numpy(C0).cuda())
            d.convert_tiles()
        d.run(2.0, -1.0)
        got = d.unpack_tiles("C").cpu().numpy()
        assert np.array_equal(got, want.astype(np.float64)), what
        torch.cuda.synchronize()


def test_random_small_integer_problems_over_all_formats_are_exact():
    """A hundred seeded problems with every format on A, B (MXFP8 included) and C (FP16 / FP8 /
    BF16 C tiles included), sizes on and off the tile grid, operands given directly or transposed, both
    policies, copies made on the sender side where a BF16 or MXFP8 tile needs them or at random.  One
    nonzero per row of A and per column of B inside each reduction tile keeps every result an
    integer of magnitude at most 15, which every format holds, so C must be exact."""
    import torch
    from paper_2508_14848_amd import gemm_mp as G
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(20250815)
    for case in range(100):
        nb = int(rng.choice([128, 256, 384, 512]))
        MT, NT, KT = int(rng.integers(1, 4)), int(rng.integers(1, 4)), int(rng.integers(1, 5))
        Mf, Nf, Kf = MT * nb, NT * nb, KT * nb
        A = np.zeros((Mf, Kf))
        B = np.zeros((Kf, Nf))
        cols = rng.integers(0, nb, (Mf, KT)) + nb * np.arange(KT)
        A[np.arange(Mf)[:, None], cols] = rng.integers(-2, 3, (Mf, KT))
        rows = rng.integers(0, nb, (KT, Nf)) + nb * np.arange(KT)[:, None]
        B[rows, np.arange(Nf)[None, :]] = rng.integers(-1, 2, (KT, Nf))
        ragged = rng.random() < 0.3
        M = Mf - (int(rng.integers(1, nb)) if ragged else 0)
        N = Nf - (int(rng.integers(1, nb)) if ragged else 0)
        K = Kf - (int(rng.integers(1, nb)) if ragged else 0)
        A, B = np.ascontiguousarray(A[:M, :K]), np.ascontiguousarray(B[:K, :N])
        C0 = rng.integers(-3, 4, (M, N)).astype(np.float64)
        mA, mB, mC = rng.integers(0, 8, (MT, KT)), rng.integers(0, 8, (KT, NT)), rng.integers(0, 5, (MT, NT))
        if case % 10 == 3:                               # one block-scaled format everywhere: its kernel where the tile size allows
            mA[:], mB[:] = ((MXFP8, MXFP8), (MXFP4, MXFP4), (MXFP6, MXFP6))[(case // 10) % 3]
            mC[:] = rng.integers(1, 5, (MT, NT))
        policy, tA, tB = int(rng.integers(0, 2)), int(rng.integers(0, 2)), int(rng.integers(0, 2))
        alpha, beta = float(rng.choice([-2, -1, 1, 2])), float(rng.choice([-1, 0, 1]))
        what = dict(case=case, nb=nb, M=M, N=N, K=K, policy=policy, tA=tA, tB=tB, alpha=alpha, beta=beta)
        if case % 20 == 0:
            _say("all formats, random integers", what)
        want = alpha * (A @ B) + beta * C0
        assert np.abs(want).max() <= 15
        d = DeviceGemmMP(M, N, K, nb, policy=policy)
        d.set_transposed("A", tA)
        d.set_transposed("B", tB)
        for which, m, X, t in (("A", mA, A, tA), ("B", mB, B, tB), ("C", mC, C0, 0)):
            d.set_precision_map(which, m.astype(np.uint16))
            d.pack_tiles(which, _even_ld(np.ascontiguousarray(X.T) if t else X))
        sender = rng.random() < 0.3
        if sender and d.ctx.conversion_bytes():
            d.convert_tiles()
        d.run(alpha, beta)                             # no format asks for copies: every tile is widened by its consumer
        got = d.unpack_tiles("C").cpu().numpy()
        assert np.array_equal(got, want), what
    torch.cuda.synchronize()


def test_256_regions_visit_every_chunk_once_at_tile_sizes_with_six_and_eight_chunks():
    """The 256 x 256 kernels start each region's pass over a product's chunks at a chunk of its
    own.  Integer problems (exact whatever the order of the additions) with block-wise different
    magnitudes, at tile sizes where a product has six or eight chunks so that every starting chunk
    and the wrap-around occur, over two products so that the scales of the next product are
    fetched across the boundary: FP8, MXFP8 and MXFP4 tiles, C in FP32 with the old C at work."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(131)
    # the block-scaled kernels have two instances: up to tile size 1024 the scale bytes travel through
    # LDS, two buffers used in turn from product to product (three products: every buffer is reused;
    # 256 / 512: a product is a single chunk pair), above it they are loaded from global memory
    cases = ((FP8, 768, 2), (FP8, 1024, 2), (MXFP8, 768, 2), (MXFP8, 1024, 2), (MXFP4, 1536, 2), (MXFP4, 2048, 2), (MXFP6, 768, 2),
             (MXFP6, 1024, 2), (MXFP8, 256, 3), (MXFP6, 256, 3), (MXFP4, 512, 3), (MXFP4, 1024, 3), (MXFP8, 1280, 2), (MXFP6, 1280, 2))
    for fmt, nb, kt in cases:
        M, N, K = nb, nb, kt * nb
        _say("256 x 256 regions, integers:", {FP8: "FP8", MXFP8: "MXFP8", MXFP4: "MXFP4", MXFP6: "MXFP6"}[fmt], (M, N, K, nb))
        if fmt == FP8:                                   # one scale per tile: the same magnitude everywhere
            A = rng.integers(-3, 4, (M, K)).astype(np.float64)
            B = rng.integers(-3, 4, (K, N)).astype(np.float64)
        else:
            A = rng.integers(-3, 4, (M, K)) * 2.0 ** rng.integers(0, 3, (M, K // 32)).repeat(32, axis=1)
            B = rng.integers(-3, 4, (K, N)) * 2.0 ** rng.integers(0, 3, (K // 32, N)).repeat(32, axis=0)
        C0 = rng.integers(-5, 6, (M, N)).astype(np.float64)
        d = DeviceGemmMP(M, N, K, nb)
        d.set_precision_map("A", np.full((1, kt), fmt, dtype=np.uint16))
        d.set_precision_map("B", np.full((kt, 1), fmt, dtype=np.uint16))
        d.set_precision_map("C", np.full((1, 1), FP32, dtype=np.uint16))
        for which, X in (("A", A), ("B", B), ("C", C0)):
            d.pack_tiles(which, torch.from_numpy(np.ascontiguousarray(X)).cuda())
        assert np.array_equal(d.unpack_tiles("A").cpu().numpy(), A) and np.array_equal(d.unpack_tiles("B").cpu().numpy(), B)
        assert d.ctx.get_stats()["work_items"] == (nb // 256) ** 2          # the 256 x 256 kernel
        d.run(1.0, -1.0)
        assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), A @ B - C0)
        torch.cuda.synchronize()


def test_owner_regions_in_blocks_of_four_by_eight_cover_a_tile_once():
    """Where a tile has more than eight columns of 128 x 128 regions the schedule hands them out in
    blocks of 4 x 8 (what an XCD works on at a time) instead of row by row.  Integer problems (exact)
    at tile sizes 2048 and 3072 (16 and 24 region columns), one FP64 and one FP32 C tile side by
    side, C poisoned beforehand: a region left out or visited twice shows."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(977)
    for nb in (2048, 3072):
        M, N, K = nb, 2 * nb, nb
        _say("owner regions in 4 x 8 blocks:", (M, N, K, nb))
        A = rng.integers(-3, 4, (M, K)).astype(np.float64)
        B = rng.integers(-3, 4, (K, N)).astype(np.float64)
        d = DeviceGemmMP(M, N, K, nb)
        d.set_precision_map("A", np.full((1, 1), FP32, dtype=np.uint16))
        d.set_precision_map("B", np.full((1, 2), FP32, dtype=np.uint16))
        d.set_precision_map("C", np.array([[FP64, FP32]], dtype=np.uint16))
        d.pack_tiles("A", torch.from_numpy(A).cuda())
        d.pack_tiles("B", torch.from_numpy(B).cuda())
        d.pack_tiles("C", torch.full((M, N), float("nan"), dtype=torch.float64, device="cuda"))
        assert d.ctx.get_stats()["work_items"] == 2 * (nb // 128) ** 2
        d.run(1.0, 0.0)
        assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), A @ B)
        torch.cuda.synchronize()


def test_mxfp8_tiles_pack_bit_for_bit_and_multiply_on_the_block_scaled_instruction():
    """MXFP8 tiles: element and scale bytes equal the oracle's block quantisation (blocks along the
    rows of A tiles and down the columns of B tiles, i.e. along the reduction index; a size off
    the tile grid included), unpack returns the values they stand for; all-MXFP8 products of small
    integers are exact through the block-scaled matrix instruction (scales differ from block to
    block by construction), and general data stays within the per-tile bounds of the oracle."""
    import torch
    from paper_2508_14848_amd import gemm_mp as G
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(61)
    # storage
    nb = 256
    M, N, K = 2 * nb, 2 * nb - 70, 3 * nb - 33
    A = rng.standard_normal((M, K)) * np.exp(rng.uniform(-30, 30, (M, K)))
    B = rng.standard_normal((K, N)) * np.exp(rng.uniform(-30, 30, (K, N)))
    A[5, 64:96] = 0.0                                            # a zero block
    d = DeviceGemmMP(M, N, K, nb)
    d.set_precision_map("A", np.full((2, 3), MXFP8, dtype=np.uint16))
    d.set_precision_map("B", np.full((3, 2), MXFP8, dtype=np.uint16))
    d.pack_tiles("A", _even_ld(A))
    d.pack_tiles("B", _even_ld(B))
    Ap, Bp = orc.pad_to_tiles(A, nb), orc.pad_to_tiles(B, nb)
    for which, Xp, tiles in (("A", Ap, [(0, 0), (1, 2)]), ("B", Bp, [(0, 0), (2, 1)])):
        for (I, J) in tiles:
            got, prec = d.tile_bytes(which, I, J)
            tile = Xp[I * nb:(I + 1) * nb, J * nb:(J + 1) * nb]
            rows = np.ascontiguousarray(tile.T if which == "B" else tile)        # packed rows: the reduction index runs along them
            _, codes, scales = orc.mx_blocks(rows)
            assert prec == MXFP8
            assert np.array_equal(got[:nb * nb], codes.ravel()), (which, I, J)
            assert np.array_equal(got[nb * nb:], scales), (which, I, J)
    Ya, _ = orc.store_tiles(Ap, nb, np.full((2, 3), MXFP8, dtype=np.uint16), mx_axis=0)
    Yb, _ = orc.store_tiles(Bp, nb, np.full((3, 2), MXFP8, dtype=np.uint16), mx_axis=1)
    assert np.array_equal(d.unpack_tiles("A").cpu().numpy(), Ya[:M, :K])
    assert np.array_equal(d.unpack_tiles("B").cpu().numpy(), Yb[:K, :N])
    # outside the block-scaled kernel (here: FP64 C tiles) the consumer widens the tiles on the fly;
    # from sender-side copies the result is the same bit for bit
    d.set_precision_map("C", np.full((2, 2), FP64, dtype=np.uint16))
    d.run(1.0, 0.0)
    C_receiver = d.unpack_tiles("C").cpu().numpy()
    assert d.convert_tiles() == (6 + 6) * nb * nb * 4            # an FP32 copy of every MXFP8 tile
    d.run(1.0, 0.0)
    assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), C_receiver)
    Cg = np.zeros((2 * nb, 2 * nb))
    Cg[:M, :N] = C_receiver
    w = W.Workload("mx64", 2 * nb, 2 * nb, 3 * nb, nb, 1.0, 0.0)
    w.mapA, w.mapB = np.full((2, 3), MXFP8, dtype=np.uint16), np.full((3, 2), MXFP8, dtype=np.uint16)
    w.mapC = np.full((2, 2), FP64, dtype=np.uint16)
    side = OracleSide(w, Ap, Bp, None)
    jobs = _all_jobs(w)
    compare_jobs(side, jobs, 0, 1.0, 0.0, Cg, side.gemm(jobs, alpha=1.0, beta=0.0))
    # integers: exact; every block gets its own scale from a different largest entry
    for nb, MT, NT, KT in ((256, 2, 1, 3), (512, 1, 2, 2)):
        M, N, K = MT * nb, NT * nb, KT * nb
        _say("MXFP8 integers", (M, N, K, nb))
        mag = 2.0 ** rng.integers(0, 3, (M, K // 32)).repeat(32, axis=1)         # 1, 2 or 4 per block of A's rows
        A = rng.integers(-3, 4, (M, K)) * mag
        magb = 2.0 ** rng.integers(0, 3, (K // 32, N)).repeat(32, axis=0)
        B = rng.integers(-3, 4, (K, N)) * magb
        C0 = rng.integers(-5, 6, (M, N)).astype(np.float64)
        for pC in (FP32, FP16 if nb == 256 else BF16):
            d = DeviceGemmMP(M, N, K, nb)
            d.set_precision_map("A", np.full((MT, KT), MXFP8, dtype=np.uint16))
            d.set_precision_map("B", np.full((KT, NT), MXFP8, dtype=np.uint16))
            d.set_precision_map("C", np.full((MT, NT), pC, dtype=np.uint16))
            for which, X in (("A", A), ("B", B), ("C", C0)):
                d.pack_tiles(which, torch.from_numpy(np.ascontiguousarray(X, dtype=np.float64)).cuda())
            assert np.array_equal(d.unpack_tiles("A").cpu().numpy(), A) and np.array_equal(d.unpack_tiles("B").cpu().numpy(), B)
            st = d.ctx.get_stats()
            assert st["products_mxfp8"] == MT * NT * KT and st["work_items"] == MT * NT * (nb // 256) ** 2
            if pC == FP32:
                d.run(1.0, -1.0)
                want = A @ B - C0
                assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), want)
            else:                                      # a low-precision C tile cannot hold these sums exactly
                d.run(1.0, 0.0)
                want = A @ B
                got = d.unpack_tiles("C").cpu().numpy()
                assert np.abs(got - want).max() <= (2.0 ** -11 if pC == FP16 else 2.0 ** -8) * np.abs(want).max()
    # general data against the oracle
    w = W.tiny()
    w.mapA = np.full_like(w.mapA, MXFP8)
    w.mapB = np.full_like(w.mapB, MXFP8)
    w.mapC = np.full_like(w.mapC, FP32)
    w.alpha, w.beta = 1.0, 0.0
    A, B, _ = _dense(w)
    side = OracleSide(w, A, B, None)
    d, dev = gpu_problem(w, A, B, None)
    assert np.array_equal(d.unpack_tiles("A").cpu().numpy(), side.Ay) and np.array_equal(d.unpack_tiles("B").cpu().numpy(), side.By)
    d.run(1.0, 0.0)
    C_gpu = d.unpack_tiles("C").cpu().numpy()
    jobs = _all_jobs(w)
    worst = compare_jobs(side, jobs, 0, 1.0, 0.0, C_gpu, side.gemm(jobs))
    _say("  worst error / bound:", worst)
    torch.cuda.synchronize()


def _fp6_bytes(codes, nb):
    """The element bytes of an MXFP6 tile from its six-bit codes (nb packed rows of nb codes), as the
    interface describes them: four codes to three bytes, code k of a group in bits 6k .. 6k+5 of the
    group's 24; the tile stored panel by panel of 128 reduction indices, row after row inside a
    panel, the blocks of 32 inside a row of a panel rotated by (row // 8)."""
    c = codes.reshape(nb, nb // 4, 4).astype(np.uint32)
    w = c[:, :, 0] | (c[:, :, 1] << 6) | (c[:, :, 2] << 12) | (c[:, :, 3] << 18)
    groups = np.stack([w & 255, (w >> 8) & 255, (w >> 16) & 255], axis=2).astype(np.uint8)      # [row][group of 4][3]
    out = np.zeros(nb * nb * 3 // 4, dtype=np.uint8)
    for p0 in range(0, nb, 128):
        width = min(128, nb - p0)
        nblk = width // 32
        for r in range(nb):
            for b in range(nblk):
                at = (p0 // 128) * nb * 96 + r * (width * 3 // 4) + ((b + r // 8) % nblk) * 24
                g0 = (p0 + 32 * b) // 4
                out[at:at + 24] = groups[r, g0:g0 + 8].ravel()
    return out


def test_mxfp6_tiles_pack_bit_for_bit_and_multiply_on_the_block_scaled_instruction():
    """MXFP6 tiles: six-bit e2m3 codes (a block of 32 in 24 bytes, code k at bits 6k .. 6k+5) and
    scale bytes equal the oracle's, both orientations, a size off the tile grid included; unpack
    returns the values; under FP64 C tiles the consumer widens them, with the same result as
    sender-side copies and within the oracle's bounds; all-MXFP6 problems of small integers with
    block-wise different magnitudes are exact on the block-scaled instruction, with FP32 and with
    narrow C tiles; general data within the bounds."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(63)
    nb = 256
    M, N, K = 2 * nb, 2 * nb - 50, 3 * nb - 31
    A = rng.standard_normal((M, K)) * np.exp(rng.uniform(-20, 20, (M, K)))
    B = rng.standard_normal((K, N)) * np.exp(rng.uniform(-20, 20, (K, N)))
    A[7, 32:64] = 0.0                                            # a zero block
    d = DeviceGemmMP(M, N, K, nb)
    d.set_precision_map("A", np.full((2, 3), MXFP6, dtype=np.uint16))
    d.set_precision_map("B", np.full((3, 2), MXFP6, dtype=np.uint16))
    d.pack_tiles("A", _even_ld(A))
    d.pack_tiles("B", _even_ld(B))
    Ap, Bp = orc.pad_to_tiles(A, nb), orc.pad_to_tiles(B, nb)
    for which, Xp, tiles in (("A", Ap, [(0, 0), (1, 2)]), ("B", Bp, [(0, 0), (2, 1)])):
        for (I, J) in tiles:
            got, prec = d.tile_bytes(which, I, J)
            tile = Xp[I * nb:(I + 1) * nb, J * nb:(J + 1) * nb]
            rows = np.ascontiguousarray(tile.T if which == "B" else tile)
            _, codes, scales = orc.mx6_blocks(rows)
            assert prec == MXFP6 and got.size == nb * nb * 3 // 4 + nb * nb // 32
            assert np.array_equal(got[:nb * nb * 3 // 4], _fp6_bytes(codes, nb)), (which, I, J)
            assert np.array_equal(got[nb * nb * 3 // 4:], scales), (which, I, J)
    Ya, _ = orc.store_tiles(Ap, nb, np.full((2, 3), MXFP6, dtype=np.uint16), mx_axis=0)
    Yb, _ = orc.store_tiles(Bp, nb, np.full((3, 2), MXFP6, dtype=np.uint16), mx_axis=1)
    assert np.array_equal(d.unpack_tiles("A").cpu().numpy(), Ya[:M, :K])
    assert np.array_equal(d.unpack_tiles("B").cpu().numpy(), Yb[:K, :N])
    # FP64 C tiles: no block-scaled kernel; the consumer widens the tiles (FP32 products folded into
    # FP64), and sender-side copies give the same bits
    d.set_precision_map("C", np.full((2, 2), FP64, dtype=np.uint16))
    d.run(1.0, 0.0)
    C_receiver = d.unpack_tiles("C").cpu().numpy()
    assert d.convert_tiles() == (6 + 6) * nb * nb * 4
    d.run(1.0, 0.0)
    assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), C_receiver)
    Cg = np.zeros((2 * nb, 2 * nb))
    Cg[:M, :N] = C_receiver
    w = W.Workload("mx6-64", 2 * nb, 2 * nb, 3 * nb, nb, 1.0, 0.0)
    w.mapA, w.mapB = np.full((2, 3), MXFP6, dtype=np.uint16), np.full((3, 2), MXFP6, dtype=np.uint16)
    w.mapC = np.full((2, 2), FP64, dtype=np.uint16)
    side = OracleSide(w, Ap, Bp, None)
    jobs = _all_jobs(w)
    compare_jobs(side, jobs, 0, 1.0, 0.0, Cg, side.gemm(jobs, alpha=1.0, beta=0.0))
    # ... and beside FP64 / FP32 tiles (FP64 and FP32 products with one MXFP6 operand)
    for other in (FP64, FP32):
        w2 = W.Workload("mx6-mixed", 2 * nb, 2 * nb, 3 * nb, nb, 1.0, 0.0)
        w2.mapA = np.full((2, 3), MXFP6, dtype=np.uint16)
        w2.mapB = np.full((3, 2), other, dtype=np.uint16)
        w2.mapA[1, 1], w2.mapB[0, 1] = other, MXFP6
        w2.mapC = np.array([[FP64, FP32], [FP32, FP64]], dtype=np.uint16)
        A2 = rng.standard_normal((2 * nb, 3 * nb))
        B2 = rng.standard_normal((3 * nb, 2 * nb))
        side2 = OracleSide(w2, A2, B2, None)
        d2, _ = gpu_problem(w2, A2, B2, None)
        d2.run(1.0, 0.0)
        jobs2 = _all_jobs(w2)
        compare_jobs(side2, jobs2, 0, 1.0, 0.0, d2.unpack_tiles("C").cpu().numpy(), side2.gemm(jobs2, alpha=1.0, beta=0.0))
    # integers: exact; every block gets its own scale from a different largest entry
    for nb, MT, NT, KT in ((256, 2, 1, 3), (512, 1, 2, 2)):
        M, N, K = MT * nb, NT * nb, KT * nb
        _say("MXFP6 integers", (M, N, K, nb))
        A = rng.integers(-7, 8, (M, K)) * 2.0 ** rng.integers(0, 3, (M, K // 32)).repeat(32, axis=1)
        B = rng.integers(-7, 8, (K, N)) * 2.0 ** rng.integers(0, 3, (K // 32, N)).repeat(32, axis=0)
        C0 = rng.integers(-5, 6, (M, N)).astype(np.float64)
        for pC in (FP32, FP16 if nb == 256 else MXFP6):
            d = DeviceGemmMP(M, N, K, nb)
            d.set_precision_map("A", np.full((MT, KT), MXFP6, dtype=np.uint16))
            d.set_precision_map("B", np.full((KT, NT), MXFP6, dtype=np.uint16))
            d.set_precision_map("C", np.full((MT, NT), pC, dtype=np.uint16))
            for which, X in (("A", A), ("B", B), ("C", C0)):
                d.pack_tiles(which, torch.from_numpy(np.ascontiguousarray(X, dtype=np.float64)).cuda())
            assert np.array_equal(d.unpack_tiles("A").cpu().numpy(), A) and np.array_equal(d.unpack_tiles("B").cpu().numpy(), B)
            st = d.ctx.get_stats()
            assert st["products_mxfp6"] == MT * NT * KT and st["work_items"] == MT * NT * (nb // 256) ** 2
            assert st["launch_items"][7] == st["work_items"] and d.ctx.conversion_bytes() == 0
            if pC == FP32:
                d.run(1.0, -1.0)
                assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), A @ B - C0)
            else:                                      # a narrow C tile cannot hold these sums exactly
                d.run(1.0, 0.0)
                want = A @ B
                got = d.unpack_tiles("C").cpu().numpy()
                if pC == FP16:
                    assert np.abs(got - want).max() <= 2.0 ** -11 * np.abs(want).max()
                else:                                  # each block of 32 along a row is rounded relative to its own largest entry
                    top = np.abs(want).reshape(M, -1, 32).max(axis=2).repeat(32, axis=1)
                    assert np.all(np.abs(got - want) <= 2.0 ** -3 * top)
                    assert np.abs(got - want).max() > 0
    # general data against the oracle (the block-scaled kernel)
    w = W.tiny()
    w.mapA = np.full_like(w.mapA, MXFP6)
    w.mapB = np.full_like(w.mapB, MXFP6)
    w.mapC = np.full_like(w.mapC, FP32)
    w.alpha, w.beta = 1.0, 0.0
    A, B, _ = _dense(w)
    side = OracleSide(w, A, B, None)
    d, dev = gpu_problem(w, A, B, None)
    assert np.array_equal(d.unpack_tiles("A").cpu().numpy(), side.Ay) and np.array_equal(d.unpack_tiles("B").cpu().numpy(), side.By)
    assert d.ctx.get_stats()["launch_items"][7] > 0
    d.run(1.0, 0.0)
    C_gpu = d.unpack_tiles("C").cpu().numpy()
    jobs = _all_jobs(w)
    worst = compare_jobs(side, jobs, 0, 1.0, 0.0, C_gpu, side.gemm(jobs))
    _say("  worst error / bound:", worst)
    torch.cuda.synchronize()


def test_mxfp4_tiles_pack_bit_for_bit_and_multiply_on_the_block_scaled_instruction():
    """MXFP4 tiles: four-bit e2m1 codes (two a byte, the lower reduction index in the low bits) and
    scale bytes equal the oracle's, both orientations; unpack returns the values; all-MXFP4
    problems of small integers with block-wise different magnitudes are exact on the block-scaled
    instruction (tile 512) and through FP32 copies (tile 256); general data within the bounds."""
    import torch
    from paper_2508_14848_amd import gemm_mp as G
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(62)
    nb = 256
    M, N, K = 2 * nb, nb - 50, 2 * nb - 31
    A = rng.standard_normal((M, K)) * np.exp(rng.uniform(-20, 20, (M, K)))
    B = rng.standard_normal((K, N)) * np.exp(rng.uniform(-20, 20, (K, N)))
    d = DeviceGemmMP(M, N, K, nb)
    d.set_precision_map("A", np.full((2, 2), MXFP4, dtype=np.uint16))
    d.set_precision_map("B", np.full((2, 1), MXFP4, dtype=np.uint16))
    d.pack_tiles("A", _even_ld(A))
    d.pack_tiles("B", _even_ld(B))
    Ap, Bp = orc.pad_to_tiles(A, nb), orc.pad_to_tiles(B, nb)
    for which, Xp, tiles in (("A", Ap, [(0, 0), (1, 1)]), ("B", Bp, [(0, 0), (1, 0)])):
        for (I, J) in tiles:
            got, prec = d.tile_bytes(which, I, J)
            tile = Xp[I * nb:(I + 1) * nb, J * nb:(J + 1) * nb]
            rows = np.ascontiguousarray(tile.T if which == "B" else tile)
            _, codes, scales = orc.mx4_blocks(rows)
            codes = codes.ravel()
            assert prec == MXFP4
            assert np.array_equal(got[:nb * nb // 2], codes[0::2] | (codes[1::2] << 4)), (which, I, J)
            assert np.array_equal(got[nb * nb // 2:], scales), (which, I, J)
    Ya, _ = orc.store_tiles(Ap, nb, np.full((2, 2), MXFP4, dtype=np.uint16), mx_axis=0)
    Yb, _ = orc.store_tiles(Bp, nb, np.full((2, 1), MXFP4, dtype=np.uint16), mx_axis=1)
    assert np.array_equal(d.unpack_tiles("A").cpu().numpy(), Ya[:M, :K])
    assert np.array_equal(d.unpack_tiles("B").cpu().numpy(), Yb[:K, :N])
    for nb, MT, NT, KT in ((512, 2, 1, 2), (1024, 1, 1, 1), (256, 1, 2, 2)):
        M, N, K = MT * nb, NT * nb, KT * nb
        _say("MXFP4 integers", (M, N, K, nb))
        A = rng.integers(-3, 4, (M, K)) * 2.0 ** rng.integers(0, 3, (M, K // 32)).repeat(32, axis=1)
        B = rng.integers(-3, 4, (K, N)) * 2.0 ** rng.integers(0, 3, (K // 32, N)).repeat(32, axis=0)
        C0 = rng.integers(-5, 6, (M, N)).astype(np.float64)
        d = DeviceGemmMP(M, N, K, nb)
        d.set_precision_map("A", np.full((MT, KT), MXFP4, dtype=np.uint16))
        d.set_precision_map("B", np.full((KT, NT), MXFP4, dtype=np.uint16))
        d.set_precision_map("C", np.full((MT, NT), FP32, dtype=np.uint16))
        for which, X in (("A", A), ("B", B), ("C", C0)):
            d.pack_tiles(which, torch.from_numpy(np.ascontiguousarray(X, dtype=np.float64)).cuda())
        assert np.array_equal(d.unpack_tiles("A").cpu().numpy(), A) and np.array_equal(d.unpack_tiles("B").cpu().numpy(), B)
        st = d.ctx.get_stats()
        assert st["products_mxfp4"] == MT * NT * KT
        if nb % 512 == 0:
            assert st["work_items"] == MT * NT * (nb // 256) ** 2 and d.ctx.conversion_bytes() == 0
        d.run(1.0, -1.0)                                 # tile 256: no block-scaled kernel, the tiles are widened on the fly
        assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), A @ B - C0)
        if nb % 512 != 0:
            d.pack_tiles("C", torch.from_numpy(C0).cuda())
            d.convert_tiles()                            # ... or read as sender-side copies: the same
            d.run(1.0, -1.0)
            assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), A @ B - C0)
    # general data against the oracle (tile 512: the block-scaled kernel)
    w = W.tiny(M=1024, N=1024, K=1024, nb=512)
    w.mapA = np.full((2, 2), MXFP4, dtype=np.uint16)
    w.mapB = np.full((2, 2), MXFP4, dtype=np.uint16)
    w.mapC = np.full((2, 2), FP32, dtype=np.uint16)
    w.alpha, w.beta = 1.0, 0.0
    A, B, _ = _dense(w)
    side = OracleSide(w, A, B, None)
    d, dev = gpu_problem(w, A, B, None)
    assert np.array_equal(d.unpack_tiles("A").cpu().numpy(), side.Ay) and np.array_equal(d.unpack_tiles("B").cpu().numpy(), side.By)
    d.run(1.0, 0.0)
    C_gpu = d.unpack_tiles("C").cpu().numpy()
    jobs = _all_jobs(w)
    worst = compare_jobs(side, jobs, 0, 1.0, 0.0, C_gpu, side.gemm(jobs))
    _say("  worst error / bound:", worst)
    torch.cuda.synchronize()


def test_bf16_products_match_the_oracle_on_general_data():
    """A and B all BF16 (no conversion anywhere: receiver-side run), C tiles of every kind: per
    tile within 4*K*u_tile with u = 2^-8, and within the FP32-accumulation bound of the oracle,
    whose BF16 products are exact FP32 multiplications of the stored operands."""
    import torch
    w = W.tiny()
    w.mapA = np.full_like(w.mapA, BF16)
    w.mapB = np.full_like(w.mapB, BF16)
    rng = np.random.default_rng(57)
    w.mapC = rng.integers(0, 5, w.mapC.shape).astype(np.uint16)
    w.mapC[0, :] = (FP64, FP32, BF16, FP8)
    w.alpha, w.beta = 1.0, 0.0
    A, B, C0 = _dense(w)
    side = OracleSide(w, A, B, None)
    d, dev = gpu_problem(w, A, B, None)
    _check_storage(d, side, "A", [(0, 0), (1, 2)])
    _check_storage(d, side, "B", [(0, 0), (2, 1)])
    assert d.ctx.get_stats()["products_bf16"] == w.MT * w.NT * w.KT
    d.run(w.alpha, w.beta)
    C_gpu = d.unpack_tiles("C").cpu().numpy()
    torch.cuda.synchronize()
    jobs = _all_jobs(w)
    C_orc, _ = finish_low_c_tiles(side, side.gemm(jobs))
    worst = compare_jobs(side, jobs, 0, w.alpha, w.beta, C_gpu, C_orc)
    _say("  worst error / bound:", worst)


@pytest.mark.parametrize("policy", [0, 1])
def test_mixed_maps_match_the_oracle_per_tile(policy):
    """All (pA, pB, pC) combinations occur; several owner regions per tile; alpha, beta general."""
    w = W.random_maps(M=512, N=768, K=1024, nb=256, probs=(0.25, 0.25, 0.25, 0.25), alpha=1.5, beta=0.5,
                      name="mixed-small")
    d, side, C_gpu, C_orc = _run_and_compare(w, policy=policy)
    # same problem again: the owner design makes the result bit-identical run to run
    import torch
    d.pack_tiles("C", torch.from_numpy(w.dense("C")).cuda())
    d.run(w.alpha, w.beta)
    again = d.unpack_tiles("C").cpu().numpy()
    assert np.array_equal(again, C_gpu)


def test_scaled_low_precision_tiles_with_wide_dynamic_range():
    """Tiles whose magnitudes differ by many orders: without the per-tile exponents FP16 / FP8
    tiles would flush to zero; C tiles FP32 and FP64."""
    w = W.tiny(M=512, N=512, K=1024, nb=128)
    w.mapA = (np.indices((w.MT, w.KT)).sum(0) % 3 + 1).astype(np.uint16)      # FP32 / FP16 / FP8
    w.mapB = (np.indices((w.KT, w.NT)).sum(0) % 2 + 2).astype(np.uint16)      # FP16 / FP8
    w.mapC = (np.indices((w.MT, w.NT)).sum(0) % 2).astype(np.uint16)
    _run_and_compare(w)


def test_beta_zero_does_not_read_c_and_alpha_zero_forms_no_product():
    import torch
    w = W.random_maps(M=256, N=256, K=512, nb=128, alpha=1.0, beta=0.0, name="conventions")
    A, B, _ = _dense(w)
    side = OracleSide(w, A, B, None)
    d, dev = gpu_problem(w, A, B, None)
    d.storage["C"].view(torch.float64)[:] = float("nan")          # poison: must never be read
    d.run(1.0, 0.0)
    C_gpu = d.unpack_tiles("C").cpu().numpy()
    jobs = _all_jobs(w)
    compare_jobs(side, jobs, 0, 1.0, 0.0, C_gpu, side.gemm(jobs, alpha=1.0, beta=0.0))
    # alpha == 0: C <- beta*C exactly, even with non-finite operands packed
    C0 = w.dense("C")
    A2 = A.copy()
    A2[3, 5] = np.inf
    d.pack_tiles("A", torch.from_numpy(A2).cuda())
    d.pack_tiles("C", torch.from_numpy(C0).cuda())
    d.run(0.0, 0.5)
    got = d.unpack_tiles("C").cpu().numpy()
    Cy, _ = orc.store_tiles(C0, w.nb, w.mapC)
    want = np.where(np.kron(w.mapC, np.ones((w.nb, w.nb))) == FP64, 0.5 * Cy,
                    (np.float32(0.5) * Cy.astype(np.float32)).astype(np.float64))
    assert np.array_equal(got, want)


def test_a_context_follows_new_maps_new_data_and_a_new_policy_between_runs():
    """The per-product table is rebuilt for every run: after the maps, the packed data (hence the
    scale exponents) or the policy change, the next run must match the oracle for the new state."""
    import torch
    w = W.random_maps(M=512, N=512, K=768, nb=128, probs=(0.25, 0.25, 0.25, 0.25), alpha=1.0, beta=0.0,
                      name="reuse")
    A, B, _ = _dense(w)
    d, _ = gpu_problem(w, A, B, None)
    jobs = _all_jobs(w)

    def check(policy):
        side = OracleSide(w, A, B, None)
        d.run(w.alpha, w.beta)
        C_gpu = d.unpack_tiles("C").cpu().numpy()
        C_orc = side.gemm(jobs, policy=policy)
        compare_jobs(side, jobs, policy, w.alpha, w.beta, C_gpu, C_orc)

    check(0)
    # new maps for A (transposed pattern) and data scaled by 2^-9 (all FP16/FP8 exponents move)
    w.mapA = np.ascontiguousarray(w.mapB.T[:w.MT, :w.KT]) if w.mapB.T.shape == w.mapA.shape else (3 - w.mapA)
    A = A * 2.0 ** -9
    d.set_precision_map("A", w.mapA)
    d.pack_tiles("A", torch.from_numpy(A).cuda())
    check(0)
    d.ctx.set_policy(1)
    check(1)


@pytest.mark.parametrize("policy", [0, 1])
def test_sender_side_conversion_gives_the_same_c_bit_for_bit(policy):
    """Converted copies hold exactly what the receiver-side path converts on the fly, so running
    from them must not change a single bit of C; they must also be dropped when A is repacked."""
    import torch
    w = W.random_maps(M=512, N=768, K=1024, nb=256, probs=(0.25, 0.25, 0.25, 0.25), alpha=1.5, beta=0.5,
                      name="sender-small")
    A, B, C0 = _dense(w)
    d, dev = gpu_problem(w, A, B, C0, policy=policy)
    d.run(w.alpha, w.beta)
    recv = d.unpack_tiles("C").cpu().numpy()
    d.pack_tiles("C", dev["C"])
    nbytes = d.convert_tiles()
    st = d.ctx.get_stats()
    assert st["converted_bytes"] == nbytes and (st["converted_tiles"] > 0) == (nbytes > 0)
    if policy == 0:
        assert nbytes > 0
    d.run(w.alpha, w.beta)
    send = d.unpack_tiles("C").cpu().numpy()
    assert np.array_equal(send, recv)
    side = OracleSide(w, A, B, C0)
    jobs = _all_jobs(w)
    compare_jobs(side, jobs, policy, w.alpha, w.beta, send, side.gemm(jobs, policy=policy))
    # new data for A: the copies are stale and must not be used
    A2 = A * 3.0
    d.pack_tiles("A", torch.from_numpy(A2).cuda())
    assert d.ctx.get_stats()["converted_tiles"] == 0
    d.pack_tiles("C", dev["C"])
    d.run(w.alpha, w.beta)
    got = d.unpack_tiles("C").cpu().numpy()
    side2 = OracleSide(w, A2, B, C0)
    compare_jobs(side2, jobs, policy, w.alpha, w.beta, got, side2.gemm(jobs, policy=policy))


def test_call_order_errors_on_the_device_path():
    import torch
    from paper_2508_14848_amd import gemm_mp as G
    from paper_2508_14848_amd.device import DeviceGemmMP
    d = DeviceGemmMP(256, 256, 256, 128)
    x = torch.zeros((256, 256), dtype=torch.float64, device="cuda")
    with pytest.raises(G.GemmMPError) as e:
        d.pack_tiles("A", x)
    assert e.value.status == G.ESTATE
    d.set_precision_map("A", np.zeros((2, 2), np.uint16))
    d.pack_tiles("A", x)
    with pytest.raises(G.GemmMPError) as e:
        d.run(1.0, 0.0)
    assert e.value.status == G.ESTATE
    with pytest.raises(G.GemmMPError) as e:
        d.ctx.pack_tiles("A", x.data_ptr() + 8, 256, None)        # misaligned dense pointer
    assert e.value.status == G.EINVAL


# ------------------------------------------------------------------------------------------
# The five configurations at full size.
def test_config_tiny_all_tiles():
    w = W.tiny()
    d, side, _, _ = _run_and_compare(w)
    assert d.ctx.get_stats()["products"] == [28, 26, 10, 0]


def test_config_random8k_all_tiles():
    w = W.random_maps()
    _run_and_compare(w, check_storage_tiles=3)


def test_config_cov16k_sampled_tiles():
    w = W.covariance()
    jobs = orc.whole_tile_jobs(w.nb, w.sample_tiles(64))
    d, side, _, _ = _run_and_compare(w, jobs=jobs, check_storage_tiles=2)
    _say("  products by precision:", d.ctx.get_stats()["products"])


def test_config_rect32k_sampled_tiles():
    w = W.decay_rect()
    jobs = orc.whole_tile_jobs(w.nb, w.sample_tiles(64))
    d, side, _, _ = _run_and_compare(w, jobs=jobs, check_storage_tiles=2)
    st = d.ctx.get_stats()
    _say("  products by precision:", st["products"])
    assert st["products"][0] == 0 and st["products"][3] > 0


@pytest.mark.parametrize("pct", [100, 80, 50, 20, 0])
def test_paper_ratio_runs_match_the_oracle(pct):
    """The paper's own experiment at a small size: aD:bS maps on A, B and C, every task at its C
    tile's precision (Section 5.2); all C tiles compared."""
    w = W.paper_ratio(pct, n=1024, nb=256)
    d, side, _, _ = _run_and_compare(w, policy=w.policy, check_storage_tiles=2)
    n64 = int((w.mapC == FP64).sum())
    assert d.ctx.get_stats()["products"] == [n64 * w.KT, (w.MT * w.NT - n64) * w.KT, 0, 0]


def test_config_cov64k_sampled_blocks():
    """The largest configuration (65536^3, 2048-wide tiles): 8 whole C tiles of the seeded sample
    and 16 rows of each of the 66 sampled tiles, the rows placed so that every one of the 16 rows
    of owner regions of a tile is met; per tile and per element."""
    w = W.CONFIGS["cov64k"]()
    tiles = sorted(set(w.sample_tiles(64)) | {(0, 0), (w.MT // 2, w.NT // 2 + 1)})
    rng = np.random.default_rng(11)
    jobs = [[I, J, 0, w.nb, 0, w.nb] for (I, J) in tiles[::len(tiles) // 8][:8]]
    for k, (I, J) in enumerate(tiles):
        r0 = (k % 16) * 128 + int(rng.integers(0, 128 - 16))
        jobs.append([I, J, r0, r0 + 16, 0, w.nb])
    assert {j[2] // 128 for j in jobs[8:]} == set(range(16))
    jobs = np.array(jobs, dtype=np.int32)
    d, side, _, _ = _run_and_compare(w, jobs=jobs, check_storage_tiles=2)
    st = d.ctx.get_stats()
    _say("  products by precision:", st["products"])
    assert (w.M // 256) * (w.N // 256) <= st["work_items"] <= (w.M // 128) * (w.N // 128)


def test_steady_state_calls_neither_allocate_nor_wait():
    """After the first pass over a shape, a loop of set map / pack / prepare / run makes no device
    or pinned allocation, and prepare and run make the host wait for nothing: the tables are
    composed in pinned memory and copied on the caller's stream."""
    import torch
    w = W.random_maps(M=1024, N=1024, K=1024, nb=256, name="random1k")
    A, B, C0 = _dense(w)
    side = OracleSide(w, A, B, C0)
    d, dev = gpu_problem(w, A, B, C0)
    d.run(w.alpha, w.beta)
    first = d.unpack_tiles("C").cpu().numpy()
    torch.cuda.synchronize()
    allocs0, waits0 = d.ctx.host_counters()
    assert allocs0 > 0
    rng = np.random.default_rng(3)
    for it in range(3):
        # new maps of the same shapes (a permutation of the rows of the old ones), new packed data
        mA, mB = w.mapA[rng.permutation(w.MT)], w.mapB[rng.permutation(w.KT)]
        d.ctx.set_precision_map("A", mA if it < 2 else w.mapA)
        d.ctx.bind_storage("A", d.storage["A"].data_ptr(), d.storage["A"].numel())
        d.ctx.set_precision_map("B", mB if it < 2 else w.mapB)
        d.ctx.bind_storage("B", d.storage["B"].data_ptr(), d.storage["B"].numel())
        d.ctx.set_precision_map("C", w.mapC)
        d.ctx.bind_storage("C", d.storage["C"].data_ptr(), d.storage["C"].numel())
        d.pack_tiles("A", dev["A"])
        d.pack_tiles("B", dev["B"])
        d.pack_tiles("C", dev["C"])
        a1, w1 = d.ctx.host_counters()
        if it == 1:
            d.prepare()
        d.run(w.alpha, w.beta)
        a2, w2 = d.ctx.host_counters()
        assert (a2, w2) == (a1, w1), "prepare / run allocated or waited: %s -> %s" % ((a1, w1), (a2, w2))
    assert d.ctx.host_counters()[0] == allocs0            # the whole loop allocated nothing
    last = d.unpack_tiles("C").cpu().numpy()
    torch.cuda.synchronize()
    assert np.array_equal(first, last)                    # the original maps again: the same C bit for bit


def test_launches_side_by_side_give_the_same_c_as_one_after_the_other(monkeypatch):
    """The kernels of a run (FP64 C tiles, FP32 C tiles, 256 x 256 regions) are forked onto side
    streams behind the product table; with GEMM_MP_SERIAL_LAUNCHES=1 they stay on the caller's
    stream.  Which workgroup computes what is the same, so C is bit for bit the same."""
    import torch
    w = W.decay_rect(M=2048, N=2048, K=1024, nb=256, eps=1e-4, name="rect2k")
    w.mapC = np.where(np.add.outer(np.arange(w.MT), np.arange(w.NT)) % 3 == 0, FP64, FP32).astype(np.uint16)
    A, B, C0 = _dense(w)
    results = []
    for serial in ("1", "0"):
        monkeypatch.setenv("GEMM_MP_SERIAL_LAUNCHES", serial)
        d, dev = gpu_problem(w, A, B, C0)
        for _ in range(2):
            d.run(w.alpha, w.beta)
        results.append(d.unpack_tiles("C").cpu().numpy())
        torch.cuda.synchronize()
        st = d.ctx.get_stats()
        assert sum(1 for n in st["launch_items"] if n) >= 3          # three kinds of launches at least
    assert np.array_equal(results[0], results[1])
    side = OracleSide(w, A, B, C0)
    jobs = orc.whole_tile_jobs(w.nb, [(0, 0), (1, 1), (w.MT - 1, w.NT - 1), (2, w.NT - 1)])
    compare_jobs(side, jobs, 0, w.alpha, w.beta, results[1], side.gemm(jobs))


def test_fp32_tiles_made_of_fp16_or_bf16_products_only():
    """C tiles accumulated in FP32 whose every product multiplies two FP16 tiles (or two BF16
    tiles) run in 256 x 256 regions on the 32x32x16 matrix instructions; the FP16 tiles' scales
    are followed by rescaling the one set of accumulators between products, and where the scales
    of a C tile's products lie too far apart the sum so far leaves through the epilogue early.
    Small integers (exact; tile sizes with 4, 8, 12 and 16 chunks, so the rotated chunk order
    wraps; general alpha and beta; FP64 and mixed tiles beside them), small integers times powers
    of two per tile (rescaling, still exact), then general data against the oracle, with tile
    magnitudes that rescale and that force the early epilogue."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP
    rng = np.random.default_rng(35)
    for fmt in (FP16, BF16):
        for (nb, MT, NT, KT) in ((256, 2, 3, 5), (512, 2, 2, 3), (768, 1, 2, 2), (1024, 1, 2, 2)):
            M, N, K = MT * nb, NT * nb, KT * nb
            A = rng.integers(-3, 4, (M, K)).astype(np.float64)
            B = rng.integers(-3, 4, (K, N)).astype(np.float64)
            C0 = rng.integers(-5, 6, (M, N)).astype(np.float64)
            shift = np.zeros(KT, dtype=np.int64)
            if fmt == FP16:                          # tile scales that differ from product to product
                shift = rng.integers(0, 4, KT)
                for L in range(KT):
                    A[:, L * nb:(L + 1) * nb] *= 2.0 ** float(shift[L])
            mA = np.full((MT, KT), fmt, dtype=np.uint16)
            mB = np.full((KT, NT), fmt, dtype=np.uint16)
            mC = np.full((MT, NT), FP32, dtype=np.uint16)
            if MT * NT > 2:
                mC[0, 0] = FP64                      # an FP64 tile: the ordinary kernel
            mB[KT - 1, NT - 1] = FP8                 # last tile column: one FP8 operand, so not that format only
            _say("16-bit-only tiles", fmt, (nb, MT, NT, KT), "shifts", shift)
            d = DeviceGemmMP(M, N, K, nb)
            for which, m, X in (("A", mA, A), ("B", mB, B), ("C", mC, C0)):
                d.set_precision_map(which, m)
                d.pack_tiles(which, torch.from_numpy(X).cuda())
            st = d.ctx.get_stats()
            big = sum(1 for I in range(MT) for J in range(NT) if mC[I, J] == FP32 and J != NT - 1)
            assert st["launch_items"][5 if fmt == FP16 else 6] == big * (nb // 256) ** 2
            d.run(2.0, -3.0)
            got = d.unpack_tiles("C").cpu().numpy()
            want = 2 * (A.astype(np.int64) @ B.astype(np.int64)) - 3 * C0.astype(np.int64)
            assert np.array_equal(got, want.astype(np.float64))
            d.pack_tiles("C", torch.from_numpy(C0).cuda())
            d.run(0.0, 1.0)                          # alpha == 0: no product is formed
            assert np.array_equal(d.unpack_tiles("C").cpu().numpy(), C0)
    # general data against the oracle; the decaying tiles of this workload give every product its own scale
    for fmt in (FP16, BF16):
        w = W.tiny(M=512, N=768, K=1024, nb=256)
        w.mapA = np.full((w.MT, w.KT), fmt, dtype=np.uint16)
        w.mapB = np.full((w.KT, w.NT), fmt, dtype=np.uint16)
        w.mapC = np.full((w.MT, w.NT), FP32, dtype=np.uint16)
        w.mapC[1, 1] = FP16                          # a narrow C tile: accumulated in its FP32 staging copy
        d, _, _, _ = _run_and_compare(w)
        assert d.ctx.get_stats()["launch_items"][5 if fmt == FP16 else 6] == w.MT * w.NT
        w.alpha, w.beta = -0.75, 1.25
        _run_and_compare(w)

    # tile magnitudes 2^0, 2^-50, 2^-90, 2^-40, 2^30 along the reduction: rescaling by up to 2^100 in
    # two steps, and jumps beyond 2^64 that force the early epilogue (with and without an old C)
    class _Jumps(type(W.tiny())):
        def panel(self, which, r0, r1):
            x = super().panel(which, r0, r1)
            if which == "A":
                for L, k in enumerate((0, -50, -90, -40, 30)):
                    x[:, L * self.nb:(L + 1) * self.nb] *= 2.0 ** k
            return x
    w = _Jumps("jumps", 512, 512, 1280, 256, 1.5, 0.5, dist="uniform")
    w.mapA = np.full((w.MT, w.KT), FP16, dtype=np.uint16)
    w.mapB = np.full((w.KT, w.NT), FP16, dtype=np.uint16)
    w.mapC = np.full((w.MT, w.NT), FP32, dtype=np.uint16)
    assert w.KT == 5
    _run_and_compare(w)
    w.alpha, w.beta = 1.0, 0.0
    _run_and_compare(w)
