"""Shared set-up for the GPU parity tests: run one workload through the oracle and through the
C ABI on the same seeded inputs, and compare per C tile with the stated tolerances."""
import numpy as np

from oracle import gemm_mp_oracle as orc

FP64, FP32, FP16, FP8, BF16, MXFP8, MXFP4 = 0, 1, 2, 3, 4, 5, 6
U = {FP64: 2.0 ** -53, FP32: 2.0 ** -24, FP16: 2.0 ** -11, FP8: 2.0 ** -4, BF16: 2.0 ** -8, MXFP8: 2.0 ** -4, MXFP4: 2.0 ** -2}


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


def compare_jobs(side, jobs, policy, alpha, beta, C_gpu, C_orc):
    """Assert the per-tile bounds; returns the worst ratios for reporting."""
    w = side.w
    nb = w.nb
    worst = dict(star=0.0, tight=0.0, rel64=0.0)
    tols = job_tolerances(side, jobs, policy, alpha)
    for (I, J, r0, r1, c0, c1), t in zip(np.asarray(jobs).reshape(-1, 6), tols):
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
        tight = t["tight"] * base + t["eta"]
        if t["pC"] >= FP16 and np.any(o != 0.0):
            # storage rounding of the finished tile, on both sides: relative u_p per entry in the
            # format's normal range, a full smallest step below it, both doubled because the two
            # sides' exponents may differ by one when their maxima straddle a power of two
            tight += 2.0 * U[t["pC"]] * np.linalg.norm(o)
            if t["pC"] in LOW_FORMAT:               # BF16 has no tile scale and FP32's range; block-scaled tiles scale per block
                E, step = LOW_FORMAT[t["pC"]]
                e_hi = np.floor(np.log2(np.abs(o).max())) - E + 1
                tight += np.sqrt(float(o.size)) * step * 2.0 ** e_hi
        worst["star"] = max(worst["star"], err / (t["tol"] * base))
        worst["tight"] = max(worst["tight"], err / tight)
        assert err <= t["tol"] * base, "tile (%d,%d): err %.3e > 4*K*u_tile bound %.3e" % (I, J, err, t["tol"] * base)
        assert err <= tight, "tile (%d,%d): err %.3e > accumulate-precision bound %.3e" % (I, J, err, tight)
    return worst


def gpu_problem(w, A, B, C0=None, policy=0, device="cuda:0"):
    """Set the workload up on the GPU through the C ABI.  Returns (DeviceGemmMP, dict of dense device tensors)."""
    import torch
    from paper_2508_14848_amd.device import DeviceGemmMP

    d = DeviceGemmMP(w.M, w.N, w.K, w.nb, device=device, policy=policy)
    dA = torch.from_numpy(A).to(device)
    dB = dA if (w.a_equals_b and B is A) else torch.from_numpy(B).to(device)
    if w.rule is not None:
        d.compute_precision_map("A", dA, w.rule["eps"], w.rule["allowed"])
        d.compute_precision_map("B", dB, w.rule["eps"], w.rule["allowed"])
    else:
        d.set_precision_map("A", w.mapA)
        d.set_precision_map("B", w.mapB)
    d.set_precision_map("C", w.mapC)
    d.pack_tiles("A", dA)
    d.pack_tiles("B", dB)
    dC = None
    if C0 is not None and w.beta != 0.0:
        dC = torch.from_numpy(C0).to(device)
        d.pack_tiles("C", dC)
    return d, dict(A=dA, B=dB, C=dC)


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
