"""Shared set-up for the GPU parity tests: run one workload through the oracle and through the
C ABI on the same seeded inputs.  The oracle's side and the tolerances live in oracle/checker.py."""
from oracle.checker import (BF16, FP8, FP16, FP32, FP64, LOW_FORMAT, MXFP4, MXFP6, MXFP8, U, OracleSide, compare_jobs,  # noqa: F401
                            finish_low_c_tiles, job_tolerances, packed_codes_expected)


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
