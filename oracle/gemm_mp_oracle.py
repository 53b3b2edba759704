"""ctypes front end of the CPU oracle (oracle/gemm_mp_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  It holds no arithmetic of its own; every number
comes from the C file, which states the passage of the paper (or the reading
of it) each function follows.  It does not import the GPU package.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gemm_mp_oracle.c")
_LIB = os.path.join(_HERE, "libgemm_mp_oracle.so")

FP64, FP32, FP16, FP8, BF16, MXFP8, MXFP4, MXFP6 = 0, 1, 2, 3, 4, 5, 6, 7
POLICY_OPERAND, POLICY_C_TILE = 0, 1
ALL_PRECISIONS_MASK = 0xF          # the four formats of the configurations
ALL_FORMATS_MASK = 0x1F            # ... and BF16


def build(force=False):
    """Compile the oracle with gcc.  -ffp-contract=off: only explicit fma() calls fuse."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O3", "-mavx2", "-mfma", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-shared", "-fPIC", "-std=c11", "-Wall", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        c_i64, c_i32, c_dbl = ctypes.c_int64, ctypes.c_int32, ctypes.c_double
        P = ctypes.c_void_p
        _lib.orc_round_fp16_array.argtypes = [P, c_i64, P, P]
        _lib.orc_round_fp8_array.argtypes = [P, c_i64, P, P]
        _lib.orc_round_bf16_array.argtypes = [P, c_i64, P, P]
        _lib.orc_mx_blocks_array.argtypes = [P, c_i64, P, P, P]
        _lib.orc_mx4_blocks_array.argtypes = [P, c_i64, P, P, P]
        _lib.orc_mx6_blocks_array.argtypes = [P, c_i64, P, P, P]
        _lib.orc_store_tiles_axis.argtypes = [P, c_i64, c_i64, c_i64, c_i32, P, P, P, c_i64, P, c_i32]
        _lib.orc_bf16_value.restype = c_dbl
        _lib.orc_bf16_value.argtypes = [ctypes.c_uint16]
        _lib.orc_fp16_value.restype = c_dbl
        _lib.orc_fp16_value.argtypes = [ctypes.c_uint16]
        _lib.orc_fp8_value.restype = c_dbl
        _lib.orc_fp8_value.argtypes = [ctypes.c_uint8]
        _lib.orc_tile_scan.argtypes = [P, c_i64, c_i64, c_i64, c_i32, P, P]
        _lib.orc_precision_rule.argtypes = [P, c_i64, c_dbl, ctypes.c_uint32, P]
        _lib.orc_scale_exponent.restype = c_i32
        _lib.orc_scale_exponent.argtypes = [c_dbl, c_i32]
        _lib.orc_store_tiles.argtypes = [P, c_i64, c_i64, c_i64, c_i32, P, P, P, c_i64, P]
        _lib.orc_product_precision.restype = c_i32
        _lib.orc_product_precision.argtypes = [c_i32, c_i32, c_i32, c_i32]
        _lib.orc_gemm_jobs.restype = c_i32
        _lib.orc_gemm_jobs.argtypes = [c_i64, c_i64, c_i64, c_i32,
                                       P, c_i64, P, P, P, c_i64, P, P, P, c_i64, P,
                                       c_dbl, c_dbl, c_i32, c_i64, P, P, c_i64,
                                       c_i64, c_i64, P, c_i32, c_i32]
        _lib.orc_stored_values.argtypes = [P, c_i64, c_i64, c_i64, c_i32, P, P, c_i64]
        _lib.orc_num_threads.restype = c_i32
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _dense(x):
    x = np.asarray(x)
    assert x.dtype == np.float64 and x.ndim == 2 and x.strides[1] == 8 and x.strides[0] % 8 == 0
    return x


def num_threads():
    return int(lib().orc_num_threads())


def round_fp16(x):
    """FP64 -> FP16 by one rounding.  Returns (values as FP64, bit patterns)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty_like(x)
    bits = np.empty(x.shape, dtype=np.uint16)
    lib().orc_round_fp16_array(_p(x), x.size, _p(y), _p(bits))
    return y, bits


def round_fp8(x):
    """FP64 -> FP8 e4m3fn by one rounding, saturating.  Returns (values, bit patterns)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty_like(x)
    bits = np.empty(x.shape, dtype=np.uint8)
    lib().orc_round_fp8_array(_p(x), x.size, _p(y), _p(bits))
    return y, bits


def mx_blocks(x):
    """MXFP8 quantisation of consecutive blocks of 32 numbers (x.size a multiple of 32).
    Returns (element numbers as FP64, element codes, scale codes = s + 127)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    assert x.size % 32 == 0
    y = np.empty_like(x)
    codes = np.empty(x.shape, dtype=np.uint8)
    scales = np.empty(x.size // 32, dtype=np.uint8)
    lib().orc_mx_blocks_array(_p(x), x.size // 32, _p(y), _p(codes), _p(scales))
    return y, codes, scales


def mx4_blocks(x):
    """MXFP4 quantisation of consecutive blocks of 32 numbers.  Returns (element numbers as FP64,
    4-bit element codes one per byte, scale codes = s + 127)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    assert x.size % 32 == 0
    y = np.empty_like(x)
    codes = np.empty(x.shape, dtype=np.uint8)
    scales = np.empty(x.size // 32, dtype=np.uint8)
    lib().orc_mx4_blocks_array(_p(x), x.size // 32, _p(y), _p(codes), _p(scales))
    return y, codes, scales


def mx6_blocks(x):
    """MXFP6 (e2m3) quantisation of consecutive blocks of 32 numbers.  Returns (element numbers as
    FP64, 6-bit element codes one per byte, scale codes = s + 127)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    assert x.size % 32 == 0
    y = np.empty_like(x)
    codes = np.empty(x.shape, dtype=np.uint8)
    scales = np.empty(x.size // 32, dtype=np.uint8)
    lib().orc_mx6_blocks_array(_p(x), x.size // 32, _p(y), _p(codes), _p(scales))
    return y, codes, scales


def round_bf16(x):
    """FP64 -> BF16 by one rounding.  Returns (values as FP64, bit patterns)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.empty_like(x)
    bits = np.empty(x.shape, dtype=np.uint16)
    lib().orc_round_bf16_array(_p(x), x.size, _p(y), _p(bits))
    return y, bits


def bf16_value(code):
    return float(lib().orc_bf16_value(int(code)))


def fp16_value(code):
    return float(lib().orc_fp16_value(int(code)))


def fp8_value(code):
    return float(lib().orc_fp8_value(int(code)))


def pad_to_tiles(X, nb):
    """A matrix whose sizes are no multiples of nb, as this build reads it (the paper's
    experiments use multiples only): the same matrix extended with zeros to whole tiles.  Zeros
    add nothing to a tile's sum of squares, to its maximum or to a product, so every function
    below is applied to the extension.  No arithmetic here."""
    X = np.asarray(X, dtype=np.float64)
    rows, cols = X.shape
    pr, pc = -rows % nb, -cols % nb
    return X if pr == 0 and pc == 0 else np.pad(X, ((0, pr), (0, pc)))


def tile_scan(X, nb):
    """Per-tile sum of squares (fixed order) and max magnitude; arrays [rows/nb][cols/nb]."""
    X = _dense(X)
    rows, cols = X.shape
    assert rows % nb == 0 and cols % nb == 0
    sumsq = np.empty((rows // nb, cols // nb), dtype=np.float64)
    maxabs = np.empty_like(sumsq)
    lib().orc_tile_scan(_p(X), X.strides[0] // 8, rows, cols, nb, _p(sumsq), _p(maxabs))
    return sumsq, maxabs


def precision_rule(sumsq, eps, allowed_mask):
    sumsq = np.ascontiguousarray(sumsq, dtype=np.float64)
    out = np.empty(sumsq.shape, dtype=np.uint16)
    lib().orc_precision_rule(_p(sumsq), sumsq.size, float(eps), int(allowed_mask), _p(out))
    return out


def scale_exponent(maxabs, p):
    return int(lib().orc_scale_exponent(float(maxabs), int(p)))


def store_tiles(X, nb, pmap, maxabs=None, out=None, mx_axis=0):
    """Storage rounding of every tile.  Returns (Y stored numbers as FP64, exps int32 per tile).
    mx_axis: the blocks of MXFP8 tiles run along the rows (0: A) or down the columns (1: B), i.e.
    along the reduction index; such tiles come back as the values they stand for, exponent 0."""
    X = _dense(X)
    rows, cols = X.shape
    pmap = np.ascontiguousarray(pmap, dtype=np.uint16)
    assert pmap.shape == (rows // nb, cols // nb)
    if maxabs is None:
        _, maxabs = tile_scan(X, nb)
    maxabs = np.ascontiguousarray(maxabs, dtype=np.float64)
    Y = np.empty_like(X) if out is None else _dense(out)
    exps = np.empty(pmap.shape, dtype=np.int32)
    lib().orc_store_tiles_axis(_p(X), X.strides[0] // 8, rows, cols, nb, _p(pmap), _p(maxabs),
                               _p(Y), Y.strides[0] // 8, _p(exps), int(mx_axis))
    return Y, exps


def stored_values(Y, nb, exps):
    """The values stored tiles stand for: stored numbers times 2^e of their tile."""
    Y = _dense(Y)
    rows, cols = Y.shape
    exps = np.ascontiguousarray(exps, dtype=np.int32)
    assert exps.shape == (rows // nb, cols // nb)
    X = np.empty_like(Y)
    lib().orc_stored_values(_p(Y), Y.strides[0] // 8, rows, cols, nb, _p(exps), _p(X), X.strides[0] // 8)
    return X


def product_precision(pA, pB, pC, policy=POLICY_OPERAND):
    return int(lib().orc_product_precision(int(pA), int(pB), int(pC), int(policy)))


def gemm_jobs(nb, Ay, mapA, eA, By, mapB, eB, Cy, mapC, alpha, beta, jobs,
              policy=POLICY_OPERAND, out=None, L_range=None, state=None, resume=False, finish=True):
    """Compute the listed jobs (rows of [I, J, r0, r1, c0, c1]) into a dense FP64 C.

    Cy may be None when beta == 0; where C tiles are stored in FP16 / FP8 it holds the values
    they stand for (stored_values), and the result for such tiles is the FP32 form that
    store_tiles then rounds, whole tile by whole tile.  Entries of the result outside the jobs are left as
    they were in `out` (NaN in a fresh array).  L_range / state / resume / finish let a
    caller split the reduction over several calls (see the C file)."""
    Ay, By = _dense(Ay), _dense(By)
    M, K = Ay.shape
    K2, N = By.shape
    assert K == K2
    mapA = np.ascontiguousarray(mapA, dtype=np.uint16)
    mapB = np.ascontiguousarray(mapB, dtype=np.uint16)
    mapC = np.ascontiguousarray(mapC, dtype=np.uint16)
    eA = np.ascontiguousarray(eA, dtype=np.int32)
    eB = np.ascontiguousarray(eB, dtype=np.int32)
    assert mapA.shape == (M // nb, K // nb) == eA.shape
    assert mapB.shape == (K // nb, N // nb) == eB.shape
    assert mapC.shape == (M // nb, N // nb)
    if Cy is None:
        assert beta == 0.0
        cy_ptr, ldc0 = None, 0
    else:
        Cy = _dense(Cy)
        assert Cy.shape == (M, N)
        cy_ptr, ldc0 = _p(Cy), Cy.strides[0] // 8
    jobs = np.ascontiguousarray(jobs, dtype=np.int32).reshape(-1, 6)
    if out is None:
        out = np.full((M, N), np.nan, dtype=np.float64)
    out = _dense(out)
    L0, L1 = (0, K // nb) if L_range is None else L_range
    if state is not None:
        assert state.dtype == np.float64 and state.flags.c_contiguous
        assert state.size == int(((jobs[:, 3] - jobs[:, 2]) * (jobs[:, 5] - jobs[:, 4])).sum())
    st_ptr = None if state is None else _p(state)
    rc = lib().orc_gemm_jobs(M, N, K, nb,
                             _p(Ay), Ay.strides[0] // 8, _p(mapA), _p(eA),
                             _p(By), By.strides[0] // 8, _p(mapB), _p(eB),
                             cy_ptr, ldc0, _p(mapC),
                             float(alpha), float(beta), int(policy),
                             jobs.shape[0], _p(jobs), _p(out), out.strides[0] // 8,
                             L0, L1, st_ptr, int(bool(resume)), int(bool(finish)))
    if rc != 0:
        raise ValueError("orc_gemm_jobs: bad argument")
    return out


def whole_tile_jobs(nb, tiles):
    """Jobs covering the given C tiles completely."""
    return np.array([[I, J, 0, nb, 0, nb] for (I, J) in tiles], dtype=np.int32)
