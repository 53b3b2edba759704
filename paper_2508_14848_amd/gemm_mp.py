"""Thin ctypes binding of libgemm_mp.so (declared in include/gemm_mp.h).

Argument marshalling only: every step of the path (tile scan, precision rule input, packing,
the tile products, unpacking) runs in the library's HIP kernels.  PyTorch is used by callers
for device memory and streams; this module itself only needs raw device pointers.

There is no CPU fallback: if the shared library is missing, loading fails loudly.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgemm_mp.so")

FP64, FP32, FP16, FP8_E4M3, BF16, MXFP8, MXFP4, MXFP6 = 0, 1, 2, 3, 4, 5, 6, 7
POLICY_OPERAND, POLICY_C_TILE = 0, 1
OK, EINVAL, ESTATE, ENOMEM, EUNSUPPORTED, EHIP, ETOOBIG = 0, -1, -2, -3, -4, -5, -6
STATIC_MAX_PRODUCTS = 65536

EXPORTS = [
    "gemm_mp_create", "gemm_mp_destroy", "gemm_mp_set_policy", "gemm_mp_set_transposed", "gemm_mp_set_precision_map",
    "gemm_mp_tile_scan", "gemm_mp_compute_precision_map", "gemm_mp_storage_bytes",
    "gemm_mp_bind_storage", "gemm_mp_pack_tiles", "gemm_mp_run", "gemm_mp_unpack_tiles",
    "gemm_mp_tile_info", "gemm_mp_get_stats", "gemm_mp_product_precision", "gemm_mp_strerror",
    "gemm_mp_conversion_bytes", "gemm_mp_convert_tiles", "gemm_mp_clear_conversion",
    "gemm_mp_prepare", "gemm_mp_host_counters", "gemm_mp_run_static",
]


class Stats(ctypes.Structure):
    _fields_ = [("products", ctypes.c_int64 * 4), ("flops", ctypes.c_double * 4),
                ("tiles", (ctypes.c_int64 * 4) * 3), ("packed_bytes", ctypes.c_uint64 * 3),
                ("work_items", ctypes.c_int64), ("converted_tiles", ctypes.c_int64),
                ("converted_bytes", ctypes.c_uint64), ("products_bf16", ctypes.c_int64),
                ("flops_bf16", ctypes.c_double), ("tiles_bf16", ctypes.c_int64 * 3),
                ("products_mxfp8", ctypes.c_int64), ("flops_mxfp8", ctypes.c_double), ("tiles_mxfp8", ctypes.c_int64 * 3),
                ("products_mxfp4", ctypes.c_int64), ("flops_mxfp4", ctypes.c_double), ("tiles_mxfp4", ctypes.c_int64 * 3),
                ("launch_items", ctypes.c_int64 * 8), ("owner_instance", ctypes.c_int32 * 2),
                ("products_mxfp6", ctypes.c_int64), ("flops_mxfp6", ctypes.c_double), ("tiles_mxfp6", ctypes.c_int64 * 3)]


class GemmMPError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: %s (%d)" % (what, strerror(status), status))


_lib = None


def lib():
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libgemm_mp.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        P, i64, i32, dbl, c = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_double, ctypes.c_char
        L.gemm_mp_create.argtypes = [ctypes.POINTER(P), i64, i64, i64, i32]
        L.gemm_mp_destroy.argtypes = [P]
        L.gemm_mp_set_policy.argtypes = [P, ctypes.c_int]
        L.gemm_mp_set_transposed.argtypes = [P, c, ctypes.c_int]
        L.gemm_mp_set_precision_map.argtypes = [P, c, P, i32, i32]
        L.gemm_mp_tile_scan.argtypes = [P, c, P, i64, P, P, P]
        L.gemm_mp_compute_precision_map.argtypes = [P, c, P, i64, dbl, ctypes.c_uint32, P, P]
        L.gemm_mp_storage_bytes.argtypes = [P, c, ctypes.POINTER(ctypes.c_size_t)]
        L.gemm_mp_bind_storage.argtypes = [P, c, P, ctypes.c_size_t]
        L.gemm_mp_pack_tiles.argtypes = [P, c, P, i64, P]
        L.gemm_mp_run.argtypes = [P, dbl, dbl, P]
        L.gemm_mp_prepare.argtypes = [P, P]
        L.gemm_mp_run_static.argtypes = [P, dbl, dbl, P]
        L.gemm_mp_host_counters.argtypes = [P, ctypes.POINTER(i64), ctypes.POINTER(i64)]
        L.gemm_mp_unpack_tiles.argtypes = [P, c, P, i64, P]
        L.gemm_mp_conversion_bytes.argtypes = [P, ctypes.POINTER(ctypes.c_size_t)]
        L.gemm_mp_convert_tiles.argtypes = [P, P, ctypes.c_size_t, P]
        L.gemm_mp_clear_conversion.argtypes = [P]
        L.gemm_mp_tile_info.argtypes = [P, c, i32, i32, ctypes.POINTER(ctypes.c_size_t),
                                        ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
        L.gemm_mp_get_stats.argtypes = [P, ctypes.POINTER(Stats)]
        L.gemm_mp_product_precision.argtypes = [ctypes.c_int] * 4
        L.gemm_mp_strerror.argtypes = [ctypes.c_int]
        L.gemm_mp_strerror.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name != "gemm_mp_strerror":
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def strerror(status):
    return lib().gemm_mp_strerror(int(status)).decode()


def product_precision(pA, pB, pC, policy=POLICY_OPERAND):
    return lib().gemm_mp_product_precision(int(pA), int(pB), int(pC), int(policy))


def _w(which):
    return which.encode() if isinstance(which, str) else which


def _check(status, what):
    if status != OK:
        raise GemmMPError(status, what)


class GemmMP:
    """One gemm_mp context.  Method names follow the C entry points (gemm_mp_<name>).

    Device pointers are plain integers (e.g. torch.Tensor.data_ptr()), streams are raw
    hipStream_t handles (e.g. torch.cuda.current_stream().cuda_stream) or 0 / None.
    """

    def __init__(self, M, N, K, tile_nb):
        self._h = ctypes.c_void_p()
        _check(lib().gemm_mp_create(ctypes.byref(self._h), M, N, K, tile_nb), "gemm_mp_create")
        self.M, self.N, self.K, self.nb = M, N, K, tile_nb
        self.MT, self.NT, self.KT = -(-M // tile_nb), -(-N // tile_nb), -(-K // tile_nb)

    def destroy(self):
        if self._h:
            lib().gemm_mp_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def tiles(self, which):
        return {"A": (self.MT, self.KT), "B": (self.KT, self.NT), "C": (self.MT, self.NT)}[which]

    def set_policy(self, policy):
        _check(lib().gemm_mp_set_policy(self._h, policy), "gemm_mp_set_policy")

    def set_transposed(self, which, transposed):
        _check(lib().gemm_mp_set_transposed(self._h, _w(which), int(bool(transposed))), "gemm_mp_set_transposed")

    def set_precision_map(self, which, pmap):
        pmap = np.ascontiguousarray(pmap, dtype=np.uint16)
        rows, cols = pmap.shape
        _check(lib().gemm_mp_set_precision_map(self._h, _w(which), pmap.ctypes.data, rows, cols),
               "gemm_mp_set_precision_map")

    def tile_scan(self, which, dense_ptr, ld, stream=None):
        rows, cols = self.tiles(which)
        sumsq = np.empty((rows, cols), dtype=np.float64)
        maxabs = np.empty((rows, cols), dtype=np.float64)
        _check(lib().gemm_mp_tile_scan(self._h, _w(which), dense_ptr, ld, stream, sumsq.ctypes.data,
                                       maxabs.ctypes.data), "gemm_mp_tile_scan")
        return sumsq, maxabs

    def compute_precision_map(self, which, dense_ptr, ld, threshold, allowed_mask, stream=None):
        rows, cols = self.tiles(which)
        out = np.empty((rows, cols), dtype=np.uint16)
        _check(lib().gemm_mp_compute_precision_map(self._h, _w(which), dense_ptr, ld, threshold, allowed_mask,
                                                   stream, out.ctypes.data), "gemm_mp_compute_precision_map")
        return out

    def storage_bytes(self, which):
        n = ctypes.c_size_t()
        _check(lib().gemm_mp_storage_bytes(self._h, _w(which), ctypes.byref(n)), "gemm_mp_storage_bytes")
        return n.value

    def bind_storage(self, which, dev_ptr, nbytes):
        _check(lib().gemm_mp_bind_storage(self._h, _w(which), dev_ptr, nbytes), "gemm_mp_bind_storage")

    def pack_tiles(self, which, dense_ptr, ld, stream=None):
        _check(lib().gemm_mp_pack_tiles(self._h, _w(which), dense_ptr, ld, stream), "gemm_mp_pack_tiles")

    def prepare(self, stream=None):
        _check(lib().gemm_mp_prepare(self._h, stream), "gemm_mp_prepare")

    def run(self, alpha, beta, stream=None):
        _check(lib().gemm_mp_run(self._h, alpha, beta, stream), "gemm_mp_run")

    def run_static(self, alpha, beta, stream=None):
        _check(lib().gemm_mp_run_static(self._h, alpha, beta, stream), "gemm_mp_run_static")

    def host_counters(self):
        """(allocations, host waits) this context has made so far."""
        a, w = ctypes.c_int64(), ctypes.c_int64()
        _check(lib().gemm_mp_host_counters(self._h, ctypes.byref(a), ctypes.byref(w)), "gemm_mp_host_counters")
        return a.value, w.value

    def conversion_bytes(self):
        n = ctypes.c_size_t()
        _check(lib().gemm_mp_conversion_bytes(self._h, ctypes.byref(n)), "gemm_mp_conversion_bytes")
        return n.value

    def convert_tiles(self, workspace_ptr, nbytes, stream=None):
        _check(lib().gemm_mp_convert_tiles(self._h, workspace_ptr, nbytes, stream), "gemm_mp_convert_tiles")

    def clear_conversion(self):
        _check(lib().gemm_mp_clear_conversion(self._h), "gemm_mp_clear_conversion")

    def unpack_tiles(self, which, dense_ptr, ld, stream=None):
        _check(lib().gemm_mp_unpack_tiles(self._h, _w(which), dense_ptr, ld, stream), "gemm_mp_unpack_tiles")

    def tile_info(self, which, I, J, want_exp=True):
        off, prec, e = ctypes.c_size_t(), ctypes.c_int(), ctypes.c_int()
        _check(lib().gemm_mp_tile_info(self._h, _w(which), I, J, ctypes.byref(off), ctypes.byref(prec),
                                       ctypes.byref(e) if want_exp else None), "gemm_mp_tile_info")
        return off.value, prec.value, (e.value if want_exp else None)

    def get_stats(self):
        s = Stats()
        _check(lib().gemm_mp_get_stats(self._h, ctypes.byref(s)), "gemm_mp_get_stats")
        return {"products": list(s.products), "flops": list(s.flops),
                "tiles": [list(s.tiles[w]) for w in range(3)], "packed_bytes": list(s.packed_bytes),
                "work_items": s.work_items, "converted_tiles": s.converted_tiles,
                "converted_bytes": s.converted_bytes, "products_bf16": s.products_bf16,
                "flops_bf16": s.flops_bf16, "tiles_bf16": list(s.tiles_bf16), "products_mxfp8": s.products_mxfp8,
                "flops_mxfp8": s.flops_mxfp8, "tiles_mxfp8": list(s.tiles_mxfp8), "products_mxfp4": s.products_mxfp4,
                "flops_mxfp4": s.flops_mxfp4, "tiles_mxfp4": list(s.tiles_mxfp4),
                "products_mxfp6": s.products_mxfp6, "flops_mxfp6": s.flops_mxfp6, "tiles_mxfp6": list(s.tiles_mxfp6),
                "launch_items": list(s.launch_items), "owner_instance": list(s.owner_instance)}
