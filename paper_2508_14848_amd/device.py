"""PyTorch plumbing around the C ABI: device buffers and the current stream.

No arithmetic happens here; tensors are only a way to own device memory and to move data
between host and device.
"""
import numpy as np
import torch

from . import gemm_mp as G


def _stream():
    return torch.cuda.current_stream().cuda_stream


class DeviceGemmMP:
    """A gemm_mp context plus the packed device buffers it is bound to."""

    def __init__(self, M, N, K, tile_nb, device="cuda:0", policy=G.POLICY_OPERAND):
        G.lib()                                  # fail loudly before touching the GPU
        if not torch.cuda.is_available():
            raise RuntimeError("gemm_mp needs a GPU; there is no CPU fallback")
        self.device = torch.device(device)
        self.ctx = G.GemmMP(M, N, K, tile_nb)
        self.ctx.set_policy(policy)
        self.storage = {}
        self.maps = {}

    def _bind(self, which):
        n = self.ctx.storage_bytes(which)
        buf = torch.empty(max(n, 256), dtype=torch.uint8, device=self.device)
        assert buf.data_ptr() % 256 == 0
        self.ctx.bind_storage(which, buf.data_ptr(), buf.numel())
        self.storage[which] = buf

    def set_transposed(self, which, transposed):
        self.ctx.set_transposed(which, transposed)
        self.transposed = getattr(self, "transposed", {})
        self.transposed[which] = bool(transposed)

    def set_precision_map(self, which, pmap):
        self.ctx.set_precision_map(which, pmap)
        self.maps[which] = np.array(pmap, dtype=np.uint16)
        self._bind(which)

    def compute_precision_map(self, which, dense, threshold, allowed_mask):
        assert dense.dtype == torch.float64 and dense.is_cuda and dense.stride(1) == 1
        pmap = self.ctx.compute_precision_map(which, dense.data_ptr(), dense.stride(0), threshold,
                                              allowed_mask, _stream())
        self.maps[which] = pmap
        self._bind(which)
        return pmap

    def tile_scan(self, which, dense):
        return self.ctx.tile_scan(which, dense.data_ptr(), dense.stride(0), _stream())

    def pack_tiles(self, which, dense):
        assert dense.dtype == torch.float64 and dense.is_cuda and dense.stride(1) == 1
        self.ctx.pack_tiles(which, dense.data_ptr(), dense.stride(0), _stream())

    def prepare(self):
        self.ctx.prepare(_stream())

    def run(self, alpha, beta):
        self.ctx.run(float(alpha), float(beta), _stream())

    def run_static(self, alpha, beta):
        self.ctx.run_static(float(alpha), float(beta), _stream())

    def convert_tiles(self):
        """Sender-side conversion: allocate the workspace and fill it; returns its size in bytes."""
        n = self.ctx.conversion_bytes()
        self.workspace = torch.empty(max(n, 256), dtype=torch.uint8, device=self.device)
        assert self.workspace.data_ptr() % 256 == 0
        self.ctx.convert_tiles(self.workspace.data_ptr(), self.workspace.numel(), _stream())
        return n

    def clear_conversion(self):
        self.ctx.clear_conversion()

    def unpack_tiles(self, which, out=None):
        rows, cols = {"A": (self.ctx.M, self.ctx.K), "B": (self.ctx.K, self.ctx.N), "C": (self.ctx.M, self.ctx.N)}[which]
        if getattr(self, "transposed", {}).get(which):
            rows, cols = cols, rows
        if out is None:                          # rows of an even length, as the library asks
            out = torch.empty((rows, cols + (cols & 1)), dtype=torch.float64, device=self.device)[:, :cols]
        self.ctx.unpack_tiles(which, out.data_ptr(), out.stride(0), _stream())
        return out

    def tile_bytes(self, which, I, J):
        """Raw stored bytes of one tile as a uint8 host array (for bit-exact checks)."""
        off, prec, _ = self.ctx.tile_info(which, I, J, want_exp=False)
        e = self.ctx.nb * self.ctx.nb
        n = {4: 2 * e, 5: e + e // 32, 6: e // 2 + e // 32, 7: e // 4 * 3 + e // 32}.get(prec, e * (8 >> min(prec, 3)))   # MX: block scales follow the elements
        torch.cuda.synchronize()
        return self.storage[which][off:off + n].cpu().numpy(), prec

    def exponents(self, which):
        rows, cols = self.ctx.tiles(which)
        return np.array([[self.ctx.tile_info(which, i, j)[2] for j in range(cols)] for i in range(rows)],
                        dtype=np.int32)
