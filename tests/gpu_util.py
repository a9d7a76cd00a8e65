"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI and fetch its outputs."""
from __future__ import annotations

import numpy as np


def torch_dtype(np_dtype):
    import torch
    return torch.float16 if np.dtype(np_dtype) == np.float16 else torch.float32


def to_device(x: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


class DeviceRun:
    """compress + decompress of one payload on cuda:0; everything copied back to numpy."""

    def __init__(self, payload, eb, R=512, S=256, LMAX=12, capacity=None, ctx=None, d_payload=None, flags=0):
        import torch
        from paper_2407_04272_amd import binding as b
        if d_payload is None:
            d_payload = to_device(payload)
        T, B, D = d_payload.shape
        dt = b.F16 if d_payload.dtype == torch.float16 else b.F32
        self.cfg = b.make_config(dt, T, B, D, R, S, LMAX, flags)
        self.ctx = ctx if ctx is not None else b.Context(self.cfg)
        self.d_payload = d_payload
        bound = b.dlc_compress_bound(self.cfg)
        cap = bound if capacity is None else capacity
        self.d_out = torch.full((max(cap, 16) + 64,), 0xA5, dtype=torch.uint8, device="cuda")  # guard bytes after cap
        self.d_sizes = torch.full((1 + T,), 77, dtype=torch.int64, device="cuda")  # (a size word nobody wrote would show)
        self.eb, _ = self.ctx.set_error_bounds(eb=eb)
        self.rc = self.ctx.compress(d_payload, self.d_out, self.d_sizes, capacity=cap)
        self.status = self.ctx.sync_status() if self.rc == 0 else self.rc
        self.sizes = self.d_sizes.cpu().numpy().astype(np.uint64)
        self.total = int(self.sizes[0])
        out = self.d_out.cpu().numpy()
        self.guard_ok = bool(np.all(out[cap:] == 0xA5))
        self.data = out[:self.total].copy()
        self.cap = cap

    def decompress(self, data=None, comp_bytes=None):
        import torch
        d_comp = self.d_out if data is None else to_device(np.concatenate([data, np.zeros(16, np.uint8)]))
        nbytes = self.total if comp_bytes is None else comp_bytes
        if data is not None and comp_bytes is None:
            nbytes = data.size
        d_rec = torch.full_like(self.d_payload, 7.0)
        rc = self.ctx.decompress(d_comp, nbytes, d_rec)
        st = self.ctx.sync_status() if rc == 0 else rc
        return st, d_rec.cpu().numpy()
