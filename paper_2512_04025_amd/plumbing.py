"""Device-memory plumbing around the C ABI: upload/download of stored tensors and the buffers one
call sequence needs, allocated with PyTorch.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np

from . import binding as psa


def to_dev(x: np.ndarray, dtype: str):
    """Stored numpy tensor (float32, or uint16 bf16 bits) -> device tensor of the same bytes."""
    import torch
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def from_dev(t, dtype: str) -> np.ndarray:
    """Device tensor -> float64 numpy values (bf16 widened exactly)."""
    import torch
    if dtype == "bf16":
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


class Buffers:
    """Device buffers one PSA call sequence needs (pyramids, scratch, M, S, rho, O, lse)."""

    def __init__(self, gp: psa.PsaParams):
        import torch
        self.gp = gp
        self.tdtype = torch.bfloat16 if gp.dtype == psa.PSA_BF16 else torch.float32
        pyr_bytes, scratch_bytes = psa.psa_query_sizes(gp)
        esize = 2 if gp.dtype == psa.PSA_BF16 else 4
        self.Kpyr = torch.empty(max(pyr_bytes // esize, 1), dtype=self.tdtype, device="cuda")
        self.Vpyr = torch.empty(max(pyr_bytes // esize, 1), dtype=self.tdtype, device="cuda")
        self.scratch = torch.empty(max(scratch_bytes, 256), dtype=torch.uint8, device="cuda")
        self.M = torch.empty((gp.B, gp.Hq, gp.nq, gp.nk), dtype=torch.uint8, device="cuda")
        self.S = torch.empty((gp.B, gp.Hq, gp.nq, gp.nk), dtype=torch.float32, device="cuda")
        self.rho = torch.empty((gp.B, gp.Hq), dtype=torch.float32, device="cuda")
        self.O = torch.empty((gp.B, gp.Hq, gp.N, gp.d), dtype=self.tdtype, device="cuda")
        self.lse = torch.empty((gp.B, gp.Hq, gp.N), dtype=torch.float32, device="cuda")

    def level(self, pyr, h: int):
        """View of pyramid level h (2..H) as [B, Hkv, nk * (bk >> (h-1)), d]."""
        gp = self.gp
        off = 0
        for t in range(2, h):
            off += gp.B * gp.Hkv * gp.nk * (gp.bk >> (t - 1)) * gp.d
        rows = gp.nk * (gp.bk >> (h - 1))
        n = gp.B * gp.Hkv * rows * gp.d
        return pyr[off:off + n].view(gp.B, gp.Hkv, rows, gp.d)
