"""Device-memory plumbing around the two attention entry points.

PyTorch is used for allocation and streams only; the arithmetic is in the
library.  `VarlenAttention` keeps the output, gradient and workspace buffers of
one bag so that repeated calls (benchmark steps, training steps) allocate
nothing.
"""
from __future__ import annotations

from typing import Sequence

import numpy as np
import torch

from . import binding as B


def bf16_bits_to_device(bits: np.ndarray, device="cuda") -> torch.Tensor:
    """uint16 bf16 bit patterns (host) -> bf16 tensor on the device."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def bf16_device_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


class VarlenAttention:
    """Buffers + calls for one packed bag: T tokens, H heads, head dim d; `causal` selects the
    causal pair of entry points."""

    def __init__(self, cu_seqlens: Sequence[int], H: int, d: int, scale: float, device="cuda",
                 causal: bool = False):
        self.causal = bool(causal)
        cu = np.asarray(cu_seqlens, dtype=np.int32)
        self.n_seq = int(cu.shape[0] - 1)
        self.T = int(cu[-1]) if cu.shape[0] else 0
        self.H, self.d, self.scale = int(H), int(d), float(scale)
        self.device = torch.device(device)
        self.cu = torch.from_numpy(cu).to(self.device)
        shape = (self.T, self.H, self.d)
        self.out = torch.empty(shape, dtype=torch.bfloat16, device=self.device)
        self.lse = torch.empty((self.H, self.T), dtype=torch.float32, device=self.device)
        self.dq = self.dk = self.dv = None
        self.workspace = None

    def forward(self, q, k, v, stream=None):
        fwd = B.knap_varlen_attn_causal_fwd if self.causal else B.knap_varlen_attn_fwd
        fwd(q, k, v, self.cu, self.n_seq, self.H, self.d, self.scale, self.out, self.lse, stream)
        return self.out, self.lse

    def _ensure_bwd_buffers(self):
        if self.dq is None:
            shape = (self.T, self.H, self.d)
            self.dq = torch.empty(shape, dtype=torch.bfloat16, device=self.device)
            self.dk = torch.empty(shape, dtype=torch.bfloat16, device=self.device)
            self.dv = torch.empty(shape, dtype=torch.bfloat16, device=self.device)
            nbytes = B.knap_varlen_attn_bwd_workspace_bytes(self.T, self.n_seq, self.H, self.d)
            self.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=self.device)

    def backward(self, q, k, v, dout, stream=None):
        self._ensure_bwd_buffers()
        bwd = B.knap_varlen_attn_causal_bwd if self.causal else B.knap_varlen_attn_bwd
        bwd(q, k, v, self.cu, self.n_seq, self.H, self.d, self.scale, self.out, self.lse, dout,
            self.dq, self.dk, self.dv, self.T, self.workspace, None, stream)
        return self.dq, self.dk, self.dv
