"""Buffer ownership around the binding: allocates device memory with torch and forwards to the
C ABI.  No arithmetic of the method happens here."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import torch

from . import binding as cq


def to_device(layers: Sequence[Dict[str, torch.Tensor]], device="cuda") -> List[Dict[str, torch.Tensor]]:
    return [{k: v.to(device).contiguous() for k, v in L.items()} for L in layers]


class Group:
    """One packed group with its KV caches and workspace."""

    def __init__(self, dims: cq.cqil_dims, layers: Sequence[Dict[str, torch.Tensor]], b_max: int = 1,
                 device="cuda", ws_tokens: int = 1):
        self.dims = dims
        self.P = len(layers)
        self.dtype = torch.bfloat16 if dims.dtype == cq.CQIL_BF16 else torch.float32
        self.device = device
        self.b_max = b_max
        nbytes = cq.cqil_packed_bytes(dims, self.P)
        if nbytes == 0:
            raise ValueError("invalid dims / P")
        self.packed = torch.empty(nbytes, dtype=torch.uint8, device=device)
        cq.cqil_pack_group(dims, layers, self.packed)
        shape = (self.P, b_max, dims.n_heads, dims.max_seq, dims.head_dim)
        self.k = torch.zeros(shape, dtype=self.dtype, device=device)
        self.v = torch.zeros(shape, dtype=self.dtype, device=device)
        self.kv_len = torch.zeros(b_max, dtype=torch.int32, device=device)
        self.kv = cq.make_kv(self.k, self.v, self.kv_len, 0)
        self._ws: Optional[torch.Tensor] = None
        self._ws_key = None

    def set_kv_len(self, lens) -> None:
        lens = [int(v) for v in lens]
        self.kv_len[: len(lens)] = torch.tensor(lens, dtype=torch.int32, device=self.device)
        self.kv.max_kv_len = max(lens)

    def workspace(self, B: int, T: int) -> torch.Tensor:
        need = cq.cqil_workspace_bytes(self.dims, self.P, B, T)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def forward(self, x: torch.Tensor, bypass_d: int, advance: bool = True,
                out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
        """One group step; `workspace` (uint8, cqil_workspace_bytes() long) replaces the group's own buffer."""
        B, T, _ = x.shape
        out = torch.empty_like(x) if out is None else out
        ws = self.workspace(B, T) if workspace is None else workspace
        cq.cqil_group_forward(self.dims, self.P, bypass_d, self.packed, self.kv, x, out, B, T, advance, ws)
        self._last_ws = ws
        return out

    def attn_out(self, B: int, T: int) -> torch.Tensor:
        """fp32 [P, B*T, d_model] view of the attention outputs left in the workspace by the last call."""
        off = cq.cqil_workspace_attn_out_offset(self.dims, self.P, B, T)
        n = self.P * B * T * self.dims.d_model
        return self._last_ws[off: off + 4 * n].view(torch.float32).view(self.P, B * T, self.dims.d_model)
