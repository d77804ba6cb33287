"""Allocation of one layer's buffers with torch (device memory, pinned host memory).

Plumbing only: this module owns tensors and hands their pointers to the C ABI.
"""
from __future__ import annotations

import torch

from . import binding as L


def lite_ring(X: torch.Tensor, l: int, w: int) -> torch.Tensor:
    """The rows of positions [l-w, l) of X [B,Hkv,>=l,d] in ring order: row j of the result is
    the position p with p mod w == j (a copy of rows, no arithmetic)."""
    lite = X[:, :, l - w:l, :]
    return torch.roll(lite, shifts=(l - w) % w, dims=2) if w > 0 else lite


class LayerBuffers:
    """Device + pinned-host buffers of one layer, as lrqk_decode_step expects them.

    A_K [B,Hkv,l,r] fp32 and K, V [B,Hkv,l,d] (bf16 or fp32) may live on any device;
    A_K is moved to the GPU, K and V into pinned host memory, the last w rows of K
    and V (the lite tokens) are also kept on the GPU, as a ring (lite_ring).  The cache starts
    empty and the carried selection thresholds unknown (pass LRQK_SELECT_FRESH with the first
    step of the layer).
    """

    def __init__(self, shape: L.Shape, A_K: torch.Tensor, K: torch.Tensor, V: torch.Tensor,
                 device="cuda"):
        self.shape = shape
        B, Hq, Hkv, l, C, d, w = shape.B, shape.Hq, shape.Hkv, shape.l, shape.C, shape.d, shape.w
        rows = shape.rows   # room for the context to grow when shape.l_cap > l
        assert tuple(K.shape) == (B, Hkv, l, d) == tuple(V.shape)
        if rows == l:
            self.A_K = A_K.to(device).contiguous()
        else:
            self.A_K = torch.zeros((B, Hkv, rows, shape.r), dtype=torch.float32, device=device)
            self.A_K[:, :, :l].copy_(A_K)
        self.K_host = torch.empty((B, Hkv, rows, d), dtype=K.dtype, pin_memory=True)
        self.V_host = torch.empty((B, Hkv, rows, d), dtype=V.dtype, pin_memory=True)
        self.K_host[:, :, :l].copy_(K)
        self.V_host[:, :, :l].copy_(V)
        self.K_host[:, :, l:].zero_()
        self.V_host[:, :, l:].zero_()
        self.liteK = lite_ring(K, l, w).to(device).contiguous()
        self.liteV = lite_ring(V, l, w).to(device).contiguous()
        i32 = dict(dtype=torch.int32, device=device)
        self.slot_of = torch.empty((B, Hq, rows), **i32)
        self.token_of = torch.empty((B, Hq, C), **i32)
        self.last_used = torch.empty((B, Hq, C), **i32)
        self.cacheK = torch.zeros((B, Hq, C, d), dtype=K.dtype, device=device)
        self.cacheV = torch.zeros((B, Hq, C, d), dtype=K.dtype, device=device)
        self.sel_thr = torch.empty((B, Hq), dtype=torch.float32, device=device)
        L.lrqk_cache_init(shape, self.slot_of, self.token_of, self.last_used)
        L.lrqk_select_state_init(shape, self.sel_thr)
        self.struct = L.make_layer(A_K=self.A_K, K_host=self.K_host, V_host=self.V_host,
                                   liteK=self.liteK, liteV=self.liteV, slot_of=self.slot_of,
                                   token_of=self.token_of, last_used=self.last_used,
                                   cacheK=self.cacheK, cacheV=self.cacheV, sel_thr=self.sel_thr)
