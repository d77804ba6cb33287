"""Glue for the GPU parity tests: puts one layer of a synthetic workload on the
device (through the Python binding of the C ABI) and, beside it, the same layer
as numpy arrays for the CPU oracle.  No arithmetic of the method happens here."""
from __future__ import annotations

import numpy as np
import torch

import paper_2510_23649_amd as L
from gen import as_numpy
from oracle import lrqk_oracle as orc

DEV = "cuda"


def lite_ring(X: torch.Tensor, l: int, w: int) -> torch.Tensor:
    """Rows of the positions [l-w, l) of X [B,Hkv,>=l,d] as the library keeps them: row j of the
    result holds the position p of the window with p mod w == j."""
    if w == 0:
        return X[:, :, l:l, :]
    row_of = {p % w: p for p in range(l - w, l)}      # position p sits at row p mod w
    return X[:, :, torch.tensor([row_of[j] for j in range(w)]), :]


def shape_of(cfg) -> L.Shape:
    return L.Shape.make(B=cfg.B, Hq=cfg.Hq, Hkv=cfg.Hkv, l=cfg.l, r=cfg.r, k=cfg.k, w=cfg.w,
                        C_slots=cfg.C, d=cfg.d,
                        kv_dtype=L.LRQK_KV_BF16 if cfg.kv_dtype == "bf16" else L.LRQK_KV_F32,
                        scale=cfg.scale)


def workspace(nbytes: int) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=DEV)


class DeviceLayer:
    """Device + pinned-host buffers of one layer, and the matching oracle-side copies."""

    def __init__(self, cfg, data, identity: bool = False, carry: bool = True):
        """carry: give the layer a carried-threshold array (lrqk_layer.sel_thr), set to unknown."""
        self.cfg = cfg
        B, Hq, Hkv, l, C, d, G = cfg.B, cfg.Hq, cfg.Hkv, cfg.l, cfg.C, cfg.d, cfg.G
        kvdt = data.K.dtype
        self.A_K = data.A_K.to(DEV).contiguous()
        self.K_host = data.K.cpu().contiguous().pin_memory()
        self.V_host = data.V.cpu().contiguous().pin_memory()
        self.liteK = lite_ring(data.K, l, cfg.w).to(DEV).contiguous()
        self.liteV = lite_ring(data.V, l, cfg.w).to(DEV).contiguous()
        self.slot_of = torch.empty((B, Hq, l), dtype=torch.int32, device=DEV)
        self.token_of = torch.empty((B, Hq, C), dtype=torch.int32, device=DEV)
        self.last_used = torch.empty((B, Hq, C), dtype=torch.int32, device=DEV)
        self.cacheK = torch.zeros((B, Hq, C, d), dtype=kvdt, device=DEV)
        self.cacheV = torch.zeros((B, Hq, C, d), dtype=kvdt, device=DEV)
        self.shape = shape_of(cfg)
        L.lrqk_cache_init(self.shape, self.slot_of, self.token_of, self.last_used)
        self.sel_thr = None
        if carry:
            self.sel_thr = torch.zeros((B, Hq), dtype=torch.float32, device=DEV)
            L.lrqk_select_state_init(self.shape, self.sel_thr)
        # oracle side
        self.np = dict(A_K=as_numpy(data.A_K), K=as_numpy(data.K), V=as_numpy(data.V))
        self.ost = orc.CacheState(B, Hq, l, C)
        self.ocK = np.zeros((B, Hq, C, d), self.np["K"].dtype)
        self.ocV = np.zeros_like(self.ocK)
        if identity:
            assert C == l
            ar = torch.arange(l, dtype=torch.int32, device=DEV)
            self.slot_of[:] = ar
            self.token_of[:] = ar
            self.last_used[:] = 0
            Kd, Vd = data.K.to(DEV), data.V.to(DEV)
            for h in range(Hq):
                self.cacheK[:, h] = Kd[:, h // G]
                self.cacheV[:, h] = Vd[:, h // G]
            self.ost = orc.CacheState.identity(B, Hq, l)
            for h in range(Hq):
                self.ocK[:, h] = self.np["K"][:, h // G]
                self.ocV[:, h] = self.np["V"][:, h // G]
        torch.cuda.synchronize()

    def struct(self) -> L.Layer:
        from paper_2510_23649_amd.binding import make_layer
        return make_layer(A_K=self.A_K, K_host=self.K_host, V_host=self.V_host, liteK=self.liteK,
                          liteV=self.liteV, slot_of=self.slot_of, token_of=self.token_of,
                          last_used=self.last_used, cacheK=self.cacheK, cacheV=self.cacheV,
                          sel_thr=self.sel_thr)

    def state_np(self):
        torch.cuda.synchronize()
        return dict(slot_of=self.slot_of.cpu().numpy(), token_of=self.token_of.cpu().numpy(),
                    last_used=self.last_used.cpu().numpy(), cacheK=as_numpy(self.cacheK),
                    cacheV=as_numpy(self.cacheV))


class StepBuffers:
    """Outputs of the selection / resolution calls, on the device."""

    def __init__(self, cfg):
        B, Hq, k = cfg.B, cfg.Hq, cfg.k
        i32 = dict(dtype=torch.int32, device=DEV)
        self.sel_idx = torch.full((B, Hq, k), -7, **i32)
        self.sel_slot = torch.full((B, Hq, k), -7, **i32)
        self.hit = torch.full((B, Hq, k), 9, dtype=torch.uint8, device=DEV)
        self.miss_tok = torch.full((B, Hq, k), -7, **i32)
        self.miss_slot = torch.full((B, Hq, k), -7, **i32)
        self.n_miss = torch.full((B, Hq), -7, **i32)
        self.link_rows = torch.full((B, cfg.Hkv), -7, **i32)

    def debug(self):
        return dict(sel_idx=self.sel_idx, sel_slot=self.sel_slot, hit=self.hit,
                    miss_tok=self.miss_tok, miss_slot=self.miss_slot, n_miss=self.n_miss,
                    link_rows=self.link_rows)

    def to_np(self):
        torch.cuda.synchronize()
        return {n: getattr(self, n).cpu().numpy() for n in
                ("sel_idx", "sel_slot", "hit", "miss_tok", "miss_slot", "n_miss", "link_rows")}


def compare_resolution(got: dict, ref: dict, where: str = ""):
    """Bit-exact comparison of the integer results of a3 (only the first n_miss
    entries of the miss lists are defined)."""
    assert np.array_equal(got["n_miss"], ref["n_miss"]), f"{where}: n_miss differs"
    assert np.array_equal(got["sel_slot"], ref["sel_slot"]), f"{where}: sel_slot differs"
    assert np.array_equal(got["hit"], ref["hit"]), f"{where}: hit map differs"
    B, Hq = got["n_miss"].shape
    for b in range(B):
        for h in range(Hq):
            nm = max(int(ref["n_miss"][b, h]), 0)
            assert np.array_equal(got["miss_tok"][b, h, :nm], ref["miss_tok"][b, h, :nm]), where
            assert np.array_equal(got["miss_slot"][b, h, :nm], ref["miss_slot"][b, h, :nm]), where


def compare_state(dl: DeviceLayer, where: str = "", rows_for=None):
    """Cache maps bit-exact; cache rows bit-exact on the slots in use."""
    st = dl.state_np()
    assert np.array_equal(st["slot_of"], dl.ost.slot_of), f"{where}: slot_of differs"
    assert np.array_equal(st["token_of"], dl.ost.token_of), f"{where}: token_of differs"
    assert np.array_equal(st["last_used"], dl.ost.last_used), f"{where}: last_used differs"
    used = dl.ost.token_of >= 0
    assert np.array_equal(st["cacheK"][used], dl.ocK[used]), f"{where}: cached K rows differ"
    assert np.array_equal(st["cacheV"][used], dl.ocV[used]), f"{where}: cached V rows differ"
