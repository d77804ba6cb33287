"""GPU test of lrqk_sparse_attend_noalloc, the attention entry point that allocates nothing:
its output must equal lrqk_sparse_attend's (same kernels, partial states in the library's
fixed device array instead of a caller's workspace) and agree with the oracle to the
attention tolerance, on two calls in a row, the second one smaller (so stale partials of
the first call lie beyond what the second one writes)."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2510_23649_amd as L
from gen import as_numpy
from oracle import lrqk_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda"
TOL = {"bf16": 2e-3, "fp32": 1e-5}


def say(msg):
    print(msg, flush=True)


def attend_case(kvd, B, Hq, Hkv, C_slots, k, w, seed):
    d = 128
    tdt = torch.bfloat16 if kvd == "bf16" else torch.float32
    g = torch.Generator().manual_seed(seed)
    rng = np.random.default_rng(seed)
    cK = torch.randn(B, Hq, C_slots, d, generator=g).to(tdt)
    cV = torch.randn(B, Hq, C_slots, d, generator=g).to(tdt)
    lK = torch.randn(B, Hkv, w, d, generator=g).to(tdt)
    lV = torch.randn(B, Hkv, w, d, generator=g).to(tdt)
    q = (torch.randn(B, Hq, d, generator=g) * 1.5).float()
    sel_slot = np.stack([np.stack([rng.permutation(C_slots)[:k] for _ in range(Hq)])
                         for _ in range(B)]).astype(np.int32)
    shp = L.Shape.make(B=B, Hq=Hq, Hkv=Hkv, l=max(k + w, C_slots) + 8, r=4, k=k, w=w,
                       C_slots=C_slots,
                       kv_dtype=L.LRQK_KV_BF16 if kvd == "bf16" else L.LRQK_KV_F32)
    return shp, q, cK, cV, sel_slot, lK, lV


def run_both(case, kvd):
    shp, q, cK, cV, sel_slot, lK, lV = case
    dq, dK, dV = q.to(DEV), cK.to(DEV), cV.to(DEV)
    dsel = torch.from_numpy(sel_slot).to(DEV)
    dlK, dlV = lK.to(DEV), lV.to(DEV)
    ws = torch.empty(L.lrqk_workspace_bytes(shp, L.LRQK_WS_ATTEND), dtype=torch.uint8, device=DEV)
    out_ws = torch.full((shp.B, shp.Hq, 128), float("nan"), device=DEV)
    out_na = torch.full((shp.B, shp.Hq, 128), float("nan"), device=DEV)
    L.lrqk_sparse_attend(shp, dq, dK, dV, dsel, dlK, dlV, out_ws, ws)
    torch.cuda.synchronize()
    mem_before = torch.cuda.memory_allocated()
    L.lrqk_sparse_attend_noalloc(shp, dq, dK, dV, dsel, dlK, dlV, out_na)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == mem_before
    a, b = out_ws.cpu().numpy(), out_na.cpu().numpy()
    assert np.array_equal(a, b), "noalloc entry point differs from lrqk_sparse_attend"
    ref = orc.sparse_attend(q.numpy(), as_numpy(cK), as_numpy(cV), sel_slot, as_numpy(lK),
                            as_numpy(lV), float(shp.scale))
    err = np.abs(b.astype(np.float64) - ref).max()
    say(f"   max abs err vs oracle {err:.3e}")
    assert err <= TOL[kvd]


@pytest.mark.parametrize("kvd", ["bf16", "fp32"])
def test_noalloc_attend_two_calls_second_smaller(kvd):
    say(f"noalloc attend kv={kvd}: 8 heads k=700 w=33, then 2 heads k=90 w=5")
    run_both(attend_case(kvd, 1, 8, 2, 1024, 700, 33, seed=101), kvd)
    run_both(attend_case(kvd, 1, 2, 1, 128, 90, 5, seed=102), kvd)


def test_noalloc_attend_rejects_oversize_and_bad_pointers():
    raw = L.load_library()
    A = 0x10000   # aligned fake address: never dereferenced on these paths
    # partial states of 16384 heads at k = 4096 exceed the fixed array
    big = L.Shape.make(B=2048, Hq=8, Hkv=8, l=8192, r=4, k=4096, w=0, C_slots=4096)
    assert L.lrqk_workspace_bytes(big, L.LRQK_WS_ATTEND) > (4 << 20)
    assert raw.lrqk_sparse_attend_noalloc(C.byref(big), A, A, A, A, A, A, A, None) == -4
    ok = L.Shape.make(B=1, Hq=8, Hkv=2, l=4096, r=4, k=256, w=16, C_slots=512)
    assert raw.lrqk_sparse_attend_noalloc(C.byref(ok), None, A, A, A, A, A, A, None) == -1
    assert raw.lrqk_sparse_attend_noalloc(C.byref(ok), A, A, A, A, None, A, A, None) == -1
