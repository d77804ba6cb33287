"""GPU parity of the decode-time factor update (lrqk_factor_update) against the CPU oracle
(oracle/lrqk_update_oracle.py), through the C ABI.

The update is fp32 linear algebra (Gram sums over the k + w rows of Omega, r x r Cholesky
solves); the oracle is float64.  Tolerance: the forward error of a backward-stable fp32
solve is about r * 2^-24 * cond(M) relative to the solution's norm; the synthetic workloads
have cond(M) of a few tens (A_Om^T A_Om dominates M, and its spectrum is that of k + w
Gaussian rows plus the planted plane), so with r <= 64 the bound is 64 * 6e-8 * ~10 = 4e-5.
The tests allow REL_TOL = 5e-5 of the largest entry of each output array and print what
they see (1e-6 .. 4e-6 on MI355X).
"""
import numpy as np
import pytest
import torch

import paper_2510_23649_amd as L
from gen import get_config, make_layer, QueryStream, as_numpy
from oracle import lrqk_update_oracle as upd
from gpu_harness import DEV, DeviceLayer, StepBuffers, workspace

pytestmark = pytest.mark.gpu

REL_TOL = 5e-5


def say(msg):
    print(msg, flush=True)


def upd_cfg(**kw):
    base = dict(B=2, Hq=8, Hkv=2, l=3000, r=32, k=300, w=40, C=600, n_heavy=32, pool_mult=4)
    base.update(kw)
    return get_config("c2").with_(**base)


def factors_for(cfg, data, seed, perturb=0.05):
    """B_K near the generator's basis, B_Q near its dual basis (what a prefill would hand over),
    both perturbed so that no term of the objective vanishes; a fresh key row k_t."""
    g = torch.Generator().manual_seed(seed)
    Bm = data.Bmat.cpu().double()                                     # [B,Hkv,r,d]
    dual = torch.linalg.solve(Bm @ Bm.transpose(-1, -2), Bm)          # (B B^T)^-1 B
    B_K = (Bm + perturb * torch.randn(Bm.shape, generator=g, dtype=torch.float64)).float()
    B_Q = dual.repeat_interleave(cfg.G, dim=1)
    B_Q = (B_Q + perturb * torch.randn(B_Q.shape, generator=g, dtype=torch.float64)).float()
    kvdt = torch.bfloat16 if cfg.kv_dtype == "bf16" else torch.float32
    k_hat_true = torch.randn(cfg.B, cfg.Hkv, cfg.r, generator=g, dtype=torch.float64)
    k_new = (torch.einsum("bhr,bhrd->bhd", k_hat_true, Bm) +
             0.05 * torch.randn(cfg.B, cfg.Hkv, cfg.d, generator=g, dtype=torch.float64)).to(kvdt)
    return B_Q.contiguous(), B_K.contiguous(), k_new.contiguous()


def run_update_case(cfg, lam1=1.0, lam2=1.0, n_iter=2, warm_steps=2, seed=7, drop=0):
    data = make_layer(cfg)
    dl = DeviceLayer(cfg, data)
    plan = L.Plan(dl.shape)
    qs = QueryStream(data)
    sb = StepBuffers(cfg)
    out = torch.empty((cfg.B, cfg.Hq, cfg.d), device=DEV)
    for step in range(1, warm_steps + 1):          # fills the cache; leaves the previous selection
        q, q_hat = qs.next()
        L.lrqk_decode_step(plan, dl.shape, step, dl.struct(), q_hat.to(DEV), q.to(DEV), out,
                           L.LRQK_FETCH_DIRECT, sb.debug())
    prev = sb.to_np()
    assert (prev["sel_slot"] >= 0).all()
    q, _ = qs.next()
    B_Q, B_K, k_new = factors_for(cfg, data, seed)
    omega = upd.omega_positions(prev["sel_idx"], cfg.l, cfg.w)
    if drop:
        # entries of the previous selection without a usable slot are left out of Omega
        rng = np.random.default_rng(seed)
        keep = np.ones(omega.shape, bool)
        slots = prev["sel_slot"].copy()
        for b in range(cfg.B):
            for h in range(cfg.Hq):
                gone = rng.choice(cfg.k, size=drop, replace=False)
                keep[b, h, gone] = False
                slots[b, h, gone[: drop // 2]] = -1
                slots[b, h, gone[drop // 2:]] = cfg.C + 3
        omega = omega[keep].reshape(cfg.B, cfg.Hq, -1)
        sb.sel_slot.copy_(torch.from_numpy(slots))
    ref = upd.factor_update(as_numpy(q), as_numpy(k_new), as_numpy(B_Q), as_numpy(B_K),
                            dl.np["A_K"], dl.np["K"], omega, lam1, lam2, n_iter)
    dBQ, dBK = B_Q.to(DEV), B_K.to(DEV)
    q_hat_d = torch.full((cfg.B, cfg.Hq, cfg.r), float("nan"), device=DEV)
    k_hat_d = torch.full((cfg.B, cfg.Hkv, cfg.r), float("nan"), device=DEV)
    ws = workspace(L.lrqk_workspace_bytes(dl.shape, L.LRQK_WS_UPDATE))
    L.lrqk_factor_update(dl.shape, dl.struct(), sb.sel_idx, sb.sel_slot, q.to(DEV), k_new.to(DEV),
                         dBQ, dBK, lam1, lam2, n_iter, q_hat_d, k_hat_d, ws)
    torch.cuda.synchronize()
    got = dict(q_hat=q_hat_d.cpu().numpy(), k_hat=k_hat_d.cpu().numpy(),
               B_Q=dBQ.cpu().numpy(), B_K=dBK.cpu().numpy())
    worst = 0.0
    for name, arr in got.items():
        assert np.all(np.isfinite(arr)), name
        rel = np.abs(arr - ref[name]).max() / np.abs(ref[name]).max()
        say(f"   {name}: max rel err {rel:.2e}")
        worst = max(worst, rel)
        assert rel <= REL_TOL, f"{name}: {rel}"
    # the step must really have moved B (the comparison above is not vacuous)
    assert np.abs(got["B_Q"] - as_numpy(B_Q)).max() > 1e-3
    assert np.abs(got["B_K"] - as_numpy(B_K)).max() > 1e-3
    plan.close()
    return worst


@pytest.mark.parametrize("r", [8, 16, 32, 64])
def test_factor_update_ranks(r):
    say(f"factor update r={r}")
    run_update_case(upd_cfg(r=r))


@pytest.mark.parametrize("G,Hkv", [(1, 3), (2, 2), (7, 1), (8, 1)])
def test_factor_update_group_sizes(G, Hkv):
    say(f"factor update G={G}")
    run_update_case(upd_cfg(B=1, Hq=G * Hkv, Hkv=Hkv, r=16))


def test_factor_update_fp32_rows_and_ragged_sizes():
    say("factor update, fp32 K rows, sizes that leave ragged chunks")
    run_update_case(upd_cfg(B=1, Hq=4, Hkv=2, l=2777, k=263, w=37, C=263, kv_dtype="f32"))


@pytest.mark.parametrize("lam1,lam2,n_iter", [(0.0, 0.0, 1), (1.0, 0.0, 2), (0.0, 1.0, 1),
                                              (0.5, 2.0, 4)])
def test_factor_update_lambdas_and_rounds(lam1, lam2, n_iter):
    say(f"factor update lambda_d1={lam1} lambda_d2={lam2} rounds={n_iter}")
    run_update_case(upd_cfg(B=1, Hq=4, Hkv=2, r=16), lam1, lam2, n_iter)


def test_factor_update_skips_entries_without_a_slot():
    say("factor update, 6 entries per head of the previous selection have no valid slot")
    run_update_case(upd_cfg(B=1, Hq=4, Hkv=2, r=16), drop=6)


def test_factor_update_no_lite_window():
    say("factor update with w = 0")
    run_update_case(upd_cfg(B=1, Hq=2, Hkv=1, r=16, w=0))


def test_factor_update_at_the_headline_shape():
    say("factor update at l = 131072, k = 2048, w = 64, r = 32, 32 / 8 heads")
    run_update_case(get_config("c3").with_(layers=1))


def test_factor_update_rejects_bad_arguments():
    cfg = upd_cfg(B=1, Hq=2, Hkv=1, r=12)
    shp = L.Shape.make(B=1, Hq=2, Hkv=1, l=cfg.l, r=12, k=cfg.k, w=cfg.w, C_slots=cfg.C)
    assert L.lrqk_workspace_bytes(shp, L.LRQK_WS_UPDATE) == 0
    t = torch.zeros(4096, device=DEV)
    ti = torch.zeros(4096, dtype=torch.int32, device=DEV)
    lay = L.make_layer(A_K=t, K_host=None, V_host=None, liteK=t, liteV=t, slot_of=ti,
                       token_of=ti, last_used=ti, cacheK=t, cacheV=t)
    with pytest.raises(L.LrqkError) as e:
        L.lrqk_factor_update(shp, lay, ti, ti, t, t, t, t, 1.0, 1.0, 2, t, t, workspace(1 << 20))
    assert e.value.status == -2
    shp16 = L.Shape.make(B=1, Hq=2, Hkv=1, l=cfg.l, r=16, k=cfg.k, w=cfg.w, C_slots=cfg.C)
    for bad in (dict(n_iter=0), dict(lam1=-1.0), dict(lam2=float("inf"))):
        with pytest.raises(L.LrqkError) as e:
            L.lrqk_factor_update(shp16, lay, ti, ti, t, t, t, t, bad.get("lam1", 1.0),
                                 bad.get("lam2", 1.0), bad.get("n_iter", 2), t, t,
                                 workspace(1 << 24))
        assert e.value.status == -1
    with pytest.raises(L.LrqkError) as e:
        L.lrqk_factor_update(shp16, lay, ti, ti, t, t, t, t, 1.0, 1.0, 2, t, t, workspace(256))
    assert e.value.status == -4


# ------------------------------------------------------------------ the whole of Alg. 2, l growing

def grow(ost, n_new_cols=1):
    """Oracle-side cache state for a context that is one token longer (new token: not cached)."""
    B, Hq, _ = ost.slot_of.shape
    ost.slot_of = np.concatenate(
        [ost.slot_of, np.full((B, Hq, n_new_cols), -1, np.int32)], axis=2)


@pytest.mark.parametrize("mode", ["direct", "staged"])
def test_alg2_steps_with_a_growing_context(mode):
    say(f"Alg. 2 with 40 appended tokens ({mode})")
    cfg = upd_cfg(B=1, Hq=4, Hkv=2, l=1500, r=16, k=128, w=24, C=256, n_heavy=16)
    new_selected, new_fetched = run_alg2_growing(cfg, 40, mode)
    assert new_selected > 0 and new_fetched > 0


def test_alg2_steps_at_the_headline_shape():
    say("Alg. 2 with 3 appended tokens at l = 131072, k = 2048, w = 64, r = 32, 32 / 8 heads")
    run_alg2_growing(get_config("c3").with_(layers=1), 3, "direct")


def run_alg2_growing(cfg, n_new, mode, lam1=1.0, lam2=1.0):
    """update -> append -> proxy scores / top-k / hit-miss / fetch / attention, for n_new new
    tokens.  Each step is compared with the oracle on its own: the oracle's update starts from
    the factors the GPU holds, and its integer decisions use the GPU's q_hat and k_hat (the
    paper's fp32), so rounding differences of the fp32 algebra are measured, never amplified
    into a different selection."""
    from oracle import lrqk_oracle as orc
    from gpu_harness import lite_ring
    from gpu_harness import compare_resolution
    l_cap = cfg.l + n_new
    data = make_layer(cfg)
    kvd = L.LRQK_KV_BF16
    shape0 = L.Shape.make(B=cfg.B, Hq=cfg.Hq, Hkv=cfg.Hkv, l=cfg.l, r=cfg.r, k=cfg.k, w=cfg.w,
                          C_slots=cfg.C, kv_dtype=kvd, scale=cfg.scale, l_cap=l_cap)
    lb = L.LayerBuffers(shape0, data.A_K, data.K, data.V)
    plan = L.Plan(shape0.with_l(l_cap))
    fmode = L.LRQK_FETCH_STAGED if mode == "staged" else L.LRQK_FETCH_DIRECT
    B, Hq, Hkv, G, r, d, w, k = cfg.B, cfg.Hq, cfg.Hkv, cfg.G, cfg.r, cfg.d, cfg.w, cfg.k
    # oracle side: arrays with room for the new rows
    A_np = np.zeros((B, Hkv, l_cap, r), np.float32)
    K_np = np.zeros((B, Hkv, l_cap, d), np.uint16)
    V_np = np.zeros_like(K_np)
    A_np[:, :, :cfg.l], K_np[:, :, :cfg.l], V_np[:, :, :cfg.l] = (as_numpy(data.A_K),
                                                                 as_numpy(data.K), as_numpy(data.V))
    ost = orc.CacheState(B, Hq, cfg.l, cfg.C)
    ocK = np.zeros((B, Hq, cfg.C, d), np.uint16)
    ocV = np.zeros_like(ocK)
    qs = QueryStream(data)
    sb = StepBuffers(cfg)
    out = torch.empty((B, Hq, d), device=DEV)
    B_Q, B_K, _ = factors_for(cfg, data, seed=11, perturb=0.02)
    dBQ, dBK = B_Q.to(DEV), B_K.to(DEV)
    q_hat_d = torch.zeros((B, Hq, r), device=DEV)
    k_hat_d = torch.zeros((B, Hkv, r), device=DEV)
    ws = workspace(L.lrqk_workspace_bytes(shape0.with_l(l_cap), L.LRQK_WS_UPDATE))
    gen = torch.Generator().manual_seed(99)
    Bm = data.Bmat.cpu().double()

    def step_and_compare(l, step, q, q_hat_t):
        shp = shape0.with_l(l)
        L.lrqk_decode_step(plan, shp, step, lb.struct, q_hat_t, q.to(DEV), out, fmode, sb.debug())
        got = sb.to_np()
        ref = orc.decode_step(np.ascontiguousarray(A_np[:, :, :l]), as_numpy(q_hat_t),
                              as_numpy(q), np.ascontiguousarray(K_np[:, :, :l]),
                              np.ascontiguousarray(V_np[:, :, :l]), ost, ocK, ocV, step, k, w,
                              cfg.scale)
        assert ref["ok"]
        assert np.array_equal(got["sel_idx"], ref["sel_idx"]), f"l={l}: selection differs"
        compare_resolution(got, ref, f"l={l}")
        assert np.array_equal(lb.slot_of.cpu().numpy()[:, :, :l], ost.slot_of), f"l={l}: slot_of"
        assert np.array_equal(lb.token_of.cpu().numpy(), ost.token_of), f"l={l}: token_of"
        assert np.array_equal(lb.last_used.cpu().numpy(), ost.last_used), f"l={l}: last_used"
        used = ost.token_of >= 0
        assert np.array_equal(as_numpy(lb.cacheK)[used], ocK[used]), f"l={l}: cached K rows"
        assert np.array_equal(as_numpy(lb.cacheV)[used], ocV[used]), f"l={l}: cached V rows"
        err = np.abs(out.cpu().numpy() - ref["out"]).max()
        assert err <= 2e-3, f"l={l}: attention error {err}"
        return got, ref

    step = 0
    for _ in range(2):                              # warm the cache with the generator's q_hat
        step += 1
        q, q_hat = qs.next()
        prev, _ = step_and_compare(cfg.l, step, q, q_hat.to(DEV))
    prev_q_hat = as_numpy(q_hat)
    new_selected = new_fetched = 0
    worst = 0.0
    for t in range(n_new):
        l = cfg.l + t
        shp = shape0.with_l(l)
        q, _ = qs.next()
        # the new key: near the span of B, its factor aligned with the group's first query head
        # (so that it is selected once it has left the lite window)
        dirs = torch.from_numpy(prev_q_hat[:, ::G, :].astype(np.float64))
        k_fac = 3.0 * dirs / dirs.norm(dim=-1, keepdim=True) + 0.3 * torch.randn(
            B, Hkv, r, generator=gen, dtype=torch.float64)
        k_new = (torch.einsum("bhr,bhrd->bhd", k_fac, Bm) +
                 0.05 * torch.randn(B, Hkv, d, generator=gen, dtype=torch.float64)).bfloat16()
        v_new = torch.randn(B, Hkv, d, generator=gen).bfloat16()
        BQ_before, BK_before = dBQ.cpu().numpy(), dBK.cpu().numpy()
        # u1
        L.lrqk_factor_update(shp, lb.struct, sb.sel_idx, sb.sel_slot, q.to(DEV), k_new.to(DEV),
                             dBQ, dBK, lam1, lam2, 2, q_hat_d, k_hat_d, ws)
        ref = upd.factor_update(as_numpy(q), as_numpy(k_new), BQ_before, BK_before, A_np, K_np,
                                upd.omega_positions(prev["sel_idx"], l, w), lam1, lam2, 2)
        got = dict(q_hat=q_hat_d.cpu().numpy(), k_hat=k_hat_d.cpu().numpy(),
                   B_Q=dBQ.cpu().numpy(), B_K=dBK.cpu().numpy())
        for name, arr in got.items():
            rel = np.abs(arr - ref[name]).max() / np.abs(ref[name]).max()
            worst = max(worst, rel)
            assert rel <= REL_TOL, f"l={l} {name}: {rel}"
        # u2
        L.lrqk_append_token(shp, lb.struct, k_hat_d, k_new.to(DEV), v_new.to(DEV))
        upd.append_token(A_np, K_np, V_np, l, got["k_hat"], as_numpy(k_new), as_numpy(v_new))
        torch.cuda.synchronize()
        assert np.array_equal(lb.A_K.cpu().numpy(), A_np), f"l={l}: A_K after append"
        assert np.array_equal(as_numpy(lb.K_host), K_np), f"l={l}: K store after append"
        assert np.array_equal(as_numpy(lb.V_host), V_np), f"l={l}: V store after append"
        ring = lite_ring(torch.from_numpy(K_np.view(np.int16)), l + 1, w).numpy().view(np.uint16)
        assert np.array_equal(as_numpy(lb.liteK), ring), f"l={l}: lite ring after append"
        grow(ost)
        # a1..a5 at length l + 1 with the GPU's q_hat
        step += 1
        prev, r2 = step_and_compare(l + 1, step, q, q_hat_d)
        prev_q_hat = got["q_hat"]
        new_selected += int((r2["sel_idx"] >= cfg.l).sum())
        for bh in range(B * Hq):
            nm = int(r2["n_miss"].reshape(-1)[bh])
            new_fetched += int((r2["miss_tok"].reshape(B * Hq, k)[bh, :nm] >= cfg.l).sum())
    say(f"   worst update error {worst:.2e}; appended tokens selected {new_selected} times, "
        f"fetched from the host store {new_fetched} times")
    plan.close()
    return new_selected, new_fetched
