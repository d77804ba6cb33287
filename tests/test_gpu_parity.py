"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element,
on seeded synthetic inputs.  Needs an MI355X: every test is marked `gpu`.

Bars: integer results (selection, hit/miss map, slots, miss lists, cache maps,
fetched rows) bit-exact; proxy scores bit-exact with the oracle's fp32 fma chain;
attention output max-abs error <= 2e-3 with bf16 K/V and <= 1e-5 with fp32 K/V.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2510_23649_amd as L
    from gpu_harness import (DEV, DeviceLayer, StepBuffers, compare_resolution, compare_state,
                             shape_of, workspace)

from gen import get_config, make_layer, QueryStream, as_numpy
from oracle import lrqk_oracle as orc
from helpers import check_topk_sets

TOL = {"bf16": 2e-3, "f32": 1e-5}


def small_cfg(**kw):
    base = dict(B=2, Hq=8, Hkv=2, l=3000, r=32, k=200, w=24, C=320, n_heavy=16, pool_mult=4,
                phase_spread=1.0, prefill="warm", rho=0.9)
    base.update(kw)
    return get_config("c1").with_(**base)


def say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------------------- a1

@pytest.mark.parametrize("r,G,l,B,Hkv", [
    (32, 4, 4096, 1, 8), (32, 4, 5000, 2, 2), (16, 4, 1031, 1, 2), (64, 4, 2049, 1, 2),
    (32, 7, 3001, 2, 1), (32, 1, 777, 1, 3), (32, 2, 255, 1, 2), (32, 8, 512, 1, 1),
    (16, 7, 300, 1, 1), (64, 1, 1000, 1, 1),
    (4, 4, 1000, 1, 2), (8, 3, 1500, 2, 2), (48, 5, 999, 1, 2), (128, 8, 700, 1, 1), (100, 6, 130, 1, 1),
])
def test_proxy_scores_bit_exact(r, G, l, B, Hkv):
    say(f"proxy_scores r={r} G={G} l={l} B={B} Hkv={Hkv}")
    rng = np.random.default_rng(r * 1000 + G * 10 + l)
    Hq = Hkv * G
    A_K = rng.standard_normal((B, Hkv, l, r)).astype(np.float32)
    q_hat = rng.standard_normal((B, Hq, r)).astype(np.float32)
    shp = L.Shape.make(B=B, Hq=Hq, Hkv=Hkv, l=l, r=r, k=1, w=0, C_slots=1)
    scores = torch.full((B, Hq, l), float("nan"), device=DEV)
    L.lrqk_proxy_scores(shp, torch.from_numpy(A_K).to(DEV), torch.from_numpy(q_hat).to(DEV), scores)
    torch.cuda.synchronize()
    _, s32 = orc.proxy_scores(A_K, q_hat)
    assert np.array_equal(scores.cpu().numpy().view(np.uint32), s32.view(np.uint32))


# ------------------------------------------------------------------------------- a2

def run_select(scores_np, k, w):
    B, Hq, l = scores_np.shape
    shp = L.Shape.make(B=B, Hq=Hq, Hkv=Hq, l=l, r=4, k=k, w=w, C_slots=max(k, 1))
    ws = workspace(L.lrqk_workspace_bytes(shp, L.LRQK_WS_SELECT))
    sel = torch.full((B, Hq, k), -1, dtype=torch.int32, device=DEV)
    L.lrqk_select_topk(shp, torch.from_numpy(scores_np).to(DEV), sel, ws)
    torch.cuda.synchronize()
    return sel.cpu().numpy()


@pytest.mark.parametrize("l,w,k,B,Hq", [
    (4096, 16, 256, 1, 8), (10000, 64, 1024, 2, 3), (70001, 64, 2048, 1, 4), (300, 0, 300, 1, 2),
    (257, 1, 1, 1, 2), (5000, 1000, 4000, 1, 2), (131072, 64, 2048, 1, 2), (4097, 0, 4096, 1, 1),
    (524288, 64, 2048, 1, 2),      # largest power of two handled by the one-workgroup kernel
    (800003, 64, 2048, 1, 2),      # beyond it: the multi-workgroup kernels
])
def test_select_topk_random(l, w, k, B, Hq):
    say(f"select_topk random l={l} w={w} k={k} B={B} Hq={Hq}")
    rng = np.random.default_rng(l + k)
    s = (rng.standard_normal((B, Hq, l)) * 11.3).astype(np.float32)
    s[:, :, l - w:] = 1e6      # the lite window must never be listed
    got = run_select(s, k, w)
    assert np.array_equal(got, orc.select_topk(s, k, w))


def test_select_topk_ties_zeros_and_massive_duplicates():
    say("select_topk ties / signed zeros / all-equal (threshold-bin overflow path)")
    rng = np.random.default_rng(5)
    l, w, k = 20000, 32, 1500
    s = np.empty((1, 6, l), np.float32)
    s[0, 0] = np.round(rng.standard_normal(l) * 4) / 4            # heavy exact ties
    s[0, 1] = 3.25                                                # all equal: lowest positions win
    s[0, 2] = rng.choice(np.array([0.0, -0.0], np.float32), l)    # +0 and -0 are equal
    s[0, 3] = -np.abs(rng.standard_normal(l)).astype(np.float32)  # all negative
    s[0, 4] = rng.choice(np.array([1.0, 1.0 + 2 ** -23, 1.0 - 2 ** -24], np.float32), l)  # one bin, 3 keys
    s[0, 5] = np.where(rng.random(l) < 0.02, 50.0, 0.5).astype(np.float32)  # few above, rest tied
    got = run_select(s, k, w)
    assert np.array_equal(got, orc.select_topk(s, k, w))
    assert np.array_equal(got[0, 1], np.arange(k))


def test_select_topk_sampled_estimate_is_verified_not_trusted():
    say("select_topk, long heads: inputs built to mislead the 1-in-8 sample, and heavy ties")
    rng = np.random.default_rng(9)
    l, w, k = 150000, 64, 2048
    e = np.arange(l)
    sampled = ((e // 4096) & 7) == (((e % 4096) // 256) & 7)     # positions the first pass looks at
    s = np.empty((1, 8, l), np.float32)
    base = (rng.standard_normal(l) * 11.3).astype(np.float32)
    s[0, 0] = np.where(sampled, -1.0, base)                      # sample sees one value only
    s[0, 1] = np.where(sampled, base + 200.0, base)              # sample far above the rest
    s[0, 2] = np.where(sampled, base - 200.0, base)              # sample far below the rest
    s[0, 3] = 7.5                                                # every score equal
    s[0, 4] = np.round(base)                                     # heavy ties around the threshold
    s[0, 5] = np.where(rng.random(l) < 0.01, 1e3, -1e3)          # 1500 large, rest equal: k cuts the ties
    s[0, 6] = base
    s[0, 6, :3000] = 1e4                                         # more than k at the top, all tied
    s[0, 7] = -np.abs(base) - 1.0
    got = run_select(s, k, w)
    assert np.array_equal(got, orc.select_topk(s, k, w))


# ------------------------------------------------------------------------------- a3 + a4

@pytest.mark.parametrize("mode", ["staged", "direct"])
@pytest.mark.parametrize("kvd,C", [("bf16", 320), ("bf16", 200), ("f32", 256)])
def test_resolve_and_fetch_over_steps(kvd, C, mode):
    say(f"cache_resolve + fetch_misses kv={kvd} C={C} mode={mode}")
    cfg = small_cfg(kv_dtype=kvd, C=C)
    data = make_layer(cfg)
    dl = DeviceLayer(cfg, data)
    plan = L.Plan(dl.shape)
    sb = StepBuffers(cfg)
    rng = np.random.default_rng(C)
    pool = rng.permutation(cfg.l - cfg.w)[: 3 * cfg.k]     # selections overlap from step to step
    fmode = L.LRQK_FETCH_STAGED if mode == "staged" else L.LRQK_FETCH_DIRECT
    for step in range(6):
        sel = np.sort(np.stack([np.stack([rng.choice(pool, cfg.k, replace=False)
                                          for _ in range(cfg.Hq)]) for _ in range(cfg.B)]),
                      axis=-1).astype(np.int32)
        sb.sel_idx.copy_(torch.from_numpy(sel))
        L.lrqk_cache_resolve(dl.shape, sb.sel_idx, step, dl.slot_of, dl.token_of, dl.last_used,
                             sb.sel_slot, sb.hit, sb.miss_tok, sb.miss_slot, sb.n_miss)
        total = L.lrqk_fetch_misses(plan, dl.shape, dl.K_host, dl.V_host, sb.miss_tok,
                                    sb.miss_slot, sb.n_miss, dl.cacheK, dl.cacheV, fmode)
        ref = orc.cache_resolve(sel, step, dl.ost)
        assert ref["ok"]
        orc.fetch(dl.np["K"], dl.np["V"], ref["miss_tok"], ref["miss_slot"], ref["n_miss"],
                  dl.ocK, dl.ocV)
        compare_resolution(sb.to_np(), ref, f"step {step}")
        compare_state(dl, f"step {step}")
        if mode == "staged":
            assert total == int(ref["n_miss"].sum())
        if mode == "group":     # rows over the host link: the oracle's shared fetch of the same lists
            scratchK, scratchV = np.zeros_like(dl.ocK), np.zeros_like(dl.ocV)
            want_rows, _ = orc.group_fetch(dl.np["K"], dl.np["V"], ref["miss_tok"], ref["miss_slot"],
                                           ref["n_miss"], scratchK, scratchV)
            assert np.array_equal(got["link_rows"], want_rows), f"step {step}: rows over the link"
            link_rows_seen.append((int(want_rows.sum()), int(ref["n_miss"].sum())))
        if step > 0:
            assert 0 < ref["n_miss"].sum() < sel.size     # the case has both hits and misses
    plan.close()


def test_resolve_contract_violations_do_not_fault():
    say("cache_resolve with a reused step and an out-of-range position")
    cfg = small_cfg(B=1, Hq=2, Hkv=1, l=500, k=8, w=4, C=8)
    shp = shape_of(cfg)
    dl = DeviceLayer(cfg, make_layer(cfg))
    sb = StepBuffers(cfg)
    sel = np.array([[[1, 2, 3, 4, 5, 6, 7, 8], [10, 20, 30, 40, 50, 60, 70, 9999]]], np.int32)
    sb.sel_idx.copy_(torch.from_numpy(sel))
    L.lrqk_cache_resolve(shp, sb.sel_idx, 3, dl.slot_of, dl.token_of, dl.last_used, sb.sel_slot,
                         sb.hit, sb.miss_tok, sb.miss_slot, sb.n_miss)
    got = sb.to_np()
    assert got["n_miss"][0, 0] == 8 and got["n_miss"][0, 1] == -1
    assert got["sel_slot"][0, 1, 7] == -1
    sel2 = np.array([[[11, 12, 13, 14, 15, 16, 17, 18], [1, 2, 3, 4, 5, 6, 7, 8]]], np.int32)
    sb.sel_idx.copy_(torch.from_numpy(sel2))
    L.lrqk_cache_resolve(shp, sb.sel_idx, 3, dl.slot_of, dl.token_of, dl.last_used, sb.sel_slot,
                         sb.hit, sb.miss_tok, sb.miss_slot, sb.n_miss)     # same step again
    got = sb.to_np()
    assert got["n_miss"][0, 0] == -1           # every slot is protected: no victims
    assert (got["sel_slot"][0, 0] == -1).all()
    # the staged fetch sees the lists on the host and refuses them; the device-side fetches skip
    plan = L.Plan(shp)
    with pytest.raises(L.LrqkError) as e:
        L.lrqk_fetch_misses(plan, shp, dl.K_host, dl.V_host, sb.miss_tok, sb.miss_slot, sb.n_miss,
                            dl.cacheK, dl.cacheV, L.LRQK_FETCH_STAGED)
    assert e.value.status == -5
    for mode in (L.LRQK_FETCH_DIRECT, L.LRQK_FETCH_GROUP):
        L.lrqk_fetch_misses(plan, shp, dl.K_host, dl.V_host, sb.miss_tok, sb.miss_slot, sb.n_miss,
                            dl.cacheK, dl.cacheV, mode)
    torch.cuda.synchronize()
    plan.close()


# ------------------------------------------------------------------------------- a5

@pytest.mark.parametrize("kvd", ["bf16", "f32"])
@pytest.mark.parametrize("k,w,C,B,Hq,Hkv", [
    (200, 24, 320, 2, 8, 2), (1, 0, 1, 1, 1, 1), (64, 0, 64, 1, 4, 4), (2048, 64, 4096, 1, 8, 2),
    (33, 1000, 40, 1, 7, 1), (1000, 13, 1000, 2, 4, 2),
])
def test_sparse_attend(kvd, k, w, C, B, Hq, Hkv):
    say(f"sparse_attend kv={kvd} k={k} w={w} C={C} B={B} Hq={Hq} Hkv={Hkv}")
    rng = np.random.default_rng(k + w)
    d = 128
    tdt = torch.bfloat16 if kvd == "bf16" else torch.float32
    g = torch.Generator().manual_seed(k * 7 + w)
    cK = torch.randn(B, Hq, C, d, generator=g).to(tdt)
    cV = torch.randn(B, Hq, C, d, generator=g).to(tdt)
    lK = torch.randn(B, Hkv, w, d, generator=g).to(tdt)
    lV = torch.randn(B, Hkv, w, d, generator=g).to(tdt)
    q = (torch.randn(B, Hq, d, generator=g) * 1.5).float()
    sel_slot = np.stack([np.stack([rng.permutation(C)[:k] for _ in range(Hq)])
                         for _ in range(B)]).astype(np.int32)
    if k > 4:
        sel_slot[0, 0, 3] = -1          # skipped rows
        sel_slot[0, 0, 4] = C + 5
    shp = L.Shape.make(B=B, Hq=Hq, Hkv=Hkv, l=max(k + w, C) + 8, r=4, k=k, w=w, C_slots=C,
                       kv_dtype=L.LRQK_KV_BF16 if kvd == "bf16" else L.LRQK_KV_F32)
    ws = workspace(L.lrqk_workspace_bytes(shp, L.LRQK_WS_ATTEND))
    out = torch.full((B, Hq, d), float("nan"), device=DEV)
    L.lrqk_sparse_attend(shp, q.to(DEV), cK.to(DEV), cV.to(DEV), torch.from_numpy(sel_slot).to(DEV),
                         lK.to(DEV) if w else None, lV.to(DEV) if w else None, out, ws)
    torch.cuda.synchronize()
    lKn = as_numpy(lK) if w else np.zeros((B, Hkv, 0, d), as_numpy(cK).dtype)
    lVn = as_numpy(lV) if w else np.zeros((B, Hkv, 0, d), as_numpy(cK).dtype)
    ref = orc.sparse_attend(q.numpy(), as_numpy(cK), as_numpy(cV), sel_slot, lKn, lVn,
                            float(shp.scale))
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref).max()
    say(f"   max abs err {err:.3e}")
    assert err <= TOL[kvd]


def test_sparse_attend_closed_forms():
    say("sparse_attend: equal keys -> mean of V; dominant logit -> that row")
    d, C, k = 128, 300, 300
    g = torch.Generator().manual_seed(11)
    q = torch.randn(1, 1, d, generator=g)
    V = torch.randn(1, 1, C, d, generator=g)
    K = torch.randn(1, 1, 1, d, generator=g).expand(1, 1, C, d).contiguous()
    shp = L.Shape.make(B=1, Hq=1, Hkv=1, l=C, r=4, k=k, w=0, C_slots=C, kv_dtype=L.LRQK_KV_F32)
    ws = workspace(L.lrqk_workspace_bytes(shp, L.LRQK_WS_ATTEND))
    sel = torch.arange(k, dtype=torch.int32, device=DEV).reshape(1, 1, k)
    out = torch.empty(1, 1, d, device=DEV)
    L.lrqk_sparse_attend(shp, q.to(DEV), K.to(DEV), V.to(DEV), sel, None, None, out, ws)
    assert np.abs(out.cpu().numpy()[0, 0] - V[0, 0].double().mean(0).numpy()).max() < 1e-5
    K2 = 0.01 * torch.randn(1, 1, C, d, generator=g)
    K2[0, 0, 123] = 300.0 * q[0, 0] / (q[0, 0] @ q[0, 0])     # logit 300/sqrt(128) above the rest
    L.lrqk_sparse_attend(shp, q.to(DEV), K2.to(DEV), V.to(DEV), sel, None, None, out, ws)
    assert np.abs(out.cpu().numpy()[0, 0] - V[0, 0, 123].numpy()).max() < 1e-5


# ------------------------------------------------------------------------------- a1..a5

def run_steps_against_oracle(cfg, n_steps, mode, identity=False, data=None, check_unfused=True,
                             carry="fresh_first", step_number=None, quiet=False):
    """Drive lrqk_decode_step for n_steps and compare every step with the oracle.
    carry: how the selection's candidate thresholds are obtained -- "off": estimated from a sample
    in every step (no lrqk_layer.sel_thr); "fresh_first": from a sample in the first step
    (LRQK_SELECT_FRESH), carried from step to step afterwards; "unknown_first": carried, the first
    step starting from unknown (NaN) thresholds, which sends every head down the exact route."""
    data = data or make_layer(cfg)
    dl = DeviceLayer(cfg, data, identity=identity, carry=carry != "off")
    plan = L.Plan(dl.shape)
    lay = dl.struct()
    qs = QueryStream(data)
    sb = StepBuffers(cfg)
    out = torch.empty((cfg.B, cfg.Hq, cfg.d), device=DEV)
    fmode = {"staged": L.LRQK_FETCH_STAGED, "direct": L.LRQK_FETCH_DIRECT,
             "group": L.LRQK_FETCH_GROUP}[mode]
    miss_rates = []
    link_rows_seen = []
    for index in range(1, n_steps + 1):
        step = step_number(index) if step_number else index   # the caller's step counter
        q, q_hat = qs.next()
        qd, qhd = q.to(DEV), q_hat.to(DEV)
        if check_unfused and index == 1:
            unfused = run_unfused(cfg, dl, qd, qhd, step)      # on copies of the state
        flags = L.LRQK_SELECT_FRESH if (carry == "fresh_first" and index == 1) else 0
        total = L.lrqk_decode_step(plan, dl.shape, step, lay, qhd, qd, out, fmode | flags,
                                   sb.debug())
        got = sb.to_np()
        ref = orc.decode_step(dl.np["A_K"], as_numpy(q_hat), as_numpy(q), dl.np["K"], dl.np["V"],
                              dl.ost, dl.ocK, dl.ocV, step, cfg.k, cfg.w, cfg.scale)
        assert ref["ok"]
        assert np.array_equal(got["sel_idx"], ref["sel_idx"]), (
            f"step {step}: selection differs; near-tie heads: "
            f"{check_topk_sets(got['sel_idx'], ref['sel_idx'], ref['s64'], cfg.w)}")
        compare_resolution(got, ref, f"step {step}")
        compare_state(dl, f"step {step}")
        err = np.abs(out.cpu().numpy().astype(np.float64) - ref["out"]).max()
        if not quiet:
            say(f"   step {step}: miss rate {ref['miss_rate']:.3f}  max abs err {err:.3e}")
        assert err <= TOL[cfg.kv_dtype], f"step {step}: attention error {err}"
        if mode == "staged":
            assert total == int(ref["n_miss"].sum())
        if mode == "group":     # rows over the host link: the oracle's shared fetch of the same lists
            scratchK, scratchV = np.zeros_like(dl.ocK), np.zeros_like(dl.ocV)
            want_rows, _ = orc.group_fetch(dl.np["K"], dl.np["V"], ref["miss_tok"], ref["miss_slot"],
                                           ref["n_miss"], scratchK, scratchV)
            assert np.array_equal(got["link_rows"], want_rows), f"step {step}: rows over the link"
            link_rows_seen.append((int(want_rows.sum()), int(ref["n_miss"].sum())))
        if check_unfused and index == 1:
            for name in ("sel_idx", "sel_slot", "hit", "n_miss"):
                assert np.array_equal(unfused[name], got[name]), f"fused/unfused {name} differ"
            assert np.abs(unfused["out"] - out.cpu().numpy()).max() <= 1e-5
        miss_rates.append(ref["miss_rate"])
    plan.close()
    if mode == "group":
        return miss_rates, link_rows_seen
    return miss_rates


def run_unfused(cfg, dl, q, q_hat, step):
    """a1, a2, a3, a4, a5 as five separate calls on clones of the cache state."""
    shp = dl.shape
    scores = torch.empty((cfg.B, cfg.Hq, cfg.l), device=DEV)
    sb = StepBuffers(cfg)
    slot_of, token_of, last_used = dl.slot_of.clone(), dl.token_of.clone(), dl.last_used.clone()
    cK, cV = dl.cacheK.clone(), dl.cacheV.clone()
    plan = L.Plan(shp)
    L.lrqk_proxy_scores(shp, dl.A_K, q_hat, scores)
    L.lrqk_select_topk(shp, scores, sb.sel_idx, workspace(L.lrqk_workspace_bytes(shp, L.LRQK_WS_SELECT)))
    L.lrqk_cache_resolve(shp, sb.sel_idx, step, slot_of, token_of, last_used, sb.sel_slot, sb.hit,
                         sb.miss_tok, sb.miss_slot, sb.n_miss)
    L.lrqk_fetch_misses(plan, shp, dl.K_host, dl.V_host, sb.miss_tok, sb.miss_slot, sb.n_miss,
                        cK, cV, L.LRQK_FETCH_STAGED)
    out = torch.empty((cfg.B, cfg.Hq, cfg.d), device=DEV)
    L.lrqk_sparse_attend(shp, q, cK, cV, sb.sel_slot, dl.liteK, dl.liteV, out,
                         workspace(L.lrqk_workspace_bytes(shp, L.LRQK_WS_ATTEND)))
    res = sb.to_np()
    res["out"] = out.cpu().numpy()
    plan.close()
    return res


@pytest.mark.parametrize("mode", ["staged", "direct"])
@pytest.mark.parametrize("kvd", ["bf16", "f32"])
def test_decode_step_small(kvd, mode):
    say(f"decode_step small kv={kvd} mode={mode}")
    rates = run_steps_against_oracle(small_cfg(kv_dtype=kvd), 5, mode)
    assert rates[0] == 1.0 and rates[-1] < 1.0


@pytest.mark.parametrize("share,kvd", [(0.0, "bf16"), (0.5, "bf16"), (1.0, "f32")])
def test_decode_step_group_shared_fetch(share, kvd):
    say(f"decode_step, fetch shared inside the KV groups, group_share={share} kv={kvd}")
    cfg = small_cfg(kv_dtype=kvd, group_share=share, Hq=8, Hkv=2)
    rates, link = run_steps_against_oracle(cfg, 6, "group", check_unfused=False)
    union, total = sum(u for u, _ in link[1:]), sum(t for _, t in link[1:])
    say(f"   rows over the link / rows missed (after the first step): {union} / {total}")
    if share == 0.0:
        assert union > 0.9 * total
    if share == 1.0:
        assert union * cfg.G == total        # identical queries in a group: one fetch serves all


def test_group_fetch_alone_fills_the_same_caches_as_the_oracle():
    say("lrqk_fetch_misses, LRQK_FETCH_GROUP: caches and shared rows vs the oracle")
    rng = np.random.default_rng(31)
    B, Hkv, G, l, C, k, d = 2, 2, 4, 5000, 600, 500, 128
    Hq = Hkv * G
    K = torch.randn(B, Hkv, l, d, generator=torch.Generator().manual_seed(1)).bfloat16()
    V = torch.randn(B, Hkv, l, d, generator=torch.Generator().manual_seed(2)).bfloat16()
    miss_tok = np.full((B, Hq, k), -1, np.int32)
    miss_slot = np.full((B, Hq, k), -1, np.int32)
    n_miss = rng.integers(0, k + 1, size=(B, Hq)).astype(np.int32)
    n_miss[1, 2] = 0
    for b in range(B):
        for kv in range(Hkv):
            common = rng.choice(l, size=k, replace=False)          # what the group tends to want
            for h in range(kv * G, (kv + 1) * G):
                n = n_miss[b, h]
                mix = np.unique(np.concatenate([rng.choice(common, size=n // 2, replace=False),
                                                rng.choice(l, size=n - n // 2, replace=False)]))
                n_miss[b, h] = len(mix)
                miss_tok[b, h, :len(mix)] = mix
                miss_slot[b, h, :len(mix)] = rng.permutation(C)[:len(mix)]
    shp = L.Shape.make(B=B, Hq=Hq, Hkv=Hkv, l=l, r=4, k=k, w=0, C_slots=C)
    plan = L.Plan(shp)
    cK = torch.zeros(B, Hq, C, d, dtype=torch.bfloat16, device=DEV)
    cV = torch.zeros_like(cK)
    L.lrqk_fetch_misses(plan, shp, K.pin_memory(), V.pin_memory(), torch.from_numpy(miss_tok).to(DEV),
                        torch.from_numpy(miss_slot).to(DEV), torch.from_numpy(n_miss).to(DEV),
                        cK, cV, L.LRQK_FETCH_GROUP)
    torch.cuda.synchronize()
    oK = np.zeros((B, Hq, C, d), np.uint16)
    oV = np.zeros_like(oK)
    rows, _ = orc.group_fetch(as_numpy(K), as_numpy(V), miss_tok, miss_slot, n_miss, oK, oV)
    assert np.array_equal(as_numpy(cK), oK) and np.array_equal(as_numpy(cV), oV)
    assert rows.sum() < n_miss.sum()             # the lists do overlap
    plan.close()


@pytest.mark.parametrize("shape", [
    dict(B=1, Hq=1, Hkv=1, l=300, r=16, k=1, w=0, C=1),             # one token, one slot
    dict(B=1, Hq=2, Hkv=2, l=777, r=64, k=700, w=77, C=700),        # k + w = l: dense selection
    dict(B=3, Hq=8, Hkv=1, l=5000, r=32, k=64, w=1, C=64),          # G = 8, cache of exactly k slots
    dict(B=1, Hq=4, Hkv=2, l=9000, r=16, k=1500, w=1000, C=8192),   # largest cache, widest window
    dict(B=2, Hq=7, Hkv=1, l=4097, r=32, k=333, w=5, C=400),        # G = 7, ragged everything
    dict(B=1, Hq=2, Hkv=1, l=150000, r=16, k=4096, w=64, C=4096),   # largest k, three groups per thread
    dict(B=1, Hq=2, Hkv=2, l=70000, r=8, k=500, w=16, C=1000),      # rank outside the filtered pass
    dict(B=1, Hq=6, Hkv=2, l=3000, r=32, k=100, w=10, C=150),       # G = 3: generic proxy kernel
    dict(B=1, Hq=2, Hkv=1, l=16384, r=32, k=4096, w=64, C=4096),    # a quarter of the context selected
    dict(B=1, Hq=2, Hkv=1, l=12000, r=32, k=1400, w=64, C=2048),    # about 10 candidates per group
    dict(B=2, Hq=4, Hkv=4, l=70, r=16, k=20, w=3, C=25),            # a context of two 64-position groups
    dict(B=1, Hq=8, Hkv=2, l=64, r=32, k=64, w=0, C=64),            # one group, everything selected, no lite rows
])
@pytest.mark.parametrize("mode", ["direct", "group", "staged"])
def test_decode_step_shape_sweep(shape, mode):
    say(f"decode_step shape sweep {shape} ({mode})")
    G = shape["Hq"] // shape["Hkv"]
    n_heavy = max(1, min(64, shape["k"] // 4, (shape["l"] - shape["w"]) // (4 * G)))
    cfg = small_cfg(n_heavy=n_heavy, **shape)
    run_steps_against_oracle(cfg, 4, mode, check_unfused=False, quiet=True)


def test_decode_step_step_counter_far_ahead_of_the_slots_ages():
    say("decode_step with step numbers that jump by thousands (ages beyond the victim histogram)")
    # steps 1, 2, 3, then 5000, 5001, 9000, 9001: the slots' ages exceed the 2048 classes of the
    # age histogram, which then cannot order them; the all-slots ordering must give the same
    # least-recently-selected victims as the oracle
    numbers = {1: 1, 2: 2, 3: 3, 4: 5000, 5: 5001, 6: 9000, 7: 9001}
    rates = run_steps_against_oracle(small_cfg(), 7, "direct", check_unfused=False,
                                     step_number=lambda i: numbers[i])
    assert all(r > 0 for r in rates)


def _crafted_steps(cfg, data, queries, mutate=None):
    """lrqk_decode_step (direct fetch, thresholds sampled in the first step, carried afterwards)
    against the oracle for the given (q, q_hat) pairs; mutate(i, dl) may change the layer before
    step i."""
    dl = DeviceLayer(cfg, data)
    plan = L.Plan(dl.shape)
    sb = StepBuffers(cfg)
    out = torch.empty((cfg.B, cfg.Hq, cfg.d), device=DEV)
    for i, (q, q_hat) in enumerate(queries, start=1):
        if mutate:
            mutate(i, dl)
        L.lrqk_decode_step(plan, dl.shape, i, dl.struct(), q_hat.to(DEV), q.to(DEV), out,
                           L.LRQK_FETCH_DIRECT | (L.LRQK_SELECT_FRESH if i == 1 else 0), sb.debug())
        got = sb.to_np()
        ref = orc.decode_step(dl.np["A_K"], as_numpy(q_hat), as_numpy(q), dl.np["K"], dl.np["V"],
                              dl.ost, dl.ocK, dl.ocV, i, cfg.k, cfg.w, cfg.scale)
        assert np.array_equal(got["sel_idx"], ref["sel_idx"]), f"step {i}: selection differs"
        compare_resolution(got, ref, f"step {i}")
        compare_state(dl, f"step {i}")
        assert np.abs(out.cpu().numpy() - ref["out"]).max() <= TOL[cfg.kv_dtype]
    plan.close()


def test_decode_step_scores_with_massive_ties():
    say("decode_step: only 97 distinct rows in A_K, every score repeated hundreds of times")
    cfg = small_cfg(B=1, Hq=4, Hkv=2, l=70000, r=32, k=1024, w=64, C=2048, n_heavy=64)
    data = make_layer(cfg)
    n = cfg.l
    data.A_K[:] = data.A_K[:, :, torch.arange(n) % 97, :]      # the k-th largest sits inside a tie
    qs = QueryStream(data)
    _crafted_steps(cfg, data, [qs.next() for _ in range(3)])


def test_decode_step_all_scores_negative():
    say("decode_step: every proxy score negative (threshold keys below zero)")
    cfg = small_cfg(B=1, Hq=4, Hkv=2, l=70000, r=32, k=1024, w=64, C=2048, n_heavy=64)
    data = make_layer(cfg)
    data.A_K.abs_()
    qs = QueryStream(data)
    queries = [(q, -q_hat.abs()) for q, q_hat in (qs.next() for _ in range(3))]
    _crafted_steps(cfg, data, queries)


def test_decode_step_selection_far_above_a_stale_threshold():
    say("decode_step: the k largest scores jump a hundredfold above the carried threshold")
    cfg = small_cfg(B=1, Hq=4, Hkv=2, l=70000, r=32, k=1024, w=64, C=2048, n_heavy=64)
    data = make_layer(cfg)
    qs = QueryStream(data)
    rng = np.random.default_rng(3)
    boosted = torch.from_numpy(np.sort(rng.choice(cfg.l - cfg.w, 3500, replace=False)))

    def mutate(i, dl):
        if i == 2:       # 3500 rows times 100, all others times 0.01: about 1750 positive giants,
            scale = torch.full((cfg.l, 1), 0.01)           # more than k, few enough to stay candidates
            scale[boosted] = 100.0
            dl.A_K.mul_(scale.to(DEV))
            dl.np["A_K"] = dl.A_K.cpu().numpy()
    _crafted_steps(cfg, data, [qs.next() for _ in range(3)], mutate)


@pytest.mark.parametrize("n_classes", [3, 50])
def test_decode_step_victims_spread_over_age_classes(n_classes):
    say(f"decode_step: one step with about 300 misses, victims drawn from {n_classes} age classes")
    # the cache starts full of tokens the step will not select, their slots last used at
    # n_classes different earlier steps (8 .. 130 slots a class): the victims have to come out in
    # (last_used, slot) order across all of them
    cfg = small_cfg(B=1, Hq=4, Hkv=2, l=6000, k=300, w=16, C=400, n_heavy=64)
    data = make_layer(cfg)
    dl = DeviceLayer(cfg, data)
    G = cfg.G
    slots = np.arange(cfg.C, dtype=np.int32)
    toks = 5000 + slots                                    # positions the proxy scores rank low
    data.A_K[:, :, 5000:5000 + cfg.C, :] *= 0.01
    dl.A_K.copy_(data.A_K)
    dl.np["A_K"] = as_numpy(data.A_K)
    last = (1 + (slots * 7) % n_classes).astype(np.int32)
    for b in range(cfg.B):
        for h in range(cfg.Hq):
            dl.ost.token_of[b, h] = toks
            dl.ost.last_used[b, h] = last
            dl.ost.slot_of[b, h, toks] = slots
            dl.ocK[b, h] = dl.np["K"][b, h // G, toks]
            dl.ocV[b, h] = dl.np["V"][b, h // G, toks]
    dl.token_of.copy_(torch.from_numpy(dl.ost.token_of))
    dl.last_used.copy_(torch.from_numpy(dl.ost.last_used))
    dl.slot_of.copy_(torch.from_numpy(dl.ost.slot_of))
    dl.cacheK.copy_(torch.from_numpy(dl.ocK.view(np.int16)).view(torch.bfloat16))
    dl.cacheV.copy_(torch.from_numpy(dl.ocV.view(np.int16)).view(torch.bfloat16))
    plan = L.Plan(dl.shape)
    qs = QueryStream(data)
    sb = StepBuffers(cfg)
    out = torch.empty((cfg.B, cfg.Hq, cfg.d), device=DEV)
    for step in (60, 61):
        q, q_hat = qs.next()
        L.lrqk_decode_step(plan, dl.shape, step, dl.struct(), q_hat.to(DEV), q.to(DEV), out,
                           L.LRQK_FETCH_DIRECT | (L.LRQK_SELECT_FRESH if step == 60 else 0),
                           sb.debug())
        got = sb.to_np()
        ref = orc.decode_step(dl.np["A_K"], as_numpy(q_hat), as_numpy(q), dl.np["K"], dl.np["V"],
                              dl.ost, dl.ocK, dl.ocV, step, cfg.k, cfg.w, cfg.scale)
        assert np.array_equal(got["sel_idx"], ref["sel_idx"])
        compare_resolution(got, ref, f"step {step}")
        compare_state(dl, f"step {step}")
        assert np.abs(out.cpu().numpy() - ref["out"]).max() <= TOL[cfg.kv_dtype]
        if step == 60:
            assert ref["n_miss"].min() > 250          # nearly everything misses
    plan.close()


@pytest.mark.parametrize("seed", [11, 12])
def test_decode_step_random_shapes(seed):
    say(f"decode_step on 30 random shapes, fetch modes and threshold sources (seed {seed})")
    rng = np.random.default_rng(seed)
    for it in range(30):
        G, Hkv, B = int(rng.choice([1, 2, 3, 4, 7, 8])), int(rng.integers(1, 3)), int(rng.integers(1, 3))
        r = int(rng.choice([8, 16, 32, 64, 12, 48]))
        l = int(rng.choice([int(rng.integers(70, 400)), int(rng.integers(400, 9000)),
                            int(rng.integers(9000, 90000))]))
        w = int(rng.integers(0, min(l // 3, 200)))
        kmax = min(l - w, 4096)
        k = int(rng.choice([1, int(rng.integers(1, max(2, kmax // 20))), int(rng.integers(1, kmax + 1))]))
        C = int(min(8192, k + rng.choice([0, 1, int(rng.integers(0, 2 * k + 2))])))
        mode = str(rng.choice(["direct", "group", "staged"]))
        carry = str(rng.choice(["fresh_first", "off", "unknown_first"]))
        shape = dict(B=B, Hq=G * Hkv, Hkv=Hkv, l=l, r=r, k=k, w=w, C=C,
                     kv_dtype=str(rng.choice(["bf16", "f32"])))
        say(f"   {it}: {shape} {mode} {carry}")
        cfg = small_cfg(n_heavy=max(1, min(64, k // 4, (l - w) // (4 * G))), **shape)
        run_steps_against_oracle(cfg, 3, mode, check_unfused=False, carry=carry, quiet=True)


@pytest.mark.parametrize("carry", ["off", "unknown_first"])
def test_decode_step_threshold_sources(carry):
    say(f"decode_step small, candidate thresholds: {carry}")
    run_steps_against_oracle(small_cfg(), 5, "direct", carry=carry, check_unfused=False)


def test_decode_step_carried_threshold_survives_a_change_of_scale():
    say("decode_step: the carried threshold meets scores 40x larger, then 1000x smaller")
    cfg = small_cfg(B=1, Hq=8, Hkv=2, l=70000, r=32, k=1024, w=64, C=2048, n_heavy=64)
    data = make_layer(cfg)
    dl = DeviceLayer(cfg, data)
    plan = L.Plan(dl.shape)
    qs = QueryStream(data)
    sb = StepBuffers(cfg)
    out = torch.empty((cfg.B, cfg.Hq, cfg.d), device=DEV)
    thr_seen = []
    for step, factor in enumerate([1.0, 1.0, 40.0, 40.0, 0.04, 0.04, 1.0], start=1):
        q, q_hat = qs.next()
        # heads 0..3 keep their scale: only |q_hat| of heads 4..7 jumps, and with it (the carried
        # value is per unit of |q_hat|) nothing should go wrong; A_K is then rescaled for real
        q_hat = q_hat.clone()
        q_hat[:, 4:] *= factor
        if step == 5:
            dl.A_K[:, 0] *= 0.001          # every score of KV head 0 shrinks: thresholds far too high
            dl.np["A_K"] = dl.A_K.cpu().numpy()
        flags = L.LRQK_SELECT_FRESH if step == 1 else 0
        L.lrqk_decode_step(plan, dl.shape, step, dl.struct(), q_hat.to(DEV), q.to(DEV), out,
                           L.LRQK_FETCH_DIRECT | flags, sb.debug())
        got = sb.to_np()
        ref = orc.decode_step(dl.np["A_K"], as_numpy(q_hat), as_numpy(q), dl.np["K"], dl.np["V"],
                              dl.ost, dl.ocK, dl.ocV, step, cfg.k, cfg.w, cfg.scale)
        assert np.array_equal(got["sel_idx"], ref["sel_idx"]), f"step {step}: selection differs"
        compare_resolution(got, ref, f"step {step}")
        compare_state(dl, f"step {step}")
        assert np.abs(out.cpu().numpy() - ref["out"]).max() <= TOL[cfg.kv_dtype]
        thr_seen.append(dl.sel_thr.cpu().numpy().copy())
    assert all(np.isfinite(t).all() for t in thr_seen)
    plan.close()


@pytest.mark.parametrize("mode", ["staged", "direct"])
def test_decode_step_full_selection_is_dense_attention(mode):
    say(f"decode_step with k + w = l ({mode}): equals dense attention")
    from helpers import dense_attention
    cfg = small_cfg(B=1, Hq=4, Hkv=2, l=700, k=636, w=64, C=636, kv_dtype="f32")
    data = make_layer(cfg)
    dl = DeviceLayer(cfg, data)
    plan = L.Plan(dl.shape)
    q, q_hat = QueryStream(data).next()
    out = torch.empty((cfg.B, cfg.Hq, cfg.d), device=DEV)
    L.lrqk_decode_step(plan, dl.shape, 0, dl.struct(), q_hat.to(DEV), q.to(DEV), out,
                       L.LRQK_FETCH_STAGED if mode == "staged" else L.LRQK_FETCH_DIRECT)
    want = dense_attention(as_numpy(q), dl.np["K"], dl.np["V"], cfg.scale)
    assert np.abs(out.cpu().numpy() - want).max() <= 1e-5
    plan.close()


def test_decode_step_very_long_context():
    say("decode_step at l = 800000 (selection by the multi-workgroup kernels)")
    cfg = small_cfg(B=1, Hq=2, Hkv=1, l=800000, r=8, k=512, w=64, C=1024, n_heavy=64)
    run_steps_against_oracle(cfg, 3, "direct", check_unfused=False)


@pytest.mark.parametrize("factor", [0.0, 50.0])
def test_decode_step_misleading_threshold_sample(factor):
    say(f"decode_step where the rows the threshold estimate samples are scaled by {factor}")
    cfg = small_cfg(B=1, Hq=8, Hkv=2, l=70000, r=32, k=1024, w=64, C=2048, n_heavy=64)
    data = make_layer(cfg)
    n = cfg.l - cfg.w
    ss = 1
    while ss < 256 and n // (ss * 2) >= 8192:      # the library's sampling stride for this n
        ss *= 2
    assert ss == 8
    data.A_K[:, :, ss // 2:n:ss, :] *= factor      # every row the estimate looks at
    run_steps_against_oracle(cfg, 2, "direct", data=data, check_unfused=False)


def test_decode_step_clustered_candidates():
    say("decode_step with more than 8 candidates inside single 64-position groups")
    cfg = small_cfg(B=1, Hq=8, Hkv=2, l=70000, r=32, k=1024, w=64, C=2048, n_heavy=64)
    data = make_layer(cfg)
    data.A_K[:, :, 5000:5200, :] *= 6.0          # 200 consecutive rows with large |score|
    data.A_K[:, :, 64000:64064, :] *= 9.0        # one whole group
    run_steps_against_oracle(cfg, 2, "direct", data=data, check_unfused=False)


def test_config1_all_hits():
    say("config 1: l=4096 r=32 k=256 w=16, identity cache (all hits)")
    cfg = get_config("c1")
    rates = run_steps_against_oracle(cfg, 2, "staged", identity=True)
    assert rates == [0.0, 0.0]


@pytest.mark.parametrize("mode", ["staged", "direct", "group"])
def test_config2_shape(mode):
    say(f"config 2: l=32768 k=1024 w=64 C=2048 ({mode})")
    run_steps_against_oracle(get_config("c2"), 4, mode, check_unfused=False)


@pytest.mark.parametrize("mode", ["staged", "direct"])
@pytest.mark.parametrize("r", [16, 32, 64])
def test_config3_one_layer_full_size(r, mode):
    say(f"config 3, one layer at full size: l=131072 k=2048 w=64 C=4096 r={r} ({mode})")
    run_steps_against_oracle(get_config("c3", r=r, layers=1), 3, mode, check_unfused=False)


def test_config4_qwen_shape_reduced_batch():
    say("config 4 shape (28 q / 4 kv heads, G = 7), batch 2 of 8")
    run_steps_against_oracle(get_config("c4", B=2), 3, "direct", check_unfused=False)


@pytest.mark.timeout(600)
def test_config4_full_batch():
    say("config 4 at full size: batch 8, 28 q / 4 kv heads, l = 65536, k = 1024, C = 2048")
    cfg = get_config("c4")
    rates = run_steps_against_oracle(cfg, 4, "direct", data=make_layer(cfg, 0, device=DEV),
                                     check_unfused=False)
    assert 0.10 < rates[-1] < 0.25            # the workload asks for about 85 % hits


@pytest.mark.timeout(900)
def test_config5_miss_heavy_full_batch():
    say("config 5 at full size: batch 16, l = 131072, k = 2048, heavy set re-drawn every 4 steps")
    cfg = get_config("c5")
    rates = run_steps_against_oracle(cfg, 6, "direct", data=make_layer(cfg, 0, device=DEV),
                                     check_unfused=False)
    assert all(0.2 < r < 0.8 for r in rates[1:])    # 30-60 % misses on average, more at a re-draw
    assert 0.30 <= sum(rates[1:]) / len(rates[1:]) <= 0.60


def test_per_kernel_timing_of_the_step():
    say("lrqk_plan_profile: kernel slots of sampled, carried and staged steps")
    cfg = small_cfg()
    data = make_layer(cfg)
    dl = DeviceLayer(cfg, data)
    plan = L.Plan(dl.shape)
    qs = QueryStream(data)
    out = torch.empty((cfg.B, cfg.Hq, cfg.d), device=DEV)

    def timed_step(step, mode):
        plan.profile(1)
        q, q_hat = qs.next()
        L.lrqk_decode_step(plan, dl.shape, step, dl.struct(), q_hat.to(DEV), q.to(DEV), out, mode)
        ms, n = plan.profile_read()
        plan.profile(0)
        assert n == 1
        return {k for k, v in ms.items() if v > 0.0}, ms

    used, ms = timed_step(1, L.LRQK_FETCH_DIRECT | L.LRQK_SELECT_FRESH)
    assert used == {"sample", "threshold", "proxy_scores", "select", "attend", "combine"}
    assert all(0.0 < ms[k] < 5.0 for k in used)              # milliseconds; these are tiny kernels
    used, _ = timed_step(2, L.LRQK_FETCH_DIRECT)              # thresholds carried: no estimate kernels
    assert used == {"proxy_scores", "select", "attend", "combine"}
    used, _ = timed_step(3, L.LRQK_FETCH_STAGED)
    assert used >= {"proxy_scores", "select", "attend", "fetch_scatter", "attend_missed_rows"}
    used, _ = timed_step(4, L.LRQK_FETCH_GROUP)
    assert used == {"proxy_scores", "select", "attend", "attend_missed_rows", "combine"}
    us = plan.time_proxy_pass(dl.shape, [dl.A_K], qs.next()[1].to(DEV), 8, sel_thr=dl.sel_thr)
    assert 0.0 < us < 1000.0
    plan.close()


def test_rerun_is_deterministic():
    say("two runs of the same steps give identical bits")
    cfg = small_cfg()
    data = make_layer(cfg)
    outs = []
    for _ in range(2):
        dl = DeviceLayer(cfg, data)
        plan = L.Plan(dl.shape)
        qs = QueryStream(data)
        out = torch.empty((cfg.B, cfg.Hq, cfg.d), device=DEV)
        acc = []
        for step in range(3):
            q, q_hat = qs.next()
            L.lrqk_decode_step(plan, dl.shape, step, dl.struct(), q_hat.to(DEV), q.to(DEV), out,
                               L.LRQK_FETCH_DIRECT)
            acc.append(out.cpu().numpy().copy())
        outs.append((np.stack(acc), dl.state_np()))
        plan.close()
    assert np.array_equal(outs[0][0].view(np.uint32), outs[1][0].view(np.uint32))
    for name in ("slot_of", "token_of", "last_used", "cacheK", "cacheV"):
        assert np.array_equal(outs[0][1][name], outs[1][1][name])
