"""Pins of the CPU oracle: closed forms, library routines, brute force, invariants
and a hand-worked example.  None of them re-types the oracle's own formulas:
each states a fact the paper or the mathematics fixes and that a plausible
mistake in the oracle (dropped term, wrong sign or index, transposed operand,
wrong head mapping) would break.  CPU only.
"""
import os

import numpy as np
import pytest

from gen import get_config, make_layer, QueryStream, as_numpy
from oracle import lrqk_oracle as orc
from helpers import (bf16_to_f64, f32_to_bf16_bits, dense_attention, topk_by_lexsort,
                     kv_to_f64)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_cfg(**kw):
    base = dict(B=2, Hq=4, Hkv=2, l=96, r=8, k=80, w=16, C=80, n_heavy=4, pool_mult=2)
    base.update(kw)
    return get_config("c1").with_(prefill="warm", phase_spread=1.0, **base)


def layer_np(cfg, layer=0):
    data = make_layer(cfg, layer)
    qs = QueryStream(data)
    q, q_hat = qs.next()
    return data, qs, dict(A_K=as_numpy(data.A_K), K=as_numpy(data.K), V=as_numpy(data.V),
                          q=as_numpy(q), q_hat=as_numpy(q_hat))


# --------------------------------------------------------------------------- scores

def test_scores_hand_example_and_head_mapping():
    # 1 batch, 2 KV heads, 4 query heads (G = 2), l = 2, r = 2; worked by hand.
    A_K = np.array([[[[1, 2], [3, 4]], [[-1, 0.5], [2, -2]]]], np.float32)   # [1,2,2,2]
    q_hat = np.array([[[0.5, -1], [1, 1], [2, 0], [0, 4]]], np.float32)      # [1,4,2]
    s64, s32 = orc.proxy_scores(A_K, q_hat)
    want = np.array([[[-1.5, -2.5], [3, 7], [-2, 4], [2, -8]]])
    assert np.array_equal(s64, want)
    assert np.array_equal(s32.astype(np.float64), want)


@pytest.mark.parametrize("r", [4, 8, 32, 64])
def test_scores_equal_matmul_and_fp32_bound(r):
    rng = np.random.default_rng(r)
    B, Hkv, G, l = 2, 3, 2, 257
    A_K = rng.standard_normal((B, Hkv, l, r)).astype(np.float32)
    q_hat = rng.standard_normal((B, Hkv * G, r)).astype(np.float32)
    s64, s32 = orc.proxy_scores(A_K, q_hat)
    # library routine: float64 matmul with repeat-KV head alignment (Sec. 4 preliminaries)
    A_rep = np.repeat(A_K.astype(np.float64), G, axis=1)
    want = np.einsum("bhlr,bhr->bhl", A_rep, q_hat.astype(np.float64))
    np.testing.assert_allclose(s64, want, rtol=1e-13, atol=1e-13)
    # fp32 chain stays within the standard running-sum bound of the exact value
    mag = np.einsum("bhlr,bhr->bhl", np.abs(A_rep), np.abs(q_hat.astype(np.float64)))
    assert np.all(np.abs(s32 - s64) <= r * 2.0 ** -24 * mag + 1e-30)


def test_scores_fp32_chain_is_an_fma_chain():
    # products that are inexact in fp32: a fused chain and a mul-then-add chain differ
    A_K = np.array([[[[1 + 2.0 ** -12, 1 - 2.0 ** -12, 3.0]]]], np.float32)
    q_hat = np.array([[[1 + 2.0 ** -12, 1 + 2.0 ** -13, -1.0 / 3.0]]], np.float32)
    _, s32 = orc.proxy_scores(A_K, q_hat)
    acc = 0.0  # emulate fma exactly: double holds each fp32 product exactly; one rounding per step
    for a, b in zip(A_K[0, 0, 0], q_hat[0, 0]):
        acc = float(np.float32(float(a) * float(b) + acc))
    assert s32[0, 0, 0] == np.float32(acc)


# --------------------------------------------------------------------------- selection

def test_topk_matches_numpy_lexsort_random_and_ties():
    rng = np.random.default_rng(1)
    B, Hq, l, w, k = 2, 3, 300, 17, 40
    s = rng.standard_normal((B, Hq, l))
    s[0, 0] = np.round(s[0, 0] * 2) / 2          # many exact ties
    s[0, 1] = 0.25                                # all equal: the k lowest positions win
    s[1, 2, l - w:] = 100.0                       # large scores inside the lite window: ignored
    sel = orc.select_topk(s, k, w)
    assert np.array_equal(sel, topk_by_lexsort(s, k, w))
    assert np.array_equal(sel[0, 1], np.arange(k))
    assert sel.max() < l - w


def test_topk_brute_force_definition():
    # position i is selected iff fewer than k positions beat it (higher score, or equal and lower)
    rng = np.random.default_rng(2)
    l, w, k = 64, 8, 10
    s = np.round(rng.standard_normal((1, 1, l)) * 3) / 3
    sel = set(orc.select_topk(s, k, w)[0, 0].tolist())
    for i in range(l - w):
        beats = sum(1 for j in range(l - w)
                    if s[0, 0, j] > s[0, 0, i] or (s[0, 0, j] == s[0, 0, i] and j < i))
        assert (i in sel) == (beats < k)


def test_lowrank_keys_make_proxy_topk_the_true_topk():
    # With K exactly A_K B (no residual, fp32 rows) and q_hat = q B^T, the proxy score equals
    # the true logit q.K_i, so Omega_k is the top-k of exact attention logits (Eq. 3, Eq. 4).
    cfg = tiny_cfg(l=400, k=32, w=8, C=64, noise=0.0, kv_dtype="f32", r=8, B=1)
    data, qs, a = layer_np(cfg)
    s64, _ = orc.proxy_scores(a["A_K"], a["q_hat"])
    G = cfg.G
    logits = np.einsum("bhld,bhd->bhl", np.repeat(a["K"].astype(np.float64), G, axis=1),
                       a["q"].astype(np.float64))
    np.testing.assert_allclose(s64, logits, rtol=0, atol=5e-4)
    assert np.array_equal(orc.select_topk(s64, cfg.k, cfg.w), topk_by_lexsort(logits, cfg.k, cfg.w))


# --------------------------------------------------------------------------- whole path

@pytest.mark.parametrize("kvd", ["bf16", "f32"])
@pytest.mark.parametrize("l,w", [(48, 16), (96, 0), (512, 64)])
def test_full_selection_equals_dense_attention(kvd, l, w):
    # k + w = l: every row is attended, so the step must reproduce dense attention exactly
    # (Sec. 4.3: exact attention on the selected rows with the original q, K, V).
    cfg = tiny_cfg(l=l, w=w, k=l - w, C=l - w, kv_dtype=kvd)
    data, qs, a = layer_np(cfg)
    st = orc.CacheState(cfg.B, cfg.Hq, cfg.l, cfg.C)
    cK = np.zeros((cfg.B, cfg.Hq, cfg.C, cfg.d), a["K"].dtype)
    cV = np.zeros_like(cK)
    res = orc.decode_step(a["A_K"], a["q_hat"], a["q"], a["K"], a["V"], st, cK, cV, step=0,
                          k=cfg.k, w=cfg.w, scale=cfg.scale)
    want = dense_attention(a["q"], a["K"], a["V"], cfg.scale)
    np.testing.assert_allclose(res["out"], want, rtol=1e-12, atol=1e-13)
    assert np.array_equal(res["sel_idx"][0, 0], np.arange(l - w))
    assert res["miss_rate"] == 1.0   # empty cache: every selected row is fetched


def test_partial_selection_equals_dense_attention_on_subset():
    # Omega smaller than l: equals textbook attention restricted to the rows of Omega
    cfg = tiny_cfg(l=200, w=8, k=24, C=32)
    data, qs, a = layer_np(cfg)
    st = orc.CacheState(cfg.B, cfg.Hq, cfg.l, cfg.C)
    cK = np.zeros((cfg.B, cfg.Hq, cfg.C, cfg.d), np.uint16)
    cV = np.zeros_like(cK)
    res = orc.decode_step(a["A_K"], a["q_hat"], a["q"], a["K"], a["V"], st, cK, cV, step=0,
                          k=cfg.k, w=cfg.w, scale=cfg.scale)
    G = cfg.G
    for b in range(cfg.B):
        for h in range(cfg.Hq):
            rows = np.concatenate([res["sel_idx"][b, h], np.arange(cfg.l - cfg.w, cfg.l)])
            want = dense_attention(a["q"][b:b + 1, h:h + 1], a["K"][b:b + 1, h // G:h // G + 1, rows],
                                   a["V"][b:b + 1, h // G:h // G + 1, rows], cfg.scale)
            np.testing.assert_allclose(res["out"][b, h], want[0, 0], rtol=1e-12, atol=1e-13)


# --------------------------------------------------------------------------- attention closed forms

def _attend_simple(q, Krows, Vrows, scale, w=0):
    """Run the oracle's attention with an identity cache over the given rows (1 head)."""
    n, d = Krows.shape
    cK = np.ascontiguousarray(Krows[None, None, : n - w])
    cV = np.ascontiguousarray(Vrows[None, None, : n - w])
    lK = np.ascontiguousarray(Krows[None, None, n - w:])
    lV = np.ascontiguousarray(Vrows[None, None, n - w:])
    sel = np.arange(n - w, dtype=np.int32)[None, None]
    return orc.sparse_attend(q[None, None].astype(np.float32), cK, cV, sel, lK, lV, scale)[0, 0]


def test_attention_equal_keys_gives_mean_of_values():
    rng = np.random.default_rng(3)
    d, n = 128, 37
    q = rng.standard_normal(d).astype(np.float32)
    K = np.tile(rng.standard_normal(d).astype(np.float32), (n, 1))
    V = rng.standard_normal((n, d)).astype(np.float32)
    out = _attend_simple(q, K, V, 0.3, w=5)
    np.testing.assert_allclose(out, V.astype(np.float64).mean(0), rtol=1e-12, atol=1e-13)


def test_attention_dominant_logit_returns_that_value_row():
    rng = np.random.default_rng(4)
    d, n = 128, 50
    q = rng.standard_normal(d).astype(np.float32)
    K = 0.01 * rng.standard_normal((n, d)).astype(np.float32)
    K[17] = 40.0 * q / np.dot(q, q)              # logit 40*scale vs ~0 for the rest
    V = rng.standard_normal((n, d)).astype(np.float32)
    out = _attend_simple(q, K, V, 2.0)
    np.testing.assert_allclose(out, V[17], atol=1e-30 + 60 * np.exp(-75.0))


def test_attention_permutation_and_shift_invariance():
    rng = np.random.default_rng(5)
    d, n = 128, 64
    q = rng.standard_normal(d).astype(np.float32)
    K = rng.standard_normal((n, d)).astype(np.float32)
    V = rng.standard_normal((n, d)).astype(np.float32)
    base = _attend_simple(q, K, V, 0.1, w=8)
    p = rng.permutation(n)
    np.testing.assert_allclose(_attend_simple(q, K[p], V[p], 0.1, w=8), base, rtol=1e-11, atol=1e-13)
    # adding c*q/|q|^2 to every key adds the same constant to every logit: softmax unchanged.
    # Use values exactly representable so the shift itself is exact: q = e_0 * 2
    q2 = np.zeros(d, np.float32); q2[0] = 2.0
    Kq = K.copy(); Kq[:, 0] = np.round(Kq[:, 0] * 1024) / 1024   # so that +8 is exact in fp32
    Ks = Kq.copy(); Ks[:, 0] += 8.0              # logit shift = scale * 16 for every row
    np.testing.assert_allclose(_attend_simple(q2, Ks, V, 0.1), _attend_simple(q2, Kq, V, 0.1),
                               rtol=1e-10, atol=1e-12)


def test_attention_two_rows_closed_form_and_scale_sign():
    # two rows: out = sigmoid(scale*(a-b)) V0 + (1 - sigmoid) V1
    d = 128
    q = np.zeros(d, np.float32); q[3] = 1.0
    K = np.zeros((2, d), np.float32); K[0, 3] = 1.5; K[1, 3] = -0.5
    V = np.zeros((2, d), np.float32); V[0, 0] = 1.0; V[1, 1] = 1.0
    out = _attend_simple(q, K, V, 0.7)
    p0 = 1.0 / (1.0 + np.exp(-0.7 * 2.0))
    np.testing.assert_allclose(out[:2], [p0, 1 - p0], rtol=1e-14)


def test_bf16_rows_are_decoded_as_upper_half_of_fp32():
    x = np.array([1.0, -2.5, 0.15625, 3.0e-3, -1.0e4], np.float32)
    bits = f32_to_bf16_bits(x)
    d = 128
    q = np.zeros(d, np.float32); q[0] = 1.0
    K = np.zeros((1, d), np.uint16)
    V = np.zeros((1, d), np.uint16); V[0, :5] = bits
    out = _attend_simple(q, K, V, 1.0)
    assert np.array_equal(out[:5], bf16_to_f64(bits))
    assert np.array_equal(bf16_to_f64(bits)[:3], [1.0, -2.5, 0.15625])


# --------------------------------------------------------------------------- cache

def test_lru_hand_worked_example():
    rows = [ln for ln in open(os.path.join(GOLDEN, "lru_worked_example.txt"))
            if ln.strip() and not ln.startswith("#")]
    st = orc.CacheState(1, 1, 10, 4)
    for ln in rows:
        f = [np.array(x.split(), np.int64) for x in ln.split("|")]
        step, sel, want_slot, want_hit, want_tok, want_lu = int(f[0][0]), f[1], f[2], f[3], f[4], f[5]
        res = orc.cache_resolve(sel.astype(np.int32)[None, None], step, st)
        assert res["ok"]
        assert np.array_equal(res["sel_slot"][0, 0], want_slot), ln
        assert np.array_equal(res["hit"][0, 0], want_hit), ln
        assert np.array_equal(st.token_of[0, 0], want_tok), ln
        assert np.array_equal(st.last_used[0, 0], want_lu), ln
        assert res["n_miss"][0, 0] == int((want_hit == 0).sum())


def _run_steps(cfg, n_steps, Cslots=None, reset_each_step=False):
    """Drive the oracle for several steps; yield per-step records for invariant checks."""
    data = make_layer(cfg)
    qs = QueryStream(data)
    A_K, K, V = as_numpy(data.A_K), as_numpy(data.K), as_numpy(data.V)
    Cs = Cslots or cfg.C
    st = orc.CacheState(cfg.B, cfg.Hq, cfg.l, Cs)
    cK = np.zeros((cfg.B, cfg.Hq, Cs, cfg.d), K.dtype)
    cV = np.zeros_like(cK)
    for t in range(n_steps):
        q, q_hat = (as_numpy(x) for x in qs.next())
        if reset_each_step:
            st = orc.CacheState(cfg.B, cfg.Hq, cfg.l, Cs)
        before = st.copy()
        res = orc.decode_step(A_K, q_hat, q, K, V, st, cK, cV, step=t, k=cfg.k, w=cfg.w,
                              scale=cfg.scale)
        yield t, before, st, res, dict(q=q, K=K, V=V, cK=cK, cV=cV)


@pytest.mark.parametrize("Cmult", [1, 2])
def test_cache_invariants_over_steps(Cmult):
    cfg = tiny_cfg(B=1, Hq=4, Hkv=2, l=600, r=8, k=48, w=8, n_heavy=8, pool_mult=4, rho=0.9)
    Cs = cfg.k * Cmult
    total_miss = 0
    for t, before, st, res, a in _run_steps(cfg, 6, Cslots=Cs):
        sel = res["sel_idx"]
        for h in range(cfg.Hq):
            resident_before = set(before.token_of[0, h][before.token_of[0, h] >= 0].tolist())
            resident_after = set(st.token_of[0, h][st.token_of[0, h] >= 0].tolist())
            omega = set(sel[0, h].tolist())
            # the selected set ends up resident; hits + misses = k; misses = newly needed rows
            assert omega <= resident_after
            nm = int(res["n_miss"][0, h])
            assert nm == len(omega - resident_before)
            assert int(res["hit"][0, h].sum()) + nm == cfg.k
            assert np.array_equal(res["miss_tok"][0, h, :nm], np.array(sorted(omega - resident_before)))
            # slot_of / token_of are mutually inverse on the resident set
            for s in range(Cs):
                tok = st.token_of[0, h, s]
                if tok >= 0:
                    assert st.slot_of[0, h, tok] == s
            assert int((st.slot_of[0, h] >= 0).sum()) == len(resident_after)
            # nothing selected in this step was evicted, and every selected row sits in its slot
            assert np.array_equal(st.token_of[0, h][res["sel_slot"][0, h]], sel[0, h])
            assert np.all(st.last_used[0, h][res["sel_slot"][0, h]] == t)
            if Cmult == 1:   # the paper's cache: exactly the active tokens
                assert resident_after == omega
            # the cache rows are bit copies of the store rows
            G = cfg.G
            assert np.array_equal(a["cK"][0, h][res["sel_slot"][0, h]], a["K"][0, h // G][sel[0, h]])
            assert np.array_equal(a["cV"][0, h][res["sel_slot"][0, h]], a["V"][0, h // G][sel[0, h]])
        # transparency: attention through the cache == attention straight from the store, bit for bit
        direct = orc.attend_store(a["q"], a["K"], a["V"], sel, cfg.w, cfg.scale)
        assert np.array_equal(direct, res["out"])
        total_miss += int(res["n_miss"].sum())
        if t == 0:
            assert res["miss_rate"] == 1.0
    assert total_miss < 6 * cfg.k * cfg.Hq   # later steps do hit


def test_no_hit_miss_mode_has_miss_rate_one():
    # Without the hit/miss buffer every selected row is transferred again (App. C.1 variant).
    cfg = tiny_cfg(B=1, l=300, k=32, w=8, C=32)
    for t, before, st, res, a in _run_steps(cfg, 3, reset_each_step=True):
        assert res["miss_rate"] == 1.0


def test_identity_cache_is_all_hits():
    cfg = tiny_cfg(B=1, l=256, k=32, w=8)
    data, qs, a = layer_np(cfg)
    st = orc.CacheState.identity(cfg.B, cfg.Hq, cfg.l)
    sel = orc.select_topk(orc.proxy_scores(a["A_K"], a["q_hat"])[1], cfg.k, cfg.w)
    res = orc.cache_resolve(sel, 1, st)
    assert res["ok"] and res["n_miss"].sum() == 0 and res["hit"].all()
    assert np.array_equal(res["sel_slot"], sel)


def test_resolve_flags_contract_violations_without_crashing():
    st = orc.CacheState(1, 1, 10, 2)
    res = orc.cache_resolve(np.array([[[3, 11]]], np.int32), 0, st)     # position outside [0, l)
    assert not res["ok"] and res["n_miss"][0, 0] == -1
    st = orc.CacheState(1, 1, 10, 2)
    orc.cache_resolve(np.array([[[1, 2]]], np.int32), 5, st)
    res = orc.cache_resolve(np.array([[[3, 4]]], np.int32), 5, st)      # step reused: no victims
    assert not res["ok"] and res["n_miss"][0, 0] == -1


# --------------------------------------------------------------------------- input preparation

def test_qhat_closed_form_is_least_squares_and_stationary():
    rng = np.random.default_rng(7)
    r, d = 8, 128
    B_Q = rng.standard_normal((r, d))
    q = rng.standard_normal((5, d))
    qh = orc.qhat_closed_form(q, B_Q)
    want = np.linalg.lstsq(B_Q.T, q.T, rcond=None)[0].T      # min || q_hat B_Q - q ||
    np.testing.assert_allclose(qh, want, rtol=1e-10, atol=1e-12)
    grad = (qh @ B_Q - q) @ B_Q.T                             # dL_dec/dq_hat at lambda = 0
    assert np.abs(grad).max() < 1e-10


def test_generator_qhat_is_the_closed_form_with_dual_basis():
    # The workload's q_hat = q B^T is Eq. 9 at lambda = 0 with B_K = B and B_Q the dual
    # basis (B B^T)^-1 B, which is what Q K^T ~ A_Q A_K^T with Q ~ A_Q B_Q, K ~ A_K B_K forces.
    cfg = tiny_cfg(B=1, l=128, k=16, w=8, C=16)
    data, qs, a = layer_np(cfg)
    for h in range(cfg.Hq):
        Bm = data.Bmat[0, h // cfg.G].double().numpy()
        B_Q = np.linalg.solve(Bm @ Bm.T, Bm)
        qh = orc.qhat_closed_form(a["q"][0, h], B_Q)
        np.testing.assert_allclose(a["q_hat"][0, h], qh, rtol=2e-6, atol=2e-6)


# --------------------------------------------------------------------------- workload sanity

def test_window_always_attended_and_heavy_tokens_are_found():
    cfg = get_config("c1").with_(l=1024, k=96, C=1024)
    data, qs, a = layer_np(cfg)
    s64, s32 = orc.proxy_scores(a["A_K"], a["q_hat"])
    sel = orc.select_topk(s32, cfg.k, cfg.w)
    assert sel.max() < cfg.l - cfg.w                         # window is implicit, never listed
    found = 0
    for h in range(cfg.Hq):
        found += len(set(data.pool_pos[0, h].tolist()) & set(sel[0, h].tolist()))
    assert found >= 0.75 * cfg.Hq * cfg.n_heavy              # most planted tokens are selected
    # with a stronger planted component the proxy finds every one of them
    cfg = cfg.with_(beta=12.0)
    data, qs, a = layer_np(cfg)
    sel = orc.select_topk(orc.proxy_scores(a["A_K"], a["q_hat"])[1], cfg.k, cfg.w)
    for h in range(cfg.Hq):
        assert set(data.pool_pos[0, h].tolist()) <= set(sel[0, h].tolist())


# --------------------------------------------------------------------------- fetch shared by a KV group

def _miss_lists(rng, B, Hq, l, k, n_each, shared_with_first=0.0, G=1):
    """Ascending miss lists per head with distinct slots; a fraction of the entries of the heads
    h % G != 0 is taken from the list of their group's first head."""
    miss_tok = np.full((B, Hq, k), -1, np.int32)
    miss_slot = np.full((B, Hq, k), -1, np.int32)
    n_miss = np.zeros((B, Hq), np.int32)
    for b in range(B):
        for h in range(Hq):
            n = int(n_each[b, h])
            toks = rng.choice(l, size=n, replace=False)
            if h % G and shared_with_first > 0 and n:
                first = miss_tok[b, h - h % G, :n_miss[b, h - h % G]]
                take = rng.choice(first, size=min(len(first), int(shared_with_first * n)), replace=False)
                rest = np.setdiff1d(toks, take)[: n - len(take)]
                toks = np.concatenate([take, rest])
            toks = np.unique(toks)
            n_miss[b, h] = len(toks)
            miss_tok[b, h, :len(toks)] = toks
            miss_slot[b, h, :len(toks)] = rng.permutation(k)[:len(toks)]
    return miss_tok, miss_slot, n_miss


@pytest.mark.parametrize("kvd", ["bf16", "f32"])
def test_group_fetch_leaves_the_caches_of_the_per_head_fetch_and_counts_the_union(kvd):
    rng = np.random.default_rng(77)
    B, Hkv, G, l, d, k = 2, 2, 4, 300, 128, 40
    Hq = Hkv * G
    if kvd == "bf16":
        K = f32_to_bf16_bits(rng.standard_normal((B, Hkv, l, d)).astype(np.float32))
        V = f32_to_bf16_bits(rng.standard_normal((B, Hkv, l, d)).astype(np.float32))
    else:
        K = rng.standard_normal((B, Hkv, l, d)).astype(np.float32)
        V = rng.standard_normal((B, Hkv, l, d)).astype(np.float32)
    n_each = rng.integers(0, k + 1, size=(B, Hq))
    n_each[0, 1] = 0                                           # a head that misses nothing
    miss_tok, miss_slot, n_miss = _miss_lists(rng, B, Hq, l, k, n_each, 0.6, G)
    cK1, cV1 = np.zeros((B, Hq, k, d), K.dtype), np.zeros((B, Hq, k, d), K.dtype)
    cK2, cV2 = cK1.copy(), cV1.copy()
    orc.fetch(K, V, miss_tok, miss_slot, n_miss, cK1, cV1)
    link_rows, union = orc.group_fetch(K, V, miss_tok, miss_slot, n_miss, cK2, cV2)
    assert np.array_equal(cK1, cK2) and np.array_equal(cV1, cV2)
    # every fetched slot holds the bits of its host row (head h reads KV head h // G)
    for b in range(B):
        for h in range(Hq):
            for j in range(n_miss[b, h]):
                assert np.array_equal(cK2[b, h, miss_slot[b, h, j]], K[b, h // G, miss_tok[b, h, j]])
                assert np.array_equal(cV2[b, h, miss_slot[b, h, j]], V[b, h // G, miss_tok[b, h, j]])
    # rows over the link = size of the union of the group's lists (numpy's set union)
    shared_somewhere = False
    for b in range(B):
        for kv in range(Hkv):
            lists = [miss_tok[b, h, :n_miss[b, h]] for h in range(kv * G, (kv + 1) * G)]
            want = np.unique(np.concatenate(lists))
            assert np.array_equal(union[b * Hkv + kv], want)
            assert link_rows[b, kv] == len(want) <= sum(len(x) for x in lists)
            shared_somewhere |= len(want) < sum(len(x) for x in lists)
    assert shared_somewhere


def test_group_fetch_special_cases():
    rng = np.random.default_rng(78)
    B, l, d, k = 1, 200, 128, 30
    K = rng.standard_normal((B, 1, l, d)).astype(np.float32)
    V = rng.standard_normal((B, 1, l, d)).astype(np.float32)
    # G = 1: nothing to share, the count is the list length
    mt, ms, nm = _miss_lists(rng, B, 1, l, k, np.array([[17]]))
    cK, cV = np.zeros((B, 1, k, d), np.float32), np.zeros((B, 1, k, d), np.float32)
    rows, _ = orc.group_fetch(K, V, mt, ms, nm, cK, cV)
    assert rows[0, 0] == 17
    # G = 3, identical lists: one list's worth of rows, all three caches filled
    mt3 = np.repeat(mt, 3, axis=1)
    ms3 = np.stack([rng.permutation(k) for _ in range(3)])[None].astype(np.int32)
    nm3 = np.repeat(nm, 3, axis=1)
    cK, cV = np.zeros((B, 3, k, d), np.float32), np.zeros((B, 3, k, d), np.float32)
    rows, _ = orc.group_fetch(K, V, mt3, ms3, nm3, cK, cV)
    assert rows[0, 0] == 17
    for h in range(3):
        for j in range(17):
            assert np.array_equal(cK[0, h, ms3[0, h, j]], K[0, 0, mt3[0, h, j]])
    # G = 2, disjoint lists: the counts add up
    mt2 = np.full((B, 2, k), -1, np.int32)
    mt2[0, 0, :5] = [1, 3, 5, 7, 9]
    mt2[0, 1, :4] = [0, 2, 4, 6]
    ms2 = np.tile(np.arange(k, dtype=np.int32), (B, 2, 1))
    cK, cV = np.zeros((B, 2, k, d), np.float32), np.zeros((B, 2, k, d), np.float32)
    rows, _ = orc.group_fetch(K, V, mt2, ms2, np.array([[5, 4]], np.int32), cK, cV)
    assert rows[0, 0] == 9


def test_group_share_knob_makes_heads_of_a_group_miss_the_same_rows():
    """The generator's group_share: with 0 the heads of a group miss (almost) disjoint rows, with
    1 the rows fetched for one head are mostly wanted by the others in the same step."""
    def union_over_total(share):
        cfg = get_config("c2").with_(B=1, Hq=8, Hkv=2, l=6000, r=16, k=256, w=16, C=512,
                                     n_heavy=64, pool_mult=4, group_share=share)
        data = make_layer(cfg)
        qs = QueryStream(data)
        A_K, K, V = as_numpy(data.A_K), as_numpy(data.K), as_numpy(data.V)
        st = orc.CacheState(cfg.B, cfg.Hq, cfg.l, cfg.C)
        cK = np.zeros((cfg.B, cfg.Hq, cfg.C, cfg.d), K.dtype)
        cV = np.zeros_like(cK)
        tot = uni = 0
        for step in range(1, 7):
            q, q_hat = qs.next()
            s64, s32 = orc.proxy_scores(A_K, as_numpy(q_hat))
            sel = orc.select_topk(s32, cfg.k, cfg.w)
            res = orc.cache_resolve(sel, step, st)
            rows, _ = orc.group_fetch(K, V, res["miss_tok"], res["miss_slot"], res["n_miss"], cK, cV)
            if step > 2:
                tot += int(res["n_miss"].sum())
                uni += int(rows.sum())
        return uni / tot
    assert union_over_total(0.0) > 0.9
    assert union_over_total(1.0) < 0.75


def test_group_fetch_hand_worked_example():
    lines = [ln.strip() for ln in open(os.path.join(GOLDEN, "group_fetch_worked_example.txt"))
             if ln.strip() and not ln.startswith("#")]
    B, Hkv, G, l, C, d, k = 1, 2, 3, 12, 5, 128, 4
    Hq = Hkv * G
    miss_tok = np.full((B, Hq, k), -1, np.int32)
    miss_slot = np.full((B, Hq, k), -1, np.int32)
    n_miss = np.zeros((B, Hq), np.int32)
    want_rows, want_cache = None, None
    for ln in lines:
        f = [x.split() for x in ln.split("|")]
        if f[0][0] == "link_rows":
            want_rows = np.array(f[1], np.int64)
        elif f[0][0] == "cache":
            want_cache = [tuple(int(v) for v in x) for x in f[1:]]
        else:
            h = int(f[0][0])
            n_miss[0, h] = len(f[1])
            miss_tok[0, h, :len(f[1])] = [int(v) for v in f[1]]
            miss_slot[0, h, :len(f[2])] = [int(v) for v in f[2]]
    # rows that can be told apart: row p of KV head kv holds the value 100 kv + p in every element
    K = np.empty((B, Hkv, l, d), np.float32)
    for kv in range(Hkv):
        for p in range(l):
            K[0, kv, p] = 100 * kv + p
    V = -K
    cK = np.full((B, Hq, C, d), -7.0, np.float32)
    cV = np.full((B, Hq, C, d), -7.0, np.float32)
    rows, union = orc.group_fetch(K, V, miss_tok, miss_slot, n_miss, cK, cV)
    assert np.array_equal(rows[0], want_rows)
    assert [list(u) for u in union] == [[2, 5, 9, 11], [0, 1, 7]]
    touched = set()
    for h, slot, pos in want_cache:
        assert np.all(cK[0, h, slot] == 100 * (h // G) + pos) and np.all(cV[0, h, slot] == -(100 * (h // G) + pos))
        touched.add((h, slot))
    for h in range(Hq):
        for slot in range(C):
            if (h, slot) not in touched:
                assert np.all(cK[0, h, slot] == -7.0) and np.all(cV[0, h, slot] == -7.0)
