"""Pins of the factor-update oracle (oracle/lrqk_update_oracle.py).  CPU only.

Each test states a fact that the decode objective of Sec. 4.2 (its Lagrangian, App. A.2)
or plain linear algebra fixes, evaluated with code of the test's own: the Lagrangian and
its partial derivatives written head by head with repeat-KV alignment, numpy.linalg.lstsq,
scipy.optimize, numbers worked by hand.  None calls the oracle to produce its own expected
value, and none re-types the oracle's solution formulas.
"""
import numpy as np
import pytest
from scipy import optimize

from oracle import lrqk_update_oracle as upd
from helpers import f32_to_bf16_bits, bf16_to_f64


def problem(seed, B=2, Hkv=2, G=2, r=4, d=8, L=40, n_om=12, bf16=False, noise=0.3):
    """A random, deliberately inconsistent instance (nothing is near a special point)."""
    rng = np.random.default_rng(seed)
    Hq = Hkv * G
    A_K = rng.standard_normal((B, Hkv, L, r)).astype(np.float32)
    B_K = (rng.standard_normal((B, Hkv, r, d)) / np.sqrt(r)).astype(np.float32)
    B_Q = (rng.standard_normal((B, Hq, r, d)) / np.sqrt(r)).astype(np.float32)
    K = np.einsum("bhlr,bhrd->bhld", A_K, B_K) + noise * rng.standard_normal((B, Hkv, L, d))
    K = K.astype(np.float32)
    q = rng.standard_normal((B, Hq, d)).astype(np.float32)
    k_new = rng.standard_normal((B, Hkv, d)).astype(np.float32)
    if bf16:
        K = f32_to_bf16_bits(K)
        k_new = f32_to_bf16_bits(k_new)
    omega = np.stack([np.stack([rng.permutation(L)[:n_om] for _ in range(Hq)])
                      for _ in range(B)]).astype(np.int64)
    return dict(q=q, k_new=k_new, B_Q=B_Q, B_K=B_K, A_K=A_K, K_store=K, omega=omega)


def as64(x):
    return bf16_to_f64(x) if x.dtype == np.uint16 else x.astype(np.float64)


def lagrangian_of_head(p, b, h, G, q_hat, k_hat, lam1, lam2):
    """L_dec of Sec. 4.2 for query head h (KV head h // G), written term by term."""
    kv = h // G
    q = as64(p["q"][b, h]); k = as64(p["k_new"][b, kv])
    BQ = as64(p["B_Q"][b, h]); BK = as64(p["B_K"][b, kv])
    pos = p["omega"][b, h]
    A = as64(p["A_K"][b, kv][pos]); K = as64(p["K_store"][b, kv][pos])
    t1 = 0.5 * np.sum((q_hat @ BQ - q) ** 2)
    t2 = 0.5 * np.sum((k_hat @ BK - k) ** 2)
    t3 = 0.5 * lam1 * (q_hat @ k_hat - q @ k) ** 2
    t4 = 0.5 * lam2 * np.sum((A @ q_hat - K @ q) ** 2)
    return t1, t2, t3, t4


def group_objective(p, b, kv, G, q_hats, k_hat, lam1, lam2):
    """What one KV group minimises: the key term once, every query head's other terms."""
    tot = 0.0
    for g in range(G):
        t1, t2, t3, t4 = lagrangian_of_head(p, b, kv * G + g, G, q_hats[g], k_hat, lam1, lam2)
        tot += t1 + t3 + t4
    return tot + t2


def numeric_grad(f, x, eps=1e-6):
    g = np.zeros_like(x)
    for i in range(x.size):
        e = np.zeros_like(x); e[i] = eps
        g[i] = (f(x + e) - f(x - e)) / (2 * eps)
    return g


# ------------------------------------------------------------------ special cases

def test_lambda_zero_is_plain_least_squares():
    p = problem(1)
    out = upd.factor_update(**p, lam1=0.0, lam2=0.0, n_iter=2)
    B, Hq, _ = p["q"].shape
    G = Hq // p["B_K"].shape[1]
    for b in range(B):
        for h in range(Hq):
            want = np.linalg.lstsq(as64(p["B_Q"][b, h]).T, as64(p["q"][b, h]), rcond=None)[0]
            np.testing.assert_allclose(out["q_hat"][b, h], want, rtol=1e-9, atol=1e-11)
        for kv in range(Hq // G):
            want = np.linalg.lstsq(as64(p["B_K"][b, kv]).T, as64(p["k_new"][b, kv]), rcond=None)[0]
            np.testing.assert_allclose(out["k_hat"][b, kv], want, rtol=1e-9, atol=1e-11)


def test_large_lambda2_enforces_the_proxy_constraint():
    # lambda_d2 -> infinity: q_hat A_Om^T = q K_Om^T in the least-squares sense
    p = problem(2, n_om=20)
    out = upd.factor_update(**p, lam1=0.0, lam2=1e9, n_iter=1)
    B, Hq, _ = p["q"].shape
    G = Hq // p["B_K"].shape[1]
    for b in range(B):
        for h in range(Hq):
            pos = p["omega"][b, h]
            A = as64(p["A_K"][b, h // G][pos]); K = as64(p["K_store"][b, h // G][pos])
            want = np.linalg.lstsq(A, K @ as64(p["q"][b, h]), rcond=None)[0]
            np.testing.assert_allclose(out["q_hat"][b, h], want, rtol=1e-6, atol=1e-7)


def test_scalar_case_worked_by_hand_with_two_heads_in_a_group():
    # r = d = 1, one KV head, two query heads, lambda_d1 = 1, lambda_d2 = 0, one round.
    #   k_hat0 = k bk / bk^2 = 4*2/4 = 2
    #   q_hat1 = (q1 bq1 + (q1 k) k_hat0) / (bq1^2 + k_hat0^2) = (1 + 4*2) / (1 + 4) = 1.8
    #   q_hat2 = (q2 bq2 + (q2 k) k_hat0) / (bq2^2 + k_hat0^2) = (-2 - 4*2) / (4 + 4) = -1.25
    #   k_hat  = (k bk + (q1 k) q_hat1 + (q2 k) q_hat2) / (bk^2 + q_hat1^2 + q_hat2^2)
    #          = (8 + 7.2 + 5) / (4 + 3.24 + 1.5625) = 20.2 / 8.8025
    one = lambda v: np.array(v, np.float32)
    out = upd.factor_update(q=one([[[1.0], [-1.0]]]), k_new=one([[[4.0]]]),
                            B_Q=one([[[[1.0]], [[2.0]]]]), B_K=one([[[[2.0]]]]),
                            A_K=np.zeros((1, 1, 1, 1), np.float32),
                            K_store=np.zeros((1, 1, 1, 1), np.float32),
                            omega=np.zeros((1, 2, 1), np.int64), lam1=1.0, lam2=0.0, n_iter=1)
    np.testing.assert_allclose(out["q_hat"][0, :, 0], [1.8, -1.25], rtol=1e-14)
    np.testing.assert_allclose(out["k_hat"][0, 0, 0], 20.2 / 8.8025, rtol=1e-14)
    # line search in the scalar case: B_new = x / x_hat exactly
    np.testing.assert_allclose(out["B_Q"][0, :, 0, 0], [1.0 / 1.8, -1.0 / -1.25], rtol=1e-14)
    np.testing.assert_allclose(out["B_K"][0, 0, 0, 0], 4.0 / (20.2 / 8.8025), rtol=1e-14)


def test_exact_recovery_on_consistent_data():
    # K = A_K B_K, B_Q the dual basis of B_K (B_Q B_K^T = I), q = q* B_Q, k = k* B_K:
    # every term of the Lagrangian vanishes at (q*, k*), for any lambda and any round count.
    rng = np.random.default_rng(3)
    B, Hkv, G, r, d, L = 1, 2, 2, 4, 8, 30
    Hq = Hkv * G
    A_K = rng.integers(-4, 5, (B, Hkv, L, r)).astype(np.float32)
    B_K64 = rng.standard_normal((B, Hkv, r, d))
    B_K = B_K64.astype(np.float32)
    K = np.einsum("bhlr,bhrd->bhld", A_K.astype(np.float64), B_K.astype(np.float64))
    dual = np.stack([[np.linalg.solve(as64(B_K[b, kv]) @ as64(B_K[b, kv]).T, as64(B_K[b, kv]))
                      for kv in range(Hkv)] for b in range(B)])
    B_Q = np.repeat(dual, G, axis=1).astype(np.float32)
    q_star = rng.standard_normal((B, Hq, r))
    k_star = rng.standard_normal((B, Hkv, r))
    q = np.einsum("bhr,bhrd->bhd", q_star, B_Q.astype(np.float64)).astype(np.float32)
    k_new = np.einsum("bhr,bhrd->bhd", k_star, B_K.astype(np.float64)).astype(np.float32)
    omega = np.stack([np.stack([rng.permutation(L)[:10] for _ in range(Hq)]) for _ in range(B)])
    for lam1, lam2, n_iter in [(1.0, 1.0, 2), (0.3, 5.0, 1), (4.0, 0.0, 3)]:
        out = upd.factor_update(q, k_new, B_Q, B_K, A_K, K.astype(np.float32), omega,
                                lam1, lam2, n_iter)
        # inputs were rounded to float32 once, hence 1e-5 rather than 1e-12
        np.testing.assert_allclose(out["q_hat"], q_star, rtol=0, atol=2e-5)
        np.testing.assert_allclose(out["k_hat"], k_star, rtol=0, atol=2e-5)
        np.testing.assert_allclose(out["B_Q"], B_Q, rtol=0, atol=2e-5)
        np.testing.assert_allclose(out["B_K"], B_K, rtol=0, atol=2e-5)


# ------------------------------------------------------------------ optimality

@pytest.mark.parametrize("G,bf16", [(1, False), (2, True), (4, False)])
def test_each_block_update_is_stationary(G, bf16):
    # after round n: q_hat_n minimises its head's Lagrangian with k_hat_{n-1} held fixed,
    # and k_hat_n minimises the group objective with the q_hat_n held fixed
    p = problem(10 + G, Hkv=2, G=G, bf16=bf16)
    lam1, lam2 = 0.7, 1.3
    prev = upd.factor_update(**p, lam1=lam1, lam2=lam2, n_iter=1)
    cur = upd.factor_update(**p, lam1=lam1, lam2=lam2, n_iter=2)
    B, Hq, _ = p["q"].shape
    for b in range(B):
        for h in range(Hq):
            f = lambda x: sum(lagrangian_of_head(p, b, h, G, x, prev["k_hat"][b, h // G],
                                                 lam1, lam2))
            g = numeric_grad(f, cur["q_hat"][b, h].copy())
            scale = max(1.0, abs(f(cur["q_hat"][b, h])))
            assert np.max(np.abs(g)) <= 1e-6 * scale
        for kv in range(Hq // G):
            qh = [cur["q_hat"][b, kv * G + g] for g in range(G)]
            f = lambda x: group_objective(p, b, kv, G, qh, x, lam1, lam2)
            g = numeric_grad(f, cur["k_hat"][b, kv].copy())
            assert np.max(np.abs(g)) <= 1e-6 * max(1.0, abs(f(cur["k_hat"][b, kv])))


def test_q_hat_update_equals_a_numerical_minimiser():
    p = problem(21, B=1, Hkv=1, G=1, r=3, d=5, L=12, n_om=6)
    lam1, lam2 = 1.0, 1.0
    prev = upd.factor_update(**p, lam1=lam1, lam2=lam2, n_iter=1)
    cur = upd.factor_update(**p, lam1=lam1, lam2=lam2, n_iter=2)
    f = lambda x: sum(lagrangian_of_head(p, 0, 0, 1, x, prev["k_hat"][0, 0], lam1, lam2))
    res = optimize.minimize(f, np.zeros(3), method="BFGS", options=dict(gtol=1e-10))
    np.testing.assert_allclose(cur["q_hat"][0, 0], res.x, rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("G", [1, 2])
def test_rounds_never_increase_the_objective(G):
    p = problem(30 + G, G=G)
    lam1, lam2 = 1.0, 1.0
    B, Hq, _ = p["q"].shape
    vals = []
    for n in (1, 2, 3, 6):
        o = upd.factor_update(**p, lam1=lam1, lam2=lam2, n_iter=n)
        vals.append(sum(group_objective(p, b, kv, G,
                                        [o["q_hat"][b, kv * G + g] for g in range(G)],
                                        o["k_hat"][b, kv], lam1, lam2)
                        for b in range(B) for kv in range(Hq // G)))
    assert all(vals[i + 1] <= vals[i] * (1 + 1e-12) for i in range(len(vals) - 1)), vals
    assert vals[-1] < vals[0]


def test_many_rounds_reach_a_joint_stationary_point():
    p = problem(40, B=1, Hkv=1, G=2)
    lam1, lam2 = 0.5, 0.5
    o = upd.factor_update(**p, lam1=lam1, lam2=lam2, n_iter=400)
    x0 = np.concatenate([o["q_hat"][0, 0], o["q_hat"][0, 1], o["k_hat"][0, 0]])
    r = o["k_hat"].shape[-1]
    f = lambda x: group_objective(p, 0, 0, 2, [x[:r], x[r:2 * r]], x[2 * r:], lam1, lam2)
    assert np.max(np.abs(numeric_grad(f, x0))) <= 1e-5 * max(1.0, f(x0))


# ------------------------------------------------------------------ B_Q / B_K step

def test_line_search_step_closed_forms():
    p = problem(50, bf16=True)
    o = upd.factor_update(**p, lam1=1.0, lam2=1.0, n_iter=2)
    B, Hq, _ = p["q"].shape
    G = Hq // p["B_K"].shape[1]
    for b in range(B):
        for h in range(Hq):
            x_hat, x, Bold = o["q_hat"][b, h], as64(p["q"][b, h]), as64(p["B_Q"][b, h])
            # the gradient is rank one along x_hat, so the optimal step is 1 / |x_hat|^2 ...
            np.testing.assert_allclose(o["eta_Q"][b, h], 1.0 / (x_hat @ x_hat), rtol=1e-10)
            # ... and it removes the residual entirely
            np.testing.assert_allclose(x_hat @ o["B_Q"][b, h], x, rtol=0, atol=1e-12)
            # B moves only along x_hat: directions orthogonal to x_hat keep their image
            y = np.linalg.svd(x_hat[None, :])[2][1:]          # basis of the complement
            np.testing.assert_allclose(y @ o["B_Q"][b, h], y @ Bold, rtol=0, atol=1e-12)
        for kv in range(Hq // G):
            x_hat, x = o["k_hat"][b, kv], as64(p["k_new"][b, kv])
            np.testing.assert_allclose(o["eta_K"][b, kv], 1.0 / (x_hat @ x_hat), rtol=1e-10)
            np.testing.assert_allclose(x_hat @ o["B_K"][b, kv], x, rtol=0, atol=1e-12)


def test_step_length_is_the_minimiser_along_the_gradient():
    p = problem(51, B=1, Hkv=1, G=1)
    o = upd.factor_update(**p, lam1=1.0, lam2=1.0, n_iter=2)
    x_hat, x, Bold = o["q_hat"][0, 0], as64(p["q"][0, 0]), as64(p["B_Q"][0, 0])
    grad = (o["B_Q"][0, 0] - Bold) / -o["eta_Q"][0, 0]
    # the direction is the gradient of the reconstruction term (central differences)
    f = lambda M: 0.5 * np.sum((x_hat @ M.reshape(Bold.shape) - x) ** 2)
    np.testing.assert_allclose(grad.ravel(), numeric_grad(f, Bold.ravel().copy()), rtol=1e-5,
                               atol=1e-7)
    best = optimize.minimize_scalar(lambda e: f(Bold - e * grad), bracket=(0.0, 1.0),
                                    tol=1e-12)
    np.testing.assert_allclose(o["eta_Q"][0, 0], best.x, rtol=1e-6)


def test_zero_residual_leaves_B_unchanged():
    # q in the row space of B_Q and no other term: the residual is zero, the step is 0/0
    rng = np.random.default_rng(52)
    r, d = 3, 6
    B_Q = rng.integers(-3, 4, (1, 1, r, d)).astype(np.float32)
    B_K = B_Q.copy()
    q = (np.array([1.0, -2.0, 0.5]) @ B_Q[0, 0].astype(np.float64)).astype(np.float32)[None, None]
    o = upd.factor_update(q, q.copy(), B_Q, B_K, np.zeros((1, 1, 2, r), np.float32),
                          np.zeros((1, 1, 2, d), np.float32), np.zeros((1, 1, 1), np.int64),
                          lam1=0.0, lam2=0.0, n_iter=1)
    assert np.all(np.isfinite(o["B_Q"])) and np.all(np.isfinite(o["B_K"]))
    np.testing.assert_allclose(o["B_Q"], B_Q, rtol=0, atol=1e-12)


# ------------------------------------------------------------------ Omega and data handling

def test_only_the_rows_of_omega_matter_and_their_order_does_not():
    p = problem(60)
    base = upd.factor_update(**p, lam1=1.0, lam2=1.0)
    p2 = {k: v.copy() for k, v in p.items()}
    B, Hq, _ = p["q"].shape
    G = Hq // p["B_K"].shape[1]
    L = p["A_K"].shape[2]
    for b in range(B):
        for kv in range(Hq // G):
            used = set()
            for g in range(G):
                used |= set(p["omega"][b, kv * G + g].tolist())
            free = [i for i in range(L) if i not in used]
            p2["A_K"][b, kv, free] += 100.0
            p2["K_store"][b, kv, free] -= 50.0
    p2["omega"] = p["omega"][:, :, ::-1].copy()
    other = upd.factor_update(**p2, lam1=1.0, lam2=1.0)
    for key in ("q_hat", "k_hat", "B_Q", "B_K"):
        np.testing.assert_allclose(other[key], base[key], rtol=1e-10, atol=1e-12)


def test_omega_is_previous_selection_plus_lite_window():
    sel = np.array([[[0, 3, 7], [1, 2, 9]]], np.int32)
    om = upd.omega_positions(sel, l=16, w=4)
    assert om.shape == (1, 2, 7)
    assert om[0, 0].tolist() == [0, 3, 7, 12, 13, 14, 15]
    assert om[0, 1].tolist() == [1, 2, 9, 12, 13, 14, 15]


def test_bf16_rows_are_decoded_not_reinterpreted():
    p = problem(61, bf16=True)
    p32 = dict(p)
    p32["K_store"] = bf16_to_f64(p["K_store"]).astype(np.float32)
    p32["k_new"] = bf16_to_f64(p["k_new"]).astype(np.float32)
    a = upd.factor_update(**p, lam1=1.0, lam2=1.0)
    b = upd.factor_update(**p32, lam1=1.0, lam2=1.0)
    for key in a:
        assert np.array_equal(a[key], b[key])


def test_append_writes_row_l_only():
    rng = np.random.default_rng(62)
    B, Hkv, L, r, d, l = 2, 2, 10, 4, 8, 7
    A_K = rng.standard_normal((B, Hkv, L, r)).astype(np.float32)
    K = f32_to_bf16_bits(rng.standard_normal((B, Hkv, L, d)).astype(np.float32))
    V = f32_to_bf16_bits(rng.standard_normal((B, Hkv, L, d)).astype(np.float32))
    A0, K0, V0 = A_K.copy(), K.copy(), V.copy()
    k_hat = rng.standard_normal((B, Hkv, r))
    k_new = f32_to_bf16_bits(rng.standard_normal((B, Hkv, d)).astype(np.float32))
    v_new = f32_to_bf16_bits(rng.standard_normal((B, Hkv, d)).astype(np.float32))
    upd.append_token(A_K, K, V, l, k_hat, k_new, v_new)
    keep = [i for i in range(L) if i != l]
    assert np.array_equal(A_K[:, :, keep], A0[:, :, keep])
    assert np.array_equal(K[:, :, keep], K0[:, :, keep]) and np.array_equal(V[:, :, keep], V0[:, :, keep])
    assert np.array_equal(A_K[:, :, l], k_hat.astype(np.float32))
    assert np.array_equal(K[:, :, l], k_new) and np.array_equal(V[:, :, l], v_new)
