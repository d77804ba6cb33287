"""Pins of the prefill oracle (oracle/lrqk_prefill_oracle.py).  CPU only.

Each test states a fact that the prefill objective of Sec. 4.1 (its Lagrangian, App. A.1) or
plain linear algebra fixes, evaluated with code of the test's own: the Lagrangian written out
with explicit l x l score matrices, numpy.linalg.lstsq, numbers worked by hand.  None calls
the oracle for its own expected value and none re-types its update formulas.
"""
import numpy as np
import pytest

from oracle import lrqk_prefill_oracle as pre
from helpers import f32_to_bf16_bits, bf16_to_f64


def as64(x):
    return bf16_to_f64(x) if x.dtype == np.uint16 else x.astype(np.float64)


def problem(seed, B=1, Hkv=2, G=2, l=12, d=6, r=3, bf16=False, low_rank=False):
    rng = np.random.default_rng(seed)
    Hq = Hkv * G
    if low_rank:   # rank(Q), rank(K) <= r exactly (up to the float32 rounding of the inputs)
        Q = np.einsum("bhlr,bhrd->bhld", rng.standard_normal((B, Hq, l, r)),
                      rng.standard_normal((B, Hq, r, d)))
        K = np.einsum("bhlr,bhrd->bhld", rng.standard_normal((B, Hkv, l, r)),
                      rng.standard_normal((B, Hkv, r, d)))
    else:
        Q = rng.standard_normal((B, Hq, l, d))
        K = rng.standard_normal((B, Hkv, l, d))
    Q, K = Q.astype(np.float32), K.astype(np.float32)
    if bf16:
        Q, K = f32_to_bf16_bits(Q), f32_to_bf16_bits(K)
    A_Q0 = rng.standard_normal((B, Hq, l, r)).astype(np.float32)
    A_K0 = rng.standard_normal((B, Hkv, l, r)).astype(np.float32)
    return dict(Q=Q, K=K, A_Q0=A_Q0, A_K0=A_K0)


def group_lagrangian(p, b, kv, G, A_Q, A_K, B_Q, B_K, lq, lk):
    """Sum over the group's query heads of L_pre (Sec. 4.1), the key term counted once.
    A_Q, B_Q: lists over the group's heads."""
    K = as64(p["K"][b, kv])
    tot = 0.5 * lk * np.sum((K - A_K @ B_K) ** 2)
    for g in range(G):
        Q = as64(p["Q"][b, kv * G + g])
        tot += 0.5 * np.sum((Q @ K.T - A_Q[g] @ A_K.T) ** 2)
        tot += 0.5 * lq * np.sum((Q - A_Q[g] @ B_Q[g]) ** 2)
    return tot


def numeric_grad(f, X, eps=1e-6):
    g = np.zeros_like(X)
    it = np.nditer(X, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        E = np.zeros_like(X); E[i] = eps
        g[i] = (f(X + E) - f(X - E)) / (2 * eps)
    return g


def test_scalar_case_worked_by_hand():
    # l = d = r = 1, one head: q = 2, k = 3, A_Q0 = A_K0 = 1, lambdas = 1, one round.
    #   B_Q = q / a = 2, B_K = k / c = 3
    #   A_K = k (q a + B_K) / (a^2 + B_K^2) = 3 * 5 / 10 = 1.5
    #   A_Q = q (k A_K + B_Q) / (A_K^2 + B_Q^2) = 2 * 6.5 / 6.25 = 2.08
    one = lambda v: np.array(v, np.float32).reshape(1, 1, 1, 1)
    o = pre.prefill_factorize(one(2.0), one(3.0), one(1.0), one(1.0), 1.0, 1.0, 1)
    assert o["B_Q"].item() == 2.0 and o["B_K"].item() == 3.0
    np.testing.assert_allclose(o["A_K"].item(), 1.5, rtol=1e-15)
    np.testing.assert_allclose(o["A_Q"].item(), 2.08, rtol=1e-15)


def test_scalar_case_with_two_query_heads_sharing_a_kv_head():
    # q1 = 2, a1 = 1; q2 = -1, a2 = 2; k = 3, c = 1; lambdas = 1; one round.
    #   B_Q1 = 2, B_Q2 = -0.5, B_K = 3
    #   A_K  = k (q1 a1 + q2 a2 + B_K) / (a1^2 + a2^2 + B_K^2) = 3 * 3 / 14 = 9/14
    #   A_Q1 = q1 (k A_K + B_Q1) / (A_K^2 + B_Q1^2);  A_Q2 = q2 (k A_K + B_Q2) / (A_K^2 + B_Q2^2)
    Q = np.array([2.0, -1.0], np.float32).reshape(1, 2, 1, 1)
    A_Q0 = np.array([1.0, 2.0], np.float32).reshape(1, 2, 1, 1)
    one = lambda v: np.array(v, np.float32).reshape(1, 1, 1, 1)
    o = pre.prefill_factorize(Q, one(3.0), A_Q0, one(1.0), 1.0, 1.0, 1)
    ak = 9.0 / 14.0
    np.testing.assert_allclose(o["B_Q"].ravel(), [2.0, -0.5], rtol=1e-15)
    np.testing.assert_allclose(o["A_K"].item(), ak, rtol=1e-15)
    np.testing.assert_allclose(o["A_Q"].ravel(), [2 * (3 * ak + 2) / (ak * ak + 4),
                                                  -1 * (3 * ak - 0.5) / (ak * ak + 0.25)],
                               rtol=1e-14)


def test_B_updates_are_least_squares_fits():
    p = problem(1, bf16=True)
    o = pre.prefill_factorize(**p, lam_pQ=0.7, lam_pK=1.3, n_iter=1)
    B, Hq, l, d = p["Q"].shape
    for b in range(B):
        for h in range(Hq):
            want = np.linalg.lstsq(as64(p["A_Q0"][b, h]), as64(p["Q"][b, h]), rcond=None)[0]
            np.testing.assert_allclose(o["B_Q"][b, h], want, rtol=1e-9, atol=1e-11)
        for kv in range(p["K"].shape[1]):
            want = np.linalg.lstsq(as64(p["A_K0"][b, kv]), as64(p["K"][b, kv]), rcond=None)[0]
            np.testing.assert_allclose(o["B_K"][b, kv], want, rtol=1e-9, atol=1e-11)


def test_A_K_update_without_the_key_term_is_a_least_squares_fit_of_the_scores():
    # lambda_pK = 0, one query head per KV head: A_K^T = argmin |Q K^T - A_Q A_K^T|
    p = problem(2, G=1)
    o = pre.prefill_factorize(**p, lam_pQ=1.0, lam_pK=0.0, n_iter=1)
    for kv in range(p["K"].shape[1]):
        S = as64(p["Q"][0, kv]) @ as64(p["K"][0, kv]).T            # l x l scores
        want = np.linalg.lstsq(as64(p["A_Q0"][0, kv]), S, rcond=None)[0].T
        np.testing.assert_allclose(o["A_K"][0, kv], want, rtol=1e-8, atol=1e-10)


@pytest.mark.parametrize("G,bf16", [(1, False), (2, True), (3, False)])
def test_every_block_update_is_stationary(G, bf16):
    p = problem(10 + G, Hkv=2, G=G, bf16=bf16)
    lq, lk = 0.8, 1.7
    o = pre.prefill_factorize(**p, lam_pQ=lq, lam_pK=lk, n_iter=1)
    for kv in range(2):
        hs = [kv * G + g for g in range(G)]
        A_Q0 = [as64(p["A_Q0"][0, h]) for h in hs]
        A_Q1 = [o["A_Q"][0, h] for h in hs]
        B_Q = [o["B_Q"][0, h] for h in hs]
        B_K, A_K1 = o["B_K"][0, kv], o["A_K"][0, kv]
        A_K0 = as64(p["A_K0"][0, kv])
        scale = group_lagrangian(p, 0, kv, G, A_Q0, A_K0, B_Q, B_K, lq, lk)
        # B_K given the initial A_K; B_Q,g given the initial A_Q,g
        g = numeric_grad(lambda X: group_lagrangian(p, 0, kv, G, A_Q0, A_K0, B_Q, X, lq, lk), B_K.copy())
        assert np.abs(g).max() <= 1e-6 * scale
        for i in range(G):
            def f(X, i=i):
                return group_lagrangian(p, 0, kv, G, A_Q0, A_K0, B_Q[:i] + [X] + B_Q[i + 1:], B_K, lq, lk)
            assert np.abs(numeric_grad(f, B_Q[i].copy())).max() <= 1e-6 * scale
        # A_K given the initial A_Q and the new B's
        g = numeric_grad(lambda X: group_lagrangian(p, 0, kv, G, A_Q0, X, B_Q, B_K, lq, lk), A_K1.copy())
        assert np.abs(g).max() <= 1e-6 * scale
        # A_Q,g given the new A_K
        for i in range(G):
            def f(X, i=i):
                return group_lagrangian(p, 0, kv, G, A_Q0[:i] + [X] + A_Q0[i + 1:], A_K1, B_Q, B_K, lq, lk)
            assert np.abs(numeric_grad(f, A_Q1[i].copy())).max() <= 1e-6 * scale


@pytest.mark.parametrize("G", [1, 2])
def test_rounds_never_increase_the_lagrangian(G):
    p = problem(20 + G, G=G)
    lq = lk = 1.0
    vals = []
    for n in (1, 2, 3, 6, 12):
        o = pre.prefill_factorize(**p, lam_pQ=lq, lam_pK=lk, n_iter=n)
        vals.append(sum(group_lagrangian(p, 0, kv, G, [o["A_Q"][0, kv * G + g] for g in range(G)],
                                         o["A_K"][0, kv], [o["B_Q"][0, kv * G + g] for g in range(G)],
                                         o["B_K"][0, kv], lq, lk) for kv in range(2)))
    assert all(vals[i + 1] <= vals[i] * (1 + 1e-12) for i in range(len(vals) - 1)), vals
    assert vals[-1] < vals[0]


def test_low_rank_inputs_are_recovered():
    # rank(Q), rank(K) <= r: a zero of the Lagrangian exists (A_K spanning K's column space,
    # A_Q = Q K^T A_K (A_K^T A_K)^-1); the alternating updates reach it
    p = problem(30, G=1, l=20, d=8, r=3, low_rank=True)
    o = pre.prefill_factorize(**p, lam_pQ=1.0, lam_pK=1.0, n_iter=200)
    for kv in range(2):
        Q, K = as64(p["Q"][0, kv]), as64(p["K"][0, kv])
        S = Q @ K.T
        assert np.abs(o["A_Q"][0, kv] @ o["A_K"][0, kv].T - S).max() <= 1e-5 * np.abs(S).max()
        assert np.abs(o["A_K"][0, kv] @ o["B_K"][0, kv] - K).max() <= 1e-5 * np.abs(K).max()
        assert np.abs(o["A_Q"][0, kv] @ o["B_Q"][0, kv] - Q).max() <= 1e-5 * np.abs(Q).max()


def test_bf16_rows_are_decoded_not_reinterpreted():
    p = problem(40, bf16=True)
    p32 = dict(p, Q=bf16_to_f64(p["Q"]).astype(np.float32), K=bf16_to_f64(p["K"]).astype(np.float32))
    a = pre.prefill_factorize(**p, lam_pQ=1.0, lam_pK=1.0)
    b = pre.prefill_factorize(**p32, lam_pQ=1.0, lam_pK=1.0)
    for key in a:
        assert np.array_equal(a[key], b[key])


def test_groups_are_independent_and_heads_map_to_their_kv_head():
    p = problem(41, Hkv=2, G=2)
    base = pre.prefill_factorize(**p, lam_pQ=1.0, lam_pK=1.0)
    p2 = {k: v.copy() for k, v in p.items()}
    p2["K"][0, 1] += 3.0            # touch only the second group
    p2["Q"][0, 3] -= 2.0
    other = pre.prefill_factorize(**p2, lam_pQ=1.0, lam_pK=1.0)
    for key, idx in (("A_K", 0), ("B_K", 0)):
        assert np.array_equal(other[key][0, idx], base[key][0, idx])
    for h in (0, 1):
        assert np.array_equal(other["A_Q"][0, h], base["A_Q"][0, h])
    assert not np.allclose(other["A_K"][0, 1], base["A_K"][0, 1])
    assert not np.allclose(other["A_Q"][0, 2], base["A_Q"][0, 2])   # same group as head 3
