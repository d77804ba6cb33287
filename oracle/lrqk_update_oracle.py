"""CPU oracle of the decode-time factor update of LRQK (Alg. 2, the steps before
"compute proxy attention"; Sec. 4.2 decode objective and its update rules; App. A.2).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  Nothing in the product package imports it, and it
imports nothing from the product package.

Plain numpy in float64, one (batch, KV head) group at a time, the steps in the
order and notation of Alg. 2.  The only library primitive is numpy.linalg.solve
for the r x r systems.

What one update computes, for new projections q_t (per query head) and k_t (per KV head):

    k_hat   <- k B_K^T (B_K B_K^T)^-1                                  (initial guess, lambda_d1 = 0)
    repeat n_iter times:
        q_hat <- m_lq M_rq^-1                                          (per query head)
            m_lq = q B_Q^T + lambda_d1 (q.k) k_hat + lambda_d2 (q K_Om^T) A_Om
            M_rq = B_Q B_Q^T + lambda_d1 k_hat^T k_hat + lambda_d2 A_Om^T A_Om
        k_hat <- (k B_K^T + lambda_d1 sum_g (q_g.k) q_hat_g)
                 (B_K B_K^T + lambda_d1 sum_g q_hat_g^T q_hat_g)^-1    (per KV head)
    B_Q <- B_Q - eta_Q grad_Q,  grad_Q = q_hat^T (q_hat B_Q - q)       (one exact line-search step)
    B_K <- B_K - eta_K grad_K,  grad_K = k_hat^T (k_hat B_K - k)
        eta = <residual, x_hat grad> / <x_hat grad, x_hat grad>        (App. A.2, optimal step)

Readings of points the paper leaves open (each also listed in the design notes)
  - Grouped-query attention: B_Q and q_hat are per query head; B_K, k_hat and the row
    appended to A_K are per KV head.  The lambda_d1 term ties k_hat to every query head of
    its group, so the k_hat rule above minimises the SUM of the group's Lagrangians; with
    one query head per KV head it is the paper's rule.
  - Omega, "the KV cache retained on the GPU at step t-1", is the set attended at the
    previous step: the previous top-k selection plus the lite window [l-w, l) as it stands
    before the new token is appended.
  - q K_Om^T is the raw dot product (no softmax scale): it is matched against q_hat A_Om^T.
  - The loop runs exactly n_iter rounds (the paper's maximum, 2); there is no tolerance
    test, which would only skip work and make the result depend on rounding.
  - A zero gradient (the residual is already zero) leaves B unchanged: eta = 0 instead of 0/0.

Pins: tests/test_update_oracle_pins.py (stationarity of the Lagrangian, least-squares
special cases via numpy.linalg.lstsq, exact recovery on consistent data, monotone decrease,
the closed form of the line search, a brute-force minimiser on a tiny case).
"""
from __future__ import annotations

import numpy as np


def _rows_as_f64(rows: np.ndarray) -> np.ndarray:
    """K/V rows as float64: uint16 arrays hold bf16 bit patterns, float32 arrays values."""
    if rows.dtype == np.uint16:
        return (rows.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    if rows.dtype == np.float32:
        return rows.astype(np.float64)
    raise TypeError(f"rows must be uint16 (bf16 bits) or float32, got {rows.dtype}")


def omega_positions(sel_idx_prev: np.ndarray, l: int, w: int) -> np.ndarray:
    """Omega of the update: previous selection [B,Hq,k] followed by the lite window [l-w, l)."""
    B, Hq, _ = sel_idx_prev.shape
    lite = np.broadcast_to(np.arange(l - w, l, dtype=np.int64), (B, Hq, w))
    return np.concatenate([sel_idx_prev.astype(np.int64), lite], axis=2)


def _solve_right(m: np.ndarray, M: np.ndarray) -> np.ndarray:
    """The row vector x with x M = m."""
    return np.linalg.solve(M.T, m)


def _line_search_step(x_hat: np.ndarray, Bm: np.ndarray, x: np.ndarray):
    """One gradient step on 1/2 |x_hat B - x|^2 with the optimal step length (App. A.2)."""
    resid = x_hat @ Bm - x                      # 1 x d
    grad = np.outer(x_hat, resid)               # r x d
    xg = x_hat @ grad                           # 1 x d
    den = float(xg @ xg)
    eta = float(resid @ xg) / den if den > 0.0 else 0.0
    return Bm - eta * grad, eta


def factor_update(q, k_new, B_Q, B_K, A_K, K_store, omega, lam1: float, lam2: float,
                  n_iter: int = 2):
    """One decode-time update.

    q       float32 [B,Hq,d]          k_new   uint16|float32 [B,Hkv,d]
    B_Q     float32 [B,Hq,r,d]        B_K     float32 [B,Hkv,r,d]
    A_K     float32 [B,Hkv,L,r]       K_store uint16|float32 [B,Hkv,L,d]
    omega   int     [B,Hq,n_omega]    positions of the rows of Omega (all < L)
    Returns a dict of float64 arrays: q_hat [B,Hq,r], k_hat [B,Hkv,r], B_Q [B,Hq,r,d],
    B_K [B,Hkv,r,d], eta_Q [B,Hq], eta_K [B,Hkv].
    """
    assert n_iter >= 1
    B, Hq, d = q.shape
    Hkv = B_K.shape[1]
    r = B_K.shape[2]
    G = Hq // Hkv
    assert Hq == G * Hkv and B_Q.shape == (B, Hq, r, d) and B_K.shape == (B, Hkv, r, d)
    out = dict(q_hat=np.zeros((B, Hq, r)), k_hat=np.zeros((B, Hkv, r)),
               B_Q=np.zeros((B, Hq, r, d)), B_K=np.zeros((B, Hkv, r, d)),
               eta_Q=np.zeros((B, Hq)), eta_K=np.zeros((B, Hkv)))
    for b in range(B):
        for kv in range(Hkv):
            BK = B_K[b, kv].astype(np.float64)
            kt = _rows_as_f64(k_new[b, kv])
            BKBKt = BK @ BK.T
            kBKt = kt @ BK.T
            k_hat = _solve_right(kBKt, BKBKt)            # initial guess: lambda_d1 = 0
            heads = range(kv * G, (kv + 1) * G)
            per_head = {}
            for h in heads:
                BQ = B_Q[b, h].astype(np.float64)
                qt = q[b, h].astype(np.float64)
                pos = np.asarray(omega[b, h], dtype=np.int64)
                A_om = A_K[b, kv, pos, :].astype(np.float64)         # n_omega x r
                K_om = _rows_as_f64(K_store[b, kv, pos, :])          # n_omega x d
                per_head[h] = dict(BQ=BQ, qt=qt, qk=float(qt @ kt), qBQt=qt @ BQ.T,
                                   BQBQt=BQ @ BQ.T, qKtA=(qt @ K_om.T) @ A_om,
                                   AtA=A_om.T @ A_om, q_hat=None)
            for _ in range(n_iter):
                for h in heads:
                    t = per_head[h]
                    m_lq = t["qBQt"] + lam1 * t["qk"] * k_hat + lam2 * t["qKtA"]
                    M_rq = t["BQBQt"] + lam1 * np.outer(k_hat, k_hat) + lam2 * t["AtA"]
                    t["q_hat"] = _solve_right(m_lq, M_rq)
                rhs = kBKt.copy()
                lhs = BKBKt.copy()
                for h in heads:
                    t = per_head[h]
                    rhs += lam1 * t["qk"] * t["q_hat"]
                    lhs += lam1 * np.outer(t["q_hat"], t["q_hat"])
                k_hat = _solve_right(rhs, lhs)
            for h in heads:
                t = per_head[h]
                out["q_hat"][b, h] = t["q_hat"]
                out["B_Q"][b, h], out["eta_Q"][b, h] = _line_search_step(t["q_hat"], t["BQ"],
                                                                          t["qt"])
            out["k_hat"][b, kv] = k_hat
            out["B_K"][b, kv], out["eta_K"][b, kv] = _line_search_step(k_hat, BK, kt)
    return out


def append_token(A_K, K_store, V_store, l: int, k_hat, k_new, v_new):
    """Alg. 2, "concatenate" and "Async k_t, v_t to CPU": row l of A_K, K and V (arrays with
    room for it) receive k_hat (rounded once to float32) and the new key / value rows (bit
    copies).  In place; the context length becomes l + 1."""
    assert A_K.shape[2] > l and K_store.shape[2] > l and V_store.shape[2] > l
    assert k_new.dtype == K_store.dtype and v_new.dtype == V_store.dtype
    A_K[:, :, l, :] = np.asarray(k_hat, dtype=np.float64).astype(np.float32)
    K_store[:, :, l, :] = k_new
    V_store[:, :, l, :] = v_new
