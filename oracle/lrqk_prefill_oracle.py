"""CPU oracle of the prefill factorisation of LRQK (Alg. 1; Sec. 4.1 "Prefill": objective,
Lagrangian and the four update rules; App. A.1).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  Nothing in the product package imports it, and it imports nothing from
the product package.

Plain numpy in float64, one (batch, KV head) group at a time, the updates in the order of
Alg. 1.  Library primitives: matrix products and numpy.linalg.solve for the r x r systems.

What it computes, for Q (l x d per query head) and K (l x d per KV head), starting from the
given A_Q, A_K (the paper draws them from N(0,1); the draws are inputs here):

    repeat n_iter times:
        B_Q <- (A_Q^T A_Q)^-1 A_Q^T Q                                           (per query head)
        B_K <- (A_K^T A_K)^-1 A_K^T K                                           (per KV head)
        A_K <- K (sum_g Q_g^T A_Q,g + lambda_pK B_K^T)
                 (sum_g A_Q,g^T A_Q,g + lambda_pK B_K B_K^T)^-1                 (per KV head)
        A_Q <- Q (K^T A_K + lambda_pQ B_Q^T) (A_K^T A_K + lambda_pQ B_Q B_Q^T)^-1   (per query head)

Readings of points the paper leaves open (each also listed in the design notes)
  - Grouped-query attention: A_Q, B_Q per query head; A_K, B_K per KV head.  The term
    |Q K^T - A_Q A_K^T|^2 exists once per query head of the group, so the A_K rule minimises
    the SUM of the group's Lagrangians (the key term counted once); with one query head per
    KV head it is the paper's rule.
  - The loop runs exactly n_iter rounds (the paper's maximum is 2); no convergence test.
  - B_Q, B_K are returned as computed at the top of the last round (Alg. 1 does not refresh
    them after the last A update).
  - (Q K^T) A is evaluated as Q (K^T A), as Sec. 4.1 recommends; in exact arithmetic the
    same thing.

Pins: tests/test_prefill_oracle_pins.py.
"""
from __future__ import annotations

import numpy as np


def _rows_as_f64(rows: np.ndarray) -> np.ndarray:
    """Q/K rows as float64: uint16 arrays hold bf16 bit patterns, float32 arrays values."""
    if rows.dtype == np.uint16:
        return (rows.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    if rows.dtype == np.float32:
        return rows.astype(np.float64)
    raise TypeError(f"rows must be uint16 (bf16 bits) or float32, got {rows.dtype}")


def _right_solve(X: np.ndarray, M: np.ndarray) -> np.ndarray:
    """X M^-1 for a square M."""
    return np.linalg.solve(M.T, X.T).T


def prefill_factorize(Q, K, A_Q0, A_K0, lam_pQ: float, lam_pK: float, n_iter: int = 2):
    """Alg. 1.

    Q     uint16|float32 [B,Hq,l,d]      K     uint16|float32 [B,Hkv,l,d]
    A_Q0  float32 [B,Hq,l,r]             A_K0  float32 [B,Hkv,l,r]        (initial values)
    Returns a dict of float64 arrays A_Q [B,Hq,l,r], A_K [B,Hkv,l,r], B_Q [B,Hq,r,d],
    B_K [B,Hkv,r,d].
    """
    assert n_iter >= 1
    B, Hq, l, d = Q.shape
    Hkv = K.shape[1]
    r = A_K0.shape[3]
    G = Hq // Hkv
    assert Hq == G * Hkv and A_Q0.shape == (B, Hq, l, r) and A_K0.shape == (B, Hkv, l, r)
    out = dict(A_Q=np.zeros((B, Hq, l, r)), A_K=np.zeros((B, Hkv, l, r)),
               B_Q=np.zeros((B, Hq, r, d)), B_K=np.zeros((B, Hkv, r, d)))
    for b in range(B):
        for kv in range(Hkv):
            heads = list(range(kv * G, (kv + 1) * G))
            Kf = _rows_as_f64(K[b, kv])
            Qf = {h: _rows_as_f64(Q[b, h]) for h in heads}
            A_K = A_K0[b, kv].astype(np.float64)
            A_Q = {h: A_Q0[b, h].astype(np.float64) for h in heads}
            B_Q, B_K = {}, None
            for _ in range(n_iter):
                for h in heads:
                    B_Q[h] = np.linalg.solve(A_Q[h].T @ A_Q[h], A_Q[h].T @ Qf[h])
                B_K = np.linalg.solve(A_K.T @ A_K, A_K.T @ Kf)
                W = lam_pK * B_K.T
                S = lam_pK * (B_K @ B_K.T)
                for h in heads:
                    W = W + Qf[h].T @ A_Q[h]
                    S = S + A_Q[h].T @ A_Q[h]
                A_K = _right_solve(Kf @ W, S)
                KtA = Kf.T @ A_K
                AtA = A_K.T @ A_K
                for h in heads:
                    A_Q[h] = _right_solve(Qf[h] @ (KtA + lam_pQ * B_Q[h].T),
                                          AtA + lam_pQ * (B_Q[h] @ B_Q[h].T))
            out["A_K"][b, kv] = A_K
            out["B_K"][b, kv] = B_K
            for h in heads:
                out["A_Q"][b, h] = A_Q[h]
                out["B_Q"][b, h] = B_Q[h]
    return out
