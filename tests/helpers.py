"""Shared test helpers: textbook formulas written with numpy/scipy only.

These are the *pins*: independent statements of what the oracle (and through
it the HIP path) must reproduce.  They call neither the oracle nor the HIP
library.
"""
from __future__ import annotations

import numpy as np
from scipy.special import softmax


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float64 values."""
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def kv_to_f64(a: np.ndarray) -> np.ndarray:
    return bf16_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


def dense_attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> np.ndarray:
    """Textbook softmax(scale q K^T) V over ALL rows, GQA by head // G.
    q [B,Hq,d] fp32, K,V [B,Hkv,l,d] (bf16 bits or fp32) -> float64 [B,Hq,d]."""
    B, Hq, d = q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    Kf, Vf = kv_to_f64(K), kv_to_f64(V)
    out = np.empty((B, Hq, d))
    for b in range(B):
        for h in range(Hq):
            logits = scale * (Kf[b, h // G] @ q[b, h].astype(np.float64))
            out[b, h] = softmax(logits) @ Vf[b, h // G]
    return out


def topk_by_lexsort(scores: np.ndarray, k: int, w: int) -> np.ndarray:
    """Top-k of scores[..., :l-w], ties to the lower position, ascending output (numpy only)."""
    B, Hq, l = scores.shape
    out = np.empty((B, Hq, k), np.int32)
    for b in range(B):
        for h in range(Hq):
            s = scores[b, h, : l - w]
            order = np.lexsort((np.arange(l - w), -s))  # primary: -s, secondary: position
            out[b, h] = np.sort(order[:k])
    return out


def check_topk_sets(sel: np.ndarray, ref: np.ndarray, s64: np.ndarray, w: int,
                    rel: float = 1e-5) -> int:
    """Compare two selections head by head.  They must be equal, except that
    positions whose double-precision score lies within `rel` (relative) of the
    k-th largest score may be swapped for one another.  Returns the number of
    heads that used the exception; raises AssertionError on any real mismatch."""
    B, Hq, k = sel.shape
    l = s64.shape[2]
    used = 0
    for b in range(B):
        for h in range(Hq):
            a, r = sel[b, h], ref[b, h]
            assert a.min() >= 0 and a.max() < l - w, "selected position outside [0, l-w)"
            assert np.all(np.diff(a) > 0), "selection not strictly ascending"
            if np.array_equal(a, r):
                continue
            used += 1
            s = s64[b, h]
            tau = np.sort(s[: l - w])[::-1][k - 1]
            band = rel * np.maximum(np.abs(s), abs(tau))
            only_a = np.setdiff1d(a, r)
            only_r = np.setdiff1d(r, a)
            for i in np.concatenate([only_a, only_r]):
                assert abs(s[i] - tau) <= band[i], (
                    f"head ({b},{h}): position {i} differs and is not a near-tie "
                    f"(score {s[i]!r}, threshold {tau!r})")
    return used
