"""numpy front end of the CPU oracle (oracle/lrqk_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  Nothing in the product package imports it, and
it imports nothing from the product package.

Arrays are numpy, C-contiguous.  bf16 K/V rows are passed as uint16 arrays
(kv_dtype 0), fp32 rows as float32 (kv_dtype 1).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lrqk_oracle.c")
_LIB = os.path.join(_HERE, "liblrqk_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over heads). Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-mfma", "-fPIC", "-shared",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_num_threads.restype = C.c_int
        _lib.oracle_cache_resolve.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _p(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"], "array must be C-contiguous"
    return a.ctypes.data_as(C.c_void_p)


def _kv_dtype(a: np.ndarray) -> int:
    if a.dtype == np.uint16:
        return 0
    if a.dtype == np.float32:
        return 1
    raise TypeError(f"K/V rows must be uint16 (bf16 bits) or float32, got {a.dtype}")


def proxy_scores(A_K: np.ndarray, q_hat: np.ndarray):
    """Alg. 2 proxy attention. Returns (s64 [B,Hq,l] float64, s32 [B,Hq,l] float32)."""
    B, Hkv, l, r = A_K.shape
    Hq = q_hat.shape[1]
    assert A_K.dtype == np.float32 and q_hat.dtype == np.float32
    assert q_hat.shape == (B, Hq, r) and Hq % Hkv == 0
    s64 = np.empty((B, Hq, l), np.float64)
    s32 = np.empty((B, Hq, l), np.float32)
    lib().oracle_proxy_scores(B, Hq, Hkv, l, r, _p(A_K), _p(q_hat), _p(s64), _p(s32))
    return s64, s32


def select_topk(scores: np.ndarray, k: int, w: int) -> np.ndarray:
    """Omega_k per head from scores [B,Hq,l] (any float dtype). int32 [B,Hq,k], ascending."""
    B, Hq, l = scores.shape
    assert 1 <= k <= l - w
    s = np.ascontiguousarray(scores, dtype=np.float64)
    sel = np.empty((B, Hq, k), np.int32)
    lib().oracle_select_topk(B * Hq, l, w, k, _p(s), _p(sel))
    return sel


class CacheState:
    """slot_of [B,Hq,l], token_of [B,Hq,C], last_used [B,Hq,C] (int32), all -1 when empty."""

    def __init__(self, B: int, Hq: int, l: int, Cslots: int):
        self.slot_of = np.full((B, Hq, l), -1, np.int32)
        self.token_of = np.full((B, Hq, Cslots), -1, np.int32)
        self.last_used = np.full((B, Hq, Cslots), -1, np.int32)

    @classmethod
    def identity(cls, B: int, Hq: int, l: int) -> "CacheState":
        """Slot i holds token i (a cache as large as the context, everything resident)."""
        st = cls(B, Hq, l, l)
        st.slot_of[:] = np.arange(l, dtype=np.int32)
        st.token_of[:] = np.arange(l, dtype=np.int32)
        st.last_used[:] = 0
        return st

    def copy(self) -> "CacheState":
        c = object.__new__(CacheState)
        c.slot_of, c.token_of, c.last_used = (self.slot_of.copy(), self.token_of.copy(),
                                              self.last_used.copy())
        return c


def cache_resolve(sel_idx: np.ndarray, step: int, st: CacheState):
    """Sec. 4.1 hit/miss resolution; updates `st` in place.
    Returns dict(sel_slot, hit, miss_tok, miss_slot, n_miss, ok)."""
    B, Hq, k = sel_idx.shape
    l, Cs = st.slot_of.shape[2], st.token_of.shape[2]
    sel_slot = np.full((B, Hq, k), -1, np.int32)
    hit = np.zeros((B, Hq, k), np.uint8)
    miss_tok = np.full((B, Hq, k), -1, np.int32)
    miss_slot = np.full((B, Hq, k), -1, np.int32)
    n_miss = np.zeros((B, Hq), np.int32)
    rc = lib().oracle_cache_resolve(B * Hq, l, Cs, k, _p(np.ascontiguousarray(sel_idx)),
                                    C.c_int32(step), _p(st.slot_of), _p(st.token_of),
                                    _p(st.last_used), _p(sel_slot), _p(hit), _p(miss_tok),
                                    _p(miss_slot), _p(n_miss))
    return dict(sel_slot=sel_slot, hit=hit, miss_tok=miss_tok, miss_slot=miss_slot,
                n_miss=n_miss, ok=(rc == 0))


def fetch(K_store, V_store, miss_tok, miss_slot, n_miss, cacheK, cacheV):
    """Alg. 2 fetch + merge: copy the missing rows into their slots (in place)."""
    B, Hkv, l, d = K_store.shape
    Hq, Cs = cacheK.shape[1], cacheK.shape[2]
    k = miss_tok.shape[2]
    kvd = _kv_dtype(K_store)
    assert _kv_dtype(cacheK) == kvd and cacheK.shape == (B, Hq, Cs, d) == cacheV.shape
    lib().oracle_fetch(B, Hq, Hkv, l, Cs, d, k, kvd, _p(K_store), _p(V_store), _p(miss_tok),
                       _p(miss_slot), _p(n_miss), _p(cacheK), _p(cacheV))


def group_fetch(K_store, V_store, miss_tok, miss_slot, n_miss, cacheK, cacheV):
    """Alg. 2 fetch + merge with the host link shared inside a KV group.  K and V are stored
    once per KV head and the paper aligns heads by repeating them (Sec. 4, preliminaries), so a
    position that several query heads of one group miss in the same step is the SAME host row:
    it is read from the store once and written into the slot each of those heads gave it.
    The caches end up exactly as with `fetch`; what changes is the number of rows that cross
    the link: the size of the union of the group's miss lists instead of their total length
    (Sec. 5.3 counts fetched rows; this is the count per KV head).

    Plain loops over (batch, KV head), positions in ascending order.  Updates cacheK, cacheV in
    place.  Returns (link_rows int64 [B,Hkv], union: list over (b, kv) of the sorted positions)."""
    B, Hkv, l, d = K_store.shape
    Hq = cacheK.shape[1]
    G = Hq // Hkv
    assert Hq == G * Hkv and cacheK.shape == cacheV.shape and cacheK.dtype == K_store.dtype
    link_rows = np.zeros((B, Hkv), np.int64)
    union = []
    for b in range(B):
        for kv in range(Hkv):
            wanted = {}                              # position -> [(head, slot), ...]
            for h in range(kv * G, (kv + 1) * G):
                for j in range(max(int(n_miss[b, h]), 0)):
                    wanted.setdefault(int(miss_tok[b, h, j]), []).append((h, int(miss_slot[b, h, j])))
            positions = sorted(wanted)
            for pos in positions:
                k_row, v_row = K_store[b, kv, pos].copy(), V_store[b, kv, pos].copy()  # one read
                for h, slot in wanted[pos]:
                    cacheK[b, h, slot] = k_row
                    cacheV[b, h, slot] = v_row
            link_rows[b, kv] = len(positions)
            union.append(np.array(positions, np.int64))
    return link_rows, union


def sparse_attend(q, cacheK, cacheV, sel_slot, liteK, liteV, scale: float) -> np.ndarray:
    """Sec. 4.3 attention over the k cache rows + w lite rows. float64 [B,Hq,d]."""
    B, Hq, d = q.shape
    Cs, k = cacheK.shape[2], sel_slot.shape[2]
    Hkv, w = liteK.shape[1], liteK.shape[2]
    kvd = _kv_dtype(cacheK)
    assert q.dtype == np.float32
    out = np.empty((B, Hq, d), np.float64)
    lib().oracle_sparse_attend(B, Hq, Hkv, Cs, d, k, w, kvd, C.c_double(scale), _p(q),
                               _p(cacheK), _p(cacheV), _p(np.ascontiguousarray(sel_slot)),
                               _p(liteK), _p(liteV), _p(out))
    return out


def attend_store(q, K_store, V_store, sel_idx, w: int, scale: float) -> np.ndarray:
    """The same attention with rows read from the full store (no cache). float64 [B,Hq,d]."""
    B, Hq, d = q.shape
    Hkv, l = K_store.shape[1], K_store.shape[2]
    k = sel_idx.shape[2]
    out = np.empty((B, Hq, d), np.float64)
    lib().oracle_attend_store(B, Hq, Hkv, l, d, k, w, _kv_dtype(K_store), C.c_double(scale),
                              _p(q), _p(K_store), _p(V_store),
                              _p(np.ascontiguousarray(sel_idx)), _p(out))
    return out


def decode_step(A_K, q_hat, q, K_store, V_store, st: CacheState, cacheK, cacheV, step: int,
                k: int, w: int, scale: float, sel_idx=None, score_precision: str = "s32"):
    """One full step a1..a5 in the paper's order (Alg. 2 proxy/top-k, fetch, merge; Sec. 4.3).

    Updates `st`, cacheK, cacheV in place.  `sel_idx` may be forced (to follow a
    selection made elsewhere); otherwise the top-k decision is taken on the fp32
    fma-chain scores ("s32") or on the double scores ("s64").
    """
    l = A_K.shape[2]
    s64, s32 = proxy_scores(A_K, q_hat)
    if sel_idx is None:
        sel_idx = select_topk(s32 if score_precision == "s32" else s64, k, w)
    res = cache_resolve(sel_idx, step, st)
    fetch(K_store, V_store, res["miss_tok"], res["miss_slot"], np.maximum(res["n_miss"], 0),
          cacheK, cacheV)
    liteK = np.ascontiguousarray(K_store[:, :, l - w:, :])
    liteV = np.ascontiguousarray(V_store[:, :, l - w:, :])
    out = sparse_attend(q, cacheK, cacheV, res["sel_slot"], liteK, liteV, scale)
    res.update(s64=s64, s32=s32, sel_idx=sel_idx, out=out,
               miss_rate=float(np.maximum(res["n_miss"], 0).sum()) / (sel_idx.size))
    return res


def qhat_closed_form(q: np.ndarray, B_Q: np.ndarray) -> np.ndarray:
    """Decode update of q_hat (Eq. 9) with lambda_d1 = lambda_d2 = 0:
    q_hat = (q B_Q^T)(B_Q B_Q^T)^-1, the least-squares solution of q_hat B_Q = q.
    q [..., d], B_Q [r, d] -> [..., r], float64."""
    q = np.asarray(q, np.float64)
    BQ = np.asarray(B_Q, np.float64)
    M = BQ @ BQ.T
    rhs = q @ BQ.T
    return np.linalg.solve(M, rhs.reshape(-1, BQ.shape[0]).T).T.reshape(rhs.shape)
