"""ctypes binding of liblrqk.so.  Marshalling only; no arithmetic on this side."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch  # loaded first so that the library binds to the HIP runtime torch uses

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "liblrqk.so")
_lib = None

LRQK_KV_BF16, LRQK_KV_F32 = 0, 1
LRQK_FETCH_STAGED, LRQK_FETCH_DIRECT, LRQK_FETCH_GROUP = 0, 1, 2
LRQK_SELECT_FRESH = 0x100
LRQK_WS_SELECT, LRQK_WS_ATTEND, LRQK_WS_UPDATE, LRQK_WS_PREFILL = 1, 2, 3, 4


class LrqkError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load_library().lrqk_status_string(status).decode()
        hip = load_library().lrqk_last_hip_error() if status == -3 else 0
        super().__init__(f"{where}: {msg} (status {status}" + (f", hipError {hip})" if hip else ")"))


class Shape(C.Structure):
    """lrqk_shape."""
    _fields_ = [(n, C.c_int32) for n in ("B", "Hq", "Hkv", "d", "l", "r", "k", "w", "C", "kv_dtype")]
    _fields_.append(("scale", C.c_float))
    _fields_.append(("l_cap", C.c_int32))

    @classmethod
    def make(cls, *, B, Hq, Hkv, l, r, k, w, C_slots, d=128, kv_dtype=LRQK_KV_BF16, scale=None,
             l_cap=0):
        return cls(B, Hq, Hkv, d, l, r, k, w, C_slots, kv_dtype,
                   float(scale if scale is not None else d ** -0.5), l_cap)

    def with_l(self, l: int) -> "Shape":
        """The same shape at another context length (same l_cap)."""
        return Shape(self.B, self.Hq, self.Hkv, self.d, l, self.r, self.k, self.w, self.C,
                     self.kv_dtype, self.scale, self.l_cap)

    @property
    def rows(self) -> int:
        """Rows allocated per head in A_K, the K/V store and slot_of."""
        return self.l_cap if self.l_cap > 0 else self.l


class Layer(C.Structure):
    """lrqk_layer: raw pointers of one layer's buffers."""
    _fields_ = [(n, C.c_void_p) for n in ("A_K", "K_host", "V_host", "liteK", "liteV", "slot_of",
                                          "token_of", "last_used", "cacheK", "cacheV",
                                          "sel_thr")]


class _StepDebug(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("sel_idx", "sel_slot", "hit", "miss_tok", "miss_slot",
                                          "n_miss", "link_rows")]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load liblrqk.so (built in-tree by `python -m paper_2510_23649_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2510_23649_amd.build` "
            "(there is no CPU or PyTorch fallback)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    sp = C.POINTER(Shape)
    sigs = {
        "lrqk_version": (C.c_int, []),
        "lrqk_status_string": (C.c_char_p, [C.c_int]),
        "lrqk_last_hip_error": (C.c_int, []),
        "lrqk_validate_shape": (C.c_int, [sp]),
        "lrqk_workspace_bytes": (sz, [sp, C.c_int]),
        "lrqk_proxy_scores": (C.c_int, [sp, vp, vp, vp, vp]),
        "lrqk_select_topk": (C.c_int, [sp, vp, vp, vp, sz, vp]),
        "lrqk_cache_init": (C.c_int, [sp, vp, vp, vp, vp]),
        "lrqk_select_state_init": (C.c_int, [sp, vp, vp]),
        "lrqk_cache_resolve": (C.c_int, [sp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]),
        "lrqk_sparse_attend": (C.c_int, [sp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]),
        "lrqk_sparse_attend_noalloc": (C.c_int, [sp, vp, vp, vp, vp, vp, vp, vp, vp]),
        "lrqk_factor_update": (C.c_int, [sp, C.POINTER(Layer), vp, vp, vp, vp, vp, vp, C.c_float,
                                         C.c_float, i32, vp, vp, vp, sz, vp]),
        "lrqk_append_token": (C.c_int, [sp, C.POINTER(Layer), vp, vp, vp, vp]),
        "lrqk_prefill_factorize": (C.c_int, [sp, vp, vp, vp, vp, vp, vp, C.c_float, C.c_float,
                                             i32, vp, sz, vp]),
        "lrqk_plan_create": (C.c_int, [sp, C.POINTER(vp)]),
        "lrqk_plan_destroy": (C.c_int, [vp]),
        "lrqk_fetch_misses": (C.c_int, [vp, sp, vp, vp, vp, vp, vp, vp, vp, C.c_int,
                                        C.POINTER(C.c_int64), vp]),
        "lrqk_decode_step": (C.c_int, [vp, sp, i32, C.POINTER(Layer), vp, vp, vp, C.c_int,
                                       C.POINTER(_StepDebug), C.POINTER(C.c_int64), vp]),
        "lrqk_calib_copy": (C.c_int, [vp, vp, sz, vp]),
        "lrqk_plan_time_proxy_pass": (C.c_int, [vp, sp, C.POINTER(vp), C.c_int, vp, vp, C.c_int,
                                                C.POINTER(C.c_float), vp]),
        "lrqk_plan_profile": (C.c_int, [vp, C.c_int]),
        "lrqk_plan_profile_read": (C.c_int, [vp, C.POINTER(C.c_double), C.POINTER(C.c_int)]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)   # AttributeError if the library does not export it
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


EXPORTS = ["lrqk_version", "lrqk_status_string", "lrqk_last_hip_error", "lrqk_validate_shape",
           "lrqk_workspace_bytes", "lrqk_proxy_scores", "lrqk_select_topk", "lrqk_cache_init",
           "lrqk_cache_resolve", "lrqk_sparse_attend", "lrqk_plan_create", "lrqk_plan_destroy",
           "lrqk_fetch_misses", "lrqk_decode_step", "lrqk_plan_profile", "lrqk_plan_profile_read", "lrqk_calib_copy",
           "lrqk_plan_time_proxy_pass", "lrqk_factor_update", "lrqk_append_token",
           "lrqk_prefill_factorize", "lrqk_sparse_attend_noalloc", "lrqk_select_state_init"]


def _check(status: int, where: str):
    if status != 0:
        raise LrqkError(status, where)


def _dev(t: Optional[torch.Tensor], dtype=None):
    """Device pointer of a contiguous CUDA/HIP tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def _pinned(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if t.is_cuda or not t.is_pinned() or not t.is_contiguous():
        raise ValueError("expected a contiguous pinned host tensor")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def lrqk_version() -> int:
    return load_library().lrqk_version()


def lrqk_status_string(status: int) -> str:
    return load_library().lrqk_status_string(status).decode()


def lrqk_last_hip_error() -> int:
    return load_library().lrqk_last_hip_error()


def lrqk_validate_shape(shape: Shape) -> int:
    return load_library().lrqk_validate_shape(C.byref(shape))


def lrqk_workspace_bytes(shape: Shape, which: int) -> int:
    return load_library().lrqk_workspace_bytes(C.byref(shape), which)


def lrqk_proxy_scores(shape, A_K, q_hat, scores, stream=None):
    _check(load_library().lrqk_proxy_scores(C.byref(shape), _dev(A_K, torch.float32),
                                            _dev(q_hat, torch.float32),
                                            _dev(scores, torch.float32), _stream(stream)),
           "lrqk_proxy_scores")


def lrqk_select_topk(shape, scores, sel_idx, workspace, stream=None):
    _check(load_library().lrqk_select_topk(C.byref(shape), _dev(scores, torch.float32),
                                           _dev(sel_idx, torch.int32), _dev(workspace),
                                           workspace.numel() * workspace.element_size(),
                                           _stream(stream)), "lrqk_select_topk")


def lrqk_cache_init(shape, slot_of, token_of, last_used, stream=None):
    _check(load_library().lrqk_cache_init(C.byref(shape), _dev(slot_of, torch.int32),
                                          _dev(token_of, torch.int32),
                                          _dev(last_used, torch.int32), _stream(stream)),
           "lrqk_cache_init")


def lrqk_select_state_init(shape, sel_thr, stream=None):
    _check(load_library().lrqk_select_state_init(C.byref(shape), _dev(sel_thr, torch.float32),
                                                 _stream(stream)), "lrqk_select_state_init")


def lrqk_cache_resolve(shape, sel_idx, step, slot_of, token_of, last_used, sel_slot, hit,
                       miss_tok, miss_slot, n_miss, stream=None):
    _check(load_library().lrqk_cache_resolve(
        C.byref(shape), _dev(sel_idx, torch.int32), int(step), _dev(slot_of, torch.int32),
        _dev(token_of, torch.int32), _dev(last_used, torch.int32), _dev(sel_slot, torch.int32),
        _dev(hit, torch.uint8), _dev(miss_tok, torch.int32), _dev(miss_slot, torch.int32),
        _dev(n_miss, torch.int32), _stream(stream)), "lrqk_cache_resolve")


def lrqk_sparse_attend(shape, q, cacheK, cacheV, sel_slot, liteK, liteV, out, workspace,
                       stream=None):
    _check(load_library().lrqk_sparse_attend(
        C.byref(shape), _dev(q, torch.float32), _dev(cacheK), _dev(cacheV),
        _dev(sel_slot, torch.int32), _dev(liteK), _dev(liteV), _dev(out, torch.float32),
        _dev(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
        "lrqk_sparse_attend")


def lrqk_sparse_attend_noalloc(shape, q, cacheK, cacheV, sel_slot, liteK, liteV, out, stream=None):
    _check(load_library().lrqk_sparse_attend_noalloc(
        C.byref(shape), _dev(q, torch.float32), _dev(cacheK), _dev(cacheV),
        _dev(sel_slot, torch.int32), _dev(liteK), _dev(liteV), _dev(out, torch.float32),
        _stream(stream)), "lrqk_sparse_attend_noalloc")


def lrqk_factor_update(shape, layer, sel_idx_prev, sel_slot_prev, q, k_new, B_Q, B_K, lambda_d1,
                       lambda_d2, n_iter, q_hat, k_hat, workspace, stream=None):
    _check(load_library().lrqk_factor_update(
        C.byref(shape), C.byref(layer), _dev(sel_idx_prev, torch.int32),
        _dev(sel_slot_prev, torch.int32), _dev(q, torch.float32), _dev(k_new),
        _dev(B_Q, torch.float32), _dev(B_K, torch.float32), float(lambda_d1), float(lambda_d2),
        int(n_iter), _dev(q_hat, torch.float32), _dev(k_hat, torch.float32), _dev(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)), "lrqk_factor_update")


def lrqk_prefill_factorize(shape, Q, K, A_Q, A_K, B_Q, B_K, lambda_pQ, lambda_pK, n_iter,
                           workspace, stream=None):
    _check(load_library().lrqk_prefill_factorize(
        C.byref(shape), _dev(Q), _dev(K), _dev(A_Q, torch.float32), _dev(A_K, torch.float32),
        _dev(B_Q, torch.float32), _dev(B_K, torch.float32), float(lambda_pQ), float(lambda_pK),
        int(n_iter), _dev(workspace), workspace.numel() * workspace.element_size(),
        _stream(stream)), "lrqk_prefill_factorize")


def lrqk_append_token(shape, layer, k_hat, k_new, v_new, stream=None):
    _check(load_library().lrqk_append_token(C.byref(shape), C.byref(layer),
                                            _dev(k_hat, torch.float32), _dev(k_new), _dev(v_new),
                                            _stream(stream)), "lrqk_append_token")


def lrqk_calib_copy(dst, src, stream=None):
    """Plain device copy of known traffic (counter calibration)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() >= nbytes
    _check(load_library().lrqk_calib_copy(_dev(dst), _dev(src), nbytes, _stream(stream)),
           "lrqk_calib_copy")


class Plan:
    """Owner of an lrqk_plan handle (lrqk_plan_create / lrqk_plan_destroy)."""

    def __init__(self, max_shape: Shape):
        h = C.c_void_p()
        _check(load_library().lrqk_plan_create(C.byref(max_shape), C.byref(h)), "lrqk_plan_create")
        self.handle = h

    KERNELS = ("sample", "threshold", "proxy_scores", "select", "resolve", "fetch_scatter",
               "attend", "attend_missed_rows", "combine")

    def profile(self, n_steps: int):
        """lrqk_plan_profile: time the kernels of the next n_steps fused steps (0 = off)."""
        _check(load_library().lrqk_plan_profile(self.handle, int(n_steps)), "lrqk_plan_profile")

    def profile_read(self):
        """lrqk_plan_profile_read -> (dict kernel slot -> summed ms, number of steps)."""
        ms = (C.c_double * len(self.KERNELS))()
        n = C.c_int(0)
        _check(load_library().lrqk_plan_profile_read(self.handle, ms, C.byref(n)),
               "lrqk_plan_profile_read")
        return dict(zip(self.KERNELS, list(ms))), n.value

    def time_proxy_pass(self, shape, A_K_list, q_hat, n_launches, sel_thr=None,
                        stream=None) -> float:
        """lrqk_plan_time_proxy_pass: microseconds per launch of step a1's pass over A_K."""
        ptrs = (C.c_void_p * len(A_K_list))(*[_dev(a, torch.float32) for a in A_K_list])
        us = C.c_float(0.0)
        _check(load_library().lrqk_plan_time_proxy_pass(
            self.handle, C.byref(shape), ptrs, len(A_K_list), _dev(q_hat, torch.float32),
            _dev(sel_thr, torch.float32), int(n_launches), C.byref(us), _stream(stream)),
            "lrqk_plan_time_proxy_pass")
        return us.value

    def close(self):
        if getattr(self, "handle", None):
            load_library().lrqk_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def lrqk_fetch_misses(plan: Plan, shape, K_host, V_host, miss_tok, miss_slot, n_miss, cacheK,
                      cacheV, mode=LRQK_FETCH_STAGED, stream=None) -> int:
    total = C.c_int64(0)
    _check(load_library().lrqk_fetch_misses(
        plan.handle, C.byref(shape), _pinned(K_host), _pinned(V_host),
        _dev(miss_tok, torch.int32), _dev(miss_slot, torch.int32), _dev(n_miss, torch.int32),
        _dev(cacheK), _dev(cacheV), int(mode), C.byref(total), _stream(stream)),
        "lrqk_fetch_misses")
    return total.value


def make_layer(*, A_K, K_host, V_host, liteK, liteV, slot_of, token_of, last_used, cacheK,
               cacheV, sel_thr=None) -> Layer:
    return Layer(_dev(A_K, torch.float32), _pinned(K_host), _pinned(V_host), _dev(liteK),
                 _dev(liteV), _dev(slot_of, torch.int32), _dev(token_of, torch.int32),
                 _dev(last_used, torch.int32), _dev(cacheK), _dev(cacheV),
                 _dev(sel_thr, torch.float32))


def lrqk_decode_step(plan: Plan, shape, step, layer: Layer, q_hat, q, out,
                     mode=LRQK_FETCH_STAGED, debug: Optional[dict] = None, stream=None) -> int:
    dbg = None
    if debug is not None:
        dbg = _StepDebug(*[_dev(debug.get(n)) for n in ("sel_idx", "sel_slot", "hit", "miss_tok",
                                                        "miss_slot", "n_miss", "link_rows")])
    total = C.c_int64(0)
    _check(load_library().lrqk_decode_step(
        plan.handle, C.byref(shape), int(step), C.byref(layer), _dev(q_hat, torch.float32),
        _dev(q, torch.float32), _dev(out, torch.float32), int(mode),
        C.byref(dbg) if dbg is not None else None, C.byref(total), _stream(stream)),
        "lrqk_decode_step")
    return total.value
