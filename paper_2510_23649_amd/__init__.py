"""LRQK decode-step hot path for AMD MI355X: thin Python binding over liblrqk.so.

Every function here has the name and the arguments of its C entry point
(include/lrqk.h) and does argument marshalling only: torch tensors supply the
device memory and the stream, all computation happens in the HIP library.
There is no fallback: if the library has not been built, importing the binding
functions raises.
"""
from .binding import (  # noqa: F401
    LRQK_FETCH_DIRECT, LRQK_FETCH_GROUP, LRQK_FETCH_STAGED, LRQK_SELECT_FRESH, lrqk_select_state_init, LRQK_KV_BF16, LRQK_KV_F32, LRQK_WS_ATTEND,
    LRQK_WS_SELECT, LRQK_WS_UPDATE, LRQK_WS_PREFILL, lrqk_factor_update, lrqk_append_token,
    lrqk_prefill_factorize, LrqkError, Layer, Plan, Shape, library_path, load_library,
    lrqk_cache_init, lrqk_cache_resolve, lrqk_calib_copy, lrqk_decode_step, lrqk_fetch_misses,
    lrqk_last_hip_error, lrqk_proxy_scores, lrqk_select_topk, lrqk_sparse_attend,
    lrqk_sparse_attend_noalloc,
    lrqk_status_string, lrqk_validate_shape, lrqk_version, lrqk_workspace_bytes, make_layer,
)
from .state import LayerBuffers  # noqa: F401
