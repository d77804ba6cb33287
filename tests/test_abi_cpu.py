"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching a device.  No GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2510_23649_amd as L
    from paper_2510_23649_amd import build as B
    if not B.is_built():
        B.build(verbose=False)
    return L


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "lrqk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lrqk_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    raw = C.CDLL(lib.library_path())
    names = declared_symbols()
    assert len(names) >= 14 and "lrqk_decode_step" in names and "lrqk_proxy_scores" in names
    for n in names:
        assert hasattr(raw, n), f"liblrqk.so does not export {n}"
    from paper_2510_23649_amd.binding import EXPORTS
    assert sorted(EXPORTS) == names


def test_version_and_status_strings(lib):
    assert lib.lrqk_version() == 200
    assert lib.lrqk_status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert lib.lrqk_status_string(code) not in ("ok", "unknown status")


def test_binding_constants_match_the_header(lib):
    text = open(os.path.join(ROOT, "include", "lrqk.h")).read()
    def const(name):
        m = re.search(r"\b%s\s*=\s*(-?\w+)" % name, text) or re.search(r"#define\s+%s\s+(\w+)" % name, text)
        return int(m.group(1), 0)
    from paper_2510_23649_amd import binding
    assert const("LRQK_PROFILE_SLOTS") == len(binding.Plan.KERNELS)
    for name in ("LRQK_FETCH_STAGED", "LRQK_FETCH_DIRECT", "LRQK_FETCH_GROUP", "LRQK_SELECT_FRESH",
                 "LRQK_KV_BF16", "LRQK_KV_F32", "LRQK_WS_SELECT", "LRQK_WS_ATTEND", "LRQK_WS_UPDATE",
                 "LRQK_WS_PREFILL"):
        assert const(name) == getattr(binding, name), name
    assert const("LRQK_VERSION") == lib.lrqk_version()
    # the structures the binding mirrors
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    n_layer = len(re.search(r"typedef struct lrqk_layer \{(.*?)\} lrqk_layer;", text, re.S).group(1).split(";")) - 1
    n_dbg = len(re.search(r"typedef struct lrqk_step_debug \{(.*?)\} lrqk_step_debug;", text, re.S).group(1).split(";")) - 1
    assert n_layer == len(binding.Layer._fields_) and n_dbg == len(binding._StepDebug._fields_)


def good(lib, **kw):
    base = dict(B=1, Hq=32, Hkv=8, l=4096, r=32, k=256, w=16, C_slots=4096)
    base.update(kw)
    return lib.Shape.make(**base)


def test_shape_validation(lib):
    assert lib.lrqk_validate_shape(good(lib)) == 0
    bad = [dict(Hq=30), dict(Hq=72, Hkv=8), dict(d=64), dict(r=30), dict(r=0), dict(r=132),
           dict(k=0), dict(k=4081), dict(k=5000, l=100000, C_slots=8000), dict(w=-1), dict(w=2000),
           dict(C_slots=255), dict(C_slots=10000), dict(l=1 << 24), dict(B=0),
           dict(scale=float("nan"))]
    for kw in bad:
        assert lib.lrqk_validate_shape(good(lib, **kw)) == -2, kw
    assert lib.lrqk_validate_shape(good(lib, kv_dtype=3)) == -1
    assert lib.lrqk_workspace_bytes(good(lib, r=30), lib.LRQK_WS_SELECT) == 0
    assert lib.lrqk_workspace_bytes(good(lib), lib.LRQK_WS_SELECT) > 0
    assert lib.lrqk_workspace_bytes(good(lib), lib.LRQK_WS_ATTEND) > 0
    assert lib.lrqk_workspace_bytes(good(lib), 99) == 0


def test_entry_points_reject_bad_arguments_before_any_device_work(lib):
    raw = lib.load_library()
    s = good(lib)
    A = 0x10000  # a well-aligned fake address: never dereferenced on these paths
    # null and misaligned pointers
    assert raw.lrqk_proxy_scores(C.byref(s), None, A, A, None) == -1
    assert raw.lrqk_proxy_scores(C.byref(s), A + 4, A, A, None) == -1
    assert raw.lrqk_select_topk(C.byref(s), A, A, A + 16, 1 << 30, None) == -1   # workspace not 256-aligned
    assert raw.lrqk_cache_resolve(C.byref(s), A, -1, A, A, A, A, A, A, A, A, None) == -1  # step < 0
    assert raw.lrqk_sparse_attend(C.byref(s), A, A, A, A, None, A, A, A, 1 << 30, None) == -1  # liteK null, w > 0
    # workspace too small
    assert raw.lrqk_select_topk(C.byref(s), A, A, A, 16, None) == -4
    assert raw.lrqk_sparse_attend(C.byref(s), A, A, A, A, A, A, A, A, 16, None) == -4
    # the entry point without a workspace: null pointer, then partial states beyond its fixed array
    assert raw.lrqk_sparse_attend_noalloc(C.byref(s), None, A, A, A, A, A, A, None) == -1
    big = lib.Shape.make(B=2048, Hq=8, Hkv=8, l=8192, r=4, k=4096, w=0, C_slots=4096)
    assert raw.lrqk_sparse_attend_noalloc(C.byref(big), A, A, A, A, A, A, A, None) == -4
    # bad shape wins over everything else
    b = good(lib, r=30)
    assert raw.lrqk_proxy_scores(C.byref(b), A, A, A, None) == -2
    assert raw.lrqk_decode_step(None, C.byref(b), 0, None, A, A, A, 0, None, None, None) == -2
    # null plan / layer, bad mode
    lay = lib.Layer(*([A] * 10))
    assert raw.lrqk_decode_step(None, C.byref(s), 0, C.byref(lay), A, A, A, 0, None, None, None) == -1
    assert raw.lrqk_decode_step(None, C.byref(s), 0, None, A, A, A, 0, None, None, None) == -1
    assert raw.lrqk_decode_step(None, C.byref(s), 0, C.byref(lay), A, A, A, 7, None, None, None) == -1
    assert raw.lrqk_fetch_misses(None, C.byref(s), A, A, A, A, A, A, A, 0, None, None) == -1
    assert raw.lrqk_fetch_misses(None, C.byref(s), A, A, A, A, A, A, A, 3, None, None) == -1   # mode
    assert raw.lrqk_select_state_init(C.byref(s), None, None) == -1
    assert raw.lrqk_select_state_init(C.byref(s), A + 4, None) == -1
    assert raw.lrqk_select_state_init(C.byref(b), A, None) == -2
    lay_bad = lib.Layer(*([A] * 10 + [A + 4]))                      # misaligned sel_thr
    assert raw.lrqk_decode_step(None, C.byref(s), 0, C.byref(lay_bad), A, A, A,
                                lib.LRQK_FETCH_DIRECT | lib.LRQK_SELECT_FRESH, None, None, None) == -1
    assert raw.lrqk_plan_destroy(None) == -1
    assert raw.lrqk_plan_create(C.byref(b), C.byref(C.c_void_p())) == -2


def test_update_append_prefill_reject_bad_arguments_before_any_device_work(lib):
    raw = lib.load_library()
    A = 0x10000
    s = good(lib)
    lay = lib.Layer(*([A] * 10))
    f32 = C.c_float
    upd = raw.lrqk_factor_update
    ok_tail = (f32(1.0), f32(1.0), 2, A, A, A, 1 << 30, None)
    assert upd(C.byref(good(lib, r=12)), C.byref(lay), A, A, A, A, A, A, *ok_tail) == -2   # rank
    assert upd(C.byref(s), None, A, A, A, A, A, A, *ok_tail) == -1                         # layer
    assert upd(C.byref(s), C.byref(lay), A, A, A, A, A, A, f32(1.0), f32(1.0), 0, A, A, A,
               1 << 30, None) == -1                                                        # rounds
    assert upd(C.byref(s), C.byref(lay), A, A, A, A, A, A, f32(-1.0), f32(1.0), 2, A, A, A,
               1 << 30, None) == -1                                                        # lambda
    assert upd(C.byref(s), C.byref(lay), A, A, A, A + 4, A, A, *ok_tail) == -1             # alignment
    assert upd(C.byref(s), C.byref(lay), A, A, A, A, A, A, f32(1.0), f32(1.0), 2, A, A, A, 64,
               None) == -4                                                                 # workspace
    assert lib.lrqk_workspace_bytes(s, lib.LRQK_WS_UPDATE) > 0
    assert lib.lrqk_workspace_bytes(good(lib, r=12), lib.LRQK_WS_UPDATE) == 0
    # append needs room for row l
    app = raw.lrqk_append_token
    assert app(C.byref(s), C.byref(lay), A, A, A, None) == -2                  # l_cap == l
    assert app(C.byref(good(lib, l_cap=4000)), C.byref(lay), A, A, A, None) == -2   # l_cap < l
    roomy = good(lib, l_cap=4100)
    assert lib.lrqk_validate_shape(roomy) == 0
    assert app(C.byref(roomy), None, A, A, A, None) == -1
    assert app(C.byref(roomy), C.byref(lay), None, A, A, None) == -1
    # prefill
    pf = raw.lrqk_prefill_factorize
    assert pf(C.byref(good(lib, r=24)), A, A, A, A, A, A, f32(1.0), f32(1.0), 2, A, 1 << 30, None) == -2
    assert pf(C.byref(s), A, None, A, A, A, A, f32(1.0), f32(1.0), 2, A, 1 << 30, None) == -1
    assert pf(C.byref(s), A, A, A, A, A, A, f32(1.0), f32(float("inf")), 2, A, 1 << 30, None) == -1
    assert pf(C.byref(s), A, A, A, A, A, A, f32(1.0), f32(1.0), 65, A, 1 << 30, None) == -1
    assert pf(C.byref(s), A, A, A, A, A, A, f32(1.0), f32(1.0), 2, A, 64, None) == -4
    assert lib.lrqk_workspace_bytes(s, lib.LRQK_WS_PREFILL) > 0


def test_product_never_touches_the_oracle():
    """The package, the header and the kernels must not import, include or name oracle/."""
    pkg = os.path.join(ROOT, "paper_2510_23649_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
    for dirpath, _, files in os.walk(os.path.join(ROOT, "oracle")):
        for f in files:
            if f.endswith((".py", ".c", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "paper_2510_23649_amd" not in text and "lrqk.h" not in text
