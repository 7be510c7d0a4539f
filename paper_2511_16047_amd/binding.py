"""ctypes binding of libamskv.so: the same calls as include/amskv.h, argument marshalling only.

Device buffers are torch tensors (PyTorch is used for device memory and streams, nothing
else); every step of the path runs in the library's HIP kernels.  There is no fallback: if
the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
# AMSKV_LIBRARY points at another build of the same library (e.g. a tuning variant)
LIB_PATH = os.environ.get("AMSKV_LIBRARY") or os.path.join(HERE, "libamskv.so")

AMSKV_OK = 0
AMSKV_ERR_INVALID_ARG = -1
AMSKV_ERR_ORDER = -2
AMSKV_ERR_EVICTED = -3
AMSKV_ERR_ARENA_TOO_SMALL = -4
AMSKV_ERR_HIP = -5
AMSKV_ERR_NO_DEVICE_MEMORY = -6
AMSKV_ERR_STATIC_LIMIT = -7
AMSKV_ERR_NO_HOST_MEMORY = -8
AMSKV_STATIC_MAX_UNITS = 16384
AMSKV_DTYPE_F32, AMSKV_DTYPE_BF16 = 0, 1
AMSKV_LAYOUT_COMPACT, AMSKV_LAYOUT_PLANNED = 0, 1
AMSKV_MODE_SCALE_WINDOW, AMSKV_MODE_TOKEN_BUDGET, AMSKV_MODE_TOKEN_WINDOW = 0, 1, 2
AMSKV_IO_HEAD_MAJOR, AMSKV_IO_TOKEN_MAJOR = 0, 1
AMSKV_MAX_SCALES = 16
_MAX_SEGMENTS = AMSKV_MAX_SCALES + 2

EXPORTED = [
    "amskv_cache_required_bytes", "amskv_cache_create", "amskv_append_scale", "amskv_attend",
    "amskv_interscale_similarity", "amskv_cache_layout", "amskv_cache_last_evicted",
    "amskv_cache_bytes_held", "amskv_cache_capacity_tokens", "amskv_cache_export",
    "amskv_cache_reset", "amskv_cache_destroy", "amskv_status_string",
    "amskv_cache_segments", "amskv_cache_budget_tokens", "amskv_cache_settle", "amskv_attention_density",
    "amskv_attention_density_enqueue", "amskv_attend_density",
    "amskv_cache_set_io_layout", "amskv_interscale_similarity_enqueue", "amskv_interscale_similarity_collect",
    "amskv_interscale_similarity_enqueue_static",
]


class AmskvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, status_string(status), status))


class _Schedule(C.Structure):
    _fields_ = [("n_scales", C.c_int32), ("side_h", C.POINTER(C.c_int32)), ("side_w", C.POINTER(C.c_int32)),
                ("batch", C.c_int32), ("dtype", C.c_int32)]


class _LayerPolicy(C.Structure):
    _fields_ = [("n_condensed", C.c_int32), ("window", C.c_int32), ("keep_all", C.c_int32)]


class _LayerBudget(C.Structure):
    _fields_ = [("c_min", C.c_int32), ("c_max", C.c_int32), ("c_cds", C.c_int32), ("theta", C.c_float)]


class _Policy(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("layer", C.POINTER(_LayerPolicy)), ("softmax_scale", C.c_float),
                ("layout", C.c_int32), ("borrow_unretained", C.c_int32), ("fuse_append", C.c_int32),
                ("mode", C.c_int32), ("budget", C.POINTER(_LayerBudget))]


_lib = None


def load_library() -> C.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libamskv.so is not built (%s); run `python -m paper_2511_16047_amd.build`" % LIB_PATH)
    # PyTorch owns the device memory and the streams handed to the library, so both must talk
    # to the same HIP runtime instance: torch bundles its own libamdhip64 and must load first,
    # then the library's dependency on that soname resolves to the copy already in the process.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
    ps, pp = C.POINTER(_Schedule), C.POINTER(_Policy)
    lib.amskv_cache_required_bytes.argtypes = [i32, i32, i32, ps, pp, C.POINTER(u64)]
    lib.amskv_cache_required_bytes.restype = i32
    lib.amskv_cache_create.argtypes = [i32, i32, i32, ps, pp, vp, u64, C.POINTER(vp)]
    lib.amskv_cache_create.restype = i32
    lib.amskv_append_scale.argtypes = [vp, i32, i32, vp, vp, vp]
    lib.amskv_append_scale.restype = i32
    lib.amskv_attend.argtypes = [vp, i32, i32, vp, vp, vp]
    lib.amskv_attend.restype = i32
    pf = C.POINTER(C.c_float)
    lib.amskv_interscale_similarity.argtypes = [vp, i32, i32, pf, pf, pf, vp]
    lib.amskv_interscale_similarity.restype = i32
    lib.amskv_cache_layout.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i64), C.POINTER(i32)]
    lib.amskv_cache_layout.restype = i32
    lib.amskv_cache_last_evicted.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32)]
    lib.amskv_cache_last_evicted.restype = i32
    lib.amskv_cache_bytes_held.argtypes = [vp, i32, i32]
    lib.amskv_cache_bytes_held.restype = i64
    lib.amskv_cache_capacity_tokens.argtypes = [vp, i32]
    lib.amskv_cache_capacity_tokens.restype = i64
    lib.amskv_cache_export.argtypes = [vp, i32, vp, vp, vp]
    lib.amskv_cache_export.restype = i32
    lib.amskv_cache_reset.argtypes = [vp]
    lib.amskv_cache_reset.restype = i32
    lib.amskv_cache_destroy.argtypes = [vp]
    lib.amskv_cache_destroy.restype = None
    lib.amskv_status_string.argtypes = [i32]
    lib.amskv_status_string.restype = C.c_char_p
    lib.amskv_cache_segments.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32), C.POINTER(i64),
                                         C.POINTER(i32)]
    lib.amskv_cache_segments.restype = i32
    lib.amskv_cache_budget_tokens.argtypes = [vp, i32]
    lib.amskv_cache_budget_tokens.restype = i64
    lib.amskv_cache_settle.argtypes = [vp, i32, vp]
    lib.amskv_cache_settle.restype = i32
    lib.amskv_attention_density.argtypes = [vp, i32, i32, vp, pf, pf, C.POINTER(i32), vp]
    lib.amskv_attention_density.restype = i32
    lib.amskv_attention_density_enqueue.argtypes = [vp, i32, i32, vp, vp, C.POINTER(i32), C.POINTER(i32), vp]
    lib.amskv_attention_density_enqueue.restype = i32
    lib.amskv_attend_density.argtypes = [vp, i32, i32, vp, vp, vp, C.POINTER(i32), C.POINTER(i32), vp]
    lib.amskv_attend_density.restype = i32
    lib.amskv_cache_set_io_layout.argtypes = [vp, i32, i64, i64, i64]
    lib.amskv_cache_set_io_layout.restype = i32
    lib.amskv_interscale_similarity_enqueue.argtypes = [vp, i32, i32, i32, vp]
    lib.amskv_interscale_similarity_enqueue.restype = i32
    lib.amskv_interscale_similarity_collect.argtypes = [vp, pf, pf, pf, vp]
    lib.amskv_interscale_similarity_collect.restype = i32
    lib.amskv_interscale_similarity_enqueue_static.argtypes = [vp, i32, i32, i32, vp, vp]
    lib.amskv_interscale_similarity_enqueue_static.restype = i32
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().amskv_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != AMSKV_OK:
        raise AmskvError(int(status), where)


def _structs(sides_h, sides_w, batch, dtype, policies, softmax_scale, layout, borrow_unretained=False, fuse_append=False,
             budgets=None, windows=None):
    """policies: [(n_condensed, window, keep_all)] per layer (scale-window mode), or None with
    budgets: [(c_min, c_max, c_cds, theta)] per layer (token-budget mode), or None with
    windows: [(window_tokens, n_sink)] per layer (token-window mode)."""
    mode = AMSKV_MODE_SCALE_WINDOW
    if budgets is not None:
        mode = AMSKV_MODE_TOKEN_BUDGET
    if windows is not None:
        mode = AMSKV_MODE_TOKEN_WINDOW
        budgets = [(int(w), int(w), int(k), 0.0) for w, k in windows]
    n = len(sides_h)
    ah = (C.c_int32 * n)(*[int(x) for x in sides_h])
    aw = (C.c_int32 * n)(*[int(x) for x in sides_w])
    sc = _Schedule(n, ah, aw, int(batch), int(dtype))
    lp = bp = None
    if policies is not None:
        lp = (_LayerPolicy * len(policies))(*[_LayerPolicy(int(c), int(w), int(bool(k))) for c, w, k in policies])
    if budgets is not None:
        bp = (_LayerBudget * len(budgets))(*[_LayerBudget(int(a), int(b), int(c), float(t)) for a, b, c, t in budgets])
    n_layers = len(budgets) if budgets is not None else len(policies)
    po = _Policy(n_layers, lp, float(softmax_scale), int(layout), int(bool(borrow_unretained)), int(bool(fuse_append)),
                 mode, bp)
    return sc, po, (ah, aw, lp, bp)


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor (or a raw address passed through)."""
    if t is None or isinstance(t, int):
        return t
    return int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if isinstance(stream, int):
        return stream or None
    if stream is None:
        import torch
        if torch.cuda.is_available():
            return int(torch.cuda.current_stream().cuda_stream) or None
        return None
    return int(getattr(stream, "cuda_stream", stream)) or None


# ------------------------------------------------------------------ the calls of amskv.h
def amskv_cache_required_bytes(layers, heads, head_dim, sides_h, sides_w, batch, dtype, policies,
                               softmax_scale=0.0, layout=AMSKV_LAYOUT_COMPACT, borrow_unretained=False, fuse_append=False,
                               budgets=None, windows=None) -> int:
    sc, po, _keep = _structs(sides_h, sides_w, batch, dtype, policies, softmax_scale, layout, borrow_unretained, fuse_append,
                             budgets, windows)
    out = C.c_uint64(0)
    _check(load_library().amskv_cache_required_bytes(layers, heads, head_dim, C.byref(sc), C.byref(po),
                                                     C.byref(out)), "amskv_cache_required_bytes")
    return int(out.value)


def amskv_cache_create(layers, heads, head_dim, sides_h, sides_w, batch, dtype, policies,
                       softmax_scale=0.0, layout=AMSKV_LAYOUT_COMPACT, arena=None, arena_bytes=None,
                       borrow_unretained=False, fuse_append=False, budgets=None, windows=None):
    """arena: torch uint8 device tensor (kept alive by the caller) or None for a plan-only cache.
    budgets (with policies=None) selects the token-budget mode, windows (with policies=None) the token-window mode.
    Returns the opaque handle (an int)."""
    sc, po, _keep = _structs(sides_h, sides_w, batch, dtype, policies, softmax_scale, layout, borrow_unretained, fuse_append,
                             budgets, windows)
    h = C.c_void_p(None)
    nbytes = 0 if arena is None else (int(arena.numel() * arena.element_size()) if arena_bytes is None else int(arena_bytes))
    _check(load_library().amskv_cache_create(layers, heads, head_dim, C.byref(sc), C.byref(po), _ptr(arena),
                                             nbytes, C.byref(h)), "amskv_cache_create")
    return h.value


def amskv_append_scale(cache, layer, s, K=None, V=None, stream=None):
    _check(load_library().amskv_append_scale(cache, layer, s, _ptr(K), _ptr(V), _stream(stream)),
           "amskv_append_scale")


def amskv_attend(cache, layer, s, Q, O, stream=None):
    _check(load_library().amskv_attend(cache, layer, s, _ptr(Q), _ptr(O), _stream(stream)), "amskv_attend")


def amskv_interscale_similarity(cache, layer, s, heads, want_v=True, want_sums=True, stream=None):
    """Returns (cosK[H], cosV[H] or None, sums[H][3] or None) as Python lists of floats."""
    ck = (C.c_float * heads)()
    cv = (C.c_float * heads)() if want_v else None
    sm = (C.c_float * (3 * heads))() if want_sums else None
    _check(load_library().amskv_interscale_similarity(cache, layer, s, ck, cv, sm, _stream(stream)),
           "amskv_interscale_similarity")
    return (list(ck), list(cv) if want_v else None,
            [[sm[3 * h + i] for i in range(3)] for h in range(heads)] if want_sums else None)


def amskv_attention_density(cache, layer, s, Q, heads, stream=None):
    """Returns (density[H][n_seg], mass[H][n_seg]) as nested Python lists of floats."""
    d = (C.c_float * (heads * AMSKV_MAX_SCALES))()
    m = (C.c_float * (heads * AMSKV_MAX_SCALES))()
    n = C.c_int32(0)
    _check(load_library().amskv_attention_density(cache, layer, s, _ptr(Q), d, m, C.byref(n), _stream(stream)),
           "amskv_attention_density")
    rows = lambda a: [[a[h * AMSKV_MAX_SCALES + i] for i in range(n.value)] for h in range(heads)]
    return rows(d), rows(m)


def amskv_attention_density_enqueue(cache, layer, s, Q, mass_out, stream=None):
    """mass_out: device float32 tensor of heads * AMSKV_MAX_SCALES elements, filled in stream order.
    Returns the key-token count of every group (density = mass / count)."""
    n = C.c_int32(0)
    ln = (C.c_int32 * _MAX_SEGMENTS)()
    _check(load_library().amskv_attention_density_enqueue(cache, layer, s, _ptr(Q), _ptr(mass_out), C.byref(n), ln,
                                                          _stream(stream)), "amskv_attention_density_enqueue")
    return [int(ln[i]) for i in range(n.value)]


def amskv_attend_density(cache, layer, s, Q, O, mass_out, stream=None):
    """amskv_attend plus the step's attention density: mass_out as for amskv_attention_density_enqueue.
    Returns the key-token count of every group."""
    n = C.c_int32(0)
    ln = (C.c_int32 * _MAX_SEGMENTS)()
    _check(load_library().amskv_attend_density(cache, layer, s, _ptr(Q), _ptr(O), _ptr(mass_out), C.byref(n), ln,
                                               _stream(stream)), "amskv_attend_density")
    return [int(ln[i]) for i in range(n.value)]


def amskv_interscale_similarity_enqueue(cache, layer, s, want_v=True, stream=None):
    _check(load_library().amskv_interscale_similarity_enqueue(cache, layer, s, int(bool(want_v)), _stream(stream)),
           "amskv_interscale_similarity_enqueue")


def amskv_interscale_similarity_enqueue_static(cache, layer, s, want_v, sums_out, stream=None):
    """sums_out: device tensor or address of (2 if want_v else 1) * heads * 4 floats."""
    _check(load_library().amskv_interscale_similarity_enqueue_static(cache, layer, s, int(bool(want_v)), _ptr(sums_out),
                                                                      _stream(stream)),
           "amskv_interscale_similarity_enqueue_static")


def amskv_interscale_similarity_collect(cache, layers, heads, want_v=True, want_sums=True, stream=None):
    """Returns (cosK[L][H], cosV[L][H] or None, sums[L][H][3] or None) as nested Python lists."""
    ck = (C.c_float * (layers * heads))()
    cv = (C.c_float * (layers * heads))() if want_v else None
    sm = (C.c_float * (3 * layers * heads))() if want_sums else None
    _check(load_library().amskv_interscale_similarity_collect(cache, ck, cv, sm, _stream(stream)),
           "amskv_interscale_similarity_collect")
    rows = lambda a: [[a[l * heads + h] for h in range(heads)] for l in range(layers)]
    return (rows(ck), rows(cv) if want_v else None,
            [[[sm[(l * heads + h) * 3 + i] for i in range(3)] for h in range(heads)] for l in range(layers)] if want_sums else None)


def amskv_cache_layout(cache, layer) -> List[Tuple[int, int, int]]:
    """[(scale_id, tok_offset, tok_len)] ascending scale id."""
    n = C.c_int32(0)
    sid = (C.c_int32 * _MAX_SEGMENTS)()
    off = (C.c_int64 * _MAX_SEGMENTS)()
    ln = (C.c_int32 * _MAX_SEGMENTS)()
    _check(load_library().amskv_cache_layout(cache, layer, C.byref(n), sid, off, ln), "amskv_cache_layout")
    return [(int(sid[i]), int(off[i]), int(ln[i])) for i in range(n.value)]


def amskv_cache_segments(cache, layer) -> List[Tuple[int, int, int, int]]:
    """[(scale_id, first_token, tok_offset, tok_len)] oldest token first."""
    n = C.c_int32(0)
    sid = (C.c_int32 * _MAX_SEGMENTS)()
    first = (C.c_int32 * _MAX_SEGMENTS)()
    off = (C.c_int64 * _MAX_SEGMENTS)()
    ln = (C.c_int32 * _MAX_SEGMENTS)()
    _check(load_library().amskv_cache_segments(cache, layer, C.byref(n), sid, first, off, ln), "amskv_cache_segments")
    return [(int(sid[i]), int(first[i]), int(off[i]), int(ln[i])) for i in range(n.value)]


def amskv_cache_budget_tokens(cache, layer) -> int:
    v = int(load_library().amskv_cache_budget_tokens(cache, layer))
    if v < 0:
        raise AmskvError(v, "amskv_cache_budget_tokens")
    return v


def amskv_cache_settle(cache, layer, stream=None):
    _check(load_library().amskv_cache_settle(cache, layer, _stream(stream)), "amskv_cache_settle")


def amskv_cache_last_evicted(cache, layer) -> List[int]:
    n = C.c_int32(0)
    sid = (C.c_int32 * AMSKV_MAX_SCALES)()
    _check(load_library().amskv_cache_last_evicted(cache, layer, C.byref(n), sid), "amskv_cache_last_evicted")
    return [int(sid[i]) for i in range(n.value)]


def amskv_cache_bytes_held(cache, layer, include_current=True) -> int:
    v = int(load_library().amskv_cache_bytes_held(cache, layer, int(bool(include_current))))
    if v < 0:
        raise AmskvError(v, "amskv_cache_bytes_held")
    return v


def amskv_cache_capacity_tokens(cache, layer) -> int:
    v = int(load_library().amskv_cache_capacity_tokens(cache, layer))
    if v < 0:
        raise AmskvError(v, "amskv_cache_capacity_tokens")
    return v


def amskv_cache_export(cache, layer, K_out=None, V_out=None, stream=None):
    _check(load_library().amskv_cache_export(cache, layer, _ptr(K_out), _ptr(V_out), _stream(stream)),
           "amskv_cache_export")


def amskv_cache_set_io_layout(cache, io_layout, q_token_stride=0, kv_token_stride=0, o_token_stride=0):
    _check(load_library().amskv_cache_set_io_layout(cache, int(io_layout), int(q_token_stride), int(kv_token_stride),
                                                    int(o_token_stride)), "amskv_cache_set_io_layout")


def amskv_cache_reset(cache):
    _check(load_library().amskv_cache_reset(cache), "amskv_cache_reset")


def amskv_cache_destroy(cache):
    load_library().amskv_cache_destroy(cache)
