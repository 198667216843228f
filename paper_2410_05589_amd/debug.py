"""ctypes binding of the testing, tuning and measurement aids (include/ps_draft_debug.h):
same names as the C ABI, argument marshalling only."""
import ctypes

from . import binding as B

PS_PLAN_FIELDS = 12
PLAN_FIELD_NAMES = ("T", "Kt", "K", "rows", "kw_log", "s_log", "Gs", "per_round", "rounds", "piece_groups",
                    "npieces", "lds_bytes")
EXPORTED_SYMBOLS = ("ps_draft_debug_plan", "ps_draft_debug_attn_plan", "ps_draft_debug_spin_limit", "ps_draft_debug_timeline",
                    "ps_verify_debug_exchange", "ps_measure_stream_read", "ps_measure_copy")

_ready = False


def _lib():
    global _ready
    lib = B.load_library()
    if not _ready:
        lib.ps_draft_debug_plan.restype = ctypes.c_int
        lib.ps_draft_debug_plan.argtypes = [ctypes.POINTER(B.ps_draft_config)] + [ctypes.c_int] * 6 + [ctypes.POINTER(ctypes.c_int)]
        lib.ps_draft_debug_attn_plan.restype = ctypes.c_int
        lib.ps_draft_debug_attn_plan.argtypes = [ctypes.POINTER(B.ps_draft_config), ctypes.c_int, ctypes.POINTER(ctypes.c_int32),
                                                 ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        lib.ps_draft_debug_spin_limit.restype = ctypes.c_int
        lib.ps_draft_debug_spin_limit.argtypes = [ctypes.c_void_p, ctypes.c_int]
        lib.ps_draft_debug_timeline.restype = ctypes.c_int
        lib.ps_draft_debug_timeline.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        lib.ps_verify_debug_exchange.restype = None
        lib.ps_verify_debug_exchange.argtypes = [ctypes.c_int, ctypes.c_int]
        lib.ps_measure_stream_read.restype = ctypes.c_int
        lib.ps_measure_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        lib.ps_measure_copy.restype = ctypes.c_int
        lib.ps_measure_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        _ready = True
    return lib


def ps_draft_debug_plan(config, batch, n_new, k, all_rows, n_cu, lds_limit):
    """Returns (status, [per phase: dict of the plan fields])."""
    out = (ctypes.c_int * (5 * PS_PLAN_FIELDS))()
    st = _lib().ps_draft_debug_plan(ctypes.byref(config), batch, n_new, k, all_rows, n_cu, lds_limit, out)
    plans = [dict(zip(PLAN_FIELD_NAMES, out[ph * PS_PLAN_FIELDS:(ph + 1) * PS_PLAN_FIELDS])) for ph in range(5)]
    return st, plans


def ps_draft_debug_attn_plan(config, kv_len, n_new, k, n_cu):
    """Returns (status, {"nk", "units", "blocks", "merge_items"})."""
    ln = (ctypes.c_int32 * len(kv_len))(*[int(v) for v in kv_len])
    out = (ctypes.c_int * 4)()
    st = _lib().ps_draft_debug_attn_plan(ctypes.byref(config), len(kv_len), ln, n_new, k, n_cu, out)
    return st, dict(zip(("nk", "units", "blocks", "merge_items"), out[:4]))


def ps_draft_debug_spin_limit(ctx, spins):
    return _lib().ps_draft_debug_spin_limit(ctx, spins)


def ps_draft_debug_timeline(ctx, buf_ptr):
    return _lib().ps_draft_debug_timeline(ctx, buf_ptr)


def ps_verify_debug_exchange(spins, ghosts):
    _lib().ps_verify_debug_exchange(spins, ghosts)


def ps_measure_stream_read(src_ptr, nbytes, stream_ptr):
    return _lib().ps_measure_stream_read(src_ptr, nbytes, stream_ptr)


def ps_measure_copy(dst_ptr, src_ptr, nbytes, stream_ptr):
    return _lib().ps_measure_copy(dst_ptr, src_ptr, nbytes, stream_ptr)
