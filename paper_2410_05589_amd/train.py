"""ctypes binding of the group-wise training attention (include/ps_train.h): same names as the C ABI,
argument marshalling only; the work runs in the HIP library."""
import ctypes

from . import binding as B

EXPORTED_SYMBOLS = ("ps_group_attention_workspace_bytes", "ps_group_attention")


class ps_group_attn_args(ctypes.Structure):
    _fields_ = [("seqs", ctypes.c_int32), ("tokens", ctypes.c_int32), ("k", ctypes.c_int32),
                ("n_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("rope_base", ctypes.c_float),
                ("q", ctypes.c_void_p), ("k_", ctypes.c_void_p), ("v", ctypes.c_void_p), ("out", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


_ready = False


def _lib():
    global _ready
    lib = B.load_library()
    if not _ready:
        lib.ps_group_attention_workspace_bytes.restype = ctypes.c_size_t
        lib.ps_group_attention_workspace_bytes.argtypes = [ctypes.POINTER(ps_group_attn_args)]
        lib.ps_group_attention.restype = ctypes.c_int
        lib.ps_group_attention.argtypes = [ctypes.POINTER(ps_group_attn_args), ctypes.c_void_p]
        _ready = True
    return lib


def make_args(seqs, tokens, k, n_heads, n_kv_heads, head_dim, dtype, rope_base):
    a = ps_group_attn_args()
    a.seqs, a.tokens, a.k = seqs, tokens, k
    a.n_heads, a.n_kv_heads, a.head_dim = n_heads, n_kv_heads, head_dim
    a.dtype = B.PS_BF16 if dtype == "bf16" else B.PS_F32
    a.rope_base = rope_base
    return a


def ps_group_attention_workspace_bytes(args):
    return int(_lib().ps_group_attention_workspace_bytes(ctypes.byref(args) if args is not None else None))


def ps_group_attention(args, stream_ptr):
    return _lib().ps_group_attention(ctypes.byref(args) if args is not None else None, stream_ptr)
