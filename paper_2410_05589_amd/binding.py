"""ctypes binding of libps_draft.so: same names as the C ABI, argument marshalling only.

Every step of the draft path runs inside the HIP library; PyTorch is used for device
memory and streams.  There is no CPU fallback: if the library is missing, loading fails.
"""
import ctypes
import os

import numpy as np

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("PS_DRAFT_LIB") or os.path.join(_PKG_DIR, "libps_draft.so")

PS_F32, PS_BF16 = 0, 1
PS_OK = 0
PS_ERR_NULL, PS_ERR_CONFIG, PS_ERR_SHAPE, PS_ERR_KV_CAPACITY = -1, -2, -3, -4
PS_ERR_OFFSETS, PS_ERR_WORKSPACE, PS_ERR_UNSUPPORTED, PS_ERR_DEVICE, PS_ERR_TIMEOUT = -5, -6, -7, -8, -9
PS_FLAG_FINAL_NORM = 1
PS_FLAG_INPUT_FC = 2

EXPORTED_SYMBOLS = ("ps_draft_workspace_bytes", "ps_draft_init", "ps_draft_step", "ps_draft_free",
                    "ps_draft_strerror", "ps_draft_set_profile_events", "ps_draft_last_status")
PS_PROFILE_EVENTS = 8
PROFILE_KERNELS = ("qkv", "attention", "oproj", "gateup", "down", "lmhead", "lm_merge")


class ps_draft_config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("hidden", "n_heads", "n_kv_heads", "head_dim", "ffn", "vocab", "k_max", "max_batch",
                 "max_new", "max_positions", "max_topk", "dtype")] + \
               [("rms_eps", ctypes.c_float), ("rope_base", ctypes.c_float), ("flags", ctypes.c_uint32)]


WEIGHT_NAMES = ("g_in", "wq", "wk", "wv", "wo", "g_post", "w_gate", "w_up", "w_down", "g_final", "w_lm", "mask_emb")
INPUT_WEIGHT_NAMES = ("embed", "w_fc", "b_fc")       # optional: the input stage


class ps_draft_weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in WEIGHT_NAMES + INPUT_WEIGHT_NAMES]


class ps_draft_step_args(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_new", ctypes.c_int32), ("k", ctypes.c_int32),
                ("topk", ctypes.c_int32), ("out_rows", ctypes.c_int32),
                ("x", ctypes.c_void_p), ("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p),
                ("kv_offsets", ctypes.POINTER(ctypes.c_int64)), ("kv_len", ctypes.POINTER(ctypes.c_int32)),
                ("top_ids", ctypes.c_void_p), ("top_p", ctypes.c_void_p), ("lse", ctypes.c_void_p),
                ("logits", ctypes.c_void_p), ("probs", ctypes.c_void_p), ("hidden_out", ctypes.c_void_p),
                ("token_ids", ctypes.c_void_p), ("features", ctypes.c_void_p),
                ("temperature", ctypes.c_float), ("sample_seed", ctypes.c_uint64),
                ("sample_ids", ctypes.c_void_p), ("sample_p", ctypes.c_void_p), ("kv_len_dev", ctypes.c_void_p),
                ("n_new_seq", ctypes.POINTER(ctypes.c_int32))]


_lib = None


def load_library():
    """Loads the in-tree HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "HIP library %s is missing: build it with `python -m paper_2410_05589_amd.build` "
            "(there is no CPU fallback)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    lib.ps_draft_workspace_bytes.restype = ctypes.c_size_t
    lib.ps_draft_workspace_bytes.argtypes = [ctypes.POINTER(ps_draft_config)]
    lib.ps_draft_init.restype = ctypes.c_int
    lib.ps_draft_init.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ps_draft_config),
                                  ctypes.POINTER(ps_draft_weights), ctypes.c_void_p, ctypes.c_size_t,
                                  ctypes.c_void_p]
    lib.ps_draft_step.restype = ctypes.c_int
    lib.ps_draft_step.argtypes = [ctypes.c_void_p, ctypes.POINTER(ps_draft_step_args), ctypes.c_void_p]
    lib.ps_draft_free.restype = None
    lib.ps_draft_free.argtypes = [ctypes.c_void_p]
    lib.ps_draft_set_profile_events.restype = ctypes.c_int
    lib.ps_draft_set_profile_events.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)]
    lib.ps_draft_last_status.restype = ctypes.c_int
    lib.ps_draft_last_status.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    lib.ps_draft_strerror.restype = ctypes.c_char_p
    lib.ps_draft_strerror.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


class PsDraftError(RuntimeError):
    def __init__(self, status):
        self.status = status
        super().__init__("ps_draft: %s (%d)" % (ps_draft_strerror(status), status))


# ------------------------------------------------------------------ the C ABI, same names
def ps_draft_strerror(status):
    return load_library().ps_draft_strerror(int(status)).decode()


def ps_draft_workspace_bytes(config):
    return int(load_library().ps_draft_workspace_bytes(ctypes.byref(config)))


def ps_draft_init(config, weights, workspace_ptr, workspace_bytes, stream_ptr):
    """Returns (status, ctx handle)."""
    h = ctypes.c_void_p()
    st = load_library().ps_draft_init(ctypes.byref(h), ctypes.byref(config) if config is not None else None,
                                      ctypes.byref(weights) if weights is not None else None,
                                      workspace_ptr, workspace_bytes, stream_ptr)
    return st, h


def ps_draft_step(ctx, args, stream_ptr):
    return load_library().ps_draft_step(ctx, ctypes.byref(args) if args is not None else None, stream_ptr)


def ps_draft_last_status(ctx, stream_ptr):
    return load_library().ps_draft_last_status(ctx, stream_ptr)


def ps_draft_free(ctx):
    load_library().ps_draft_free(ctx)


def ps_draft_set_profile_events(ctx, event_handles):
    """event_handles: None, or PS_PROFILE_EVENTS integer hipEvent_t handles."""
    if event_handles is None:
        return load_library().ps_draft_set_profile_events(ctx, None)
    arr = (ctypes.c_void_p * PS_PROFILE_EVENTS)(*event_handles)
    return load_library().ps_draft_set_profile_events(ctx, arr)


# ------------------------------------------------------------------ marshalling helpers
def make_config(shape, max_batch, max_new, max_positions, max_topk, k_max=None, input_fc=False):
    c = ps_draft_config()
    c.hidden, c.n_heads, c.n_kv_heads, c.head_dim = shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim
    c.ffn, c.vocab = shape.ffn, shape.vocab
    c.k_max = shape.k_max if k_max is None else k_max
    c.max_batch, c.max_new, c.max_positions, c.max_topk = max_batch, max_new, max_positions, max_topk
    c.dtype = PS_BF16 if shape.dtype == "bf16" else PS_F32
    c.rms_eps, c.rope_base = shape.rms_eps, shape.rope_base
    c.flags = (PS_FLAG_FINAL_NORM if shape.final_norm else 0) | (PS_FLAG_INPUT_FC if input_fc else 0)
    return c


def to_device(a, dtype, device="cuda:0"):
    """Stored numpy tensor (float32, or uint16 bf16 bit patterns) -> torch device tensor."""
    import torch
    a = np.ascontiguousarray(a)
    if dtype == "bf16" and a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def from_device(t):
    """torch device tensor -> numpy (bf16 as uint16 bit patterns)."""
    import torch
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class Drafter:
    """Holds device tensors and a context; each method is one C-ABI call plus marshalling."""

    def __init__(self, shape, weights_np, max_batch=1, max_new=1, max_positions=4096, max_topk=8,
                 k_max=None, device="cuda:0", stream=None):
        import torch
        self.torch = torch
        self.shape, self.device = shape, device
        self.config = make_config(shape, max_batch, max_new, max_positions, max_topk, k_max=k_max,
                                  input_fc="w_fc" in weights_np)
        names = WEIGHT_NAMES + tuple(n for n in INPUT_WEIGHT_NAMES if n in weights_np)
        self.weights_dev = {n: to_device(weights_np[n], shape.dtype, device) for n in names}
        self.weights = ps_draft_weights()
        for n in names:
            setattr(self.weights, n, self.weights_dev[n].data_ptr())
        nbytes = ps_draft_workspace_bytes(self.config)
        if nbytes == 0:
            st, _ = ps_draft_init(self.config, self.weights, None, 0, None)
            raise PsDraftError(st)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
        ptr = (self.workspace.data_ptr() + 255) & ~255
        sp = self._stream_ptr(stream)
        st, self.ctx = ps_draft_init(self.config, self.weights, ptr, nbytes, sp)
        if st != PS_OK:
            raise PsDraftError(st)

    def _stream_ptr(self, stream):
        s = stream if stream is not None else self.torch.cuda.current_stream(self.device)
        return ctypes.c_void_p(s.cuda_stream)

    def alloc_outputs(self, batch, n_new, k, topk, all_rows=False, logits=False, probs=False, hidden=False, sample=False):
        t = self.torch
        rows = (n_new + k) if all_rows else (k + 1)
        o = {"top_ids": t.empty((batch, rows, topk), dtype=t.int32, device=self.device),
             "top_p": t.empty((batch, rows, topk), dtype=t.float32, device=self.device),
             "lse": t.empty((batch, rows), dtype=t.float32, device=self.device)}
        if logits:
            o["logits"] = t.empty((batch, rows, self.shape.vocab), dtype=t.float32, device=self.device)
        if probs:
            o["probs"] = t.empty((batch, rows, self.shape.vocab), dtype=t.float32, device=self.device)
        if sample:
            o["sample_ids"] = t.empty((batch, rows), dtype=t.int32, device=self.device)
            o["sample_p"] = t.empty((batch, rows), dtype=t.float32, device=self.device)
        if hidden:
            o["hidden_out"] = t.empty((batch, n_new + k, self.shape.hidden), dtype=t.float32, device=self.device)
        return o

    def make_args(self, x, k_cache, v_cache, kv_offsets, kv_len, n_new, k, topk, outputs, all_rows=False,
                  token_ids=None, features=None, temperature=0.0, sample_seed=0, kv_len_dev=None, n_new_seq=None):
        """Builds the argument struct; keeps the host arrays alive on the struct.  x: hidden states, or None
        when token_ids (and features) are given."""
        a = ps_draft_step_args()
        a.batch, a.n_new, a.k, a.topk, a.out_rows = len(kv_len), n_new, k, topk, 1 if all_rows else 0
        a.x = x.data_ptr() if x is not None else None
        a.k_cache, a.v_cache = k_cache.data_ptr(), v_cache.data_ptr()
        a.token_ids = token_ids.data_ptr() if token_ids is not None else None
        a.features = features.data_ptr() if features is not None else None
        a._keep_in = (token_ids, features, kv_len_dev)
        a.temperature, a.sample_seed = temperature, sample_seed
        a.kv_len_dev = kv_len_dev.data_ptr() if kv_len_dev is not None else None
        for n in ("sample_ids", "sample_p"):
            setattr(a, n, outputs[n].data_ptr() if n in outputs else None)
        off = np.ascontiguousarray(kv_offsets, dtype=np.int64)
        ln = np.ascontiguousarray(kv_len, dtype=np.int32)
        nn = None if n_new_seq is None else np.ascontiguousarray(n_new_seq, dtype=np.int32)
        a.n_new_seq = nn.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)) if nn is not None else None
        a._keep = (off, ln, nn, x, k_cache, v_cache, outputs)
        a.kv_offsets = off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
        a.kv_len = ln.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
        for n in ("top_ids", "top_p", "lse", "logits", "probs", "hidden_out"):
            setattr(a, n, outputs[n].data_ptr() if n in outputs else None)
        return a

    def step(self, args, stream=None):
        st = ps_draft_step(self.ctx, args, self._stream_ptr(stream))
        if st != PS_OK:
            raise PsDraftError(st)

    def last_status(self, stream=None):
        return ps_draft_last_status(self.ctx, self._stream_ptr(stream))

    def close(self):
        if getattr(self, "ctx", None):
            ps_draft_free(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
