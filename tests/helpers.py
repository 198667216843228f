"""Shared test scaffolding: tiny shapes and random stored tensors (no method arithmetic)."""
import numpy as np

from paper_2410_05589_amd.configs import DrafterShape, Workload
from paper_2410_05589_amd import inputs


def tiny_shape(dtype="f32", n_kv_heads=2, **kw):
    base = dict(hidden=64, n_heads=4, n_kv_heads=n_kv_heads, head_dim=16, ffn=96, vocab=50,
                dtype=dtype, rms_eps=1e-6, rope_base=10000.0, k_max=4)
    base.update(kw)
    return DrafterShape(**base)


def tiny_workload(shape, batch=1, kv_len=(7,), n_new=2, k=3, topk=3, seed=11):
    return Workload("tiny", shape, batch=batch, kv_len=tuple(kv_len), n_new=n_new, k=k, topk=topk, seed=seed)


def scaled_weights(shape, seed, scale=5.0):
    """Weights with matrices scaled up so that attention and the MLP are far from linear/uniform."""
    w = inputs.make_weights(shape, seed)
    if shape.dtype == "f32":
        for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "w_lm"):
            w[name] = (w[name] * np.float32(scale)).astype(np.float32)
    else:
        for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "w_lm"):
            w[name] = inputs.f32_to_bf16_bits(inputs.bf16_bits_to_f32(w[name]) * np.float32(scale))
    return w


def store(a, dtype):
    return inputs.f32_to_bf16_bits(a) if dtype == "bf16" else np.asarray(a, dtype=np.float32)
