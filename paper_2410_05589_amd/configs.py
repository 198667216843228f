"""Named drafter shapes and workloads for the parallel draft step.

Only shapes, sizes and seeds live here (no arithmetic of the method): the five
workloads are the ones the benchmark definition lists; the drafter is one
Llama-style decoder layer shaped like a layer of its target model
(Section 5.1 "Models": 202M parameters for 7B targets, 317M for 13B), run on
n_new newly accepted positions plus k appended [MASK] positions
(Section 4.1 "Inference").
"""
from dataclasses import dataclass, field, replace
from typing import Tuple


@dataclass(frozen=True)
class DrafterShape:
    hidden: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    dtype: str            # "f32" | "bf16": weights, KV cache and input hidden states
    rms_eps: float
    rope_base: float
    k_max: int            # number of distinct [MASK] embedding rows
    final_norm: bool = True

    @property
    def q_dim(self):
        return self.n_heads * self.head_dim

    @property
    def kv_dim(self):
        return self.n_kv_heads * self.head_dim

    def layer_params(self):
        """Matrix parameters of the decoder layer (no gains, no LM head)."""
        return (self.hidden * self.q_dim * 2 + 2 * self.hidden * self.kv_dim
                + 3 * self.hidden * self.ffn)


@dataclass(frozen=True)
class Workload:
    name: str
    shape: DrafterShape
    batch: int
    kv_len: Tuple[int, ...]      # valid cache positions per sequence before the step
    n_new: int
    k: int
    topk: int
    seed: int
    n_new_mix: Tuple[int, ...] = ()   # accepted-length mix for multi-step runs (c2)
    kv_len_range: Tuple[int, int] = (0, 0)  # (lo, hi) when kv_len is drawn (c3)

    @property
    def m(self):
        return self.n_new + self.k

    def with_(self, **kw):
        return replace(self, **kw)


_TINY = DrafterShape(hidden=256, n_heads=4, n_kv_heads=4, head_dim=64, ffn=688, vocab=1024,
                     dtype="f32", rms_eps=1e-6, rope_base=10000.0, k_max=8)
_7B = DrafterShape(hidden=4096, n_heads=32, n_kv_heads=32, head_dim=128, ffn=11008, vocab=32000,
                   dtype="bf16", rms_eps=1e-5, rope_base=10000.0, k_max=8)
_13B = DrafterShape(hidden=5120, n_heads=40, n_kv_heads=40, head_dim=128, ffn=13824, vocab=32000,
                    dtype="bf16", rms_eps=1e-5, rope_base=10000.0, k_max=8)
_L3_8B = DrafterShape(hidden=4096, n_heads=32, n_kv_heads=8, head_dim=128, ffn=14336, vocab=128256,
                      dtype="bf16", rms_eps=1e-5, rope_base=500000.0, k_max=8)

WORKLOADS = {
    "c0": Workload("c0", _TINY, batch=1, kv_len=(64,), n_new=1, k=4, topk=4, seed=0),
    "c1": Workload("c1", _7B, batch=1, kv_len=(512,), n_new=1, k=5, topk=8, seed=1),
    "c2": Workload("c2", _13B, batch=1, kv_len=(1024,), n_new=1, k=5, topk=8, seed=2,
                   n_new_mix=(1, 2, 3, 4, 5, 6)),
    "c3": Workload("c3", _7B, batch=8, kv_len=(), n_new=1, k=5, topk=8, seed=3,
                   kv_len_range=(128, 2048)),
    "c4": Workload("c4", _L3_8B, batch=1, kv_len=(4096,), n_new=1, k=8, topk=8, seed=4),
}


def small_shape(dtype="bf16", **kw):
    """A reduced drafter for parity tests: several tiles per GEMM and ragged tails."""
    base = dict(hidden=512, n_heads=8, n_kv_heads=8, head_dim=64, ffn=1376, vocab=2064,
                dtype=dtype, rms_eps=1e-5, rope_base=10000.0, k_max=8)
    base.update(kw)
    return DrafterShape(**base)
