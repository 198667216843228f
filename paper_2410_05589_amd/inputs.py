"""Seeded synthetic inputs for the parallel draft step.

This module only draws numbers and lays them out; it holds none of the
method's arithmetic, so both the CPU oracle's tests and the HIP path's callers
may use it.  Every tensor has its own Philox stream keyed by (seed, tensor id),
so any subset can be regenerated on its own.

Value recipe (benchmark definition): matrices, mask-independent weights and the
cached K/V ~ N(0, 0.02); norm gains 1 + N(0, 0.02); input hidden states and the
[MASK] embeddings ~ N(0, 1).  For bf16 workloads every tensor is rounded to
bf16 (round to nearest even) here and handed out as uint16 bit patterns, so the
oracle and the device read exactly the same stored values.
"""
import numpy as np

_TENSOR_IDS = {
    "g_in": 1, "wq": 2, "wk": 3, "wv": 4, "wo": 5, "g_post": 6, "w_gate": 7, "w_up": 8,
    "w_down": 9, "g_final": 10, "w_lm": 11, "mask_emb": 12, "x": 13, "k_cache": 14,
    "v_cache": 15, "kv_len": 16, "n_new_mix": 17, "embed": 18, "w_fc": 19, "b_fc": 20, "token_ids": 21,
    "features": 22, "uniforms": 23, "train_q": 24, "train_k": 25, "train_v": 26,
}


def _rng(seed, name, sub=0):
    return np.random.Generator(np.random.Philox(key=[int(seed), _TENSOR_IDS[name] + 1000 * int(sub)]))


def f32_to_bf16_bits(a):
    """Round float32 to bfloat16 (nearest even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(a, dtype):
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    return np.ascontiguousarray(a, dtype=np.float32)


def _normal(seed, name, shape, std, mean, dtype, sub=0):
    g = _rng(seed, name, sub)
    a = g.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    return _store(a, dtype)


def make_weights(shape, seed):
    """All drafter weights, row-major [out, in]; bf16 tensors as uint16 bits."""
    s, dt = shape, shape.dtype
    w = {
        "g_in": _normal(seed, "g_in", (s.hidden,), 0.02, 1.0, dt),
        "wq": _normal(seed, "wq", (s.q_dim, s.hidden), 0.02, 0.0, dt),
        "wk": _normal(seed, "wk", (s.kv_dim, s.hidden), 0.02, 0.0, dt),
        "wv": _normal(seed, "wv", (s.kv_dim, s.hidden), 0.02, 0.0, dt),
        "wo": _normal(seed, "wo", (s.hidden, s.q_dim), 0.02, 0.0, dt),
        "g_post": _normal(seed, "g_post", (s.hidden,), 0.02, 1.0, dt),
        "w_gate": _normal(seed, "w_gate", (s.ffn, s.hidden), 0.02, 0.0, dt),
        "w_up": _normal(seed, "w_up", (s.ffn, s.hidden), 0.02, 0.0, dt),
        "w_down": _normal(seed, "w_down", (s.hidden, s.ffn), 0.02, 0.0, dt),
        "g_final": _normal(seed, "g_final", (s.hidden,), 0.02, 1.0, dt),
        "w_lm": _normal(seed, "w_lm", (s.vocab, s.hidden), 0.02, 0.0, dt),
        "mask_emb": _normal(seed, "mask_emb", (s.k_max, s.hidden), 1.0, 0.0, dt),
    }
    return w


def make_input_stage_weights(shape, seed, fc=True, bias=True):
    """The shared embedding table ~ N(0, 1) like the hidden states it stands for, and the input projection
    [H, 2H] ~ N(0, 0.02) * (1 / sqrt(2 H) / 0.02 ...) scaled so that its output has about unit scale, with a
    bias ~ N(0, 0.02); bf16 tensors as uint16 bits."""
    s, dt = shape, shape.dtype
    w = {"embed": _normal(seed, "embed", (s.vocab, s.hidden), 1.0, 0.0, dt)}
    if fc:
        w["w_fc"] = _normal(seed, "w_fc", (s.hidden, 2 * s.hidden), float(1.0 / np.sqrt(2.0 * s.hidden)), 0.0, dt)
        if bias:
            w["b_fc"] = _normal(seed, "b_fc", (s.hidden,), 0.02, 0.0, dt)
    return w


def make_input_stage_inputs(workload, n_new=None, sub=0):
    """Token ids uniform in [0, V) and target features ~ N(0, 1) for the real rows of a step."""
    s = workload.shape
    n_new = workload.n_new if n_new is None else n_new
    g = _rng(workload.seed, "token_ids", sub)
    ids = g.integers(0, s.vocab, size=(workload.batch, n_new)).astype(np.int32)
    feats = _normal(workload.seed, "features", (workload.batch, n_new, s.hidden), 1.0, 0.0, s.dtype, sub=sub)
    return {"token_ids": ids, "features": feats}


def make_group_attention_inputs(seed, seqs, tokens, k, n_heads, n_kv_heads, head_dim, dtype):
    """q, k, v ~ N(0, 1) of a training sequence laid out as parallel groups: [seqs, tokens (k + 1), heads, d]."""
    rows = tokens * (k + 1)
    return {"q": _normal(seed, "train_q", (seqs, rows, n_heads, head_dim), 1.0, 0.0, dtype),
            "k": _normal(seed, "train_k", (seqs, rows, n_kv_heads, head_dim), 1.0, 0.0, dtype),
            "v": _normal(seed, "train_v", (seqs, rows, n_kv_heads, head_dim), 1.0, 0.0, dtype)}


def draw_kv_len(workload):
    """Per-sequence valid cache lengths: fixed, or uniform in the stated range."""
    if workload.kv_len:
        return tuple(int(v) for v in workload.kv_len)
    lo, hi = workload.kv_len_range
    g = _rng(workload.seed, "kv_len")
    return tuple(int(v) for v in g.integers(lo, hi + 1, size=workload.batch))


def draw_n_new_mix(workload, steps):
    """Accepted-length mix: n_new per step, uniform over workload.n_new_mix."""
    g = _rng(workload.seed, "n_new_mix")
    mix = np.asarray(workload.n_new_mix if workload.n_new_mix else (workload.n_new,))
    return [int(v) for v in mix[g.integers(0, len(mix), size=steps)]]


def make_step_inputs(workload, kv_len=None, n_new=None, k=None, slack=0, sub=0):
    """Input hidden states and a ragged KV cache with an offsets array.

    Sequence b owns cache rows [kv_offsets[b], kv_offsets[b+1]); its first
    kv_len[b] rows hold N(0, 0.02) values, the remaining n_new + k (+ slack)
    rows are zero and receive this step's new K/V rows.
    """
    s = workload.shape
    kv_len = tuple(draw_kv_len(workload) if kv_len is None else kv_len)
    n_new = workload.n_new if n_new is None else n_new
    k = workload.k if k is None else k
    m = n_new + k
    cap = [l + m + slack for l in kv_len]
    off = np.zeros(len(kv_len) + 1, dtype=np.int64)
    off[1:] = np.cumsum(cap)
    total = int(off[-1])
    kc = np.zeros((total, s.n_kv_heads, s.head_dim), dtype=np.uint16 if s.dtype == "bf16" else np.float32)
    vc = np.zeros_like(kc)
    for b, l in enumerate(kv_len):
        if l == 0:
            continue
        kc[off[b]:off[b] + l] = _normal(workload.seed, "k_cache", (l, s.n_kv_heads, s.head_dim), 0.02, 0.0,
                                        s.dtype, sub=sub * 64 + b)
        vc[off[b]:off[b] + l] = _normal(workload.seed, "v_cache", (l, s.n_kv_heads, s.head_dim), 0.02, 0.0,
                                        s.dtype, sub=sub * 64 + b)
    x = _normal(workload.seed, "x", (len(kv_len), n_new, s.hidden), 1.0, 0.0, s.dtype, sub=sub)
    return {"x": x, "k_cache": kc, "v_cache": vc, "kv_offsets": off,
            "kv_len": np.asarray(kv_len, dtype=np.int32), "n_new": n_new, "k": k}


# ---------------------------------------------------------------- draft tree and acceptance walk
def draft_tree(fanout):
    """Static draft tree: fanout[t] = how many of draft row t's top tokens every node of depth t gets
    as children (node 0 = root).  Returns (parent, rank), nodes in breadth-first order, a node's
    children in ascending rank."""
    parent, rank, level = [-1], [0], [0]
    for f in fanout:
        nxt = []
        for u in level:
            for j in range(f):
                parent.append(u)
                rank.append(j)
                nxt.append(len(parent) - 1)
        level = nxt
    return np.array(parent, dtype=np.int32), np.array(rank, dtype=np.int32)


def verify_inputs(seed, batch, parent, rank, rows, topk, vocab, agreement=0.7, concentration=0.05):
    """Seeded inputs of a tree build + acceptance walk (numbers only: no step of the walk is taken here).

    The drafter's distributions q [batch, rows, vocab] are peaked (a Dirichlet with a small
    concentration, like a language model's); top_ids are q's largest entries per row (ties to the lower
    id); the target's distribution after a node of depth t is `agreement` times draft row t (so
    proposals of the next depth are often accepted) plus (1 - agreement) times an independent peaked
    draw; r is uniform in [0, 1).  Everything is float32 as stored; nothing needs to sum to exactly 1.
    """
    g = np.random.Generator(np.random.Philox(key=[int(seed), 9001]))
    n = len(parent)
    depth = np.zeros(n, dtype=np.int64)
    for s in range(1, n):
        depth[s] = depth[parent[s]] + 1

    def peaked(shape_prefix):
        a = g.standard_gamma(concentration, size=tuple(shape_prefix) + (vocab,)) + 1e-12
        return a / a.sum(axis=-1, keepdims=True)

    q = peaked((batch, rows))
    other = peaked((batch, n))
    p = np.empty((batch, n, vocab))
    for s in range(n):
        t = int(depth[s])
        p[:, s] = agreement * q[:, t] + (1.0 - agreement) * other[:, s] if t < rows else other[:, s]
    q32 = q.astype(np.float32)
    order = np.lexsort((np.broadcast_to(np.arange(vocab), q32.shape), -q32), axis=-1)
    top_ids = order[..., :topk].astype(np.int32)
    r = g.random((batch, n)).astype(np.float32)
    r = np.minimum(r, np.float32(1.0 - 2.0 ** -24))
    return {"q": q32, "p": p.astype(np.float32), "r": r, "top_ids": np.ascontiguousarray(top_ids)}
