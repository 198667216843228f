"""CPU oracle for the ParallelSpec parallel draft step.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this file; the product path never does, and this file imports nothing of the
HIP path.

What it computes (Section 4.1 "Inference"; Algorithm 1's draft line; Section 5.1
"Models"): the drafter is ONE Llama-style decoder layer shaped like a layer of
the target model, followed by the target's (shared, frozen) LM head
(Section 4.3, Medusa integration).  At a draft step the k special tokens
[MASK]_1..[MASK]_k are appended after the sequence; the representation of the
last real token decodes x_t and the representation of [MASK]_j decodes x_{t+j}:
distribution j is q(x | x_<n, [MASK]_1..j), so mask j sees the prefix and masks
1..j only (Algorithm 1).  [MASK] tokens of earlier draft rounds are never
visible (Section 4.1 "Group-wise Parallel Training"): with a KV cache this
holds because only the n_new real rows are committed after a step.

The method is exact (a Transformer layer forward), so this oracle is the plain
definition evaluated in float64 on exactly the stored input values (bf16
tensors are widened, never re-rounded), with one stated exception: this step's
new K/V rows are rounded to the cache dtype before attention reads them, so a
row gives the same answer now and when read from the cache next round.

Pins (tests/test_oracle_*.py, all CPU): full-sequence brute force with a dense
mask and no cache; PyTorch float64 library ops; chained single-row steps;
prefix rows unchanged by appending [MASK] slots; multi-round commit; RoPE shift
invariance; GQA == MHA with repeated heads; batch == each sequence alone;
closed forms for degenerate weights; the paper's printed parameter counts.
The paper prints no worked numeric example, so absolute output values are
pinned by these and by the definition only.
"""
import numpy as np


# ---------------------------------------------------------------- storage types
def widen(a, dtype):
    """Stored tensor -> float64 (bf16 tensors arrive as uint16 bit patterns)."""
    a = np.asarray(a)
    if dtype == "bf16":
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def round_to_storage(a64, dtype):
    """float64 -> stored representation of the cache dtype, one rounding only.

    bf16: round to nearest even on the 8-bit significand straight from float64
    (no intermediate float32 rounding); returns uint16 bit patterns.
    f32: ordinary float64 -> float32 conversion.
    """
    a64 = np.asarray(a64, dtype=np.float64)
    if dtype != "bf16":
        return a64.astype(np.float32)
    m, e = np.frexp(a64)                       # a = m * 2**e, 0.5 <= |m| < 1
    e_eff = np.maximum(e, -125)                # below 2**-126 the spacing is fixed (subnormals)
    q = np.rint(np.ldexp(a64, 8 - e_eff))      # np.rint rounds halves to even
    r = np.ldexp(q, e_eff - 8)                 # exactly representable in bf16, hence in float32
    return (r.astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


# ---------------------------------------------------------------- building blocks
def rms_norm(z, gain, eps):
    """z / sqrt(mean(z^2) + eps) * gain, row-wise."""
    ms = np.mean(z * z, axis=-1, keepdims=True)
    return z / np.sqrt(ms + eps) * gain


def rope(t, pos, base):
    """Rotary embedding, rotate-half pairing (j, j + d/2), angle pos * base**(-2j/d).

    t: [rows, heads, d]; pos: [rows] integer positions.
    """
    d = t.shape[-1]
    half = d // 2
    inv_freq = base ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]     # [rows, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = t[..., :half], t[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(a):
    return a / (1.0 + np.exp(-a))


def log_sum_exp(l):
    mx = np.max(l, axis=-1, keepdims=True)
    return (mx + np.log(np.sum(np.exp(l - mx), axis=-1, keepdims=True)))[..., 0]


def top_k(logits_row, k):
    """Ids of the k largest logits, descending; equal logits -> lower id first."""
    ids = np.arange(logits_row.shape[0])
    order = np.lexsort((ids, -logits_row))
    return order[:k]


# ---------------------------------------------------------------- the draft step
def draft_step(shape, weights, x, k_cache, v_cache, kv_offsets, kv_len, n_new, k, topk,
               all_rows=False, return_attn=False, x_is_float=False):
    """One parallel draft step for a batch of independent sequences.

    shape      : object with hidden, n_heads, n_kv_heads, head_dim, ffn, vocab, dtype,
                 rms_eps, rope_base, final_norm
    weights    : dict of stored tensors (g_in, wq, wk, wv, wo, g_post, w_gate, w_up,
                 w_down, g_final, w_lm, mask_emb), row-major [out, in]
    x          : [B, n_new, hidden] stored hidden states of the newly accepted positions
                 (x_is_float: float64 values instead, e.g. the output of oracle.input_stage.fused_input)
    k_cache, v_cache : [total_positions, n_kv_heads, head_dim] stored; K is post-RoPE.
                 NOT modified; updated copies are returned.
    kv_offsets : [B+1]; sequence b owns rows [off[b], off[b+1])
    kv_len     : [B] valid positions before this step
    Output rows: the last real row and the k mask rows (k+1 per sequence), or all
    n_new+k rows when all_rows.
    """
    dt = shape.dtype
    H, nq, nkv, d = shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim
    grp = nq // nkv
    B = len(kv_len)
    M = n_new + k
    W = {name: widen(w, dt) for name, w in weights.items() if w is not None}
    X = np.asarray(x, dtype=np.float64) if x_is_float else widen(x, dt)
    kc = np.array(k_cache, copy=True)
    vc = np.array(v_cache, copy=True)
    rows = list(range(M)) if all_rows else list(range(n_new - 1, M))
    R = len(rows)
    out = {
        "logits": np.zeros((B, R, shape.vocab)), "lse": np.zeros((B, R)),
        "probs": np.zeros((B, R, shape.vocab)), "top_ids": np.zeros((B, R, topk), dtype=np.int64),
        "top_p": np.zeros((B, R, topk)), "hidden_out": np.zeros((B, M, H)),
    }
    attn_rows = []
    for b in range(B):
        L, off = int(kv_len[b]), int(kv_offsets[b])
        # 1. the k [MASK] embeddings are appended after the real rows; positions continue
        Z = np.concatenate([X[b, :n_new], W["mask_emb"][:k]], axis=0)           # [M, H]
        pos = L + np.arange(M)
        # 2.-3. input norm and the three projections, split into heads
        A = rms_norm(Z, W["g_in"], shape.rms_eps)
        Q = (A @ W["wq"].T).reshape(M, nq, d)
        Kn = (A @ W["wk"].T).reshape(M, nkv, d)
        Vn = (A @ W["wv"].T).reshape(M, nkv, d)
        # 4. rotary embedding on Q and the new K rows
        Q = rope(Q, pos, shape.rope_base)
        Kn = rope(Kn, pos, shape.rope_base)
        # 5. new rows go into the cache in the cache dtype; attention reads them back
        kc[off + L: off + L + M] = round_to_storage(Kn, dt)
        vc[off + L: off + L + M] = round_to_storage(Vn, dt)
        Kall = widen(kc[off: off + L + M], dt)                                   # [L+M, nkv, d]
        Vall = widen(vc[off: off + L + M], dt)
        # 6. row i sees cache positions 0..L-1 and this step's rows 0..i
        O = np.zeros((M, nq, d))
        P_b = np.zeros((M, nq, L + M))
        for i in range(M):
            vis = L + i + 1
            for h in range(nq):
                s = Kall[:vis, h // grp, :] @ Q[i, h, :] / np.sqrt(d)
                p = np.exp(s - np.max(s))
                p = p / np.sum(p)
                O[i, h, :] = p @ Vall[:vis, h // grp, :]
                P_b[i, h, :vis] = p
        attn_rows.append(P_b)
        # 7. output projection and residual
        Y = Z + O.reshape(M, nq * d) @ W["wo"].T
        # 8. SwiGLU MLP and residual
        Bn = rms_norm(Y, W["g_post"], shape.rms_eps)
        U = silu(Bn @ W["w_gate"].T) * (Bn @ W["w_up"].T)
        Y2 = Y + U @ W["w_down"].T
        out["hidden_out"][b] = Y2
        # 9. LM head on the decoding rows
        Nf = Y2[rows]
        if shape.final_norm:
            Nf = rms_norm(Nf, W["g_final"], shape.rms_eps)
        logits = Nf @ W["w_lm"].T
        # 10. distributions and top-k candidates
        lse = log_sum_exp(logits)
        out["logits"][b] = logits
        out["lse"][b] = lse
        out["probs"][b] = np.exp(logits - lse[:, None])
        for r in range(R):
            ids = top_k(logits[r], topk)
            out["top_ids"][b, r] = ids
            out["top_p"][b, r] = out["probs"][b, r, ids]
    out["k_cache"] = kc
    out["v_cache"] = vc
    if return_attn:
        out["attn"] = attn_rows
    return out
