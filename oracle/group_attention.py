"""CPU oracle for the attention of group-wise parallel training.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this file; it imports
nothing of the HIP path.

What it computes (Section 4.1 "Group-wise Parallel Training"; captions of Figures 2 and 3).  To train the
parallel drafter without a mismatch between training and inference, a training sequence of T real tokens is
laid out as T parallel groups, each an input token followed by k [MASK] tokens:

    x_0 m_1 .. m_k | x_1 m_1 .. m_k | ... | x_{T-1} m_1 .. m_k          (T (k + 1) rows)

and attention runs over this layout with a customised causal mask: every token ignores the [MASK] tokens of
previous groups.  So row (group g, slot s; slot 0 is the real token) sees the real tokens of groups 0..g and
the [MASK] tokens 1..s of its own group - exactly what the same token sees at inference, where x_0..x_g are
the prefix and the k masks are appended after it (Section 4.1 "Inference"; Algorithm 1: distribution j is
conditioned on [MASK]_1..j).  Position indices are adjusted to match: the real token of group g stands at
position g, its mask j at position g + j.

Readings (both figures are missing from the available text): the layout order and the positions above, which
are the ones under which training and inference coincide (pinned below against the inference oracle); keys are
rounded to the storage type after the rotary embedding and values are used as stored, as the inference path
keeps them in its cache.

Pins (tests/test_oracle_group_attention.py, CPU): the mask against the sentence that defines it, pair by pair;
the whole computation against PyTorch's float64 scaled_dot_product_attention with that mask and complex-number
rotary; every group's rows against the attention probabilities of the inference oracle's draft step on the
prefix x_0..x_g (the property the layout exists for); k = 0 is ordinary causal attention; planted mistakes
(earlier groups' masks visible, positions by layout index) break the agreement with inference.
"""
import numpy as np

from oracle.ps_oracle import rope, round_to_storage, widen


def group_layout(tokens, k):
    """(group, slot, position) of every row of the training layout."""
    rows = tokens * (k + 1)
    group = np.arange(rows) // (k + 1)
    slot = np.arange(rows) % (k + 1)
    return group, slot, group + slot


def group_mask(tokens, k):
    """visible[i, j]: may row i attend to row j?  Causal, minus the [MASK] tokens of earlier groups."""
    group, slot, _ = group_layout(tokens, k)
    rows = len(group)
    vis = np.zeros((rows, rows), dtype=bool)
    for i in range(rows):
        for j in range(i + 1):                                     # causal in layout order
            earlier_groups_mask = slot[j] > 0 and group[j] < group[i]
            vis[i, j] = not earlier_groups_mask
    return vis


def group_attention(q, k_, v, tokens, k, rope_base, dtype, return_probs=False):
    """q [rows, n_heads, d], k_, v [rows, n_kv_heads, d] stored (before the rotary embedding), rows = tokens (k+1).
    Returns the attention output [rows, n_heads, d] in float64 (and the probabilities [rows, n_heads, rows])."""
    Q, K, V = widen(q, dtype), widen(k_, dtype), widen(v, dtype)
    rows, nq, d = Q.shape
    nkv = K.shape[1]
    grp = nq // nkv
    _, _, pos = group_layout(tokens, k)
    Q = rope(Q, pos, rope_base)
    K = widen(round_to_storage(rope(K, pos, rope_base), dtype), dtype)
    vis = group_mask(tokens, k)
    out = np.zeros((rows, nq, d))
    probs = np.zeros((rows, nq, rows))
    for i in range(rows):
        cols = np.nonzero(vis[i])[0]
        for h in range(nq):
            s = K[cols, h // grp, :] @ Q[i, h, :] / np.sqrt(d)
            p = np.exp(s - np.max(s))
            p = p / np.sum(p)
            out[i, h, :] = p @ V[cols, h // grp, :]
            probs[i, h, cols] = p
    return (out, probs) if return_probs else out


def visible_pairs(tokens, k):
    """Number of (query, key) pairs the mask leaves: T real tokens see 1..T real keys, every mask j of group g
    sees g + 1 real keys and j masks."""
    return int(group_mask(tokens, k).sum()) if tokens * (k + 1) <= 512 else \
        (k + 1) * tokens * (tokens + 1) // 2 + tokens * k * (k + 1) // 2
