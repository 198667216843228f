"""CPU oracle for the input stage of the parallel drafter.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this file; it imports
nothing of the HIP path.

What it computes (Section 4.3 "Integration with Popular Speculative Decoding Frameworks"):

* Medusa integration: the draft model shares the target's embedding layer, kept frozen, to which the K
  trainable [MASK] tokens were added.  The input of a real position is therefore the row of the embedding
  table that its token selects; the input of [MASK]_j is the j-th added row (the step's mask_emb).
* EAGLE integration: the draft model is a fully connected layer followed by the (now parallel) head; its
  input at a position is built from the target's last-layer hidden state f of a position and the embedding e
  of a token, pi(. | f, e): the fully connected layer maps the concatenation [f ; e] (2H values) to H values.

Readings where the paper is silent: the concatenation order is (f, e), as the paper writes the pair; a bias
is optional; which f goes with which e (EAGLE pairs f_i with the token after it) is the caller's business
and not part of this computation; [MASK] rows are the learned mask embeddings as they are (a learned input
needs no projection).  Everything is the plain definition in float64 on the stored values; the result of the
fully connected layer is NOT rounded to the storage type (it feeds the layer's RMSNorm and residual stream).

Pins (tests/test_oracle_input_stage.py, CPU): the gather against plain indexing, token by token; the
projection against PyTorch's float64 `linear` on the concatenated rows and against the sum of two separate
products; a one-hot feature selects a column of w_fc; with w_fc = [0 | I] the projection is the embedding
itself, so the fused mode reduces to the token mode, and the token mode reduces to the hidden-state mode
of the draft step bit for bit.
"""
import numpy as np

from oracle.ps_oracle import widen


def embed_tokens(embed, token_ids):
    """Rows of the stored embedding table [V, H] selected by token_ids [B, n]; stored values, unchanged."""
    embed = np.asarray(embed)
    ids = np.asarray(token_ids)
    out = np.empty(ids.shape + (embed.shape[1],), dtype=embed.dtype)
    for b in range(ids.shape[0]):
        for i in range(ids.shape[1]):
            out[b, i] = embed[int(ids[b, i])]
    return out


def fused_input(features, embed, token_ids, w_fc, b_fc, dtype):
    """w_fc . [f ; e] (+ b_fc) per real position, float64 [B, n, H].

    features [B, n, H] stored, embed [V, H] stored, w_fc [H, 2H] stored, b_fc [H] stored or None."""
    F = widen(features, dtype)
    E = widen(embed_tokens(embed, token_ids), dtype)
    W = widen(w_fc, dtype)
    cat = np.concatenate([F, E], axis=-1)                 # [B, n, 2H]: (f, e)
    out = cat @ W.T
    if b_fc is not None:
        out = out + widen(b_fc, dtype)
    return out
