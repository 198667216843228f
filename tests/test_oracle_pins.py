"""CPU pins of the oracle (no GPU): brute force, library routines, invariants, closed forms.

None of these re-types the oracle's own formulas: the brute force is a per-position
full-sequence forward with a dense mask matrix, complex-number rotary embedding and no
KV cache; the library pin composes PyTorch float64 ops; the rest are properties the
paper and the mathematics fix (Section 4.1 "Inference", Algorithm 1, Section 5.1).
"""
import cmath
import math
import os

import numpy as np
import pytest
import torch

from oracle import ps_oracle as orc
from paper_2410_05589_amd import inputs
from paper_2410_05589_amd.configs import WORKLOADS, DrafterShape
from tests.helpers import tiny_shape, tiny_workload, scaled_weights, store


# ----------------------------------------------------------------------------------------------
# Scenario: a sequence of L prefix positions (hidden states known), n_new newly accepted
# positions and k [MASK] slots.  The full-sequence references run the layer over all L+M
# positions at once; the oracle gets the prefix only through the KV cache.
# ----------------------------------------------------------------------------------------------
def _scenario(shape, L, n_new, k, seed):
    g = np.random.default_rng(seed)
    w = scaled_weights(shape, seed)
    hp = store(g.standard_normal((L, shape.hidden)).astype(np.float32), shape.dtype)
    x = store(g.standard_normal((1, n_new, shape.hidden)).astype(np.float32), shape.dtype)
    return w, hp, x


def _full_sequence_inputs(shape, w, hp, x, k):
    W = {n: orc.widen(a, shape.dtype) for n, a in w.items()}
    seq = np.concatenate([orc.widen(hp, shape.dtype), orc.widen(x, shape.dtype)[0], W["mask_emb"][:k]], axis=0)
    return W, seq


def brute_force_layer(shape, W, seq, round_kv):
    """Per-position loops, dense (T x T) visibility matrix, complex rotary, no cache.

    round_kv: function applied to K (post-rotary) and V of every position (the cache keeps
    them in the storage dtype).
    Returns (final hidden [T,H], logits [T,V], K [T,nkv,d], V [T,nkv,d]).
    """
    T, H = seq.shape
    nq, nkv, d = shape.n_heads, shape.n_kv_heads, shape.head_dim
    half = d // 2
    visible = np.zeros((T, T), dtype=bool)
    for i in range(T):
        for j in range(T):
            visible[i, j] = j <= i
    q = np.zeros((T, nq, d)); kk = np.zeros((T, nkv, d)); vv = np.zeros((T, nkv, d))
    for t in range(T):
        z = seq[t]
        a = np.array([z[c] / math.sqrt(sum(float(v) ** 2 for v in z) / H + shape.rms_eps) * W["g_in"][c]
                      for c in range(H)])
        qt = W["wq"] @ a; kt = W["wk"] @ a; vt = W["wv"] @ a
        for hh in range(nq):
            for j in range(half):
                rot = cmath.exp(1j * t * shape.rope_base ** (-2.0 * j / d))
                c = complex(qt[hh * d + j], qt[hh * d + j + half]) * rot
                q[t, hh, j], q[t, hh, j + half] = c.real, c.imag
        for hh in range(nkv):
            for j in range(half):
                rot = cmath.exp(1j * t * shape.rope_base ** (-2.0 * j / d))
                c = complex(kt[hh * d + j], kt[hh * d + j + half]) * rot
                kk[t, hh, j], kk[t, hh, j + half] = c.real, c.imag
            vv[t, hh] = vt[hh * d:(hh + 1) * d]
    kk = round_kv(kk); vv = round_kv(vv)
    o = np.zeros((T, nq * d))
    for t in range(T):
        for hh in range(nq):
            kvh = hh // (nq // nkv)
            sc = np.full(T, -np.inf)
            for j in range(T):
                if visible[t, j]:
                    sc[j] = float(np.dot(q[t, hh], kk[j, kvh])) / math.sqrt(d)
            e = np.exp(sc - sc.max())
            p = e / e.sum()
            for j in range(T):
                o[t, hh * d:(hh + 1) * d] += p[j] * vv[j, kvh]
    y = seq + o @ W["wo"].T
    hid = np.zeros_like(y)
    logits = np.zeros((T, shape.vocab))
    for t in range(T):
        bn = y[t] / math.sqrt(np.mean(y[t] ** 2) + shape.rms_eps) * W["g_post"]
        gate = W["w_gate"] @ bn; up = W["w_up"] @ bn
        u = gate / (1.0 + np.exp(-gate)) * up
        hid[t] = y[t] + W["w_down"] @ u
        n = hid[t]
        if shape.final_norm:
            n = n / math.sqrt(np.mean(n ** 2) + shape.rms_eps) * W["g_final"]
        logits[t] = W["w_lm"] @ n
    return hid, logits, kk, vv


def torch_layer(shape, W, seq, round_kv):
    """The same full-sequence forward composed from PyTorch float64 library ops."""
    F = torch.nn.functional
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).double()
    T, H = seq.shape
    nq, nkv, d = shape.n_heads, shape.n_kv_heads, shape.head_dim
    z = t(seq)
    a = F.rms_norm(z, (H,), t(W["g_in"]), eps=shape.rms_eps)
    q = F.linear(a, t(W["wq"])).view(T, nq, d).transpose(0, 1)     # [nq, T, d]
    k = F.linear(a, t(W["wk"])).view(T, nkv, d).transpose(0, 1)
    v = F.linear(a, t(W["wv"])).view(T, nkv, d).transpose(0, 1)
    inv = 1.0 / (shape.rope_base ** (torch.arange(0, d, 2).double() / d))
    fr = torch.outer(torch.arange(T).double(), inv)
    emb = torch.cat((fr, fr), dim=-1)
    cos, sin = emb.cos(), emb.sin()
    rot = lambda u: torch.cat((-u[..., d // 2:], u[..., :d // 2]), dim=-1)
    q = q * cos + rot(q) * sin
    k = k * cos + rot(k) * sin
    k = t(round_kv(k.numpy())); v = t(round_kv(v.numpy()))
    kr = k.repeat_interleave(nq // nkv, dim=0); vr = v.repeat_interleave(nq // nkv, dim=0)
    mask = torch.tril(torch.ones(T, T, dtype=torch.bool))
    o = F.scaled_dot_product_attention(q[None], kr[None], vr[None], attn_mask=mask)[0]
    o = o.transpose(0, 1).reshape(T, nq * d)
    y = z + F.linear(o, t(W["wo"]))
    bn = F.rms_norm(y, (H,), t(W["g_post"]), eps=shape.rms_eps)
    hid = y + F.linear(F.silu(F.linear(bn, t(W["w_gate"]))) * F.linear(bn, t(W["w_up"])), t(W["w_down"]))
    n = F.rms_norm(hid, (H,), t(W["g_final"]), eps=shape.rms_eps) if shape.final_norm else hid
    logits = F.linear(n, t(W["w_lm"]))
    return hid.numpy(), logits.numpy(), k.transpose(0, 1).numpy(), v.transpose(0, 1).numpy()


def _check_against_full_sequence(shape, ref_fn, L, n_new, k, seed, tol):
    w, hp, x = _scenario(shape, L, n_new, k, seed)
    W, seq = _full_sequence_inputs(shape, w, hp, x, k)
    rkv = lambda a: orc.widen(orc.round_to_storage(a, shape.dtype), shape.dtype)
    hid, logits, kk, vv = ref_fn(shape, W, seq, rkv)
    M = n_new + k
    cap = L + M
    kc = np.zeros((cap, shape.n_kv_heads, shape.head_dim), dtype=np.uint16 if shape.dtype == "bf16" else np.float32)
    vc = np.zeros_like(kc)
    kc[:L] = orc.round_to_storage(kk[:L], shape.dtype)
    vc[:L] = orc.round_to_storage(vv[:L], shape.dtype)
    out = orc.draft_step(shape, w, x, kc, vc, np.array([0, cap]), np.array([L]), n_new, k, topk=3, all_rows=True)
    np.testing.assert_allclose(out["hidden_out"][0], hid[L:], rtol=tol, atol=tol)
    np.testing.assert_allclose(out["logits"][0], logits[L:], rtol=tol, atol=tol)
    np.testing.assert_allclose(orc.widen(out["k_cache"], shape.dtype)[L:L + M], kk[L:], rtol=tol, atol=tol)
    np.testing.assert_allclose(orc.widen(out["v_cache"], shape.dtype)[L:L + M], vv[L:], rtol=tol, atol=tol)
    # softmax / top-k against the library definitions
    lt = torch.from_numpy(logits[L:])
    np.testing.assert_allclose(out["probs"][0], torch.softmax(lt, -1).numpy(), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(out["lse"][0], torch.logsumexp(lt, -1).numpy(), rtol=1e-9, atol=1e-9)
    # default rows = last real row + the k mask rows (k+1 distributions, Section 4.1)
    out_d = orc.draft_step(shape, w, x, kc, vc, np.array([0, cap]), np.array([L]), n_new, k, topk=3)
    assert out_d["logits"].shape == (1, k + 1, shape.vocab)
    np.testing.assert_allclose(out_d["logits"][0], logits[L + n_new - 1:], rtol=tol, atol=tol)


@pytest.mark.parametrize("nkv", [4, 2, 1])
def test_brute_force_full_sequence_f32(nkv):
    # f32 storage: the brute force rounds K/V to float32 like the cache does
    _check_against_full_sequence(tiny_shape("f32", n_kv_heads=nkv), brute_force_layer, L=7, n_new=2, k=3,
                                 seed=3 + nkv, tol=1e-9)


def test_brute_force_full_sequence_bf16_storage():
    _check_against_full_sequence(tiny_shape("bf16"), brute_force_layer, L=5, n_new=1, k=4, seed=9, tol=1e-9)


def test_brute_force_no_final_norm_and_no_prefix():
    _check_against_full_sequence(tiny_shape("f32", final_norm=False), brute_force_layer, L=0, n_new=3, k=2,
                                 seed=21, tol=1e-9)


@pytest.mark.parametrize("dtype,L,n_new,k", [("f32", 33, 3, 4), ("bf16", 20, 1, 4), ("f32", 12, 4, 0)])
def test_library_ops_full_sequence(dtype, L, n_new, k):
    shape = tiny_shape(dtype, hidden=128, n_heads=8, n_kv_heads=2, head_dim=16, ffn=176, vocab=97)
    _check_against_full_sequence(shape, torch_layer, L=L, n_new=n_new, k=k, seed=5, tol=1e-9)


# ----------------------------------------------------------------------------------------------
# invariants
# ----------------------------------------------------------------------------------------------
def _fresh(shape, kv_len=(7,), n_new=2, k=3, seed=11, batch=None, slack=8):
    wl = tiny_workload(shape, batch=batch or len(kv_len), kv_len=kv_len, n_new=n_new, k=k, seed=seed)
    w = scaled_weights(shape, seed)
    # the scaled-up cache makes cached keys matter in the softmax
    inp = inputs.make_step_inputs(wl, slack=slack)
    for name in ("k_cache", "v_cache"):
        a = inp[name]
        inp[name] = store(orc.widen(a, shape.dtype).astype(np.float32) * 30.0, shape.dtype)
    return wl, w, inp


def _step(shape, w, inp, n_new=None, k=None, x=None, kc=None, vc=None, kv_len=None, **kw):
    return orc.draft_step(shape, w, inp["x"] if x is None else x,
                          inp["k_cache"] if kc is None else kc, inp["v_cache"] if vc is None else vc,
                          inp["kv_offsets"], inp["kv_len"] if kv_len is None else kv_len,
                          inp["n_new"] if n_new is None else n_new, inp["k"] if k is None else k,
                          topk=kw.pop("topk", 3), **kw)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_prefix_rows_unchanged_by_appending_mask_slots(dtype):
    """Row j is conditioned on [MASK]_1..j only (Algorithm 1): fewer slots leave earlier rows alone."""
    shape = tiny_shape(dtype)
    wl, w, inp = _fresh(shape)
    full = _step(shape, w, inp, all_rows=True)
    for kk in range(0, inp["k"]):
        part = _step(shape, w, inp, k=kk, all_rows=True)
        rows = inp["n_new"] + kk
        np.testing.assert_allclose(part["logits"][0], full["logits"][0, :rows], rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(part["hidden_out"][0], full["hidden_out"][0, :rows], rtol=1e-11, atol=1e-12)
    # k = 0 is an ordinary causal decode step; its last row is the autoregressive next-token row
    ar = _step(shape, w, inp, k=0)
    assert ar["logits"].shape[1] == 1
    one = _step(shape, w, inp, k=1)
    np.testing.assert_allclose(one["logits"][0, 0], ar["logits"][0, 0], rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_parallel_step_equals_chained_single_row_steps(dtype):
    """An M-row step == M ordinary one-row decode steps fed [x..., mask_1..mask_k] one at a time."""
    shape = tiny_shape(dtype)
    wl, w, inp = _fresh(shape)
    full = _step(shape, w, inp, all_rows=True)
    feed = np.concatenate([inp["x"][0], w["mask_emb"][:inp["k"]]], axis=0)
    kc, vc, L = inp["k_cache"], inp["v_cache"], int(inp["kv_len"][0])
    for i in range(feed.shape[0]):
        o = _step(shape, w, inp, n_new=1, k=0, x=feed[None, i:i + 1], kc=kc, vc=vc, kv_len=np.array([L + i]))
        kc, vc = o["k_cache"], o["v_cache"]
        np.testing.assert_allclose(o["logits"][0, 0], full["logits"][0, i], rtol=1e-10, atol=1e-11)
    assert np.array_equal(kc, full["k_cache"]) and np.array_equal(vc, full["v_cache"])


def test_masks_of_previous_rounds_are_invisible():
    """Three rounds committing only the accepted rows == one pass over the real tokens + last masks."""
    shape = tiny_shape("f32")
    wl, w, inp = _fresh(shape, kv_len=(5,), n_new=1, k=3, slack=16)
    g = np.random.default_rng(0)
    accepted = [1, 3, 2]
    xs = [store(g.standard_normal((1, a, shape.hidden)).astype(np.float32), "f32") for a in accepted]
    kc, vc, L = inp["k_cache"], inp["v_cache"], 5
    for a, x in zip(accepted, xs):
        o = _step(shape, w, inp, n_new=a, k=3, x=x, kc=kc, vc=vc, kv_len=np.array([L]))
        kc, vc = o["k_cache"], o["v_cache"]      # rows L+a.. hold stale mask rows: never read again
        L += a
    L -= accepted[-1]
    allx = np.concatenate(xs, axis=1)
    ref = _step(shape, w, inp, n_new=sum(accepted), k=3, x=allx, kv_len=np.array([5]))
    np.testing.assert_allclose(o["logits"][0], ref["logits"][0], rtol=1e-10, atol=1e-11)
    # planted mistake: committing the mask rows as well (advancing by n_new + k) changes the answer
    kc, vc, L = inp["k_cache"], inp["v_cache"], 5
    for a, x in zip(accepted, xs):
        bad = _step(shape, w, inp, n_new=a, k=3, x=x, kc=kc, vc=vc, kv_len=np.array([L]))
        kc, vc = bad["k_cache"], bad["v_cache"]
        L += a + 3
    assert np.abs(bad["logits"][0] - ref["logits"][0]).max() > 1e-3


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_softmax_and_topk_invariants(dtype):
    shape = tiny_shape(dtype)
    wl, w, inp = _fresh(shape)
    o = _step(shape, w, inp, return_attn=True, topk=5)
    P = o["attn"][0]
    L, n_new = int(inp["kv_len"][0]), inp["n_new"]
    np.testing.assert_allclose(P.sum(-1), 1.0, rtol=0, atol=1e-12)
    for i in range(P.shape[0]):
        assert np.all(P[i, :, L + i + 1:] == 0.0) and np.all(P[i, :, :L + i + 1] > 0.0)
    np.testing.assert_allclose(o["probs"].sum(-1), 1.0, atol=1e-12)
    assert np.all(np.isfinite(o["lse"]))
    assert np.array_equal(o["top_ids"][..., 0], o["logits"].argmax(-1))
    tl = np.take_along_axis(o["logits"], o["top_ids"], axis=-1)
    assert np.all(np.diff(tl, axis=-1) <= 0)
    np.testing.assert_allclose(o["top_p"], np.take_along_axis(o["probs"], o["top_ids"], axis=-1))
    vals, ids = torch.topk(torch.from_numpy(o["logits"]), 5, dim=-1)
    assert np.array_equal(ids.numpy(), o["top_ids"])


def test_topk_ties_prefer_lower_id():
    row = np.array([0.5, 2.0, 2.0, -1.0, 2.0, 0.5])
    assert list(orc.top_k(row, 5)) == [1, 2, 4, 0, 5]


def test_rope_properties():
    g = np.random.default_rng(1)
    q = g.standard_normal((6, 3, 16)); kk = g.standard_normal((6, 3, 16))
    pos = np.array([0, 1, 5, 100, 1000, 4095])
    rq = orc.rope(q, pos, 10000.0)
    np.testing.assert_allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1), rtol=1e-12)
    np.testing.assert_array_equal(rq[0], q[0])                     # position 0 is the identity
    # relative property: <R(p1) q, R(p2) k> depends on p1 - p2 only
    a = np.einsum("rhd,rhd->rh", orc.rope(q, pos, 10000.0), orc.rope(kk, pos - 3, 10000.0))
    b = np.einsum("rhd,rhd->rh", orc.rope(q, pos + 77, 10000.0), orc.rope(kk, pos + 74, 10000.0))
    np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-9)
    # absolute definition, pair (j, j + d/2) rotated by pos * base**(-2j/d), counter-clockwise
    d = 16
    for j in range(d // 2):
        z = complex(q[3, 1, j], q[3, 1, j + d // 2]) * cmath.exp(1j * 100 * 10000.0 ** (-2.0 * j / d))
        assert abs(rq[3, 1, j] - z.real) < 1e-12 and abs(rq[3, 1, j + d // 2] - z.imag) < 1e-12


def test_gqa_equals_mha_with_repeated_kv_heads():
    sg = tiny_shape("f32", n_kv_heads=2)
    sm = tiny_shape("f32", n_kv_heads=4)
    wl, w, inp = _fresh(sg)
    d, grp = sg.head_dim, 2
    rep_rows = lambda a: np.repeat(a.reshape(sg.n_kv_heads, d, -1), grp, axis=0).reshape(sm.n_kv_heads * d, -1)
    w2 = dict(w); w2["wk"] = rep_rows(w["wk"]); w2["wv"] = rep_rows(w["wv"])
    inp2 = dict(inp)
    inp2["k_cache"] = np.repeat(inp["k_cache"], grp, axis=1); inp2["v_cache"] = np.repeat(inp["v_cache"], grp, axis=1)
    a = _step(sg, w, inp); b = _step(sm, w2, inp2)
    np.testing.assert_allclose(a["logits"], b["logits"], rtol=1e-11, atol=1e-12)
    np.testing.assert_array_equal(np.repeat(a["k_cache"], grp, axis=1), b["k_cache"])


def test_batch_equals_each_sequence_alone():
    shape = tiny_shape("bf16")
    wl, w, inp = _fresh(shape, kv_len=(7, 0, 19), n_new=2, k=3)
    o = _step(shape, w, inp)
    off = inp["kv_offsets"]
    for b in range(3):
        kc = inp["k_cache"][off[b]:off[b + 1]]; vc = inp["v_cache"][off[b]:off[b + 1]]
        ob = orc.draft_step(shape, w, inp["x"][b:b + 1], kc, vc, np.array([0, off[b + 1] - off[b]]),
                            inp["kv_len"][b:b + 1], 2, 3, topk=3)
        np.testing.assert_array_equal(ob["logits"][0], o["logits"][b])
        np.testing.assert_array_equal(ob["k_cache"], o["k_cache"][off[b]:off[b + 1]])
        np.testing.assert_array_equal(ob["top_ids"][0], o["top_ids"][b])


def test_closed_forms_for_degenerate_weights():
    shape = tiny_shape("f32")
    wl, w, inp = _fresh(shape)
    W = {n: orc.widen(a, "f32") for n, a in w.items()}
    Z = np.concatenate([orc.widen(inp["x"], "f32")[0], W["mask_emb"][:inp["k"]]], axis=0)
    # Wo = 0 and Wd = 0: the layer is the identity, logits = RMSNorm(Z) Wlm^T
    w0 = dict(w); w0["wo"] = np.zeros_like(w["wo"]); w0["w_down"] = np.zeros_like(w["w_down"])
    o = _step(shape, w0, inp, all_rows=True)
    n = Z / np.sqrt((Z ** 2).mean(-1, keepdims=True) + shape.rms_eps) * W["g_final"]
    np.testing.assert_allclose(o["hidden_out"][0], Z, rtol=0, atol=0)
    np.testing.assert_allclose(o["logits"][0], n @ W["w_lm"].T, rtol=1e-12, atol=1e-12)
    # Wq = 0: uniform attention; with Wd = 0 and Wv = 0 the new V rows are 0, so
    # O[i] = sum(cached V) / (L + i + 1) and hidden = Z + O Wo^T
    w1 = dict(w); w1["wq"] = np.zeros_like(w["wq"]); w1["wv"] = np.zeros_like(w["wv"])
    w1["w_down"] = np.zeros_like(w["w_down"])
    o = _step(shape, w1, inp, all_rows=True)
    L = int(inp["kv_len"][0])
    vsum = orc.widen(inp["v_cache"], "f32")[:L].sum(0)                       # [nkv, d]
    grp = shape.n_heads // shape.n_kv_heads
    for i in range(Z.shape[0]):
        oi = np.repeat(vsum, grp, axis=0).reshape(-1) / (L + i + 1)
        np.testing.assert_allclose(o["hidden_out"][0, i], Z[i] + W["wo"] @ oi, rtol=1e-11, atol=1e-12)
    # all cached and new V equal to one vector v (Wv = 0, cache V := 0 -> O = 0): hidden = Z + MLP(Z)
    w2 = dict(w); w2["wv"] = np.zeros_like(w["wv"])
    inp2 = dict(inp); inp2["v_cache"] = np.zeros_like(inp["v_cache"])
    o = _step(shape, w2, inp2, all_rows=True)
    bn = Z / np.sqrt((Z ** 2).mean(-1, keepdims=True) + shape.rms_eps) * W["g_post"]
    gate = bn @ W["w_gate"].T
    ref = Z + (gate / (1 + np.exp(-gate)) * (bn @ W["w_up"].T)) @ W["w_down"].T
    np.testing.assert_allclose(o["hidden_out"][0], ref, rtol=1e-11, atol=1e-12)


def test_new_kv_rows_are_stored_rounded_and_read_back_rounded():
    """The cache dtype rounding of this step's rows is visible to this step's attention."""
    shape = tiny_shape("bf16")
    wl, w, inp = _fresh(shape)
    o = _step(shape, w, inp, all_rows=True)
    L, M = int(inp["kv_len"][0]), inp["n_new"] + inp["k"]
    assert o["k_cache"].dtype == np.uint16
    assert np.array_equal(o["k_cache"][:L], inp["k_cache"][:L])               # old rows untouched
    assert np.array_equal(o["k_cache"][L + M:], inp["k_cache"][L + M:])
    # re-running row M-1 alone against the updated cache reproduces it exactly
    feed = np.concatenate([inp["x"][0], w["mask_emb"][:inp["k"]]], axis=0)
    last = _step(shape, w, inp, n_new=1, k=0, x=feed[None, M - 1:M], kc=o["k_cache"], vc=o["v_cache"],
                 kv_len=np.array([L + M - 1]))
    np.testing.assert_allclose(last["logits"][0, 0], o["logits"][0, M - 1], rtol=1e-10, atol=1e-11)


def test_round_to_storage_bf16():
    # ties to even, one rounding from float64
    one = 1.0
    ulp = 2.0 ** -7
    cases = {one + ulp / 2: one, one + 3 * ulp / 2: one + 2 * ulp, one + ulp / 2 + 1e-12: one + ulp,
             -(one + ulp / 2): -one, 0.0: 0.0, 3.0e-39: None}
    for v, want in cases.items():
        got = orc.widen(orc.round_to_storage(np.array([v]), "bf16"), "bf16")[0]
        if want is not None:
            assert got == want, (v, got, want)
    # a value whose float32 rounding lands on a bf16 tie: direct rounding must not double-round
    v = one + ulp / 2 + 2.0 ** -30
    assert orc.widen(orc.round_to_storage(np.array([v]), "bf16"), "bf16")[0] == one + ulp
    # on float32-representable inputs it agrees with the integer rounding used by the input generator
    g = np.random.default_rng(2)
    a = (g.standard_normal(20000) * np.exp(g.uniform(-20, 20, 20000))).astype(np.float32)
    assert np.array_equal(orc.round_to_storage(a.astype(np.float64), "bf16"), inputs.f32_to_bf16_bits(a))
    assert np.array_equal(orc.widen(inputs.f32_to_bf16_bits(a), "bf16").astype(np.float32),
                          inputs.bf16_bits_to_f32(inputs.f32_to_bf16_bits(a)))


def test_parameter_counts_match_the_paper():
    """Section 5.1 prints 202M (7B targets) and 317M (13B targets) for the one-layer drafter."""
    path = os.path.join(os.path.dirname(__file__), "golden", "param_counts.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    shapes = {(WORKLOADS[n].shape.hidden, WORKLOADS[n].shape.ffn): WORKLOADS[n].shape for n in ("c1", "c2")}
    for hidden, ffn, printed in rows:
        s = shapes[(int(hidden), int(ffn))]
        assert round(s.layer_params() / 1e6) == int(printed)
        w_names = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")
        dims = {"wq": s.q_dim * s.hidden, "wk": s.kv_dim * s.hidden, "wv": s.kv_dim * s.hidden,
                "wo": s.hidden * s.q_dim, "w_gate": s.ffn * s.hidden, "w_up": s.ffn * s.hidden,
                "w_down": s.hidden * s.ffn}
        assert sum(dims[n] for n in w_names) == s.layer_params()


def test_planted_mistakes_are_caught():
    """Sanity of the pins themselves: a wrong mask, position or pairing changes the answer."""
    shape = tiny_shape("f32")
    w, hp, x = _scenario(shape, 7, 2, 3, 3)
    W, seq = _full_sequence_inputs(shape, w, hp, x, 3)
    ident = lambda a: a
    hid, logits, kk, vv = brute_force_layer(shape, W, seq, ident)
    cap = 12
    kc = np.zeros((cap, shape.n_kv_heads, shape.head_dim), dtype=np.float32); vc = np.zeros_like(kc)
    kc[:7] = kk[:7]; vc[:7] = vv[:7]
    good = orc.draft_step(shape, w, x, kc, vc, np.array([0, cap]), np.array([7]), 2, 3, topk=3, all_rows=True)
    assert np.abs(good["logits"][0] - logits[7:]).max() < 1e-5
    # wrong cache length (positions shifted by one) must show
    kc2 = np.zeros((cap + 1, shape.n_kv_heads, shape.head_dim), dtype=np.float32); vc2 = np.zeros_like(kc2)
    kc2[1:8] = kk[:7]; vc2[1:8] = vv[:7]; kc2[0] = kk[0]; vc2[0] = vv[0]
    bad = orc.draft_step(shape, w, x, kc2, vc2, np.array([0, cap + 1]), np.array([8]), 2, 3, topk=3, all_rows=True)
    assert np.abs(bad["logits"][0] - logits[7:]).max() > 1e-3


def test_one_ulp_flips_of_new_cache_rows_move_logits_by_less_than_the_gpu_tests_allow(monkeypatch):
    """Evidence for the bound the GPU parity tests put on bf16 logits (5e-3, tests/gpu_util.py).  The step
    rounds its new K/V rows to bf16 before attention reads them; a device that computes those rows in float32
    lands on the neighbouring bf16 value wherever the exact value sits within float32 error of a rounding
    boundary (measured on the device: about 0.3 % of the new elements).  Here that is planted in the oracle at
    the 7B shape - 1 % of the new elements moved by one unit in the last place, three times the measured rate -
    and the logits move by more than the arithmetic error of the device path (5e-5) but stay below the bound."""
    from paper_2410_05589_amd.configs import WORKLOADS
    wl = WORKLOADS["c1"]
    shape = wl.shape
    w = inputs.make_weights(shape, wl.seed)
    inp = inputs.make_step_inputs(wl)
    args = (shape, w, inp["x"], inp["k_cache"], inp["v_cache"], inp["kv_offsets"], inp["kv_len"], wl.n_new, wl.k, wl.topk)
    ref = orc.draft_step(*args)
    exact = orc.round_to_storage
    rng = np.random.default_rng(0)

    def flipped(a, dt):
        r = exact(a, dt)
        if dt != "bf16":
            return r
        hit = rng.random(r.shape) < 0.01
        step = np.where(rng.random(r.shape) < 0.5, 1, -1)
        return np.where(hit, (r.astype(np.int32) + step).astype(np.uint16), r)

    monkeypatch.setattr(orc, "round_to_storage", flipped)
    out = orc.draft_step(*args)
    moved = float(np.abs(out["logits"] - ref["logits"]).max())
    n_flipped = int((out["k_cache"] != ref["k_cache"]).sum() + (out["v_cache"] != ref["v_cache"]).sum())
    assert n_flipped > 200
    assert 5e-5 < moved < 5e-3, moved
