"""Pins of the group-wise training attention oracle: each compares it with something it does not contain."""
import numpy as np
import pytest

from oracle import group_attention as ga
from oracle import ps_oracle as orc
from paper_2410_05589_amd import inputs
from tests.helpers import tiny_shape, tiny_workload, store


def test_mask_pair_by_pair_against_its_definition():
    T, k = 5, 3
    vis = ga.group_mask(T, k)
    rows = T * (k + 1)
    for i in range(rows):
        gi, si = divmod(i, k + 1)
        for j in range(rows):
            gj, sj = divmod(j, k + 1)
            if sj == 0:
                want = gj <= gi                                 # a real token: visible to its own group and all later ones
            else:
                want = gj == gi and sj <= si                    # a [MASK] token: only inside its group, to itself and later slots
            assert vis[i, j] == want, (i, j)
    # closed-form count of the visible pairs (also used for the FLOP count of the benchmark)
    assert vis.sum() == (k + 1) * T * (T + 1) // 2 + T * k * (k + 1) // 2 == ga.visible_pairs(T, k)
    assert ga.visible_pairs(2048, 4) == 5 * 2048 * 2049 // 2 + 2048 * 10
    group, slot, pos = ga.group_layout(T, k)
    assert pos.tolist()[:9] == [0, 1, 2, 3, 1, 2, 3, 4, 2]      # x_0 m1 m2 m3 | x_1 m1 m2 m3 | x_2 ...


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_against_the_library_attention_with_the_mask_and_complex_rotary(dtype):
    torch = pytest.importorskip("torch")
    T, k, nq, nkv, d = 6, 2, 4, 2, 16
    rows = T * (k + 1)
    g = np.random.default_rng(3)
    q = store(g.standard_normal((rows, nq, d)).astype(np.float32), dtype)
    kk = store(g.standard_normal((rows, nkv, d)).astype(np.float32), dtype)
    v = store(g.standard_normal((rows, nkv, d)).astype(np.float32), dtype)
    got = ga.group_attention(q, kk, v, T, k, 10000.0, dtype)
    pos = np.array([r // (k + 1) + r % (k + 1) for r in range(rows)], dtype=np.float64)

    def crot(t):       # rotate-half pairs (j, j + d/2) as complex numbers
        z = t[..., : d // 2] + 1j * t[..., d // 2:]
        ang = pos[:, None, None] * (10000.0 ** (-2.0 * np.arange(d // 2) / d))[None, None, :]
        z = z * np.exp(1j * ang)
        return np.concatenate([z.real, z.imag], axis=-1)

    Q = torch.from_numpy(crot(orc.widen(q, dtype))).permute(1, 0, 2)
    K = orc.widen(orc.round_to_storage(crot(orc.widen(kk, dtype)), dtype), dtype)
    K = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(nq // nkv, dim=0)
    V = torch.from_numpy(orc.widen(v, dtype)).permute(1, 0, 2).repeat_interleave(nq // nkv, dim=0)
    mask = torch.from_numpy(ga.group_mask(T, k))
    want = torch.nn.functional.scaled_dot_product_attention(Q, K, V, attn_mask=mask).permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-10)


def _inference_probabilities(shape, w, X, T, k):
    """Attention probabilities of the inference oracle: for every g, one draft step on the prefix x_0..x_g
    (cache: the real rows before x_g; new rows: x_g and the k masks), committing one row per step."""
    wl = tiny_workload(shape, batch=1, kv_len=(0,), n_new=1, k=k)
    inp = inputs.make_step_inputs(wl, slack=T + k)
    kc, vc = inp["k_cache"], inp["v_cache"]
    per_group = []
    for g_ in range(T):
        out = orc.draft_step(shape, w, X[None, g_:g_ + 1], kc, vc, inp["kv_offsets"], np.array([g_]), 1, k, 1, return_attn=True)
        per_group.append(out["attn"][0])                    # [k+1, nq, g + k + 1]
        kc, vc = out["k_cache"], out["v_cache"]
    return per_group


def _training_probabilities(shape, w, X, T, k, mask_fn=None, pos_fn=None, monkeypatch=None):
    dt = shape.dtype
    W = {n: orc.widen(t, dt) for n, t in w.items()}
    Z = np.concatenate([np.concatenate([orc.widen(X[g_:g_ + 1], dt), W["mask_emb"][:k]]) for g_ in range(T)])
    A = orc.rms_norm(Z, W["g_in"], shape.rms_eps)
    rows = T * (k + 1)
    q = (A @ W["wq"].T).reshape(rows, shape.n_heads, shape.head_dim).astype(np.float32)
    kk = (A @ W["wk"].T).reshape(rows, shape.n_kv_heads, shape.head_dim).astype(np.float32)
    v = (A @ W["wv"].T).reshape(rows, shape.n_kv_heads, shape.head_dim).astype(np.float32)
    return ga.group_attention(q, kk, v, T, k, shape.rope_base, "f32", return_probs=True)[1]


def _compare_with_inference(probs_train, per_group, T, k, atol):
    worst = 0.0
    for g_ in range(T):
        for s in range(k + 1):
            i = g_ * (k + 1) + s
            # inference key order: real tokens 0..g-1 from the cache, then this step's rows x_g, m_1..m_s
            cols = [gg * (k + 1) for gg in range(g_)] + [g_ * (k + 1) + ss for ss in range(s + 1)]
            want = per_group[g_][s][:, :g_ + s + 1]
            got = probs_train[i][:, cols]
            worst = max(worst, float(np.abs(got - want).max()))
            others = np.delete(probs_train[i], cols, axis=1)
            assert np.all(others == 0.0)
    return worst


def test_training_rows_see_what_the_same_tokens_see_at_inference(monkeypatch):
    """The property the layout, the mask and the position indices exist for (Section 4.1): the model behaves
    the same in training and evaluation."""
    shape = tiny_shape("f32")
    T, k = 6, 3
    w = inputs.make_weights(shape, 8)
    for n in ("wq", "wk"):
        w[n] = (w[n] * np.float32(8.0)).astype(np.float32)           # far from uniform attention
    X = np.random.default_rng(4).standard_normal((T, shape.hidden)).astype(np.float32)
    per_group = _inference_probabilities(shape, w, X, T, k)
    probs = _training_probabilities(shape, w, X, T, k)
    assert _compare_with_inference(probs, per_group, T, k, 1e-6) < 1e-6     # (float32 storage of q, k, v on one side)
    # planted mistakes: masks of earlier groups visible; positions by layout index
    with monkeypatch.context() as m:
        m.setattr(ga, "group_mask", lambda T_, k_: np.tril(np.ones((T_ * (k_ + 1),) * 2, dtype=bool)))
        bad = _training_probabilities(shape, w, X, T, k)
        worst = 0.0
        for g_ in range(1, T):
            i = g_ * (k + 1)
            worst = max(worst, float(bad[i][:, 1].max()))               # row x_g now attends to m_1 of group 0
        assert worst > 1e-3
    with monkeypatch.context() as m:
        m.setattr(ga, "group_layout", lambda T_, k_: (np.arange(T_ * (k_ + 1)) // (k_ + 1), np.arange(T_ * (k_ + 1)) % (k_ + 1),
                                                     np.arange(T_ * (k_ + 1))))
        bad = _training_probabilities(shape, w, X, T, k)
        cols_ok = True
        try:
            far = _compare_with_inference(bad, per_group, T, k, 1e-6)
        except AssertionError:
            far = 1.0
        assert far > 1e-3


def test_without_masks_it_is_ordinary_causal_attention():
    torch = pytest.importorskip("torch")
    T, nq, d = 9, 2, 8
    g = np.random.default_rng(5)
    q, kk, v = (g.standard_normal((T, nq, d)).astype(np.float32) for _ in range(3))
    got = ga.group_attention(q, kk, v, T, 0, 10000.0, "f32")
    pos = np.arange(T)
    Q = torch.from_numpy(orc.rope(q.astype(np.float64), pos, 10000.0)).permute(1, 0, 2)
    K = torch.from_numpy(orc.rope(kk.astype(np.float64), pos, 10000.0).astype(np.float32).astype(np.float64)).permute(1, 0, 2)
    V = torch.from_numpy(v.astype(np.float64)).permute(1, 0, 2)
    want = torch.nn.functional.scaled_dot_product_attention(Q, K, V, is_causal=True).permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-10)
