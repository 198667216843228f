"""Pins of the input-stage oracle (Section 4.3): each check compares it with something it does not contain."""
import numpy as np
import pytest

from oracle import input_stage as ist
from oracle import ps_oracle as orc
from paper_2410_05589_amd import inputs
from tests.helpers import tiny_shape, tiny_workload, store


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gather_is_indexing_the_embedding_matrix(dtype):
    shape = tiny_shape(dtype)
    w = inputs.make_input_stage_weights(shape, 3)
    ids = np.array([[0, 49, 7], [7, 7, 1]], dtype=np.int32)
    got = ist.embed_tokens(w["embed"], ids)
    assert got.dtype == w["embed"].dtype
    assert np.array_equal(got, w["embed"][ids])            # numpy fancy indexing, the library's gather
    assert np.array_equal(got[1, 0], got[0, 2])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("bias", [False, True])
def test_projection_is_the_library_linear_on_the_concatenation(dtype, bias):
    torch = pytest.importorskip("torch")
    shape = tiny_shape(dtype)
    wl = tiny_workload(shape, batch=2, kv_len=(5, 9), n_new=3, k=2)
    w = inputs.make_input_stage_weights(shape, 5, bias=bias)
    inp = inputs.make_input_stage_inputs(wl)
    got = ist.fused_input(inp["features"], w["embed"], inp["token_ids"], w["w_fc"], w.get("b_fc"), dtype)
    f = torch.from_numpy(orc.widen(inp["features"], dtype))
    e = torch.from_numpy(orc.widen(w["embed"], dtype))[torch.from_numpy(inp["token_ids"].astype(np.int64))]
    b = torch.from_numpy(orc.widen(w["b_fc"], dtype)) if bias else None
    want = torch.nn.functional.linear(torch.cat([f, e], dim=-1), torch.from_numpy(orc.widen(w["w_fc"], dtype)), b)
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-12, atol=1e-12)
    # the same as two separate products: the left half of w_fc sees the feature, the right half the embedding
    W = orc.widen(w["w_fc"], dtype)
    H = shape.hidden
    two = f.numpy() @ W[:, :H].T + e.numpy() @ W[:, H:].T + (b.numpy() if bias else 0.0)
    np.testing.assert_allclose(got, two, rtol=1e-12, atol=1e-12)


def test_one_hot_inputs_select_columns_of_the_projection():
    shape = tiny_shape("f32")
    H, V = shape.hidden, shape.vocab
    g = np.random.default_rng(0)
    w_fc = g.standard_normal((H, 2 * H)).astype(np.float32)
    embed = np.zeros((V, H), dtype=np.float32)
    embed[np.arange(V), np.arange(V) % H] = 1.0               # token t's embedding = unit vector t mod H
    feats = np.zeros((1, 2, H), dtype=np.float32)
    feats[0, 0, 3] = 1.0                                      # position 0: feature e_3; position 1: zero feature
    ids = np.array([[5, 9]], dtype=np.int32)
    out = ist.fused_input(feats, embed, ids, w_fc, None, "f32")
    np.testing.assert_array_equal(out[0, 0], w_fc[:, 3].astype(np.float64) + w_fc[:, H + 5].astype(np.float64))
    np.testing.assert_array_equal(out[0, 1], w_fc[:, H + 9].astype(np.float64))   # a swapped (e, f) order would pick column 9


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_the_three_input_modes_reduce_to_each_other(dtype):
    """w_fc = [0 | I] makes the projection return the embedding, so the fused mode equals the token mode; and
    the token mode is the hidden-state mode of the draft step fed with the gathered rows, bit for bit."""
    shape = tiny_shape(dtype)
    wl = tiny_workload(shape, batch=2, kv_len=(6, 3), n_new=2, k=3, topk=3)
    w = inputs.make_weights(shape, wl.seed)
    ws = inputs.make_input_stage_weights(shape, wl.seed, fc=False)
    inp = inputs.make_step_inputs(wl)
    tin = inputs.make_input_stage_inputs(wl)
    H = shape.hidden
    x_tok = ist.embed_tokens(ws["embed"], tin["token_ids"])
    ref = orc.draft_step(shape, w, x_tok, inp["k_cache"], inp["v_cache"], inp["kv_offsets"], inp["kv_len"], 2, 3, 3)
    w_fc = store(np.concatenate([np.zeros((H, H)), np.eye(H)], axis=1).astype(np.float32), dtype)
    x_fused = ist.fused_input(tin["features"], ws["embed"], tin["token_ids"], w_fc, None, dtype)
    assert np.array_equal(x_fused, orc.widen(x_tok, dtype))
    out = orc.draft_step(shape, w, x_fused, inp["k_cache"], inp["v_cache"], inp["kv_offsets"], inp["kv_len"], 2, 3, 3,
                         x_is_float=True)
    for name in ("logits", "hidden_out", "top_ids", "k_cache", "v_cache"):
        assert np.array_equal(out[name], ref[name]), name
    # and a feature that matters changes the result (the left half of w_fc is live)
    w_fc2 = store(np.concatenate([0.5 * np.eye(H), np.eye(H)], axis=1).astype(np.float32), dtype)
    x2 = ist.fused_input(tin["features"], ws["embed"], tin["token_ids"], w_fc2, None, dtype)
    np.testing.assert_allclose(x2, orc.widen(x_tok, dtype) + 0.5 * orc.widen(tin["features"], dtype), rtol=0, atol=1e-12)
