"""GPU parity of the input stage fused into the draft step (Section 4.3): token ids instead of hidden states
(embedding gather), and token ids + target features through the fully connected layer, through the C ABI
against the CPU oracle, at small shapes with ragged tails and at the c1 / c4 shapes."""
import numpy as np
import pytest

from oracle import input_stage as ist
from paper_2410_05589_amd import binding as B
from paper_2410_05589_amd import inputs
from paper_2410_05589_amd.configs import WORKLOADS, Workload, small_shape
from tests.gpu_util import compare_with_oracle
from oracle import ps_oracle as orc

pytestmark = pytest.mark.gpu


def _step(d, shape, inp, tin, n_new, k, topk, mode, n_new_seq=None):
    import torch
    dt = shape.dtype
    kc, vc = B.to_device(inp["k_cache"], dt), B.to_device(inp["v_cache"], dt)
    outs = d.alloc_outputs(len(inp["kv_len"]), n_new, k, topk, logits=True, probs=True, hidden=True)
    for t in outs.values():
        t.fill_(-12345) if t.dtype != torch.int32 else t.fill_(-7)
    tok = torch.from_numpy(tin["token_ids"]).to("cuda:0") if mode != "hidden" else None
    feat = B.to_device(tin["features"], dt) if mode == "fused" else None
    x = B.to_device(inp["x"], dt) if mode == "hidden" else None
    a = d.make_args(x, kc, vc, inp["kv_offsets"], inp["kv_len"], n_new, k, topk, outs, token_ids=tok, features=feat,
                    n_new_seq=n_new_seq)
    d.step(a)
    torch.cuda.synchronize()
    res = {n: t.cpu().numpy() for n, t in outs.items()}
    res["k_cache"], res["v_cache"] = B.from_device(kc), B.from_device(vc)
    return res


def _case(wl, n_new=None, label="", bias=True, modes=("tokens", "fused", "hidden", "fused", "tokens")):
    shape = wl.shape
    n_new = wl.n_new if n_new is None else n_new
    print("case", label or wl.name, "H", shape.hidden, "V", shape.vocab, "batch", wl.batch, "n_new", n_new, "k", wl.k, flush=True)
    w = inputs.make_weights(shape, wl.seed)
    w.update(inputs.make_input_stage_weights(shape, wl.seed, bias=bias))
    inp = inputs.make_step_inputs(wl, n_new=n_new)
    tin = inputs.make_input_stage_inputs(wl, n_new=n_new)
    d = B.Drafter(shape, w, max_batch=wl.batch, max_new=n_new, max_positions=int(max(inp["kv_len"])) + n_new + wl.k,
                  max_topk=8, k_max=wl.k)
    x_tok = ist.embed_tokens(w["embed"], tin["token_ids"])
    x_fused = ist.fused_input(tin["features"], w["embed"], tin["token_ids"], w["w_fc"], w.get("b_fc"), shape.dtype)
    refs = {
        "hidden": orc.draft_step(shape, w, inp["x"], inp["k_cache"], inp["v_cache"], inp["kv_offsets"], inp["kv_len"], n_new, wl.k, wl.topk),
        "tokens": orc.draft_step(shape, w, x_tok, inp["k_cache"], inp["v_cache"], inp["kv_offsets"], inp["kv_len"], n_new, wl.k, wl.topk),
        "fused": orc.draft_step(shape, w, x_fused, inp["k_cache"], inp["v_cache"], inp["kv_offsets"], inp["kv_len"], n_new, wl.k, wl.topk,
                                x_is_float=True),
    }
    for mode in modes:     # the modes take turns on one context
        res = _step(d, shape, inp, tin, n_new, wl.k, wl.topk, mode)
        print("   ", mode, compare_with_oracle(shape, res, refs[mode], inp, n_new, wl.k, wl.topk), flush=True)
    assert d.last_status() == B.PS_OK
    d.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_shapes(dtype):
    shape = small_shape(dtype, vocab=2069)
    _case(Workload("in-small", shape, batch=1, kv_len=(200,), n_new=2, k=5, topk=8, seed=81))
    _case(Workload("in-batch", shape, batch=3, kv_len=(5, 300, 129), n_new=3, k=4, topk=5, seed=82), bias=False)
    _case(Workload("in-k0", shape, batch=2, kv_len=(0, 64), n_new=1, k=0, topk=1, seed=83), label="k = 0, empty cache")


def test_many_rows_bf16():
    # 8 sequences x 6 real rows: three column tiles in the input projection as well
    shape = small_shape("bf16", hidden=1024, n_heads=8, n_kv_heads=8, head_dim=128, ffn=2752, vocab=4000)
    _case(Workload("in-rows", shape, batch=8, kv_len=(128, 700, 77, 130, 1, 500, 300, 64), n_new=6, k=2, topk=8, seed=84),
          modes=("fused", "tokens"))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sequences_with_different_accepted_lengths(dtype):
    """n_new_seq with token ids (and features): the token ids of the slots a sequence does not use are never
    looked up (they are far outside the table here) and their features (huge here) leak nowhere.  Every sequence
    against the oracle's step of that sequence alone."""
    shape = small_shape(dtype, vocab=2069)
    n_new, k, topk = 3, 4, 5
    kv, nseq = (5, 300, 129, 0), (2, 1, 3, 1)
    wl = Workload("in-ragged", shape, batch=len(kv), kv_len=kv, n_new=n_new, k=k, topk=topk, seed=86)
    w = inputs.make_weights(shape, wl.seed)
    w.update(inputs.make_input_stage_weights(shape, wl.seed))
    inp = inputs.make_step_inputs(wl)
    tin = inputs.make_input_stage_inputs(wl)
    tok, feat = tin["token_ids"].copy(), tin["features"].copy()
    for b, nb in enumerate(nseq):
        tok[b, :n_new - nb] = 2 ** 30
        feat[b, :n_new - nb] = inputs.f32_to_bf16_bits(np.full((1, shape.hidden), 3.0e4, np.float32)) if dtype == "bf16" else 3.0e4
    bad = dict(tin, token_ids=tok, features=feat)
    d = B.Drafter(shape, w, max_batch=len(kv), max_new=n_new, max_positions=max(kv) + n_new + k, max_topk=8, k_max=k)
    off = inp["kv_offsets"]
    for mode in ("tokens", "fused", "tokens"):
        res = _step(d, shape, inp, bad, n_new, k, topk, mode, n_new_seq=np.array(nseq, dtype=np.int32))
        for b, nb in enumerate(nseq):
            t_b = tin["token_ids"][b:b + 1, n_new - nb:]
            if mode == "tokens":
                x_b, is_float = ist.embed_tokens(w["embed"], t_b), False
            else:
                x_b, is_float = ist.fused_input(tin["features"][b:b + 1, n_new - nb:], w["embed"], t_b, w["w_fc"], w.get("b_fc"), shape.dtype), True
            one = dict(k_cache=inp["k_cache"][off[b]:off[b + 1]], v_cache=inp["v_cache"][off[b]:off[b + 1]],
                       kv_offsets=np.array([0, off[b + 1] - off[b]], dtype=np.int64), kv_len=inp["kv_len"][b:b + 1])
            ref = orc.draft_step(shape, w, x_b, one["k_cache"], one["v_cache"], one["kv_offsets"], one["kv_len"], nb, k, topk,
                                 x_is_float=is_float)
            got = {n: res[n][b:b + 1] for n in ("top_ids", "top_p", "lse", "logits", "probs")}
            got["hidden_out"] = res["hidden_out"][b:b + 1, n_new - nb:]
            got["k_cache"], got["v_cache"] = res["k_cache"][off[b]:off[b + 1]], res["v_cache"][off[b]:off[b + 1]]
            print(mode, "sequence", b, "n_new", nb, compare_with_oracle(shape, got, ref, one, nb, k, topk), flush=True)
    assert d.last_status() == B.PS_OK
    d.close()


@pytest.mark.parametrize("name", ["c1", "c4"])
def test_full_size_shapes(name):
    _case(WORKLOADS[name], modes=("tokens", "fused"))


def test_argument_errors():
    import torch
    shape = small_shape("bf16")
    wl = Workload("in-err", shape, batch=1, kv_len=(10,), n_new=1, k=2, topk=4, seed=85)
    w = inputs.make_weights(shape, wl.seed)
    inp = inputs.make_step_inputs(wl)
    tin = inputs.make_input_stage_inputs(wl)
    d = B.Drafter(shape, w, max_batch=1, max_new=1, max_positions=20, max_topk=4, k_max=2)     # no embedding table, no projection
    dt = shape.dtype
    x, kc, vc = (B.to_device(inp[n], dt) for n in ("x", "k_cache", "v_cache"))
    tok = torch.from_numpy(tin["token_ids"]).to("cuda:0")
    feat = B.to_device(tin["features"], dt)
    outs = d.alloc_outputs(1, 1, 2, 4)
    st = lambda **kw: B.ps_draft_step(d.ctx, d.make_args(kw.get("x"), kc, vc, inp["kv_offsets"], inp["kv_len"], 1, 2, 4, outs,
                                                           token_ids=kw.get("tok"), features=kw.get("feat")), None)
    assert st() == B.PS_ERR_NULL                               # neither x nor token ids
    assert st(x=x, tok=tok) == B.PS_ERR_SHAPE                  # both
    assert st(tok=tok) == B.PS_ERR_NULL                        # token ids without an embedding table
    assert st(x=x, feat=feat) == B.PS_ERR_SHAPE                # features without token ids
    d.close()
    w.update(inputs.make_input_stage_weights(shape, wl.seed, fc=False))
    d = B.Drafter(shape, w, max_batch=1, max_new=1, max_positions=20, max_topk=4, k_max=2)     # table, but no projection
    st = lambda **kw: B.ps_draft_step(d.ctx, d.make_args(kw.get("x"), kc, vc, inp["kv_offsets"], inp["kv_len"], 1, 2, 4, outs,
                                                           token_ids=kw.get("tok"), features=kw.get("feat")), None)
    assert st(tok=tok) == B.PS_OK
    assert st(tok=tok, feat=feat) == B.PS_ERR_SHAPE            # the configuration has no input projection
    torch.cuda.synchronize()
    d.close()
