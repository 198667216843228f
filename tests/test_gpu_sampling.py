"""GPU parity of the sampling epilogue (temperature, the in-kernel draw, lengths kept on the device) through
the C ABI against the CPU oracle."""
import numpy as np
import pytest
from scipy import stats

from oracle import ps_oracle as orc
from oracle import sampling as smp
from paper_2410_05589_amd import binding as B
from paper_2410_05589_amd import inputs
from paper_2410_05589_amd.configs import WORKLOADS, Workload, small_shape
from tests.gpu_util import compare_with_oracle

pytestmark = pytest.mark.gpu


def _tempered_ref(ref, T, topk):
    """The oracle's step with its distributions re-taken at temperature T (logits stay as they are)."""
    z, lse, p = smp.tempered(ref["logits"], T)
    out = dict(ref, lse=lse, probs=p)
    out["top_p"] = np.take_along_axis(p, ref["top_ids"], axis=-1)
    return out, z


def _run(d, shape, inp, n_new, k, topk, T=0.0, seed=0, sample=True):
    import torch
    dt = shape.dtype
    x, kc, vc = (B.to_device(inp[n], dt) for n in ("x", "k_cache", "v_cache"))
    outs = d.alloc_outputs(len(inp["kv_len"]), n_new, k, topk, logits=True, probs=True, hidden=True, sample=sample)
    for t in outs.values():
        t.fill_(-12345) if t.dtype != torch.int32 else t.fill_(-7)
    a = d.make_args(x, kc, vc, inp["kv_offsets"], inp["kv_len"], n_new, k, topk, outs, temperature=T, sample_seed=seed)
    d.step(a)
    torch.cuda.synchronize()
    res = {n: t.cpu().numpy() for n, t in outs.items()}
    res["k_cache"], res["v_cache"] = B.from_device(kc), B.from_device(vc)
    return res


def _check_draws(res, z, p, seed, logit_tol):
    """The drawn ids: exact wherever the oracle's winner leads by more than what the logits may differ by;
    otherwise the device's choice must be within that of the oracle's best perturbed value."""
    Bn, R, V = z.shape
    exact = 0
    for b in range(Bn):
        for r in range(R):
            m = b * R + r
            best, val, margin = smp.gumbel_sample(z[b, r], seed, m)
            got = int(res["sample_ids"][b, r])
            assert 0 <= got < V
            if margin > 2 * logit_tol:
                assert got == best, (b, r, got, best, margin)
                exact += 1
            else:
                v_got = z[b, r, got] + smp.gumbel(seed, m, np.array([got]))[0]
                assert val - v_got <= 2 * logit_tol
            np.testing.assert_allclose(res["sample_p"][b, r], p[b, r, got], rtol=3e-3, atol=1e-9)
    return exact


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_temperature_and_draws_small_shapes(dtype):
    shape = small_shape(dtype, vocab=2069)
    wl = Workload("smp", shape, batch=3, kv_len=(5, 300, 129), n_new=2, k=5, topk=8, seed=91)
    w = inputs.make_weights(shape, wl.seed)
    inp = inputs.make_step_inputs(wl)
    d = B.Drafter(shape, w, max_batch=3, max_new=2, max_positions=400, max_topk=8, k_max=5)
    ref = orc.draft_step(shape, w, inp["x"], inp["k_cache"], inp["v_cache"], inp["kv_offsets"], inp["kv_len"], 2, 5, 8)
    tol = 2e-4 if dtype == "f32" else 1e-2
    for T, seed in ((0.0, 1), (1.0, 2), (0.7, 3), (1.8, (5 << 32) + 4), (0.05, 5)):
        res = _run(d, shape, inp, 2, 5, 8, T=T, seed=seed)
        Teff = T if T > 0 else 1.0
        rt, z = _tempered_ref(ref, Teff, 8)
        stats_ = compare_with_oracle(shape, res, rt, inp, 2, 5, 8) if Teff >= 0.5 else {}
        exact = _check_draws(res, z, rt["probs"], seed, tol / Teff)
        print("T", T, "seed", seed, stats_, "draws exact", exact, flush=True)
        if Teff >= 0.5:
            assert exact >= 15
    # without sample_ids nothing is drawn, and a draw does not disturb the other outputs
    a = _run(d, shape, inp, 2, 5, 8, T=1.0, seed=9, sample=False)
    b = _run(d, shape, inp, 2, 5, 8, T=1.0, seed=9, sample=True)
    for name in ("logits", "probs", "top_ids", "top_p", "lse"):
        assert np.array_equal(a[name], b[name]), name
    d.close()


def test_draws_on_the_device_follow_the_softmax():
    """Many seeds, one step shape with a small vocabulary: the frequencies of the drawn tokens of a row match
    the row's (tempered) distribution from the oracle."""
    shape = small_shape("f32", hidden=256, n_heads=4, n_kv_heads=4, head_dim=64, ffn=512, vocab=24)
    wl = Workload("smp-freq", shape, batch=1, kv_len=(20,), n_new=1, k=2, topk=4, seed=92)
    w = inputs.make_weights(shape, wl.seed)
    w["w_lm"] = (w["w_lm"] * np.float32(40.0)).astype(np.float32)          # a distribution with some shape to it
    inp = inputs.make_step_inputs(wl)
    d = B.Drafter(shape, w, max_batch=1, max_new=1, max_positions=40, max_topk=4, k_max=2)
    ref = orc.draft_step(shape, w, inp["x"], inp["k_cache"], inp["v_cache"], inp["kv_offsets"], inp["kv_len"], 1, 2, 4)
    T, draws = 1.3, 6000
    _, _, p = smp.tempered(ref["logits"], T)
    counts = np.zeros((3, 24))
    import torch
    x, kc, vc = (B.to_device(inp[n], "f32") for n in ("x", "k_cache", "v_cache"))
    outs = d.alloc_outputs(1, 1, 2, 4, sample=True)
    ids = []
    for s in range(draws):
        d.step(d.make_args(x, kc, vc, inp["kv_offsets"], inp["kv_len"], 1, 2, 4, outs, temperature=T, sample_seed=77000 + s))
        ids.append(outs["sample_ids"].clone())
    torch.cuda.synchronize()
    for t in ids:
        for r, tok in enumerate(t.cpu().numpy()[0]):
            counts[r, tok] += 1
    for r in range(3):
        keep = p[0, r] * draws >= 5
        pv = stats.chisquare(np.append(counts[r][keep], counts[r][~keep].sum()), np.append(p[0, r][keep], p[0, r][~keep].sum()) * draws).pvalue
        print("row", r, "p-value", pv, flush=True)
        assert pv > 1e-4
    d.close()


@pytest.mark.parametrize("name", ["c1", "c4"])
def test_full_size_shapes(name):
    wl = WORKLOADS[name]
    shape = wl.shape
    w = inputs.make_weights(shape, wl.seed)
    inp = inputs.make_step_inputs(wl)
    d = B.Drafter(shape, w, max_batch=1, max_new=wl.n_new, max_positions=wl.kv_len[0] + wl.m, max_topk=8, k_max=wl.k)
    ref = orc.draft_step(shape, w, inp["x"], inp["k_cache"], inp["v_cache"], inp["kv_offsets"], inp["kv_len"], wl.n_new, wl.k, wl.topk)
    for T, seed in ((1.0, 11), (0.8, 12)):
        res = _run(d, shape, inp, wl.n_new, wl.k, wl.topk, T=T, seed=seed)
        rt, z = _tempered_ref(ref, T, wl.topk)
        print(name, "T", T, compare_with_oracle(shape, res, rt, inp, wl.n_new, wl.k, wl.topk),
              "draws exact", _check_draws(res, z, rt["probs"], seed, 1e-2 / T), flush=True)
    d.close()


def test_lengths_on_the_device_let_a_replayed_graph_advance():
    """A step captured once with kv_len_dev: between replays the caller commits n_new rows by adding to the
    lengths in device memory and writes new inputs; every replay matches the oracle's step at the current
    lengths, eager steps with plain host lengths in between included."""
    import torch
    shape = small_shape("bf16", vocab=2069)
    n_new, k, topk = 2, 4, 8
    wl = Workload("kvdev", shape, batch=2, kv_len=(100, 250), n_new=n_new, k=k, topk=topk, seed=93)
    w = inputs.make_weights(shape, wl.seed)
    rounds = 6
    inp = inputs.make_step_inputs(wl, slack=n_new * rounds + 8)
    bound = np.asarray(inp["kv_len"]) + n_new * rounds          # where the lengths may get to
    d = B.Drafter(shape, w, max_batch=2, max_new=n_new, max_positions=int(bound.max()) + n_new + k, max_topk=topk, k_max=k)
    dt = shape.dtype
    x, kc, vc = (B.to_device(inp[n], dt) for n in ("x", "k_cache", "v_cache"))
    lens = torch.from_numpy(np.asarray(inp["kv_len"], dtype=np.int32)).to("cuda:0")
    outs = d.alloc_outputs(2, n_new, k, topk, logits=True, probs=True, hidden=True)
    args = d.make_args(x, kc, vc, inp["kv_offsets"], bound, n_new, k, topk, outs, kv_len_dev=lens)
    d.step(args)                                                # eager once (also resolves anything lazy), at the start lengths
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            d.step(args, stream=side)
    torch.cuda.synchronize()
    kc_o, vc_o = inp["k_cache"], inp["v_cache"]
    cur = np.asarray(inp["kv_len"], dtype=np.int32).copy()
    g = np.random.default_rng(3)
    for rnd in range(rounds):
        xs = inputs.f32_to_bf16_bits(g.standard_normal((2, n_new, shape.hidden)).astype(np.float32))
        x.copy_(B.to_device(xs, dt)); kc.copy_(B.to_device(kc_o, dt)); vc.copy_(B.to_device(vc_o, dt))
        lens.copy_(torch.from_numpy(cur))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        res = {n: t.cpu().numpy() for n, t in outs.items()}
        res["k_cache"], res["v_cache"] = B.from_device(kc), B.from_device(vc)
        step_inp = dict(inp, x=xs, k_cache=kc_o, v_cache=vc_o, kv_len=cur.copy())
        ref = orc.draft_step(shape, w, xs, kc_o, vc_o, inp["kv_offsets"], cur, n_new, k, topk)
        print("replay", rnd, "lengths", cur.tolist(), compare_with_oracle(shape, res, ref, step_inp, n_new, k, topk), flush=True)
        kc_o, vc_o = ref["k_cache"], ref["v_cache"]             # commit the n_new real rows
        cur += n_new
    assert d.last_status() == B.PS_OK
    d.close()
