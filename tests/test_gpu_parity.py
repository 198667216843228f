"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Tolerances (stated by the benchmark definition): token ids bit-exact wherever the oracle's
logit gaps exceed 1e-3; logits within max-abs 1e-4 (f32) or 2e-2 relative to max |logit|
(bf16).  The tests additionally require the logit error to stay below half the id gap,
which is what makes the id guarantee hold.
"""
import ctypes

import numpy as np
import pytest

from paper_2410_05589_amd import binding as B
from paper_2410_05589_amd import inputs
from paper_2410_05589_amd.configs import WORKLOADS, DrafterShape, Workload, small_shape
from tests.gpu_util import run_gpu_step, compare_with_oracle, oracle_step

pytestmark = pytest.mark.gpu


def _drafter(shape, w, max_batch, max_new, max_positions, max_topk=8, k_max=None):
    return B.Drafter(shape, w, max_batch=max_batch, max_new=max_new, max_positions=max_positions,
                     max_topk=max_topk, k_max=k_max)


def _run_case(wl, kv_len=None, n_new=None, k=None, topk=None, all_rows=False, label=""):
    shape = wl.shape
    n_new = wl.n_new if n_new is None else n_new
    k = wl.k if k is None else k
    topk = wl.topk if topk is None else topk
    print("case", label or wl.name, "dtype", shape.dtype, "H", shape.hidden, "V", shape.vocab, "n_new", n_new,
          "k", k, "kv_len", kv_len, flush=True)
    w = inputs.make_weights(shape, wl.seed)
    inp = inputs.make_step_inputs(wl, kv_len=kv_len, n_new=n_new, k=k)
    d = _drafter(shape, w, max_batch=len(inp["kv_len"]), max_new=n_new,
                 max_positions=int(max(inp["kv_len"])) + n_new + k, max_topk=max(8, topk), k_max=k)
    res = run_gpu_step(d, inp, n_new, k, topk, all_rows=all_rows)
    ref = oracle_step(shape, w, inp, n_new, k, topk, all_rows=all_rows)
    stats = compare_with_oracle(shape, res, ref, inp, n_new, k, topk)
    print("   ", stats, flush=True)
    d.close()
    return stats


def test_c0_tiny_f32():
    _run_case(WORKLOADS["c0"])
    _run_case(WORKLOADS["c0"], all_rows=True, label="c0 all rows")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_shapes_several_tiles_and_ragged_tails(dtype):
    # vocab 2064 + 5 is not a multiple of the 16-row tile; ffn 1376 = 172 gate/up tiles; KV lengths
    # straddle the attention chunk size
    shape = small_shape(dtype, vocab=2069)
    wl = Workload("small", shape, batch=1, kv_len=(200,), n_new=2, k=5, topk=8, seed=21)
    _run_case(wl)
    _run_case(wl, kv_len=(127,), n_new=1, k=0, topk=1, label="k=0 ordinary decode step")
    _run_case(wl, kv_len=(0,), n_new=3, k=4, label="empty cache")
    _run_case(wl, kv_len=(128,), n_new=6, k=5, all_rows=True, label="chunk boundary, all rows")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gqa_head_dim_128_and_batch(dtype):
    shape = small_shape(dtype, hidden=512, n_heads=4, n_kv_heads=2, head_dim=128, ffn=1024, vocab=1000)
    wl = Workload("gqa", shape, batch=3, kv_len=(5, 300, 129), n_new=2, k=3, topk=5, seed=22)
    _run_case(wl)
    _run_case(wl, kv_len=(70,), n_new=1, k=8, label="k = k_max")


def test_ragged_batch_many_rows_bf16():
    # 8 sequences x 6 rows = 48 activation rows (three MFMA column tiles), ragged KV
    shape = small_shape("bf16", hidden=1024, n_heads=8, n_kv_heads=8, head_dim=128, ffn=2752, vocab=4000)
    wl = Workload("ragged", shape, batch=8, kv_len=(128, 2048, 777, 130, 1, 1500, 300, 64), n_new=1, k=5,
                  topk=8, seed=23)
    _run_case(wl)


@pytest.mark.parametrize("plan", [
    "qkv:1:1,oproj:1:1,gateup:1:1,down:1:1,lm:1:1",
    "qkv:1:8,oproj:2:4,gateup:4:2,down:8:1,lm:1:8",
    "qkv:1:4,oproj:4:2,gateup:2:4,down:2:2,lm:1:2",
    "qkv:1:2,oproj:8:1,gateup:8:1,down:4:2,lm:1:4",
])
def test_every_k_split_of_the_gemm_engine(plan, monkeypatch):
    """The way a phase's contraction dimension is shared (K-slices across workgroups x wavefronts per
    tile) is normally chosen by the library; PS_DRAFT_PLAN forces other splits, all of which must
    give the same results.  One and three MFMA column tiles."""
    monkeypatch.setenv("PS_DRAFT_PLAN", plan)
    shape = small_shape("bf16", hidden=1024, n_heads=8, n_kv_heads=4, head_dim=128, ffn=2752, vocab=4000)
    wl = Workload("plans", shape, batch=1, kv_len=(300,), n_new=1, k=5, topk=8, seed=31)
    _run_case(wl, label="plan " + plan)
    wl3 = Workload("plans3", shape, batch=7, kv_len=(5, 130, 64, 700, 0, 256, 33), n_new=2, k=4, topk=8, seed=32)
    _run_case(wl3, label="plan " + plan + " (42 rows)")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_new_rows_left_to_the_merge_items(dtype):
    """float32 kernels: when this step's rows alone would make up one more key block per sequence and that
    block would cost the workgroups a second round of attention work items (more items than compute units),
    the merge items take these rows instead.  8 sequences x 8 kv heads, KV lengths that are multiples of the
    block size (one of them 0): 256 block items instead of 320.  (The bf16 kernels always let the rows ride
    on the last block of cache keys: the same shapes, an empty cache among them.)"""
    shape = small_shape(dtype, hidden=1024, n_heads=8, n_kv_heads=8, head_dim=128, ffn=1376, vocab=2000)
    wl = Workload("sep", shape, batch=8, kv_len=(0, 1024, 512, 512, 512, 512, 512, 512), n_new=1, k=5, topk=8, seed=33)
    _run_case(wl)
    # grouped queries: 2 query heads per kv head, 9 rows -> 18 query rows per kv head (two passes of 16)
    shape2 = small_shape(dtype, hidden=1024, n_heads=16, n_kv_heads=8, head_dim=64, ffn=1376, vocab=2000)
    wl2 = Workload("sep gqa", shape2, batch=4, kv_len=(1024,) * 4, n_new=1, k=8, topk=8, seed=34)
    _run_case(wl2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_key_blocks_of_twice_the_size(dtype):
    """float32 kernels: more attention work items than compute units with 128-key blocks, no more than that
    with 256-key blocks: every wavefront then takes two groups of 16 keys.  One pass of query rows, and two
    (GQA).  (bf16 kernels: the host picks blocks of 128 .. 2048 keys; several blocks per sequence here.)"""
    shape = small_shape(dtype, hidden=1024, n_heads=8, n_kv_heads=8, head_dim=128, ffn=1376, vocab=2000)
    wl = Workload("nk2", shape, batch=8, kv_len=(600, 513, 700, 640, 520, 767, 600, 650), n_new=1, k=5, topk=8, seed=37)
    _run_case(wl)
    shape2 = small_shape(dtype, hidden=1024, n_heads=16, n_kv_heads=8, head_dim=64, ffn=1376, vocab=2000)
    wl2 = Workload("nk2 gqa", shape2, batch=7, kv_len=(600, 513, 700, 640, 520, 767, 600), n_new=1, k=8, topk=8, seed=38)
    _run_case(wl2)


def test_two_contexts_take_turns_on_one_stream():
    """Two drafters of different shape and type (own workspaces, own step counters) stepping alternately."""
    shape_a = small_shape("bf16", hidden=512, n_heads=4, n_kv_heads=4, head_dim=128, ffn=1024, vocab=3001)
    shape_b = small_shape("f32", vocab=1500)
    wl_a = Workload("ctx a", shape_a, batch=2, kv_len=(150, 31), n_new=2, k=4, topk=8, seed=35)
    wl_b = Workload("ctx b", shape_b, batch=1, kv_len=(77,), n_new=1, k=5, topk=4, seed=36)
    wa, wb = inputs.make_weights(shape_a, wl_a.seed), inputs.make_weights(shape_b, wl_b.seed)
    da = _drafter(shape_a, wa, max_batch=2, max_new=2, max_positions=200, k_max=4)
    db = _drafter(shape_b, wb, max_batch=1, max_new=1, max_positions=100, k_max=5)
    for rep in range(3):
        inp_a = inputs.make_step_inputs(Workload("ctx a", shape_a, batch=2, kv_len=(150, 31), n_new=2, k=4, topk=8, seed=40 + rep))
        inp_b = inputs.make_step_inputs(Workload("ctx b", shape_b, batch=1, kv_len=(77,), n_new=1, k=5, topk=4, seed=50 + rep))
        res_a = run_gpu_step(da, inp_a, 2, 4, 8)
        res_b = run_gpu_step(db, inp_b, 1, 5, 4)
        compare_with_oracle(shape_a, res_a, oracle_step(shape_a, wa, inp_a, 2, 4, 8), inp_a, 2, 4, 8)
        compare_with_oracle(shape_b, res_b, oracle_step(shape_b, wb, inp_b, 1, 5, 4), inp_b, 1, 5, 4)
    da.close()
    db.close()


def test_changing_shapes_on_one_context():
    """Row layout, column tiles and K-slice plan change from step to step on ONE context: exchange-buffer
    slots a step does not write must never look written to a later step (two alternating copies)."""
    shape = small_shape("bf16", hidden=1024, n_heads=8, n_kv_heads=8, head_dim=128, ffn=2752, vocab=2069)
    w = inputs.make_weights(shape, 31)
    d = _drafter(shape, w, max_batch=8, max_new=3, max_positions=700, k_max=5)
    seq = [(1, 1, 5, (100,)), (8, 1, 5, (128, 600, 77, 130, 1, 500, 300, 64)), (1, 1, 5, (100,)), (3, 2, 5, (5, 300, 129)),
           (3, 2, 5, (5, 300, 129)), (8, 3, 5, (30, 31, 32, 33, 34, 35, 36, 37)), (2, 1, 0, (64, 65)), (1, 1, 5, (100,)),
           (1, 3, 2, (257,)), (1, 1, 5, (100,))]
    for step, (batch, n_new, k, kv) in enumerate(seq):
        wl = Workload("shapes", shape, batch=batch, kv_len=kv, n_new=n_new, k=k, topk=4, seed=100 + step)
        inp = inputs.make_step_inputs(wl, kv_len=kv, n_new=n_new, k=k)
        res = run_gpu_step(d, inp, n_new, k, 4)
        ref = oracle_step(shape, w, inp, n_new, k, 4)
        print("step", step, (batch, n_new, k), compare_with_oracle(shape, res, ref, inp, n_new, k, 4), flush=True)
    d.close()


def test_maximum_rows_and_topk():
    # 8 sequences x 8 rows = 64 activation rows (the most the library takes), top-32, all rows decoded
    shape = small_shape("bf16", hidden=512, n_heads=8, n_kv_heads=4, head_dim=64, ffn=1376, vocab=3000)
    wl = Workload("maxrows", shape, batch=8, kv_len=(9, 200, 63, 64, 65, 0, 127, 129), n_new=3, k=5, topk=32, seed=32)
    _run_case(wl)
    _run_case(wl, all_rows=True, topk=1, label="64 rows, all decoded, top-1")


@pytest.mark.parametrize("dtype,nk", [("f32", None), ("bf16", None), ("bf16", "1")])
def test_very_long_sequence_many_key_blocks(dtype, nk, monkeypatch):
    # 33000 keys = 258 attention blocks of 128 keys (the float32 kernels' size; the bf16 kernels' when forced):
    # more than one group of 256 blocks in the combination pass; bf16 by itself: 17 blocks of 2048 keys
    if nk:
        monkeypatch.setenv("PS_DRAFT_ATTN_NK", nk)
    shape = small_shape(dtype, hidden=256, n_heads=4, n_kv_heads=2, head_dim=64, ffn=704, vocab=1024)
    wl = Workload("long", shape, batch=2, kv_len=(33000, 2100), n_new=1, k=4, topk=4, seed=33)
    _run_case(wl)


@pytest.mark.parametrize("nk", ["1", "2", "4", "8", "16"])
def test_every_block_size_of_the_bf16_attention(nk, monkeypatch):
    """The bf16 attention works on blocks of 128 NK cache keys per work unit (NK groups of 16 keys per wavefront,
    two at a time); the library picks NK, PS_DRAFT_ATTN_NK forces it.  Ragged batch with an empty cache, lengths
    around the block sizes and a long sequence; one pass of query rows (head_dim 128), then three passes (GQA, 4
    query heads per kv head x 9 rows, head_dim 64) and rows of the step spilling into a second group of 16 (17 rows)."""
    monkeypatch.setenv("PS_DRAFT_ATTN_NK", nk)
    shape = small_shape("bf16", hidden=512, n_heads=4, n_kv_heads=4, head_dim=128, ffn=1024, vocab=1000)
    wl = Workload("blocks", shape, batch=7, kv_len=(0, 1, 127, 128, 129, 2049, 700), n_new=1, k=5, topk=4, seed=61)
    _run_case(wl, label="NK " + nk)
    shape2 = small_shape("bf16", hidden=512, n_heads=8, n_kv_heads=2, head_dim=64, ffn=1024, vocab=1000)
    wl2 = Workload("blocks gqa", shape2, batch=3, kv_len=(15, 300, 4100), n_new=1, k=8, topk=4, seed=62)
    _run_case(wl2, label="NK " + nk + " (three passes)")
    shape3 = small_shape("bf16", hidden=512, n_heads=4, n_kv_heads=2, head_dim=64, ffn=1024, vocab=1000)
    wl3 = Workload("blocks 17 rows", shape3, batch=2, kv_len=(250, 31), n_new=9, k=8, topk=4, seed=63)
    _run_case(wl3, label="NK " + nk + " (17 rows per sequence)")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sequences_with_different_accepted_lengths(dtype):
    """n_new_seq: the sequences of one batch accepted 1 .. n_new tokens each (Section 3: a verification round yields
    1..gamma+1 tokens per sequence).  Sequence b uses the last n_new_seq[b] of its n_new slots; the slots in front
    hold huge values here, which must not leak anywhere.  Every sequence is compared with the oracle's step of
    that sequence alone with its own n_new (the oracle pins batch == each sequence alone): outputs, hidden rows,
    the cache rows written and the ones left alone.  Several key blocks, an empty cache, grouped queries."""
    shape = small_shape(dtype, hidden=512, n_heads=8, n_kv_heads=4, head_dim=64, ffn=1024, vocab=1500)
    n_new, k, topk = 4, 3, 4
    kv = (300, 0, 129, 17, 640)
    nseq = (1, 4, 2, 3, 1)
    wl = Workload("ragged n_new", shape, batch=len(kv), kv_len=kv, n_new=n_new, k=k, topk=topk, seed=71)
    w = inputs.make_weights(shape, wl.seed)
    inp = inputs.make_step_inputs(wl)
    x = inp["x"].copy()
    for b, nb in enumerate(nseq):      # poison the unused slots (finite: the interface asks for finite inputs)
        x[b, :n_new - nb] = inputs.f32_to_bf16_bits(np.full((1, shape.hidden), 3.0e4, np.float32)) if dtype == "bf16" else 3.0e4
    inp = dict(inp, x=x)
    d = _drafter(shape, w, max_batch=len(kv), max_new=n_new, max_positions=max(kv) + n_new + k, k_max=k)
    res = run_gpu_step(d, inp, n_new, k, topk, n_new_seq=np.array(nseq, dtype=np.int32))
    off = inp["kv_offsets"]
    for b, nb in enumerate(nseq):
        one = dict(x=inp["x"][b:b + 1, n_new - nb:], k_cache=inp["k_cache"][off[b]:off[b + 1]], v_cache=inp["v_cache"][off[b]:off[b + 1]],
                   kv_offsets=np.array([0, off[b + 1] - off[b]], dtype=np.int64), kv_len=inp["kv_len"][b:b + 1])
        ref = oracle_step(shape, w, one, nb, k, topk)
        got = {n: res[n][b:b + 1] for n in ("top_ids", "top_p", "lse", "logits", "probs")}
        got["hidden_out"] = res["hidden_out"][b:b + 1, n_new - nb:]
        got["k_cache"], got["v_cache"] = res["k_cache"][off[b]:off[b + 1]], res["v_cache"][off[b]:off[b + 1]]
        print("sequence", b, "n_new", nb, compare_with_oracle(shape, got, ref, one, nb, k, topk), flush=True)
    d.close()


def test_rounds_of_a_batch_whose_sequences_accept_different_lengths():
    """Three rounds of drafting for three sequences that accept different numbers of tokens each round (n_new_seq),
    committed by advancing every sequence's length by what it accepted: the [MASK] rows of a round are overwritten
    by the next, positions continue per sequence.  After every round each sequence is compared with the oracle run
    on that sequence alone from the oracle's own caches of the round before."""
    shape = small_shape("bf16", hidden=512, n_heads=8, n_kv_heads=4, head_dim=64, ffn=1024, vocab=1500)
    n_max, k, topk = 4, 3, 4
    kv0 = (120, 0, 33)
    wl = Workload("ragged rounds", shape, batch=3, kv_len=kv0, n_new=n_max, k=k, topk=topk, seed=72)
    w = inputs.make_weights(shape, wl.seed)
    inp = inputs.make_step_inputs(wl, slack=16)
    off = inp["kv_offsets"]
    d = _drafter(shape, w, max_batch=3, max_new=n_max, max_positions=max(kv0) + 16 + n_max + k, k_max=k)
    kc_g, vc_g = inp["k_cache"], inp["v_cache"]
    kc_o = [inp["k_cache"][off[b]:off[b + 1]] for b in range(3)]
    vc_o = [inp["v_cache"][off[b]:off[b + 1]] for b in range(3)]
    L = np.array(kv0, dtype=np.int32)
    g = np.random.default_rng(6)
    for rnd, acc in enumerate([(1, 4, 2), (3, 1, 4), (2, 2, 1)]):
        x = inputs.f32_to_bf16_bits(g.standard_normal((3, n_max, shape.hidden)).astype(np.float32))
        cur = dict(inp, x=x, k_cache=kc_g, v_cache=vc_g, kv_len=L.copy())
        res = run_gpu_step(d, cur, n_max, k, topk, n_new_seq=np.array(acc, dtype=np.int32))
        for b, nb in enumerate(acc):
            one = dict(x=x[b:b + 1, n_max - nb:], k_cache=kc_o[b], v_cache=vc_o[b],
                       kv_offsets=np.array([0, off[b + 1] - off[b]], dtype=np.int64), kv_len=L[b:b + 1].copy())
            ref = oracle_step(shape, w, one, nb, k, topk)
            got = {n: res[n][b:b + 1] for n in ("top_ids", "top_p", "lse", "logits", "probs")}
            got["hidden_out"] = res["hidden_out"][b:b + 1, n_max - nb:]
            got["k_cache"], got["v_cache"] = res["k_cache"][off[b]:off[b + 1]], res["v_cache"][off[b]:off[b + 1]]
            print("round", rnd, "sequence", b, "accepted", nb, compare_with_oracle(shape, got, ref, one, nb, k, topk, check_cache=False), flush=True)
            kc_o[b], vc_o[b] = ref["k_cache"], ref["v_cache"]
        kc_g, vc_g = res["k_cache"], res["v_cache"]
        L = L + np.array(acc, dtype=np.int32)
    d.close()


def test_without_final_norm():
    shape = small_shape("bf16", final_norm=False)
    wl = Workload("nonorm", shape, batch=2, kv_len=(33, 64), n_new=1, k=4, topk=4, seed=24)
    _run_case(wl)


def test_multi_round_commit_only_accepted_rows():
    """Rows of earlier rounds' [MASK] slots are overwritten, never read (Section 4.1)."""
    import torch
    shape = small_shape("bf16")
    wl = Workload("rounds", shape, batch=1, kv_len=(40,), n_new=1, k=4, topk=4, seed=25)
    w = inputs.make_weights(shape, wl.seed)
    inp = inputs.make_step_inputs(wl, slack=32)
    d = _drafter(shape, w, max_batch=1, max_new=5, max_positions=128, k_max=4)
    kc_g, vc_g = inp["k_cache"], inp["v_cache"]
    kc_o, vc_o = inp["k_cache"], inp["v_cache"]
    L = 40
    g = np.random.default_rng(5)
    for rnd, acc in enumerate([1, 4, 2, 5]):
        x = inputs.f32_to_bf16_bits(g.standard_normal((1, acc, shape.hidden)).astype(np.float32))
        cur = dict(inp, x=x, k_cache=kc_g, v_cache=vc_g, kv_len=np.array([L], dtype=np.int32))
        res = run_gpu_step(d, cur, acc, 4, 4)
        cur_o = dict(cur, k_cache=kc_o, v_cache=vc_o)
        ref = oracle_step(shape, w, cur_o, acc, 4, 4)
        print("round", rnd, compare_with_oracle(shape, res, ref, cur_o, acc, 4, 4, check_cache=False), flush=True)
        kc_g, vc_g, kc_o, vc_o = res["k_cache"], res["v_cache"], ref["k_cache"], ref["v_cache"]
        L += acc
    d.close()


def test_repeated_steps_are_bitwise_identical():
    """Fixed-order reductions: the same step twice gives the same bits (also a race detector)."""
    shape = small_shape("bf16", vocab=4096)
    wl = Workload("det", shape, batch=2, kv_len=(300, 17), n_new=2, k=5, topk=8, seed=26)
    w = inputs.make_weights(shape, wl.seed)
    inp = inputs.make_step_inputs(wl)
    d = _drafter(shape, w, max_batch=2, max_new=2, max_positions=400, k_max=5)
    first = run_gpu_step(d, inp, 2, 5, 8)
    for _ in range(3):
        again = run_gpu_step(d, inp, 2, 5, 8)
        for name in first:
            assert np.array_equal(first[name], again[name]), name
    d.close()


def test_step_replayed_from_a_graph():
    """A captured ps_draft_step can be replayed: the step's sequence number lives on the device.  Replays
    alternate with eager steps of the same context and with new inputs written into the captured buffers;
    every replay is compared with the oracle."""
    import torch
    shape = small_shape("bf16", vocab=2069)
    wl = Workload("graph", shape, batch=2, kv_len=(200, 70), n_new=1, k=5, topk=8, seed=41)
    w = inputs.make_weights(shape, wl.seed)
    d = _drafter(shape, w, max_batch=2, max_new=1, max_positions=300, k_max=5)
    inp0 = inputs.make_step_inputs(wl)
    dt = shape.dtype
    x = B.to_device(inp0["x"], dt)
    kc = B.to_device(inp0["k_cache"], dt)
    vc = B.to_device(inp0["v_cache"], dt)
    outs = d.alloc_outputs(2, 1, 5, 8, logits=True, probs=True, hidden=True)
    args = d.make_args(x, kc, vc, inp0["kv_offsets"], inp0["kv_len"], 1, 5, 8, outs)
    d.step(args)                               # eager warm-up (first use of the context)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            d.step(args, stream=side)
    torch.cuda.synchronize()
    for rep in range(5):
        wl_r = Workload("graph", shape, batch=2, kv_len=(200, 70), n_new=1, k=5, topk=8, seed=50 + rep)
        inp = inputs.make_step_inputs(wl_r)
        x.copy_(B.to_device(inp["x"], dt)); kc.copy_(B.to_device(inp["k_cache"], dt)); vc.copy_(B.to_device(inp["v_cache"], dt))
        for t in outs.values():
            t.fill_(-12345) if t.dtype != torch.int32 else t.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        res = {n: t.cpu().numpy() for n, t in outs.items()}
        res["k_cache"] = B.from_device(kc); res["v_cache"] = B.from_device(vc)
        ref = oracle_step(shape, w, inp, 1, 5, 8)
        print("replay", rep, compare_with_oracle(shape, res, ref, inp, 1, 5, 8), flush=True)
        if rep % 2 == 0:                       # an eager step of the same context in between
            other = run_gpu_step(d, inp0, 1, 5, 8)
            ref0 = oracle_step(shape, w, inp0, 1, 5, 8)
            compare_with_oracle(shape, other, ref0, inp0, 1, 5, 8)
    d.close()


def test_replayed_small_step_among_eager_steps_of_other_shapes():
    """The copies of the exchange buffers are kept clean on the device (each step resets what the previous
    step left beyond its own footprint), so a captured small step can be replayed between eager steps with
    more rows, more column tiles and other K-slice plans, in any order, without the host knowing."""
    import torch
    shape = small_shape("bf16", vocab=2069)
    w = inputs.make_weights(shape, 61)
    d = _drafter(shape, w, max_batch=4, max_new=6, max_positions=400, k_max=5)
    wl_s = Workload("g-small", shape, batch=1, kv_len=(150,), n_new=1, k=5, topk=8, seed=61)
    inp_s = inputs.make_step_inputs(wl_s)
    dt = shape.dtype
    x, kc, vc = (B.to_device(inp_s[n], dt) for n in ("x", "k_cache", "v_cache"))
    outs = d.alloc_outputs(1, 1, 5, 8, logits=True, probs=True, hidden=True)
    args = d.make_args(x, kc, vc, inp_s["kv_offsets"], inp_s["kv_len"], 1, 5, 8, outs)
    ref_s = oracle_step(shape, w, inp_s, 1, 5, 8)
    d.step(args)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            d.step(args, stream=side)
    torch.cuda.synchronize()
    # eager steps in between: 11 rows; 4 x 11 = 44 rows (three column tiles); 2 x 8 rows; the small shape itself
    others = [(1, (150,), 6, 5), (4, (30, 200, 129, 7), 6, 5), (2, (64, 65), 3, 5), (4, (30, 200, 129, 7), 6, 5),
              (1, (150,), 1, 5), (1, (150,), 6, 5), (1, (150,), 6, 5)]
    for i, (batch, kv, n_new, k) in enumerate(others):
        wl_o = Workload("g-other", shape, batch=batch, kv_len=kv, n_new=n_new, k=k, topk=8, seed=70 + i)
        inp_o = inputs.make_step_inputs(wl_o)
        res_o = run_gpu_step(d, inp_o, n_new, k, 8)
        print("eager", i, (batch, n_new, k), compare_with_oracle(shape, res_o, oracle_step(shape, w, inp_o, n_new, k, 8), inp_o, n_new, k, 8), flush=True)
        for rep in range(1 + i % 2):       # one or two replays in a row
            kc.copy_(B.to_device(inp_s["k_cache"], dt)); vc.copy_(B.to_device(inp_s["v_cache"], dt))
            for t in outs.values():
                t.fill_(-12345) if t.dtype != torch.int32 else t.fill_(-7)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            res = {n: t.cpu().numpy() for n, t in outs.items()}
            res["k_cache"] = B.from_device(kc); res["v_cache"] = B.from_device(vc)
            print("  replay", i, rep, compare_with_oracle(shape, res, ref_s, inp_s, 1, 5, 8), flush=True)
    assert d.last_status() == B.PS_OK
    d.close()


def test_a_step_that_gives_up_its_waits_is_marked_reported_and_recovered_from():
    """Forced from the host: with a poll limit of 1 every wait whose data is not there yet is given up, the
    way it would be after about a second if other work held compute units.  The kernel ends normally, every
    output row is marked (ids -1, probabilities 0, lse NaN), ps_draft_last_status reports it once and
    cleans up, and the following steps match the oracle again."""
    from paper_2410_05589_amd import debug as DBG
    shape = small_shape("bf16", vocab=2069)
    wl = Workload("giveup", shape, batch=2, kv_len=(300, 70), n_new=2, k=5, topk=8, seed=62)
    w = inputs.make_weights(shape, wl.seed)
    inp = inputs.make_step_inputs(wl)
    d = _drafter(shape, w, max_batch=2, max_new=2, max_positions=400, k_max=5)
    ref = oracle_step(shape, w, inp, 2, 5, 8)
    compare_with_oracle(shape, run_gpu_step(d, inp, 2, 5, 8), ref, inp, 2, 5, 8)
    assert d.last_status() == B.PS_OK
    assert DBG.ps_draft_debug_spin_limit(d.ctx, 1) == B.PS_OK
    print("step with poll limit 1", flush=True)
    bad = run_gpu_step(d, inp, 2, 5, 8, want=())
    assert (bad["top_ids"] == -1).all() and (bad["top_p"] == 0).all() and np.isnan(bad["lse"]).all()
    assert DBG.ps_draft_debug_spin_limit(d.ctx, 0) == B.PS_OK
    assert d.last_status() == B.PS_ERR_TIMEOUT
    assert d.last_status() == B.PS_OK
    for _ in range(3):
        print("   after recovery", compare_with_oracle(shape, run_gpu_step(d, inp, 2, 5, 8), ref, inp, 2, 5, 8), flush=True)
    assert d.last_status() == B.PS_OK
    d.close()


def test_optional_outputs_may_be_null():
    shape = small_shape("bf16")
    wl = Workload("opt", shape, batch=1, kv_len=(50,), n_new=1, k=3, topk=4, seed=27)
    w = inputs.make_weights(shape, wl.seed)
    inp = inputs.make_step_inputs(wl)
    d = _drafter(shape, w, max_batch=1, max_new=1, max_positions=64, k_max=3)
    full = run_gpu_step(d, inp, 1, 3, 4)
    lean = run_gpu_step(d, inp, 1, 3, 4, want=())
    only_probs = run_gpu_step(d, inp, 1, 3, 4, want=("probs",))
    for name in ("top_ids", "top_p", "lse"):
        assert np.array_equal(full[name], lean[name])
    assert np.array_equal(full["probs"], only_probs["probs"])
    d.close()


def test_step_argument_errors_enqueue_nothing():
    import torch
    shape = small_shape("bf16")
    wl = Workload("err", shape, batch=2, kv_len=(10, 20), n_new=1, k=3, topk=4, seed=28)
    w = inputs.make_weights(shape, wl.seed)
    inp = inputs.make_step_inputs(wl)
    d = _drafter(shape, w, max_batch=2, max_new=2, max_positions=40, max_topk=4, k_max=3)
    dt = shape.dtype
    x, kc, vc = (B.to_device(inp[n], dt) for n in ("x", "k_cache", "v_cache"))
    outs = d.alloc_outputs(2, 1, 3, 4)
    for t in outs.values():
        t.zero_()
    torch.cuda.synchronize()
    kc0 = B.from_device(kc).copy()

    def status(**kw):
        a = d.make_args(x, kc, vc, kw.pop("off", inp["kv_offsets"]), kw.pop("ln", inp["kv_len"]),
                        kw.pop("n_new", 1), kw.pop("k", 3), kw.pop("topk", 4), outs)
        for name, v in kw.items():
            setattr(a, name, v)
        return B.ps_draft_step(d.ctx, a, None)

    assert status(n_new=3) == B.PS_ERR_SHAPE
    assert status(n_new=0) == B.PS_ERR_SHAPE
    assert status(k=4) == B.PS_ERR_SHAPE
    assert status(topk=5) == B.PS_ERR_SHAPE
    assert status(topk=0) == B.PS_ERR_SHAPE
    assert status(out_rows=2) == B.PS_ERR_SHAPE
    assert status(x=None) == B.PS_ERR_NULL
    assert status(top_ids=None) == B.PS_ERR_NULL
    keep = [np.array(v, dtype=np.int32) for v in ((1, 0), (1, 3))]
    as_ptr = lambda arr: arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))   # noqa: E731
    assert status(n_new=2, n_new_seq=as_ptr(keep[0])) == B.PS_ERR_SHAPE         # 0 accepted tokens
    assert status(n_new=2, n_new_seq=as_ptr(keep[1])) == B.PS_ERR_SHAPE         # more than n_new
    assert status(n_new=2) == B.PS_ERR_KV_CAPACITY                                # 20 + 2 + 3 rows do not fit sequence 1's 24 cache rows
    assert status(ln=np.array([10, 21], dtype=np.int32)) == B.PS_ERR_KV_CAPACITY
    assert status(ln=np.array([10, -1], dtype=np.int32)) == B.PS_ERR_SHAPE
    assert status(off=np.array([0, 30, 20], dtype=np.int64)) == B.PS_ERR_OFFSETS
    assert status(off=np.array([0, 14, 100], dtype=np.int64), ln=np.array([10, 37], dtype=np.int32)) \
        == B.PS_ERR_KV_CAPACITY                                    # beyond max_positions
    torch.cuda.synchronize()
    assert np.array_equal(B.from_device(kc), kc0)
    assert int(outs["top_ids"].abs().sum()) == 0
    assert status() == B.PS_OK
    torch.cuda.synchronize()
    d.close()


# ---------------------------------------------------------------- the benchmark workloads at full size
@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4"])
def test_full_size_workloads(name):
    wl = WORKLOADS[name]
    if name == "c2":
        # the accepted-length mix as the benchmark runs it: one context, every n_new of the mix in turn
        shape = wl.shape
        w = inputs.make_weights(shape, wl.seed)
        d = _drafter(shape, w, max_batch=1, max_new=6, max_positions=wl.kv_len[0] + 6 + wl.k, k_max=wl.k)
        for n_new in (3, 1, 6, 2, 5, 4, 1):
            inp = inputs.make_step_inputs(wl, n_new=n_new)
            res = run_gpu_step(d, inp, n_new, wl.k, wl.topk)
            ref = oracle_step(shape, w, inp, n_new, wl.k, wl.topk)
            print("c2 n_new", n_new, compare_with_oracle(shape, res, ref, inp, n_new, wl.k, wl.topk), flush=True)
        d.close()
    else:
        _run_case(wl)
