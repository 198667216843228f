"""GPU parity of the tree construction and the acceptance walk (through the C ABI) against the CPU oracle.

Both sides decide in float64 on the same float32 inputs; they differ only in the order of the sums
over the vocabulary (relative 1e-13 at most).  So accepted nodes, accepted tokens and the last drawn
token must be bit-exact wherever the oracle's decision margins exceed MARGIN; a sample whose margin is
smaller is not compared (and there must be almost none).
"""
import numpy as np
import pytest

from oracle import verify_walk as vw
from paper_2410_05589_amd import binding as B
from paper_2410_05589_amd import inputs
from paper_2410_05589_amd import verify as VF

pytestmark = pytest.mark.gpu
MARGIN = 1e-9


def _run_gpu(parent, rank, inp, rows, topk, tokens_override=None):
    import torch
    dev = torch.device("cuda:0")
    batch, n, vocab = inp["p"].shape
    tree = VF.make_tree(parent, rank)
    top_ids = torch.from_numpy(inp["top_ids"]).to(dev)
    tokens = torch.full((batch, n), -5, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    st = VF.ps_tree_tokens(tree, batch, rows, topk, top_ids.data_ptr(), tokens.data_ptr(), stream)
    assert st == B.PS_OK, B.ps_draft_strerror(st)
    if tokens_override is not None:
        torch.cuda.synchronize()
        built = tokens.cpu().numpy()
        tokens = torch.from_numpy(np.ascontiguousarray(tokens_override, dtype=np.int32)).to(dev)
    q = torch.from_numpy(inp["q"]).to(dev)
    p = torch.from_numpy(inp["p"]).to(dev)
    r = torch.from_numpy(inp["r"]).to(dev)
    n_acc = torch.full((batch,), -7, dtype=torch.int32, device=dev)
    path = torch.full((batch, rows), -7, dtype=torch.int32, device=dev)
    out_tokens = torch.full((batch, rows + 1), -7, dtype=torch.int32, device=dev)
    a = VF.ps_verify_args()
    a.batch, a.rows, a.vocab = batch, rows, vocab
    a.tokens, a.q, a.p, a.r = tokens.data_ptr(), q.data_ptr(), p.data_ptr(), r.data_ptr()
    a.n_accepted, a.path, a.out_tokens = n_acc.data_ptr(), path.data_ptr(), out_tokens.data_ptr()
    st = VF.ps_verify_walk(tree, a, stream)
    assert st == B.PS_OK, B.ps_draft_strerror(st)
    torch.cuda.synchronize()
    res = {"tokens": tokens.cpu().numpy() if tokens_override is None else built, "n_accepted": n_acc.cpu().numpy(),
           "path": path.cpu().numpy(), "out_tokens": out_tokens.cpu().numpy()}
    if tokens_override is None:
        # the same walk with the tokens taken straight from top_ids (no ps_tree_tokens): identical outputs
        n_acc.fill_(-7); path.fill_(-7); out_tokens.fill_(-7)
        a.tokens, a.top_ids, a.topk = None, top_ids.data_ptr(), topk
        st = VF.ps_verify_walk(tree, a, stream)
        assert st == B.PS_OK, B.ps_draft_strerror(st)
        torch.cuda.synchronize()
        assert np.array_equal(n_acc.cpu().numpy(), res["n_accepted"])
        assert np.array_equal(path.cpu().numpy(), res["path"])
        assert np.array_equal(out_tokens.cpu().numpy(), res["out_tokens"])
    return res


def _check(parent, rank, inp, rows, topk, label, tokens_override=None, oracle_tokens=None):
    print("case", label, "nodes", len(parent), "rows", rows, "vocab", inp["p"].shape[2], "batch", inp["p"].shape[0], flush=True)
    gpu = _run_gpu(parent, rank, inp, rows, topk, tokens_override)
    batch = inp["p"].shape[0]
    compared = 0
    for b in range(batch):
        want_tokens = vw.tree_tokens(inp["top_ids"][b], parent, rank)
        assert gpu["tokens"][b].tolist() == want_tokens.tolist(), (label, b)
        walk_tokens = want_tokens if oracle_tokens is None else oracle_tokens[b]
        ref = vw.acceptance_walk(parent, walk_tokens, inp["q"][b], inp["p"][b], inp["r"][b])
        if ref["accept_margin"] <= MARGIN or ref["cdf_margin"] <= MARGIN:
            continue
        compared += 1
        na = ref["n_accepted"]
        assert gpu["n_accepted"][b] == na, (label, b)
        assert gpu["path"][b].tolist() == ref["path"] + [-1] * (rows - na), (label, b)
        assert gpu["out_tokens"][b].tolist() == ref["tokens"] + [-1] * (rows - na), (label, b)
    assert compared >= batch - 1 - batch // 16, (label, compared)
    return gpu


TREES = {
    "chain": [1, 1, 1, 1, 1],
    "wide": [8],
    "bushy": [4, 2, 2, 1, 1],          # 61 nodes
    "two levels": [3, 3],
}


@pytest.mark.parametrize("tree", sorted(TREES))
@pytest.mark.parametrize("vocab", [1000, 5003, 32000])
def test_walk_matches_oracle(tree, vocab):
    parent, rank = inputs.draft_tree(TREES[tree])
    rows = len(TREES[tree]) + 1
    for seed, agreement in ((1, 0.7), (2, 0.2), (3, 0.97)):
        inp = inputs.verify_inputs(100 * seed + vocab % 97, 6, parent, rank, rows, 8, vocab, agreement=agreement)
        _check(parent, rank, inp, rows, 8, "%s V%d agreement %.2f" % (tree, vocab, agreement))


def test_walk_at_the_largest_sizes():
    # Llama-3 vocabulary, the most nodes the interface takes, batch 8: the oracle walks every sequence
    parent, rank = inputs.draft_tree([7, 2, 2, 1])     # 1 + 7 + 14 + 28 + 28 = 78 > 64: cut to 64 nodes
    parent, rank = parent[:64], rank[:64]
    inp = inputs.verify_inputs(7, 8, parent, rank, 9, 8, 128256, agreement=0.8)
    _check(parent, rank, inp, 9, 8, "largest")


def test_root_only_tree_just_draws_a_token():
    parent, rank = np.array([-1], dtype=np.int32), np.array([0], dtype=np.int32)
    inp = inputs.verify_inputs(5, 4, parent, rank, 1, 4, 777)
    inp["r"][0, 0] = 0.0
    inp["r"][1, 0] = np.float32(1.0 - 2.0 ** -24)
    gpu = _check(parent, rank, inp, 1, 4, "root only")
    assert gpu["n_accepted"].tolist() == [0, 0, 0, 0]
    first = int(np.flatnonzero(inp["p"][0, 0] > 0)[0])
    assert gpu["out_tokens"][0, 0] == first              # u = 0 draws the first token with probability > 0


def test_proposals_the_drafter_gave_no_mass():
    """q(x) = 0 at proposed tokens counts as ratio 1 (accepted for every r < 1), in both kernels' paths."""
    for vocab, batch in ((32000, 6), (65536, 3)):
        parent, rank = inputs.draft_tree([3, 2])
        inp = inputs.verify_inputs(55 + vocab % 7, batch, parent, rank, 3, 8, vocab, agreement=0.3)
        tok = np.stack([vw.tree_tokens(inp["top_ids"][b], parent, rank) for b in range(batch)])
        for b in range(batch):
            for s in (1, 3, 4, 7):                 # some first children, some later ones, both depths
                inp["q"][b, 0 if s <= 3 else 1, tok[b, s]] = 0.0
        gpu = _check(parent, rank, inp, 3, 8, "q(x) = 0, V %d" % vocab)
        assert (gpu["n_accepted"] >= 1).all()      # node 1 carries a token with q = 0: always accepted


def test_token_outside_the_vocabulary_is_skipped():
    parent, rank = inputs.draft_tree([3, 1])
    inp = inputs.verify_inputs(6, 5, parent, rank, 3, 8, 2000, agreement=0.9)
    tokens = np.stack([vw.tree_tokens(inp["top_ids"][b], parent, rank) for b in range(5)])
    tokens[:, 1] = 2000          # first child of the root: out of range
    tokens[:, 2] = -3
    # the oracle sees the same tree without these two nodes (and without the child of node 1)
    keep = [0, 3, 6]
    sub_parent = np.array([-1, 0, 1], dtype=np.int32)
    gpu = _run_gpu(parent, rank, inp, 3, 8, tokens_override=tokens)
    for b in range(5):
        ref = vw.acceptance_walk(sub_parent, tokens[b, keep], inp["q"][b], inp["p"][b][keep], inp["r"][b][keep])
        if ref["accept_margin"] <= MARGIN or ref["cdf_margin"] <= MARGIN:
            continue
        assert gpu["n_accepted"][b] == ref["n_accepted"]
        assert gpu["path"][b, :ref["n_accepted"]].tolist() == [keep[s] for s in ref["path"]]
        assert gpu["out_tokens"][b, :ref["n_accepted"] + 1].tolist() == ref["tokens"]


def test_walk_after_a_draft_step_end_to_end():
    # the drafter's own output feeds the tree: top_ids and probs of a c0-sized step
    from paper_2410_05589_amd.configs import WORKLOADS
    from tests.gpu_util import run_gpu_step
    wl = WORKLOADS["c0"]
    w = inputs.make_weights(wl.shape, wl.seed)
    inp = inputs.make_step_inputs(wl, kv_len=[64, 40])
    drafter = B.Drafter(wl.shape, w, max_batch=2, max_new=wl.n_new, max_positions=256, max_topk=4)
    res = run_gpu_step(drafter, inp, wl.n_new, wl.k, 4)
    rows = wl.k + 1
    parent, rank = inputs.draft_tree([3, 2, 1, 1, 1])
    vin = inputs.verify_inputs(9, 2, parent, rank, rows, 4, wl.shape.vocab, agreement=0.0)
    q = res["probs"].reshape(2, rows, wl.shape.vocab).astype(np.float32)
    vin["q"] = q
    vin["top_ids"] = res["top_ids"].reshape(2, rows, 4).astype(np.int32)
    # a target that mostly agrees with the drafter's next row
    depth = vw.tree_depths(parent)
    for s in range(len(parent)):
        if depth[s] < rows:
            vin["p"][:, s] = (0.8 * q[:, depth[s]] + 0.2 * vin["p"][:, s]).astype(np.float32)
    _check(parent, rank, vin, rows, 4, "after a draft step")


def test_tree_and_walk_replayed_from_a_graph():
    """Both calls allocate and copy nothing, so they can be captured; replays with new inputs written into
    the captured buffers are each compared with the oracle, with eager calls in between."""
    import torch
    dev = torch.device("cuda:0")
    for vocab in (32000, 40004):          # P in registers / P recomputed from the two rows
        parent, rank = inputs.draft_tree([3, 2, 2, 1])
        rows, topk, batch, n = 5, 8, 3, len(parent)
        tree = VF.make_tree(parent, rank)
        inp = inputs.verify_inputs(20, batch, parent, rank, rows, topk, vocab)
        top_ids = torch.from_numpy(inp["top_ids"]).to(dev)
        tokens = torch.zeros((batch, n), dtype=torch.int32, device=dev)
        q, p, r = (torch.from_numpy(inp[x]).to(dev) for x in ("q", "p", "r"))
        n_acc = torch.zeros((batch,), dtype=torch.int32, device=dev)
        path = torch.zeros((batch, rows), dtype=torch.int32, device=dev)
        out_tokens = torch.zeros((batch, rows + 1), dtype=torch.int32, device=dev)
        a = VF.ps_verify_args()
        a.batch, a.rows, a.vocab = batch, rows, vocab
        a.tokens, a.q, a.p, a.r = tokens.data_ptr(), q.data_ptr(), p.data_ptr(), r.data_ptr()
        a.n_accepted, a.path, a.out_tokens = n_acc.data_ptr(), path.data_ptr(), out_tokens.data_ptr()

        def both(stream):
            assert VF.ps_tree_tokens(tree, batch, rows, topk, top_ids.data_ptr(), tokens.data_ptr(), stream) == B.PS_OK
            assert VF.ps_verify_walk(tree, a, stream) == B.PS_OK

        def check(cur, label):
            torch.cuda.synchronize()
            got_n, got_path, got_tok = n_acc.cpu().numpy(), path.cpu().numpy(), out_tokens.cpu().numpy()
            for b in range(batch):
                tok = vw.tree_tokens(cur["top_ids"][b], parent, rank)
                ref = vw.acceptance_walk(parent, tok, cur["q"][b], cur["p"][b], cur["r"][b])
                if ref["accept_margin"] <= MARGIN or ref["cdf_margin"] <= MARGIN:
                    continue
                na = ref["n_accepted"]
                assert got_n[b] == na, (label, b)
                assert got_path[b].tolist() == ref["path"] + [-1] * (rows - na), (label, b)
                assert got_tok[b].tolist() == ref["tokens"] + [-1] * (rows - na), (label, b)

        both(torch.cuda.current_stream().cuda_stream)        # eager first
        check(inp, "eager V%d" % vocab)
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                both(side.cuda_stream)
        torch.cuda.synchronize()
        for rep in range(4):
            cur = inputs.verify_inputs(30 + rep, batch, parent, rank, rows, topk, vocab, agreement=(0.3, 0.9, 0.6, 0.75)[rep])
            top_ids.copy_(torch.from_numpy(cur["top_ids"])); q.copy_(torch.from_numpy(cur["q"]))
            p.copy_(torch.from_numpy(cur["p"])); r.copy_(torch.from_numpy(cur["r"]))
            n_acc.fill_(-7); path.fill_(-7); out_tokens.fill_(-7); tokens.fill_(-7)
            torch.cuda.synchronize()
            print("replay", rep, "vocab", vocab, flush=True)
            graph.replay()
            check(cur, "replay %d V%d" % (rep, vocab))
            if rep % 2 == 0:
                both(torch.cuda.current_stream().cuda_stream)
                check(cur, "eager after replay %d V%d" % (rep, vocab))


def test_large_vocabulary_with_more_sequences_than_compute_units_allow_to_split():
    # 64 sequences x 8 workgroups would need 512 compute units: every sequence is walked by one workgroup
    parent, rank = inputs.draft_tree([2])
    inp = inputs.verify_inputs(12, 64, parent, rank, 2, 4, 131072, agreement=0.5)
    _check(parent, rank, inp, 2, 4, "large vocabulary, one workgroup per sequence")


def test_a_wait_that_runs_out_marks_the_sequence_and_the_next_call_is_fine():
    """Several workgroups per sequence: with the test hook every workgroup also waits for one that does not
    exist, with a short limit, so every wait is given up: the kernel ends normally, n_accepted = -2.  The
    call after it (hook off) gives the oracle's result."""
    from paper_2410_05589_amd import debug as DBG
    parent, rank = inputs.draft_tree([3, 2])
    inp = inputs.verify_inputs(44, 2, parent, rank, 3, 8, 40004, agreement=0.1)   # rejections are certain
    DBG.ps_verify_debug_exchange(200, 1)
    try:
        gpu = _run_gpu(parent, rank, inp, 3, 8)
    finally:
        DBG.ps_verify_debug_exchange(0, 0)
    assert gpu["n_accepted"].tolist() == [-2, -2]
    _check(parent, rank, inp, 3, 8, "after a wait that ran out")


def test_tokens_emitted_by_the_gpu_walk_follow_the_target_distribution():
    """Section 4.2's claim on the device path itself: with children that are independent samples of q, the first
    token the walk emits is distributed as the target's p(. | prefix), and the second, given the first, as the
    target's distribution after it.  32768 walks of a 3 x 2 tree over 8 tokens (512 launches of 64 sequences)."""
    import torch
    dev = torch.device("cuda:0")
    V, batch, launches = 8, 64, 512
    g = np.random.default_rng(77)
    p_root = g.dirichlet(np.full(V, 0.7))
    p_after = g.dirichlet(np.full(V, 0.7), size=V)
    noise = g.dirichlet(np.full(V, 0.7), size=2)
    q_rows = np.stack([0.5 * p_root + 0.5 * noise[0], 0.5 * p_after.mean(axis=0) + 0.5 * noise[1]]).astype(np.float32)
    q64 = q_rows.astype(np.float64)
    parent = np.array([-1, 0, 0, 0, 1, 1, 2, 2, 3, 3], dtype=np.int32)
    depth = vw.tree_depths(parent)
    n, rows = len(parent), 2
    tree = VF.make_tree(parent, np.zeros(n, dtype=np.int32))
    p_root32, p_after32 = p_root.astype(np.float32), p_after.astype(np.float32)
    q = torch.from_numpy(np.broadcast_to(q_rows, (batch, rows, V)).copy()).to(dev)
    tokens = torch.zeros((batch, n), dtype=torch.int32, device=dev)
    p = torch.zeros((batch, n, V), dtype=torch.float32, device=dev)
    r = torch.zeros((batch, n), dtype=torch.float32, device=dev)
    n_acc = torch.zeros((batch,), dtype=torch.int32, device=dev)
    path = torch.zeros((batch, rows), dtype=torch.int32, device=dev)
    out_tokens = torch.zeros((batch, rows + 1), dtype=torch.int32, device=dev)
    a = VF.ps_verify_args()
    a.batch, a.rows, a.vocab = batch, rows, V
    a.tokens, a.q, a.p, a.r = tokens.data_ptr(), q.data_ptr(), p.data_ptr(), r.data_ptr()
    a.n_accepted, a.path, a.out_tokens = n_acc.data_ptr(), path.data_ptr(), out_tokens.data_ptr()
    stream = torch.cuda.current_stream().cuda_stream
    first = np.zeros(V)
    second = np.zeros((V, V))
    accepted = 0
    for it in range(launches):
        tok = np.full((batch, n), -1, dtype=np.int32)
        for s in range(1, n):                        # children: independent samples of their depth's draft row
            tok[:, s] = g.choice(V, size=batch, p=q64[depth[s] - 1] / q64[depth[s] - 1].sum())
        pp = np.empty((batch, n, V), dtype=np.float32)
        pp[:, 0] = p_root32
        pp[:, 1:] = p_after32[tok[:, 1:]]
        tokens.copy_(torch.from_numpy(tok)); p.copy_(torch.from_numpy(pp))
        r.copy_(torch.from_numpy(np.minimum(g.random((batch, n)), 1.0 - 2.0 ** -24).astype(np.float32)))
        assert VF.ps_verify_walk(tree, a, stream) == B.PS_OK
        torch.cuda.synchronize()
        out, na = out_tokens.cpu().numpy(), n_acc.cpu().numpy()
        accepted += int(na.sum())
        np.add.at(first, out[:, 0], 1)
        has2 = na >= 1                               # a second token exists after at least one accepted one
        np.add.at(second, (out[has2, 0], out[has2, 1]), 1)
    trials = batch * launches
    assert accepted > 0.5 * trials
    f = first / trials
    assert np.all(np.abs(f - p_root) < 4.5 * np.sqrt(p_root * (1 - p_root) / trials) + 1e-6), (f, p_root)
    for x in range(V):
        m = second[x].sum()
        if m < 400:
            continue
        fx = second[x] / m
        assert np.all(np.abs(fx - p_after[x]) < 4.5 * np.sqrt(p_after[x] * (1 - p_after[x]) / m) + 1e-6), (x, fx, p_after[x])
