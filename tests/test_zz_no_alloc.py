"""The acceptance walk's entry point that allocates nothing (ps_verify_walk_static) against the entry point it
is a variant of (ps_verify_walk), through the C ABI: same outputs bit for bit, on two calls in a row of which
the second is smaller (fewer sequences, a smaller vocabulary, a smaller tree), so whatever the first call left
in the library's exchange array must not disturb the second.  Both calls use vocabularies that need the
exchange between workgroups.  Also: ps_verify_walk with a caller-owned workspace gives the same, and sizes
beyond the array's are refused."""
import numpy as np
import pytest

from oracle import verify_walk as vw
from paper_2410_05589_amd import binding as B
from paper_2410_05589_amd import inputs
from paper_2410_05589_amd import verify as VF

pytestmark = pytest.mark.gpu


def _walk(fn, parent, rank, inp, rows, topk, workspace=None):
    import torch
    dev = torch.device("cuda:0")
    batch, n, vocab = inp["p"].shape
    tree = VF.make_tree(parent, rank)
    top_ids = torch.from_numpy(inp["top_ids"]).to(dev)
    q, p, r = (torch.from_numpy(inp[x]).to(dev) for x in ("q", "p", "r"))
    n_acc = torch.full((batch,), -7, dtype=torch.int32, device=dev)
    path = torch.full((batch, rows), -7, dtype=torch.int32, device=dev)
    out_tokens = torch.full((batch, rows + 1), -7, dtype=torch.int32, device=dev)
    a = VF.ps_verify_args()
    a.batch, a.rows, a.vocab = batch, rows, vocab
    a.tokens, a.top_ids, a.topk = None, top_ids.data_ptr(), topk
    a.q, a.p, a.r = q.data_ptr(), p.data_ptr(), r.data_ptr()
    a.n_accepted, a.path, a.out_tokens = n_acc.data_ptr(), path.data_ptr(), out_tokens.data_ptr()
    if workspace is not None:
        a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel()
    st = fn(tree, a, torch.cuda.current_stream().cuda_stream)
    assert st == B.PS_OK, B.ps_draft_strerror(st)
    torch.cuda.synchronize()
    return {"n_accepted": n_acc.cpu().numpy(), "path": path.cpu().numpy(), "out_tokens": out_tokens.cpu().numpy()}


def test_static_walk_matches_the_walk_on_two_calls_the_second_smaller():
    import torch
    cases = []
    parent, rank = inputs.draft_tree([4, 2, 2, 1, 1])                       # 61 nodes
    cases.append((parent, rank, inputs.verify_inputs(91, 8, parent, rank, 6, 8, 128256, agreement=0.5), 6))
    parent2, rank2 = inputs.draft_tree([3, 2])                              # 10 nodes
    cases.append((parent2, rank2, inputs.verify_inputs(92, 3, parent2, rank2, 3, 8, 65536, agreement=0.3), 3))
    for i, (pa, rk, inp, rows) in enumerate(cases):
        print("call", i, "batch", inp["p"].shape[0], "vocab", inp["p"].shape[2], "nodes", len(pa), flush=True)
        got = _walk(VF.ps_verify_walk_static, pa, rk, inp, rows, 8)
        want = _walk(VF.ps_verify_walk, pa, rk, inp, rows, 8)
        for name in want:
            assert np.array_equal(got[name], want[name]), (i, name)
        assert (got["n_accepted"] >= 0).all()
        # and the caller-owned workspace (zeroed once, sized for the larger batch, reused for the smaller)
        if i == 0:
            ws = torch.zeros(VF.ps_verify_workspace_bytes(8, 128256), dtype=torch.uint8, device="cuda:0")
        mine = _walk(VF.ps_verify_walk, pa, rk, inp, rows, 8, workspace=ws)
        for name in want:
            assert np.array_equal(mine[name], want[name]), (i, "workspace", name)
        # the oracle agrees wherever its decisions are not on a knife's edge
        for b in range(inp["p"].shape[0]):
            tok = vw.tree_tokens(inp["top_ids"][b], pa, rk)
            ref = vw.acceptance_walk(pa, tok, inp["q"][b], inp["p"][b], inp["r"][b])
            if ref["accept_margin"] > 1e-9 and ref["cdf_margin"] > 1e-9:
                assert got["n_accepted"][b] == ref["n_accepted"]
                assert got["out_tokens"][b, :ref["n_accepted"] + 1].tolist() == ref["tokens"]


def test_static_walk_refuses_what_its_array_cannot_hold():
    import torch
    parent, rank = inputs.draft_tree([2])
    dummy = torch.zeros(16, dtype=torch.float32, device="cuda:0")
    a = VF.ps_verify_args()
    a.batch, a.rows, a.vocab = 65, 2, 128256
    for n in ("tokens", "q", "p", "r", "n_accepted", "path", "out_tokens"):
        setattr(a, n, dummy.data_ptr())
    tree = VF.make_tree(parent, rank)
    assert VF.ps_verify_walk_static(tree, a, None) == B.PS_ERR_UNSUPPORTED      # more sequences than slots
    a.batch = 40                                                                  # 40 x 8 workgroups > compute units
    assert VF.ps_verify_walk_static(tree, a, None) == B.PS_ERR_UNSUPPORTED
    torch.cuda.synchronize()
