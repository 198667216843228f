"""CPU oracle for the draft-tree construction and the acceptance walk.  TEST INFRASTRUCTURE ONLY.

Only tests/ and bench.py's baseline leg may import this file; the product path never does,
and this file imports nothing of the HIP path.

What it computes (Algorithm 1, the part after the draft line; Section 4.2): the drafter's
k+1 distributions give a token tree N whose nodes at depth t carry tokens proposed from
the distribution of draft row t-1, q(. | x_<n, [MASK]_1..t-1); the target model gives, for
every node, its next-token distribution given the path to that node.  The walk starts at
the root.  The children of the current node are tried one after the other: child s with
token x is accepted when a uniform number r is below min(1, P(x) / q_t(x)), P being the
target distribution at the current node; the walk then moves to s and P becomes the
target distribution at s.  A rejected child is removed and P becomes the normalised
positive part of P - q_t.  When a node has no children (left), the walk ends and one more
token is drawn from P.

The steps are taken in the algorithm's order, in float64.  Readings where the paper is
silent: Select() takes the children in ascending node index (the order in which the tree
lists them); all random numbers are inputs (r[s] for the test of node s; r[0], the root's
unused slot, draws the last token); the last token is drawn by inversion of the cumulative
sum in token-id order: the number of ids whose cumulative sum is <= r[0] * total, at most
V-1.

Pins (tests/test_oracle_verify.py, CPU): the first three emitted tokens follow the target
distribution when the children are independent samples of q (Monte Carlo over the oracle,
Section 4.2's claim of a preserved output distribution; the same check fails for planted
mistakes); p == q accepts every first child; a proposal
the target gives probability 0 is always rejected; inversion against numpy.searchsorted;
tree tokens against a hand-written example.
"""
import numpy as np


def tree_depths(parent):
    """Depth of every node; node 0 is the root (parent -1), parents precede their children."""
    parent = np.asarray(parent, dtype=np.int64)
    depth = np.zeros(len(parent), dtype=np.int64)
    assert parent[0] == -1
    for s in range(1, len(parent)):
        assert 0 <= parent[s] < s
        depth[s] = depth[parent[s]] + 1
    return depth


def tree_tokens(top_ids, parent, rank):
    """Token of node s = the rank[s]-th most probable token of draft row depth(s)-1.

    top_ids: [rows, topk] token ids sorted by probability; returns [n_nodes] (root: -1).
    """
    depth = tree_depths(parent)
    out = np.full(len(parent), -1, dtype=np.int64)
    for s in range(1, len(parent)):
        out[s] = top_ids[depth[s] - 1][rank[s]]
    return out


def draw_by_inversion(P, u):
    """Index drawn from the unnormalised distribution P with the uniform number u in [0, 1)."""
    c = 0.0
    target = u * float(np.sum(P))
    n = 0
    for i in range(len(P)):
        c += float(P[i])
        if c <= target:
            n += 1
    return min(n, len(P) - 1)


def acceptance_walk(parent, tokens, q, p, r):
    """One walk over the tree.

    parent [N], tokens [N] (root ignored), q [rows, V] draft distributions (row t-1 for depth t),
    p [N, V] target distributions (p[s] = next-token distribution after the path to s),
    r [N] uniform numbers.  Returns a dict: path (accepted nodes), tokens (accepted tokens and
    the last drawn one), n_accepted, and the margins of every decision (distance of r from the
    acceptance ratio; distance of the inversion target from the nearest cumulative sum, relative
    to the total) so that a comparison can tell forced differences from rounding; and how many
    rejections met P as a row of p or as a residual (for counting the bytes a walk has to touch).
    """
    parent = np.asarray(parent, dtype=np.int64)
    N = len(parent)
    depth = tree_depths(parent)
    q = np.asarray(q, dtype=np.float64)
    p = np.asarray(p, dtype=np.float64)
    u = 0
    P = p[0].copy()
    path, out_tokens, margins = [], [], []
    fresh, rejected = True, {True: 0, False: 0}              # bookkeeping only: is P still a row of p?
    while True:
        H = [s for s in range(N) if parent[s] == u]          # children, ascending index
        if not H:
            break
        moved = False
        while H:
            s = H[0]
            x = int(tokens[s])
            qt = q[depth[s] - 1]
            ratio = min(1.0, P[x] / qt[x]) if qt[x] > 0.0 else 1.0
            margins.append(abs(float(r[s]) - ratio))
            if r[s] < ratio:
                path.append(s)
                out_tokens.append(x)
                u = s
                P = p[s].copy()
                fresh = True
                moved = True
                break
            rejected[fresh] += 1
            fresh = False
            res = np.maximum(P - qt, 0.0)
            tot = float(np.sum(res))
            P = res / tot if tot > 0.0 else res
            H.pop(0)
        if not moved:
            break
    x_next = draw_by_inversion(P, float(r[0]))
    c = np.cumsum(P)
    target = float(r[0]) * float(np.sum(P))
    cdf_margin = float(np.min(np.abs(c - target))) / max(float(np.sum(P)), 1e-300)
    out_tokens.append(x_next)
    return {"path": path, "tokens": out_tokens, "n_accepted": len(path),
            "accept_margin": min(margins) if margins else 1.0, "cdf_margin": cdf_margin, "final_P": P,
            "rejected_from_row": rejected[True], "rejected_from_residual": rejected[False], "final_from_row": fresh}
