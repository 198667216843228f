"""CPU pins of the acceptance-walk oracle (Algorithm 1; Section 4.2): none re-types its formulas.

The main pin is the property the algorithm exists for: when the children of every node are
independent samples of the draft distribution of their depth, the tokens the walk emits are
distributed exactly as if the target model had generated them one by one (checked on the
first three emitted tokens; a second test plants mistakes in the oracle and shows that this
check fails for each of them).
"""
import numpy as np

from oracle import verify_walk as vw


def _dirichlet(g, n, V, conc=0.7):
    return g.dirichlet(np.full(V, conc), size=n)


def _emitted_token_statistics(trials, seed=11):
    # target: first-order Markov chain over V tokens; drafter: one distribution per depth (it does
    # not see the path, like the parallel drafter); tree: 3 children of the root, 2 children each
    V = 4
    g = np.random.default_rng(seed)
    p_root = _dirichlet(g, 1, V)[0]
    p_after = _dirichlet(g, V, V)            # p_after[a] = target distribution after token a
    noise = _dirichlet(g, 2, V)
    q = np.stack([0.5 * p_root + 0.5 * noise[0], 0.5 * p_after.mean(axis=0) + 0.5 * noise[1]])   # a drafter that is half right
    parent = np.array([-1, 0, 0, 0, 1, 1, 2, 2, 3, 3])
    depth = [0, 1, 1, 1, 2, 2, 2, 2, 2, 2]           # (written out: independent of the oracle)
    first = np.zeros(V)
    second = np.zeros((V, V))
    third = np.zeros((V, V))
    n_acc = 0
    for _ in range(trials):
        tokens = np.array([-1] + [g.choice(V, p=q[depth[s] - 1]) for s in range(1, len(parent))])
        p = np.stack([p_root] + [p_after[tokens[s]] for s in range(1, len(parent))])
        out = vw.acceptance_walk(parent, tokens, q, p, g.random(len(parent)))
        first[out["tokens"][0]] += 1
        if len(out["tokens"]) > 1:
            second[out["tokens"][0], out["tokens"][1]] += 1
        if len(out["tokens"]) > 2:                   # (the target is a Markov chain: the third follows the second)
            third[out["tokens"][1], out["tokens"][2]] += 1
        n_acc += out["n_accepted"]
    # worst deviation of an observed frequency from the target's probability, in standard deviations
    worst = float(np.max(np.abs(first / trials - p_root) / np.sqrt(p_root * (1 - p_root) / trials)))
    for counts in (second, third):
        for a in range(V):
            n = counts[a].sum()
            if n > 0.01 * trials:
                sd = np.sqrt(p_after[a] * (1 - p_after[a]) / n)
                worst = max(worst, float(np.max(np.abs(counts[a] / n - p_after[a]) / sd)))
    return n_acc / trials, worst


def test_emitted_tokens_follow_the_target_distribution():
    accepted_per_walk, worst = _emitted_token_statistics(30000)
    assert accepted_per_walk > 0.5                   # the tree is actually used
    assert worst < 4.5, worst


def test_the_distribution_pin_catches_planted_mistakes(monkeypatch):
    """The same statistics on an oracle with one step spoiled (planted here, on the CPU) are far off."""
    class NoClip:                                    # (P - q)+ without the positive part
        def __getattr__(self, name):
            return (lambda x, y: x) if name == "maximum" else getattr(np, name)
    monkeypatch.setattr(vw, "np", NoClip())
    assert _emitted_token_statistics(8000)[1] > 8.0
    monkeypatch.undo()
    real_depths = vw.tree_depths                     # every depth reads the first draft row
    monkeypatch.setattr(vw, "tree_depths", lambda parent: np.minimum(real_depths(parent), 1))
    assert _emitted_token_statistics(8000)[1] > 8.0
    monkeypatch.undo()
    class NoSum:                                     # the residual is not normalised (its sum is taken as 1)
        def __getattr__(self, name):
            return (lambda x: 1.0) if name == "sum" else getattr(np, name)
    monkeypatch.setattr(vw, "np", NoSum())
    assert _emitted_token_statistics(8000)[1] > 8.0
    monkeypatch.undo()
    real_draw = vw.draw_by_inversion                 # the last token always drawn with u = 0.5
    monkeypatch.setattr(vw, "draw_by_inversion", lambda P, u: real_draw(P, 0.5))
    assert _emitted_token_statistics(8000)[1] > 8.0


def test_single_child_chain_accepts_with_probability_sum_min_p_q():
    # textbook speculative sampling (one proposal): P(accept) = sum_x min(p(x), q(x))
    V, trials = 5, 20000
    g = np.random.default_rng(5)
    p0, q0 = _dirichlet(g, 2, V)
    parent = np.array([-1, 0])
    acc = 0
    for _ in range(trials):
        tokens = np.array([-1, g.choice(V, p=q0)])
        out = vw.acceptance_walk(parent, tokens, q0[None], np.stack([p0, p0]), g.random(2))
        acc += out["n_accepted"]
    want = np.minimum(p0, q0).sum()
    assert abs(acc / trials - want) < 4.5 * np.sqrt(want * (1 - want) / trials)


def test_equal_distributions_accept_every_first_child():
    g = np.random.default_rng(2)
    V = 7
    parent = np.array([-1, 0, 0, 1, 1, 3])
    q = _dirichlet(g, 3, V)
    depth = vw.tree_depths(parent)
    tokens = np.array([-1] + [g.integers(V) for _ in range(5)])
    # the target agrees with the drafter at every node that still has children
    p = np.stack([q[min(depth[s], 2)] for s in range(6)])
    out = vw.acceptance_walk(parent, tokens, q, p, g.random(6))
    assert out["path"] == [1, 3, 5] and out["n_accepted"] == 3
    assert out["tokens"][:3] == [tokens[1], tokens[3], tokens[5]]


def test_impossible_proposals_are_rejected_and_never_drawn():
    g = np.random.default_rng(3)
    V = 6
    parent = np.array([-1, 0, 0])
    tokens = np.array([-1, 2, 4])
    q = _dirichlet(g, 1, V)
    p0 = _dirichlet(g, 1, V)[0]
    p0[[2, 4]] = 0.0
    p0 /= p0.sum()
    for t in range(50):
        out = vw.acceptance_walk(parent, tokens, q, np.stack([p0, p0, p0]), g.random(3))
        assert out["n_accepted"] == 0 and out["path"] == []
        assert out["tokens"][0] not in (2, 4)
        assert abs(out["final_P"].sum() - 1.0) < 1e-12 and np.all(out["final_P"] >= 0)


def test_inversion_agrees_with_searchsorted():
    g = np.random.default_rng(4)
    for V in (1, 2, 17, 300):
        P = g.random(V) * (g.random(V) > 0.3)
        P[g.integers(V)] += 0.1
        for u in list(g.random(20)) + [0.0]:
            want = min(int(np.searchsorted(np.cumsum(P), u * P.sum(), side="right")), V - 1)
            assert vw.draw_by_inversion(P, u) == want


def test_tree_tokens_of_a_hand_made_tree():
    # rows of top_ids: draft row 0 (depth 1), row 1 (depth 2), row 2 (depth 3)
    top_ids = np.array([[10, 11, 12], [20, 21, 22], [30, 31, 32]])
    parent = np.array([-1, 0, 0, 1, 1, 2, 3])
    rank = np.array([0, 0, 1, 0, 2, 1, 1])
    assert vw.tree_depths(parent).tolist() == [0, 1, 1, 2, 2, 2, 3]
    assert vw.tree_tokens(top_ids, parent, rank).tolist() == [-1, 10, 11, 20, 22, 21, 31]


def test_a_proposal_the_drafter_gave_no_mass_counts_as_ratio_one():
    """The reading for q(x) = 0 (the paper does not say): the limit of min(1, P(x) / q) as q -> 0+ for a token
    the target supports.  Pinned against that limit - the same walk with q(x) a denormal instead of 0 takes
    the same decisions - and against its consequences: such a child is accepted for every r < 1, the walk moves
    on to it, and P becomes the target's row at it."""
    V = 6
    g = np.random.default_rng(21)
    parent = np.array([-1, 0, 0, 1])
    tokens = np.array([-1, 2, 4, 5])
    p = _dirichlet(g, 4, V)
    q = _dirichlet(g, 2, V)
    q[0, 2] = 0.0
    q[0] /= q[0].sum()
    q_tiny = q.copy()
    q_tiny[0, 2] = 5e-324
    for trial in range(200):
        r = g.random(4)
        r[1] = 1.0 - 2.0 ** -24 if trial == 0 else r[1]         # even the largest r a float32 uniform can be
        a = vw.acceptance_walk(parent, tokens, q, p, r)
        b = vw.acceptance_walk(parent, tokens, q_tiny, p, r)
        assert a["path"] == b["path"] and a["tokens"] == b["tokens"]
        assert a["path"][0] == 1 and a["tokens"][0] == 2         # node 1 (token 2, q = 0) is always accepted
        if a["n_accepted"] == 1:
            # its child was rejected: the final draw comes from the residual of the target's row AT NODE 1
            res = np.maximum(p[1] - q[1], 0.0)
            np.testing.assert_allclose(a["final_P"], res / res.sum(), rtol=1e-12)
