"""CPU pins of the acceptance-walk oracle (Algorithm 1; Section 4.2): none re-types its formulas.

The main pin is the property the algorithm exists for: when the children of every node are
independent samples of the draft distribution of their depth, the tokens the walk emits are
distributed exactly as if the target model had generated them one by one.
"""
import numpy as np

from oracle import verify_walk as vw


def _dirichlet(g, n, V, conc=0.7):
    return g.dirichlet(np.full(V, conc), size=n)


def test_emitted_tokens_follow_the_target_distribution():
    # target: first-order Markov chain over V tokens; drafter: one distribution per depth (it does
    # not see the path, like the parallel drafter); tree: 3 children of the root, 2 children each
    V, trials = 4, 30000
    g = np.random.default_rng(11)
    p_root = _dirichlet(g, 1, V)[0]
    p_after = _dirichlet(g, V, V)            # p_after[a] = target distribution after token a
    noise = _dirichlet(g, 2, V)
    q = np.stack([0.5 * p_root + 0.5 * noise[0], 0.5 * p_after.mean(axis=0) + 0.5 * noise[1]])   # a drafter that is half right
    parent = np.array([-1, 0, 0, 0, 1, 1, 2, 2, 3, 3])
    depth = vw.tree_depths(parent)
    first = np.zeros(V)
    second = np.zeros((V, V))
    n_acc = 0
    for _ in range(trials):
        tokens = np.array([-1] + [g.choice(V, p=q[depth[s] - 1]) for s in range(1, len(parent))])
        p = np.stack([p_root] + [p_after[tokens[s]] for s in range(1, len(parent))])
        out = vw.acceptance_walk(parent, tokens, q, p, g.random(len(parent)))
        first[out["tokens"][0]] += 1
        if len(out["tokens"]) > 1:
            second[out["tokens"][0], out["tokens"][1]] += 1
        n_acc += out["n_accepted"]
    assert n_acc > 0.5 * trials                      # the tree is actually used
    f = first / trials
    assert np.all(np.abs(f - p_root) < 4.5 * np.sqrt(p_root * (1 - p_root) / trials)), (f, p_root)
    for a in range(V):
        n = second[a].sum()
        assert n > 500
        fa = second[a] / n
        assert np.all(np.abs(fa - p_after[a]) < 4.5 * np.sqrt(p_after[a] * (1 - p_after[a]) / n)), (a, fa, p_after[a])


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
