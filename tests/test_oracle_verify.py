"""Pins of the greedy-verification oracle (oracle/verify.py): a hand example on the golden tree, the
brute-force reading of "the longest branch that agrees with the ground truth", and special cases."""
import json
import os

import numpy as np
import pytest

from oracle import opt_tree as ot
from oracle import verify as vf

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows_with_argmax(am, V, seed=0):
    g = np.random.default_rng(seed)
    x = g.standard_normal((len(am), V))
    for r, t in enumerate(am):
        x[r, t] = 10.0
    return x


def test_hand_example_on_the_golden_tree():
    # tree of tests/golden/hand_tree.json: tokens [0,1,0,2,0], parents [-1,-1,0,0,2] (node 4 = 0 -> 0 -> 0)
    g = json.load(open(os.path.join(GOLDEN, "hand_tree.json")))
    tok, par = np.array(g["token"]), np.array(g["parent"])
    # target says 0 at the root, 0 after node 0, 0 after node 2, 1 after node 4: the branch 0-2-4 is accepted whole
    A, nodes, out = vf.greedy_verify(_rows_with_argmax([0, 0, 2, 0, 1, 1], 3), tok, par, 5)
    assert (A, nodes, out) == (4, [0, 2, 4], [0, 0, 0, 1])
    # target says 0 then 2: node 3 (token 2 under node 0) is accepted, then its own row says 1
    A, nodes, out = vf.greedy_verify(_rows_with_argmax([0, 2, 2, 0, 1, 1], 3), tok, par, 5)
    assert (A, nodes, out) == (3, [0, 3], [0, 2, 1])
    # target says 2 at the root: no child of the root carries 2, only the free token is produced
    A, nodes, out = vf.greedy_verify(_rows_with_argmax([2, 0, 0, 0, 0, 0], 3), tok, par, 5)
    assert (A, nodes, out) == (1, [], [2])


def _brute_force(target_logits, token, parent, n_out):
    """A node agrees with the ground truth if its token is the target's most probable token at its parent's
    position and its parent agrees (the root agrees by definition).  The accepted branch is the set of
    agreeing nodes; it must be a chain."""
    am = [int(np.argmax(r)) for r in target_logits]
    agree = {}
    for i in range(n_out):                      # parents precede children in the builder's output order
        p = int(parent[i])
        agree[i] = (p == -1 or agree[p]) and int(token[i]) == am[p + 1]
    chain = [i for i in range(n_out) if agree[i]]
    for a, b in zip(chain, chain[1:]):
        assert int(parent[b]) == a
    last = chain[-1] if chain else -1
    return len(chain) + 1, chain, [int(token[i]) for i in chain] + [am[last + 1]]


@pytest.mark.parametrize("seed", range(6))
def test_walk_equals_brute_force_on_built_trees(seed):
    V, k, n, d = 12, 3, 14, 5
    g = np.random.default_rng(seed)
    tree = ot.build_tree(g.standard_normal((d, n, V)) * 2.0, k, n, d)
    # a target that mostly agrees with the draft: its most probable token at a position is, with probability
    # 0.7, the token of one of that position's children in the tree
    am = []
    for pos in range(-1, n):
        kids = [i for i in range(tree["n_out"]) if tree["parent"][i] == pos]
        am.append(int(tree["token"][g.choice(kids)]) if kids and g.random() < 0.7 else int(g.integers(V)))
    x = _rows_with_argmax(am, V, seed)
    got = vf.greedy_verify(x, tree["token"], tree["parent"], tree["n_out"])
    assert got == _brute_force(x, tree["token"], tree["parent"], tree["n_out"])


def test_chain_fully_accepted_and_ties_take_the_smaller_token():
    n = 6
    tok, par = np.arange(n) + 1, np.arange(n) - 1            # a chain 1-2-3-4-5-6
    x = _rows_with_argmax([1, 2, 3, 4, 5, 6, 0], 8)
    A, nodes, out = vf.greedy_verify(x, tok, par, n)
    assert (A, nodes, out) == (n + 1, list(range(n)), [1, 2, 3, 4, 5, 6, 0])
    x[0, 0] = x[0, 1]                                         # tie at the root between tokens 0 and 1 -> 0 wins
    A, nodes, out = vf.greedy_verify(x, tok, par, n)
    assert (A, nodes, out) == (1, [], [0])
    # nodes beyond n_out do not exist
    A, nodes, out = vf.greedy_verify(_rows_with_argmax([1, 2, 3, 4, 5, 6, 0], 8), tok, par, 2)
    assert (A, nodes, out) == (3, [0, 1], [1, 2, 3])


def test_kv_append_moves_the_accepted_rows_and_respects_the_capacity():
    g = np.random.default_rng(1)
    H, cap, n, D = 2, 10, 5, 4
    Kp, Vp = g.standard_normal((H, cap, D)), g.standard_normal((H, cap, D))
    Kt, Vt = g.standard_normal((H, n, D)), g.standard_normal((H, n, D))
    K0, V0 = Kp.copy(), Vp.copy()
    L = vf.kv_append(Kp, Vp, Kt, Vt, 6, [1, 3, 4])
    assert L == 9
    np.testing.assert_array_equal(Kp[:, :6], K0[:, :6])
    np.testing.assert_array_equal(Kp[:, 6:9], Kt[:, [1, 3, 4]])
    np.testing.assert_array_equal(Vp[:, 6:9], Vt[:, [1, 3, 4]])
    np.testing.assert_array_equal(Kp[:, 9:], K0[:, 9:])
    Kp, Vp = K0.copy(), V0.copy()
    assert vf.kv_append(Kp, Vp, Kt, Vt, 8, [0, 2, 4]) == cap       # only two rows fit
    np.testing.assert_array_equal(Kp[:, 8:10], Kt[:, [0, 2]])


# ---------------------------------------------------------------------------------------------------------
# Random sampling (Sec. 4, non-greedy settings; the reading stated in oracle/verify.py)

def test_sample_truth_on_a_dyadic_distribution():
    # q = (1/2, 1/4, 1/8, 1/8): boundaries of the inverse CDF at 0.5, 0.75, 0.875
    row = np.log(np.array([0.5, 0.25, 0.125, 0.125]))
    for u, want in [(0.0, 0), (0.49, 0), (0.51, 1), (0.74, 1), (0.76, 2), (0.874, 2), (0.876, 3), (0.999, 3)]:
        assert vf.sample_truth(row, 1.0, u) == want
    # temperature 1/2 squares the probabilities: (16, 4, 1, 1) / 22 -> boundaries 16/22, 20/22, 21/22
    for u, want in [(0.72, 0), (0.73, 1), (0.90, 1), (0.92, 2), (0.95, 2), (0.96, 3)]:
        assert vf.sample_truth(row, 0.5, u) == want
    # temperature 2 takes square roots: (2, sqrt 2, 1, 1) / (4 + sqrt 2) -> first boundary at 0.3694
    assert vf.sample_truth(row, 2.0, 0.36) == 0 and vf.sample_truth(row, 2.0, 0.38) == 1
    # a shift of the logits changes nothing
    assert vf.sample_truth(row + 123.0, 0.5, 0.73) == 1


def test_sample_truth_counts_follow_the_softmax():
    # over the regular grid u = (j + 1/2) / N every token is drawn N q_v times, up to one grid point per boundary
    g = np.random.default_rng(5)
    row = g.standard_normal(40) * 2.0
    row[[3, 17]] = -np.inf                      # masked tokens are never drawn
    for T in (0.3, 1.0, 1.7):
        z = row / T
        q = np.exp(z - z[np.isfinite(z)].max())
        q /= q.sum()
        N = 20000
        counts = np.bincount([vf.sample_truth(row, T, (j + 0.5) / N) for j in range(N)], minlength=40)
        assert counts[3] == 0 and counts[17] == 0
        assert np.abs(counts - N * q).max() <= 1.0 + 1e-9


def test_low_temperature_is_the_greedy_rule_and_u_spans_the_support():
    g = np.random.default_rng(9)
    x = g.standard_normal((7, 50))
    x[np.arange(7), g.integers(0, 50, 7)] += 6.0
    for r in range(7):
        for u in (0.0, 0.3, 0.999999):
            assert vf.sample_truth(x[r], 1e-3, u) == int(np.argmax(x[r]))
    row = np.array([-np.inf, 0.3, -1.0, 0.1, -np.inf])
    assert vf.sample_truth(row, 1.0, 0.0) == 1                  # the first token with a positive probability
    assert vf.sample_truth(row, 1.0, 1.0 - 1e-12) == 3          # the last one
    with pytest.raises(ValueError):
        vf.sample_truth(row, 0.0, 0.5)


def test_sampled_walk_on_the_golden_tree():
    # tokens [0,1,0,2,0], parents [-1,-1,0,0,2]; every target row is q = (1/2, 1/4, 1/4)
    g = json.load(open(os.path.join(GOLDEN, "hand_tree.json")))
    tok, par = np.array(g["token"]), np.array(g["parent"])
    rows = np.tile(np.log(np.array([0.5, 0.25, 0.25])), (6, 1))
    # u per position (root, node 0..4).  root: 0.1 -> token 0 = node 0; after node 0: 0.8 -> token 2 = node 3;
    # after node 3 (row 4): 0.6 -> token 1, node 3 has no child: 3 tokens, nodes [0, 3]
    u = np.array([0.1, 0.8, 0.0, 0.0, 0.6, 0.0])
    assert vf.sampled_verify(rows, 1.0, u, tok, par, 5) == (3, [0, 3], [0, 2, 1])
    # root: 0.6 -> token 1 = node 1; row 2 (after node 1): 0.9 -> token 2; node 1 is a leaf
    u = np.array([0.6, 0.0, 0.9, 0.0, 0.0, 0.0])
    assert vf.sampled_verify(rows, 1.0, u, tok, par, 5) == (2, [1], [1, 2])
    # root: 0.8 -> token 2: no child of the root carries it
    assert vf.sampled_verify(rows, 1.0, np.array([0.8, 0, 0, 0, 0, 0.0]), tok, par, 5) == (1, [], [2])
    # the whole branch 0 - 0 - 0, then the free token
    u = np.array([0.2, 0.3, 0.0, 0.4, 0.0, 0.7])
    assert vf.sampled_verify(rows, 1.0, u, tok, par, 5) == (4, [0, 2, 4], [0, 0, 0, 1])


@pytest.mark.parametrize("seed", range(4))
def test_sampled_walk_equals_greedy_walk_on_the_drawn_tokens(seed):
    # replacing every row by one whose arg-max is the drawn token turns the sampled walk into the greedy walk
    V, k, n, d = 12, 3, 14, 5
    g = np.random.default_rng(100 + seed)
    tree = ot.build_tree(g.standard_normal((d, n, V)) * 2.0, k, n, d)
    tok, par, n_out = np.array(tree["token"]), np.array(tree["parent"]), len(tree["token"])
    target = g.standard_normal((n + 1, V)) * 3.0
    for r in range(n + 1):                      # lean towards a child so that branches get accepted
        kids = [i for i in range(n_out) if par[i] == r - 1]
        if kids:
            target[r, tok[kids[g.integers(len(kids))]]] += 4.0
    u = g.random(n + 1)
    T = 0.8
    drawn = [vf.sample_truth(target[r], T, u[r]) for r in range(n + 1)]
    want = vf.greedy_verify(_rows_with_argmax(drawn, V, seed), tok, par, n_out)
    assert vf.sampled_verify(target, T, u, tok, par, n_out) == want


def test_sampled_verification_reproduces_the_target_distribution():
    # losslessness: over a regular grid of (u_root, u_next) the first two produced tokens occur as often as
    # q_root(a) * q_after(a)(b) says, whether or not the tree holds them
    V = 4
    tok, par = np.array([1, 2, 0, 3]), np.array([-1, -1, 0, 0])      # root -> {1, 2}; node 0 (token 1) -> {0, 3}
    g = np.random.default_rng(3)
    rows = g.standard_normal((5, V))
    T = 1.3
    q = np.exp(rows / T)
    q /= q.sum(1, keepdims=True)
    N = 120
    pair = np.zeros((V, V))
    single = np.zeros(V)
    for i in range(N):
        for j in range(N):
            u = np.array([(i + 0.5) / N] + [(j + 0.5) / N] * 4)
            A, nodes, out = vf.sampled_verify(rows, T, u, tok, par, 4)
            if A >= 2:
                pair[out[0], out[1]] += 1
            else:
                single[out[0]] += 1
    for a in range(V):
        child = [i for i in range(4) if par[i] == -1 and tok[i] == a]
        if child:                                                   # a is in the tree: the next token follows
            np.testing.assert_allclose(pair[a] / N**2, q[0, a] * q[child[0] + 1], atol=2.5 / N)
            assert single[a] == 0
        else:                                                       # a is not: the step ends with a alone
            np.testing.assert_allclose(single[a] / N**2, q[0, a], atol=1.5 / N)
            assert pair[a].sum() == 0


def test_sample_margin_is_the_distance_to_the_nearest_cdf_boundary():
    row = np.log(np.array([0.5, 0.25, 0.125, 0.125]))
    assert abs(vf.sample_margin(row, 1.0, 0.6) - 0.1) < 1e-12           # boundaries 0.5, 0.75, 0.875
    assert abs(vf.sample_margin(row, 1.0, 0.86) - 0.015) < 1e-12
    # moving u by less than the margin never changes the draw
    g = np.random.default_rng(2)
    x = g.standard_normal(30) * 2
    for u in g.random(50):
        m = vf.sample_margin(x, 0.9, u)
        assert vf.sample_truth(x, 0.9, u - 0.99 * m) == vf.sample_truth(x, 0.9, u) == vf.sample_truth(x, 0.9, u + 0.99 * m)
