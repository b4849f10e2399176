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
