"""Pins for oracle/opt_tree.py against things other than itself (CPU only)."""
import itertools
import json
import math
import os

import numpy as np
import pytest
import scipy.special

from oracle import opt_tree as ot

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- row statistics
@pytest.mark.parametrize("V,scale,seed", [(7, 1.0, 0), (1000, 3.0, 1), (32000, 4.0, 2)])
def test_row_lse_matches_scipy(V, scale, seed):
    x = np.random.default_rng(seed).standard_normal(V) * scale
    assert ot.row_logsumexp(x) == pytest.approx(float(scipy.special.logsumexp(x)), abs=1e-12)


def test_row_lse_constant_row_closed_form():
    for V, c in [(5, 0.0), (1000, -3.5), (32000, 12.25)]:
        assert ot.row_logsumexp(np.full(V, c)) == pytest.approx(c + math.log(V), abs=1e-12)
        assert list(ot.row_top_k(np.full(V, c), 4)) == [0, 1, 2, 3]


def test_row_lse_extreme_values_do_not_overflow():
    x = np.array([1e4, 1e4 - 1.0, -1e4])
    assert ot.row_logsumexp(x) == pytest.approx(1e4 + math.log1p(math.exp(-1.0)), abs=1e-9)


def test_row_top_k_against_python_sort_with_ties():
    rng = np.random.default_rng(3)
    for _ in range(20):
        V = int(rng.integers(3, 60))
        x = rng.integers(-3, 4, size=V).astype(np.float64)      # many exact ties
        k = int(rng.integers(1, V + 1))
        want = sorted(range(V), key=lambda i: (-x[i], i))[:k]
        assert list(ot.row_top_k(x, k)) == want


# ---------------------------------------------------------------- hand-derived example
def test_hand_worked_example():
    g = json.load(open(os.path.join(GOLDEN, "hand_tree.json")))
    b = ot.TreeBuilder(g["k"], g["n"])
    for t in range(g["steps"]):
        rows = np.log(np.array(g["rows"][str(t)], dtype=np.float64)) + 0.75 * (t + 1)   # softmax is shift-invariant
        tok, par = b.expand(rows)
        assert list(tok) == g["layer_tokens"][t]
        assert list(par) == g["layer_parent_slots"][t]
        np.testing.assert_allclose(np.exp(b.layers[t]["score"]), g["layer_phat"][t], rtol=1e-12)
        assert b.e_sub() == pytest.approx(g["e_sub_after_step"][t], rel=1e-12)
    out = b.finalize()
    assert out["n_out"] == g["n"]
    assert list(out["token"]) == g["token"]
    assert list(out["parent"]) == g["parent"]
    assert list(out["depth"]) == g["depth"]
    assert [int(m[0]) for m in out["mask"]] == g["mask"]
    np.testing.assert_allclose(np.exp(out["score"]), g["phat"], rtol=1e-12)
    assert out["expect"] == pytest.approx(g["expect"], rel=1e-12)


# ---------------------------------------------------------------- brute force (definition of E_sub)
def _path_row(path, V, seed):
    """Logits row of the node reached by `path` (tuple of tokens): what a draft model would emit."""
    h = np.random.SeedSequence([seed, len(path)] + [int(p) + 1 for p in path])
    return np.random.default_rng(h).standard_normal(V) * 2.0


def _universe(V, k, d, seed):
    """Full k-ary tree of depth d: children = k most probable tokens (probability space, scipy softmax)."""
    nodes = []          # (path, parent index or -1, phat)
    frontier = [((), -1, 1.0)]
    for _ in range(d):
        nxt = []
        for path, idx, phat in frontier:
            p = scipy.special.softmax(_path_row(path, V, seed))
            top = sorted(range(V), key=lambda i: (-p[i], i))[:k]
            for tkn in top:
                nodes.append((path + (tkn,), idx, phat * p[tkn]))
                nxt.append((path + (tkn,), len(nodes) - 1, phat * p[tkn]))
        frontier = nxt
    return nodes


def _best_closed_subset(nodes, n):
    """Enumerate every ancestor-closed n-subset (nodes are in BFS order: parents come first)."""
    best = (-1.0, None)
    N = len(nodes)

    def rec(i, chosen, total):
        nonlocal best
        if len(chosen) == n:
            if total > best[0]:
                best = (total, frozenset(chosen))
            return
        if i == N or len(chosen) + (N - i) < n:
            return
        par = nodes[i][1]
        if par == -1 or par in chosen:
            chosen.add(i)
            rec(i + 1, chosen, total + nodes[i][2])
            chosen.remove(i)
        rec(i + 1, chosen, total)

    rec(0, set(), 0.0)
    return best


def _run_streaming(V, k, n, d, seed):
    b = ot.TreeBuilder(k, n)
    paths = [()]
    for _ in range(d):
        rows = np.stack([_path_row(p, V, seed) for p in paths])
        tok, par = b.expand(rows)
        paths = [paths[int(pj)] + (int(tk),) for tk, pj in zip(tok, par)]
    return b, b.finalize()


@pytest.mark.parametrize("V,k,d,n,seed", [
    (6, 2, 3, 3, 0), (6, 2, 3, 5, 1), (7, 3, 3, 4, 2), (8, 3, 3, 6, 3), (6, 2, 4, 6, 4), (5, 2, 4, 7, 5),
    (8, 3, 2, 5, 6), (6, 3, 3, 1, 7), (6, 2, 3, 14, 8),
])
def test_greedy_tree_is_the_brute_force_optimum(V, k, d, n, seed):
    nodes = _universe(V, k, d, seed)
    n_eff = min(n, len(nodes))
    best_E, best_set = _best_closed_subset(nodes, n_eff)
    b, out = _run_streaming(V, k, n, d, seed)
    assert out["n_out"] == n_eff
    assert out["expect"] == pytest.approx(best_E, rel=1e-12)
    # same node set: rebuild each chosen node's token path from parent[]
    got = set()
    for i in range(out["n_out"]):
        path, j = [], i
        while j >= 0:
            path.append(int(out["token"][j]))
            j = int(out["parent"][j])
        got.add(tuple(reversed(path)))
    want = {nodes[i][0] for i in best_set}
    assert got == want


# ---------------------------------------------------------------- theorems and invariants
def _random_logits(V, k, n, d, seed, scale=3.0):
    return np.random.default_rng(seed).standard_normal((d, n, V)) * scale


@pytest.mark.parametrize("V,k,n,d,seed", [(50, 3, 8, 5, 0), (200, 4, 16, 4, 1), (64, 5, 70, 4, 2), (1000, 4, 16, 4, 3)])
def test_closure_monotone_scores_and_mask(V, k, n, d, seed):
    out = ot.build_tree(_random_logits(V, k, n, d, seed), k, n, d)
    m = out["n_out"]
    for i in range(m):
        p = int(out["parent"][i])
        assert p < i                                            # parents first
        if p >= 0:
            assert out["score"][p] > out["score"][i]            # Thm. 3.1
            assert out["depth"][i] == out["depth"][p] + 1
        else:
            assert out["depth"][i] == 1
        # mask row = walk to the root
        want, j = 0, i
        while j >= 0:
            want |= 1 << j
            j = int(out["parent"][j])
        got = sum(int(out["mask"][i][w]) << (64 * w) for w in range(out["mask"].shape[1]))
        assert got == want
        assert bin(got).count("1") == out["depth"][i]
    assert np.all(out["score"][:m] < 0)
    assert 0 < out["expect"] <= d + 1e-12                        # each layer's p^ sum to <= 1
    np.testing.assert_array_equal(out["mask"][:m], ot.ancestor_mask(out["parent"][:m])[:, : out["mask"].shape[1]])


def test_layer_probability_mass_at_most_one():
    out = ot.build_tree(_random_logits(30, 3, 9, 4, 5), 3, 9, 4)
    for layer in out["layers"]:
        assert np.exp(layer["score"]).sum() <= 1.0 + 1e-12


def test_e_sub_is_monotone_in_drafting_steps_and_prefix_stable():
    V, k, n, dmax = 40, 3, 10, 6
    logits = _random_logits(V, k, n, dmax, 11)
    prev_E, prev_layers = 0.0, None
    for d in range(1, dmax + 1):
        out = ot.build_tree(logits[:d], k, n, d)
        assert out["expect"] >= prev_E - 1e-15                  # Thm. 3.2
        if prev_layers is not None:
            for a, b_ in zip(prev_layers, out["layers"]):
                np.testing.assert_array_equal(a["token"], b_["token"])
        prev_E, prev_layers = out["expect"], out["layers"]


def test_special_case_n_equals_one_is_argmax_of_root_row():
    logits = _random_logits(100, 4, 1, 3, 7)
    out = ot.build_tree(logits, 4, 1, 3)
    assert out["n_out"] == 1 and out["token"][0] == int(np.argmax(logits[0, 0]))
    assert out["parent"][0] == -1 and out["depth"][0] == 1
    assert out["expect"] == pytest.approx(float(scipy.special.softmax(logits[0, 0]).max()), rel=1e-12)


def test_special_case_k_equals_one_is_a_greedy_chain():
    V, n, d = 50, 8, 5
    logits = _random_logits(V, 1, n, d, 9)
    out = ot.build_tree(logits, 1, n, d)
    assert out["n_out"] == d                                     # pool has only d nodes
    p = 1.0
    for t in range(d):
        assert out["token"][t] == int(np.argmax(logits[t, 0]))
        assert out["parent"][t] == t - 1
        p *= float(scipy.special.softmax(logits[t, 0]).max())
        assert math.exp(out["score"][t]) == pytest.approx(p, rel=1e-12)
    assert np.all(out["token"][d:] == -1) and np.all(out["depth"][d:] == 0)
    assert np.all(out["mask"][d:] == 0)


def test_budget_larger_than_pool_returns_whole_pool():
    V, k, d, n = 20, 2, 3, 64
    out = ot.build_tree(_random_logits(V, k, n, d, 13), k, n, d)
    assert out["n_out"] == 2 + 4 + 8


def test_planted_peaks_are_followed():
    V, k, n, d = 500, 3, 6, 4
    logits = _random_logits(V, k, n, d, 17, scale=1.0)
    peaks = [17, 230, 41, 499]
    for t in range(d):
        logits[t, 0, peaks[t]] += 40.0                           # slot 0 of each layer is the best path
    out = ot.build_tree(logits, k, n, d)
    chain = [i for i in range(out["n_out"]) if out["depth"][i] == i + 1 and (i == 0 or out["parent"][i] == i - 1)]
    assert [int(out["token"][i]) for i in range(d) if out["depth"][i] >= 1][:1] == [peaks[0]]
    # the all-peaks path is in the tree
    j, path = None, []
    for i in range(out["n_out"]):
        if out["depth"][i] == d:
            q, path = i, []
            while q >= 0:
                path.append(int(out["token"][q])); q = int(out["parent"][q])
            if list(reversed(path)) == peaks:
                j = i
    assert j is not None


def test_tie_rules_on_constant_rows():
    # every candidate of a row ties; every row ties with every other row
    V, k, n, d = 9, 3, 4, 2
    out = ot.build_tree(np.zeros((d, n, V)), k, n, d)
    assert list(out["token"][:4]) == [0, 1, 2, 0]
    assert list(out["parent"][:4]) == [-1, -1, -1, 0]
    assert list(out["depth"][:4]) == [1, 1, 1, 2]


def test_frontier_sizes():
    assert ot.frontier_sizes(10, 50, 10)[:4] == [1, 10, 50, 50]
    assert sum(ot.frontier_sizes(10, 50, 10)[:10]) == 411
    assert sum(ot.frontier_sizes(16, 256, 20)[:20]) == 4625


# ---------------------------------------------------------------- adaptive depth (Algorithm 1's loop)
def _hand_logits():
    g = json.load(open(os.path.join(GOLDEN, "hand_tree.json")))
    logits = np.full((g["steps"], g["n"], g["vocab"]), -30.0)
    for t in range(g["steps"]):
        rows = np.log(np.array(g["rows"][str(t)], dtype=np.float64))
        logits[t, :rows.shape[0]] = rows
    return g, logits


@pytest.mark.parametrize("delta,steps", [(0.05, 3), (0.5, 3), (0.8, 2), (0.9, 1), (5.0, 1)])
def test_adaptive_depth_on_the_hand_example(delta, steps):
    # E_sub after the steps is 0.9, 1.68, 1.767 (golden file): gains 0.9, 0.78, 0.087.  The loop drafts step
    # i+1 only if gain_i > delta, and never more than 3 steps here.
    g, logits = _hand_logits()
    out = ot.build_tree_adaptive(logits, g["k"], g["n"], g["steps"], delta)
    assert out["steps"] == steps
    np.testing.assert_allclose(out["e_sub_trace"], g["e_sub_after_step"][:steps], rtol=1e-12)
    if steps == 3:
        assert list(out["token"]) == g["token"] and list(out["parent"]) == g["parent"]
    if steps == 1:                      # the tree is the root's top-k children
        assert out["n_out"] == 2 and list(out["token"][:2]) == [0, 1] and list(out["depth"][:2]) == [1, 1]


def test_adaptive_depth_reduces_to_fixed_depth_and_to_one_step():
    V, k, n, dmax = 50, 3, 8, 6
    logits = _random_logits(V, k, n, dmax, 21)
    full = ot.build_tree(logits, k, n, dmax)
    neg = ot.build_tree_adaptive(logits, k, n, dmax, -1.0)      # every gain is >= 0 > -1 (Thm. 3.2): never stops early
    assert neg["steps"] == dmax
    for key in ("token", "parent", "depth", "mask"):
        np.testing.assert_array_equal(neg[key], full[key])
    assert neg["expect"] == full["expect"]
    one = ot.build_tree_adaptive(logits, k, n, dmax, 10.0)      # no gain exceeds 10 (E <= n): one step only
    assert one["steps"] == 1
    ref = ot.build_tree(logits[:1], k, n, 1)
    np.testing.assert_array_equal(one["token"], ref["token"])


def test_adaptive_depth_trace_obeys_the_loop_condition():
    V, k, n, dmax = 60, 4, 12, 8
    for seed, delta in [(3, 0.02), (4, 0.05), (5, 0.2), (6, 0.005)]:
        logits = _random_logits(V, k, n, dmax, seed)
        out = ot.build_tree_adaptive(logits, k, n, dmax, delta)
        tr = out["e_sub_trace"]
        assert len(tr) == out["steps"]
        # E_sub after t steps is the E of the fixed-depth tree of t steps (the brute-force-pinned routine)
        for t in range(1, out["steps"] + 1):
            assert tr[t - 1] == pytest.approx(ot.build_tree(logits[:t], k, n, t)["expect"], rel=1e-13)
        gains = np.diff([0.0] + tr)
        assert np.all(gains[:-1] > delta)                       # every step but the last was licensed
        if out["steps"] < dmax:
            assert gains[-1] <= delta                           # stopped because the gain fell to delta or below


def test_frontier_masks_agree_with_the_ancestor_mask_of_the_whole_pool():
    # the pool of all layers is itself a tree; relabel its nodes densely (layer by layer), take the pinned
    # ancestor_mask of that tree and map the bits back to pool indices t * n + slot
    V, k, n, d = 30, 3, 7, 5
    out = ot.build_tree(_random_logits(V, k, n, d, 13), k, n, d)
    layers = out["layers"]
    dense, parent = {}, []
    for t, layer in enumerate(layers):
        for s in range(layer["token"].shape[0]):
            dense[(t, s)] = len(parent)
            parent.append(-1 if t == 0 else dense[(t - 1, int(layer["parent_slot"][s]))])
    am = ot.ancestor_mask(np.array(parent))
    pool_index = {v: t * n + s for (t, s), v in dense.items()}
    for upto in range(1, d + 1):
        got = ot.frontier_masks(layers[:upto], n, d)
        F = layers[upto - 1]["token"].shape[0]
        for s in range(n):
            want = set()
            if s < F:
                row = am[dense[(upto - 1, s)]]
                want = {pool_index[j] for j in range(len(parent)) if (int(row[j // 64]) >> (j % 64)) & 1}
            have = {j for j in range(d * n) if (int(got[s, j // 64]) >> (j % 64)) & 1}
            assert have == want
            if s < F:
                assert len(have) == upto            # itself and one ancestor per earlier layer


def test_attention_oracle_with_more_tree_keys_than_queries_reduces_to_the_square_case():
    # padding the tree K/V with rows no mask bit points at must not change anything
    from oracle import tree_attention as ta
    g = np.random.default_rng(3)
    B, H, n, D, L, extra = 1, 2, 5, 8, 6, 9
    Q, Kp, Vp = g.standard_normal((B, H, n, D)), g.standard_normal((B, H, L, D)), g.standard_normal((B, H, L, D))
    Kt, Vt = g.standard_normal((B, H, n, D)), g.standard_normal((B, H, n, D))
    mask = ot.ancestor_mask(np.array([-1, 0, 0, 1, 3]))[None]
    ref = ta.tree_verify_attention(Q, Kp, Vp, Kt, Vt, [L], mask)
    Kt2 = np.concatenate([Kt, g.standard_normal((B, H, extra, D))], axis=2)
    Vt2 = np.concatenate([Vt, g.standard_normal((B, H, extra, D))], axis=2)
    np.testing.assert_allclose(ta.tree_verify_attention(Q, Kp, Vp, Kt2, Vt2, [L], mask), ref, rtol=0, atol=1e-15)
