"""Pins for oracle/tree_attention.py against textbook routines and invariants (CPU only)."""
import numpy as np
import pytest
import scipy.special

from oracle import opt_tree as ot
from oracle import tree_attention as ta
import workloads as wl


def _inputs(B, Hq, Hkv, n, D, Lmax, seed, lens=None):
    g = np.random.default_rng(seed)
    d = dict(
        Q=g.standard_normal((B, Hq, n, D)), K_prefix=g.standard_normal((B, Hkv, max(Lmax, 1), D)),
        V_prefix=g.standard_normal((B, Hkv, max(Lmax, 1), D)), K_tree=g.standard_normal((B, Hkv, n, D)),
        V_tree=g.standard_normal((B, Hkv, n, D)),
        prefix_len=np.array(lens if lens is not None else [Lmax] * B, dtype=np.int32))
    return d


def _masks(B, n, seed, shape="random"):
    parents = [wl.random_tree_parents(n, seed + b, shape) for b in range(B)]
    return parents, np.stack([ot.ancestor_mask(p) for p in parents])


def test_chain_tree_equals_causal_attention():
    """A chain-shaped tree over a prefix is ordinary causal self-attention on the joined sequence."""
    B, H, n, D, L = 2, 3, 7, 16, 11
    x = _inputs(B, H, H, n, D, L, 0)
    _, mask = _masks(B, n, 0, "chain")
    O = ta.tree_verify_attention(**x, mask=mask)
    for b in range(B):
        for h in range(H):
            K = np.concatenate([x["K_prefix"][b, h], x["K_tree"][b, h]])
            V = np.concatenate([x["V_prefix"][b, h], x["V_tree"][b, h]])
            Qfull = np.concatenate([np.zeros((L, D)), x["Q"][b, h]])          # only the last n rows matter
            S = Qfull @ K.T / np.sqrt(D)
            S = np.where(np.tril(np.ones((L + n, L + n), dtype=bool)), S, -np.inf)
            want = (scipy.special.softmax(S, axis=-1) @ V)[L:]
            np.testing.assert_allclose(O[b, h], want, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 2)])
def test_gather_form_dense_attention_over_prefix_and_ancestors(Hq, Hkv):
    """Node i's output equals unmasked attention over just [prefix ; ancestors of i ; i]."""
    B, n, D, L = 2, 13, 8, 9
    lens = [9, 4]
    x = _inputs(B, Hq, Hkv, n, D, L, 1, lens)
    parents, mask = _masks(B, n, 5)
    O = ta.tree_verify_attention(**x, mask=mask)
    g = Hq // Hkv
    for b in range(B):
        for h in range(Hq):
            for i in range(n):
                anc, j = [], i
                while j >= 0:
                    anc.append(j); j = int(parents[b][j])
                K = np.concatenate([x["K_prefix"][b, h // g, : lens[b]], x["K_tree"][b, h // g, anc]])
                V = np.concatenate([x["V_prefix"][b, h // g, : lens[b]], x["V_tree"][b, h // g, anc]])
                w = scipy.special.softmax(K @ x["Q"][b, h, i] / np.sqrt(D))
                np.testing.assert_allclose(O[b, h, i], w @ V, rtol=1e-12, atol=1e-13)


def test_star_tree_each_node_sees_prefix_and_itself_only():
    B, H, n, D, L = 1, 2, 5, 8, 6
    x = _inputs(B, H, H, n, D, L, 2)
    _, mask = _masks(B, n, 0, "star")
    O = ta.tree_verify_attention(**x, mask=mask)
    for i in range(n):
        y = {k: (v[:, :, i:i + 1] if k in ("Q", "K_tree", "V_tree") else v) for k, v in x.items()}
        Oi = ta.tree_verify_attention(**y, mask=np.ones((B, 1, 1), dtype=np.uint64))
        np.testing.assert_allclose(O[:, :, i], Oi[:, :, 0], rtol=1e-12)


def test_relabelling_siblings_permutes_outputs():
    B, H, n, D, L = 1, 2, 6, 8, 5
    x = _inputs(B, H, H, n, D, L, 3)
    parent = np.array([-1, -1, 0, 0, 1, 2])
    perm = np.array([1, 0, 4, 3, 2, 5])            # new index i holds old node perm[i]; still parents-first
    inv = np.argsort(perm)
    parent2 = np.array([-1 if parent[perm[i]] < 0 else inv[parent[perm[i]]] for i in range(n)])
    O1 = ta.tree_verify_attention(**x, mask=ot.ancestor_mask(parent)[None])
    y = dict(x)
    for k in ("Q", "K_tree", "V_tree"):
        y[k] = x[k][:, :, perm]
    O2 = ta.tree_verify_attention(**y, mask=ot.ancestor_mask(parent2)[None])
    np.testing.assert_allclose(O2, O1[:, :, perm], rtol=1e-12, atol=1e-14)


def test_gqa_equals_mha_with_replicated_kv_heads():
    B, Hq, Hkv, n, D, L = 1, 6, 2, 5, 8, 7
    x = _inputs(B, Hq, Hkv, n, D, L, 4)
    _, mask = _masks(B, n, 9)
    O = ta.tree_verify_attention(**x, mask=mask)
    y = dict(x)
    for k in ("K_prefix", "V_prefix", "K_tree", "V_tree"):
        y[k] = np.repeat(x[k], Hq // Hkv, axis=1)
    np.testing.assert_allclose(ta.tree_verify_attention(**y, mask=mask), O, rtol=1e-13)


def test_constant_values_give_constant_output_and_scale_override():
    B, H, n, D, L = 1, 2, 9, 4, 3
    x = _inputs(B, H, H, n, D, L, 5)
    x["V_prefix"][:] = 2.5
    x["V_tree"][:] = 2.5
    _, mask = _masks(B, n, 1)
    np.testing.assert_allclose(ta.tree_verify_attention(**x, mask=mask), 2.5, rtol=1e-13)
    # scale 0 => uniform weights over the visible keys
    x = _inputs(B, H, H, n, D, L, 6)
    parents, mask = _masks(B, n, 2)
    O = ta.tree_verify_attention(**x, mask=mask, scale=0.0)
    i = n - 1
    anc, j = [], i
    while j >= 0:
        anc.append(j); j = int(parents[0][j])
    want = (x["V_prefix"][0, 0, :L].sum(0) + x["V_tree"][0, 0, anc].sum(0)) / (L + len(anc))
    np.testing.assert_allclose(O[0, 0, i], want, rtol=1e-12)


def test_empty_prefix_and_wide_mask_words():
    B, H, n, D = 1, 1, 70, 4          # two mask words
    x = _inputs(B, H, H, n, D, 0, 7, lens=[0])
    parents, mask = _masks(B, n, 3)
    assert mask.shape == (1, n, 2)
    O = ta.tree_verify_attention(**x, mask=mask)
    roots = [i for i in range(n) if parents[0][i] < 0]
    for i in roots:                    # a root child with no prefix sees only itself
        np.testing.assert_allclose(O[0, 0, i], x["V_tree"][0, 0, i], rtol=1e-13)
