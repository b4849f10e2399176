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


# ---------------------------------------------------------------------------
# 8-bit K/V cache: the format's plumbing (workloads.py) and the oracle's reading
# ---------------------------------------------------------------------------
def test_e4m3_decode_against_the_format_definition():
    """Values written out from the format's definition: bias 7, three mantissa bits, subnormals m * 2^-9, no
    infinities, one NaN code per sign, largest finite value 448."""
    dec = wl.e4m3_bits_to_f32
    hand = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x38: 1.0, 0x39: 1.125, 0x3C: 1.5,
            0x40: 2.0, 0x7E: 448.0, 0x77: 240.0, 0xB8: -1.0, 0xFE: -448.0, 0x81: -2.0 ** -9}
    for code, val in hand.items():
        assert float(dec(np.array([code], dtype=np.uint8))[0]) == val, hex(code)
    allv = dec(np.arange(256, dtype=np.uint8))
    assert np.isnan(allv[0x7F]) and np.isnan(allv[0xFF]) and np.isfinite(np.delete(allv, [0x7F, 0xFF])).all()
    assert np.all(np.diff(allv[:0x7F]) > 0)                              # codes 0..0x7e increase strictly
    assert np.array_equal(allv[0x80:0xFF], -allv[:0x7F])                # the sign bit mirrors
    assert np.signbit(allv[0x80]) and allv[0x80] == 0.0                 # minus zero
    assert np.array_equal(allv[:0x7F].astype(np.float32).view(np.uint32) & 0xFFFF, np.zeros(0x7F, dtype=np.uint32))   # every value is a bf16 value


def test_e4m3_rounding_is_to_nearest_even_and_saturates():
    enc, dec = wl.f32_to_e4m3_bits, wl.e4m3_bits_to_f32
    codes = np.arange(256, dtype=np.uint8)
    finite = np.delete(codes, [0x7F, 0xFF])
    assert np.array_equal(enc(dec(finite)), finite)                     # every code is a fixed point
    # halfway between neighbours goes to the even code; just off halfway goes to the nearer one
    t = dec(np.arange(0x7F, dtype=np.uint8)).astype(np.float64)
    for i in range(0x7E):
        mid = np.float32((t[i] + t[i + 1]) / 2)
        if float(mid) == (t[i] + t[i + 1]) / 2:
            assert int(enc(np.array([mid]))[0]) == (i if i % 2 == 0 else i + 1)
        assert int(enc(np.array([np.float32(t[i] + 0.26 * (t[i + 1] - t[i]))]))[0]) == i
        assert int(enc(np.array([np.float32(t[i] + 0.74 * (t[i + 1] - t[i]))]))[0]) == i + 1
    assert int(enc(np.array([1e6], dtype=np.float32))[0]) == 0x7E and int(enc(np.array([-1e6], dtype=np.float32))[0]) == 0xFE
    assert int(enc(np.array([0.0], dtype=np.float32))[0]) == 0 and int(enc(np.array([-0.0], dtype=np.float32))[0]) == 0x80
    g = np.random.default_rng(3)
    x = (g.standard_normal(20000) * 3).astype(np.float32)
    err = np.abs(dec(enc(x)).astype(np.float64) - x)
    table = np.abs(dec(finite).astype(np.float64))
    nearest = np.abs(np.abs(x.astype(np.float64))[:, None] - table[None, :]).min(axis=1)
    np.testing.assert_allclose(err, nearest, rtol=0, atol=0)            # brute force: no code is nearer


def test_fp8_cache_attention_is_the_plain_attention_of_the_dequantised_cache():
    """Scales of one make it the plain oracle on the decoded bytes; scaling K by s is scaling the softmax scale by s;
    scaling V by s scales O by s (the two places a scale factor can act)."""
    B, Hq, Hkv, n, D, L = 2, 4, 2, 6, 16, 9
    g = np.random.default_rng(5)
    x = _inputs(B, Hq, Hkv, n, D, L, 7, lens=[9, 4])
    _, mask = _masks(B, n, 3)
    q8 = lambda a: wl.f32_to_e4m3_bits(a.astype(np.float32))
    K8p, V8p, K8t, V8t = q8(x["K_prefix"]), q8(x["V_prefix"]), q8(x["K_tree"]), q8(x["V_tree"])
    one = np.ones((B, Hkv))
    base = ta.tree_verify_attention_fp8kv(x["Q"], K8p, V8p, K8t, V8t, one, one, x["prefix_len"], mask, wl.e4m3_bits_to_f32)
    d = lambda a: wl.e4m3_bits_to_f32(a).astype(np.float64)
    plain = ta.tree_verify_attention(x["Q"], d(K8p), d(V8p), d(K8t), d(V8t), x["prefix_len"], mask)
    np.testing.assert_array_equal(base, plain)
    ks, vs = g.uniform(0.5, 2.0, (B, Hkv)), g.uniform(0.5, 2.0, (B, Hkv))
    got = ta.tree_verify_attention_fp8kv(x["Q"], K8p, V8p, K8t, V8t, ks, vs, x["prefix_len"], mask, wl.e4m3_bits_to_f32)
    for b in range(B):
        for hk in range(Hkv):
            hs = slice(hk * (Hq // Hkv), (hk + 1) * (Hq // Hkv))
            sub = ta.tree_verify_attention(x["Q"][b:b + 1, hs], d(K8p)[b:b + 1, hk:hk + 1], d(V8p)[b:b + 1, hk:hk + 1],
                                           d(K8t)[b:b + 1, hk:hk + 1], d(V8t)[b:b + 1, hk:hk + 1], x["prefix_len"][b:b + 1],
                                           mask[b:b + 1], scale=ks[b, hk] / np.sqrt(D))
            np.testing.assert_allclose(got[b:b + 1, hs], vs[b, hk] * sub, rtol=1e-12, atol=1e-14)
