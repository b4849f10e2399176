"""Parity of ot_verify_greedy / ot_kv_append with the oracle (needs an MI355X).  Integer results and the
moved K/V rows must be bit-exact."""
import numpy as np
import pytest

from oracle import opt_tree as ot_oracle
from oracle import verify as vf
import workloads as wl
from tests import _util as U

pytestmark = pytest.mark.gpu


def _target_rows(tree, n, V, g, agree, dtype):
    """Target logits [n + 1, V] whose most probable token at a position is, with probability `agree`, the token
    of one of that position's children in the draft tree."""
    x = (g.standard_normal((n + 1, V)) * 2.0).astype(np.float32)
    for pos in range(-1, n):
        kids = [i for i in range(tree["n_out"]) if tree["parent"][i] == pos]
        t = int(tree["token"][g.choice(kids)]) if kids and g.random() < agree else int(g.integers(V))
        x[pos + 1, t] = 12.0
    return wl.store(x, dtype)


@pytest.mark.parametrize("V,k,n,d,B,dtype,agree", [
    (1000, 4, 16, 4, 3, "f32", 0.8),
    (32000, 10, 50, 10, 2, "bf16", 0.9),       # 7B shape: 51 target rows per sequence
    (40000, 5, 70, 6, 2, "bf16", 0.95),        # two scan parts, two wavefronts of nodes
    (300, 1, 8, 8, 2, "f32", 1.0),             # a chain, accepted whole: A = n + 1
    (300, 3, 200, 3, 1, "f32", 0.5),           # n larger than the tree (n_out < n)
    (2000, 8, 256, 6, 1, "bf16", 0.9),         # maximum n
    (32000, 8, 60, 10, 16, "bf16", 0.9),       # the 70B batch: 16 sequences, 61 target rows each
])
def test_verify_and_append_match_oracle(V, k, n, d, B, dtype, agree):
    import torch
    from paper_2406_17276_amd import api
    g = np.random.default_rng(V + n)
    draft = wl.store((g.standard_normal((B, d, n, V)) * 3.0).astype(np.float32), dtype)
    trees = U.oracle_trees(draft, dtype, k, n, d)
    target = np.stack([_target_rows(trees[b], n, V, g, agree, dtype) for b in range(B)])
    want = [vf.greedy_verify(wl.to_f64(target[b], dtype), trees[b]["token"], trees[b]["parent"], trees[b]["n_out"])
            for b in range(B)]
    print("accepted lengths:", [w[0] for w in want], flush=True)

    tree_dev = api.alloc_tree(B, n)
    tree_dev.token.copy_(torch.from_numpy(np.stack([t["token"] for t in trees]).astype(np.int32)))
    tree_dev.parent.copy_(torch.from_numpy(np.stack([t["parent"] for t in trees]).astype(np.int32)))
    tree_dev.n_out.copy_(torch.tensor([t["n_out"] for t in trees], dtype=torch.int32))
    alen, anode, atok = api.verify_greedy(U.to_device(target, dtype), tree_dev)
    torch.cuda.synchronize()
    alen, anode, atok = alen.cpu().numpy(), anode.cpu().numpy(), atok.cpu().numpy()
    for b in range(B):
        A, nodes, toks = want[b]
        assert alen[b] == A
        assert list(anode[b, :A - 1]) == nodes and np.all(anode[b, A - 1:] == -1)
        assert list(atok[b, :A]) == toks and np.all(atok[b, A:] == -1)

    # K/V append: 2 KV heads, head_dim 64, room for all but the longest branch of sequence 0
    H, D, L0 = 2, 64, 37
    cap = L0 + max(1, want[0][0] - 2)
    w = wl.Workload("v", B, 8, 1, 1, n, dtype, "normal", 1.0, H, H, D, cap)
    x = wl.make_attention_inputs(w, 5)
    plen = np.full(B, L0, dtype=np.int32)
    kp, vp = U.to_device(x["K_prefix"], dtype), U.to_device(x["V_prefix"], dtype)
    kt, vt = U.to_device(x["K_tree"], dtype), U.to_device(x["V_tree"], dtype)
    new_len = api.kv_append(kp, vp, kt, vt, torch.from_numpy(plen).cuda(),
                            torch.from_numpy(alen).cuda(), torch.from_numpy(anode).cuda())
    torch.cuda.synchronize()
    got_k, got_v = U.from_device_f64(kp), U.from_device_f64(vp)
    for b in range(B):
        Kp, Vp = wl.to_f64(x["K_prefix"][b], dtype).copy(), wl.to_f64(x["V_prefix"][b], dtype).copy()
        L = vf.kv_append(Kp, Vp, wl.to_f64(x["K_tree"][b], dtype), wl.to_f64(x["V_tree"][b], dtype), L0, want[b][1])
        assert int(new_len[b]) == L
        np.testing.assert_array_equal(got_k[b], Kp)
        np.testing.assert_array_equal(got_v[b], Vp)


# ---------------------------------------------------------------------------------------------------------
# Random sampling: ot_verify_sample.  The kernel sums exp2 terms in fp32 per 16-byte vector and in fp64 above
# (relative error of a cumulative probability ~1e-6), so the uniform numbers are drawn with a margin of 1e-5
# to every boundary of the oracle's CDF; the drawn tokens and the walk must then be bit-exact.
SAMPLE_MARGIN = 1e-5


def _uniforms_with_margin(rows64, T, g):
    u = np.empty(len(rows64), dtype=np.float32)
    for r, row in enumerate(rows64):
        for _ in range(100):
            u[r] = np.float32(g.random())
            if u[r] < 1.0 and vf.sample_margin(row, T, float(u[r])) > SAMPLE_MARGIN:
                break
        else:
            raise RuntimeError("no uniform number with a margin")
    return u


def _tree_to_device(api, trees, B, n):
    import torch
    tree_dev = api.alloc_tree(B, n)
    tree_dev.token.copy_(torch.from_numpy(np.stack([t["token"] for t in trees]).astype(np.int32)))
    tree_dev.parent.copy_(torch.from_numpy(np.stack([t["parent"] for t in trees]).astype(np.int32)))
    tree_dev.n_out.copy_(torch.tensor([t["n_out"] for t in trees], dtype=torch.int32))
    return tree_dev


@pytest.mark.parametrize("V,k,n,d,B,dtype,agree,T", [
    (1000, 4, 16, 4, 3, "f32", 0.8, 1.0),
    (32000, 10, 50, 10, 2, "bf16", 0.9, 1.0),      # 7B shape
    (40000, 5, 70, 6, 2, "bf16", 0.95, 0.7),
    (300, 3, 200, 3, 1, "f32", 0.5, 1.5),          # n larger than the tree
    (32000, 8, 60, 10, 16, "bf16", 0.9, 0.8),      # the 70B batch
])
def test_sampled_verification_matches_oracle(V, k, n, d, B, dtype, agree, T):
    import torch
    from paper_2406_17276_amd import api
    g = np.random.default_rng(7 * V + n)
    draft = wl.store((g.standard_normal((B, d, n, V)) * 3.0).astype(np.float32), dtype)
    trees = U.oracle_trees(draft, dtype, k, n, d)
    target = np.stack([_target_rows(trees[b], n, V, g, agree, dtype) for b in range(B)])
    t64 = wl.to_f64(target, dtype)
    u = np.stack([_uniforms_with_margin(t64[b], T, g) for b in range(B)])
    want = [vf.sampled_verify(t64[b], T, u[b].astype(np.float64), trees[b]["token"], trees[b]["parent"],
                              trees[b]["n_out"]) for b in range(B)]
    print("accepted lengths:", [w[0] for w in want], flush=True)
    alen, anode, atok = api.verify_sample(U.to_device(target, dtype), torch.from_numpy(u).cuda(), T,
                                          _tree_to_device(api, trees, B, n))
    torch.cuda.synchronize()
    alen, anode, atok = alen.cpu().numpy(), anode.cpu().numpy(), atok.cpu().numpy()
    for b in range(B):
        A, nodes, toks = want[b]
        assert alen[b] == A
        assert list(anode[b, :A - 1]) == nodes and np.all(anode[b, A - 1:] == -1)
        assert list(atok[b, :A]) == toks and np.all(atok[b, A:] == -1)


@pytest.mark.parametrize("V,n,B,dtype,T,scale,masked", [
    (32000, 50, 2, "bf16", 1.0, 2.0, 0),           # 7B shape
    (128256, 12, 1, "bf16", 0.8, 3.0, 0),          # 251 segments: four per lane of the picking wavefront
    (262144, 3, 1, "bf16", 1.0, 3.0, 0),           # the largest supported row: 512 segments, eight per lane
    (1001, 20, 2, "f32", 1.3, 1.0, 0),             # rows not 16-byte aligned: element loads, ragged last vector
    (1003, 7, 1, "bf16", 0.9, 2.0, 0),             # the same for bf16 rows (2006 bytes apart)
    (5000, 9, 1, "bf16", 0.25, 1.5, 3000),         # 3000 tokens masked with -inf, among them whole segments
    (70, 5, 1, "f32", 4.0, 0.5, 0),                # less than one segment, nearly flat distribution
])
def test_every_row_draw_matches_oracle(V, n, B, dtype, T, scale, masked):
    """A chain whose node i carries the token the oracle draws at position i is accepted whole, so the produced
    tokens are the draws of all n + 1 rows."""
    import torch
    from paper_2406_17276_amd import api
    g = np.random.default_rng(V + n)
    x = (g.standard_normal((B, n + 1, V)) * scale).astype(np.float32)
    if masked:
        x[:, :, :2048] = -np.inf                                    # whole leading segments
        for b in range(B):
            for r in range(n + 1):
                x[b, r, g.choice(np.arange(2048, V), masked - 2048, replace=False)] = -np.inf
    target = wl.store(x, dtype)
    t64 = wl.to_f64(target, dtype)
    u = np.stack([_uniforms_with_margin(t64[b], T, g) for b in range(B)])
    u[:, 0] = 0.0                                                   # the first token with a positive probability
    draws = [[vf.sample_truth(t64[b, r], T, float(u[b, r])) for r in range(n + 1)] for b in range(B)]
    trees = [dict(token=np.array(draws[b][:n]), parent=np.arange(-1, n - 1), n_out=n) for b in range(B)]
    for b in range(B):
        assert vf.sampled_verify(t64[b], T, u[b].astype(np.float64), trees[b]["token"], trees[b]["parent"], n) == \
            (n + 1, list(range(n)), draws[b])
    alen, anode, atok = api.verify_sample(U.to_device(target, dtype), torch.from_numpy(u).cuda(), T,
                                          _tree_to_device(api, trees, B, n))
    torch.cuda.synchronize()
    assert list(alen.cpu().numpy()) == [n + 1] * B
    np.testing.assert_array_equal(atok.cpu().numpy(), np.array(draws))
    np.testing.assert_array_equal(anode.cpu().numpy(), np.tile(np.arange(n), (B, 1)))


def test_low_temperature_draw_is_the_greedy_result():
    import torch
    from paper_2406_17276_amd import api
    V, k, n, d, B, dtype = 4000, 6, 30, 5, 2, "bf16"
    g = np.random.default_rng(11)
    draft = wl.store((g.standard_normal((B, d, n, V)) * 3.0).astype(np.float32), dtype)
    trees = U.oracle_trees(draft, dtype, k, n, d)
    target = np.stack([_target_rows(trees[b], n, V, g, 0.9, dtype) for b in range(B)])
    tree_dev = _tree_to_device(api, trees, B, n)
    dev = U.to_device(target, dtype)
    u = torch.from_numpy(g.random((B, n + 1)).astype(np.float32)).cuda()
    a = api.verify_greedy(dev, tree_dev)
    b_ = api.verify_sample(dev, u, 0.02, tree_dev)                  # the boosted logit leads by > 2: e^-100
    torch.cuda.synchronize()
    for x, y in zip(a, b_):
        assert torch.equal(x, y)
