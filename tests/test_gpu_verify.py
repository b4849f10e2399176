"""Parity of ot_verify_greedy / ot_kv_append with the oracle (needs an MI355X).  Integer results and the
moved K/V rows must be bit-exact."""
import numpy as np
import pytest

from oracle import opt_tree as ot_oracle
from oracle import verify as vf
from paper_2406_17276_amd import workloads as wl
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
