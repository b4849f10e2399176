"""Three consecutive decoding steps of Algorithm 2 on the GPU, every call fed by the device outputs of the
call before it (tree -> mask of the attention; verification -> cache append -> prefix lengths of the next
step's attention), against the same chain of oracle functions on the host (needs an MI355X)."""
import numpy as np
import pytest

from oracle import tree_attention as ta_oracle
from oracle import verify as vf
import workloads as wl
from tests import _util as U

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-5, "bf16": 2e-2}


def _leaning_target(tree, n, V, g, dtype):
    x = (g.standard_normal((n + 1, V)) * 2.0).astype(np.float32)
    for pos in range(-1, n):
        kids = [i for i in range(tree["n_out"]) if tree["parent"][i] == pos]
        if kids and g.random() < 0.9:
            x[pos + 1, int(tree["token"][g.choice(kids)])] = 9.0
    return wl.store(x, dtype)


@pytest.mark.parametrize("dtype,V,k,n,d,Hq,Hkv,D", [("bf16", 2000, 5, 24, 5, 4, 2, 64), ("f32", 600, 4, 40, 4, 2, 2, 128)])
def test_three_decoding_steps_chain_like_the_oracle(dtype, V, k, n, d, Hq, Hkv, D):
    import torch
    from paper_2406_17276_amd import api
    B, cap, T = 2, 96, 0.9
    g = np.random.default_rng(V + n)
    draw = lambda *shape: wl.store(g.standard_normal(shape).astype(np.float32), dtype)
    Kp, Vp = draw(B, Hkv, cap, D), draw(B, Hkv, cap, D)
    plen = np.array([37, 50], dtype=np.int32)
    kp_d, vp_d = U.to_device(Kp, dtype), U.to_device(Vp, dtype)
    plen_d = torch.from_numpy(plen).cuda()
    Kp64, Vp64 = wl.to_f64(Kp, dtype).copy(), wl.to_f64(Vp, dtype).copy()

    for it in range(3):
        print("decoding step", it, "prefix lengths", list(plen), flush=True)
        for _ in range(8):                                           # draft logits with clear selection cuts
            draft = wl.store((g.standard_normal((B, d, n, V)) * 3.0).astype(np.float32), dtype)
            trees = U.oracle_trees(draft, dtype, k, n, d)
            if min(t["min_gap"] for t in trees) > U.GAP:
                break
        else:
            raise RuntimeError("no draft logits with the required score gap")
        tree_d = api.build_tree(U.to_device(draft, dtype), k, n, d)
        U.assert_tree_equal(tree_d, trees, n)

        Q, Kt, Vt = draw(B, Hq, n, D), draw(B, Hkv, n, D), draw(B, Hkv, n, D)
        kt_d, vt_d = U.to_device(Kt, dtype), U.to_device(Vt, dtype)
        O = api.tree_verify_attention(U.to_device(Q, dtype), kp_d, vp_d, kt_d, vt_d, plen_d, tree_d.mask)
        want_O = ta_oracle.tree_verify_attention(wl.to_f64(Q, dtype), Kp64, Vp64, wl.to_f64(Kt, dtype), wl.to_f64(Vt, dtype),
                                                 plen, np.stack([t["mask"] for t in trees]), None)
        assert np.abs(U.from_device_f64(O) - want_O).max() < TOL[dtype]

        target = np.stack([_leaning_target(trees[b], n, V, g, dtype) for b in range(B)])
        t64 = wl.to_f64(target, dtype)
        if it % 2 == 0:
            want = [vf.greedy_verify(t64[b], trees[b]["token"], trees[b]["parent"], trees[b]["n_out"]) for b in range(B)]
            alen, anode, atok = api.verify_greedy(U.to_device(target, dtype), tree_d)
        else:
            u = np.empty((B, n + 1), dtype=np.float32)
            for b in range(B):
                for r in range(n + 1):
                    while True:
                        u[b, r] = np.float32(g.random())
                        if u[b, r] < 1.0 and vf.sample_margin(t64[b, r], T, float(u[b, r])) > 1e-5:
                            break
            want = [vf.sampled_verify(t64[b], T, u[b].astype(np.float64), trees[b]["token"], trees[b]["parent"],
                                      trees[b]["n_out"]) for b in range(B)]
            alen, anode, atok = api.verify_sample(U.to_device(target, dtype), torch.from_numpy(u).cuda(), T, tree_d)
        print("  produced tokens per sequence:", [w[0] for w in want], flush=True)
        plen_d = api.kv_append(kp_d, vp_d, kt_d, vt_d, plen_d, alen, anode)
        torch.cuda.synchronize()
        for b in range(B):
            A, nodes, toks = want[b]
            assert int(alen[b]) == A
            assert list(anode[b, :A - 1].cpu().numpy()) == nodes and list(atok[b, :A].cpu().numpy()) == toks
            plen[b] = vf.kv_append(Kp64[b], Vp64[b], wl.to_f64(Kt[b], dtype), wl.to_f64(Vt[b], dtype), plen[b], nodes)
        np.testing.assert_array_equal(plen_d.cpu().numpy(), plen)
        np.testing.assert_array_equal(U.from_device_f64(kp_d), Kp64)
        np.testing.assert_array_equal(U.from_device_f64(vp_d), Vp64)
    assert plen.sum() > 37 + 50                                      # something was accepted on the way
