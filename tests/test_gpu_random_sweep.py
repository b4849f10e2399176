"""Seeded sweeps over many small random shapes: tree build (one-shot and streaming), tree attention and both
verifications against the oracle (needs an MI355X).  The shapes straddle the kernels' internal boundaries (one
wavefront / several, 64-key tiles, 16-byte vectors, segment and part sizes)."""
import numpy as np
import pytest

from oracle import opt_tree as ot_oracle
from oracle import tree_attention as ta_oracle
from oracle import verify as vf
import workloads as wl
from tests import _util as U

pytestmark = pytest.mark.gpu


def test_tree_build_sweep():
    import torch
    from paper_2406_17276_amd import api
    g = np.random.default_rng(101)
    done = 0
    for it in range(48):
        k = int(g.integers(1, 17))
        n = int(g.choice([1, 2, 3, 7, 16, 31, 32, 33, 50, 63, 64, 65, 100, 128, 200, 256]))
        d, B, V = int(g.integers(1, 13)), int(g.integers(1, 4)), int(g.integers(max(k, 2), 400))
        dtype, scale = str(g.choice(["f32", "bf16"])), float(g.choice([0.3, 1.0, 3.0, 8.0]))
        d = min(d, max(1, int(4e6 // (n * V * B))))
        x = wl.store((g.standard_normal((B, d, n, V)) * scale).astype(np.float32), dtype)
        want = U.oracle_trees(x, dtype, k, n, d)
        if min(t["min_gap"] for t in want) <= U.GAP:
            continue
        print(f"case {it}: V={V} k={k} n={n} d={d} B={B} {dtype} scale={scale}", flush=True)
        dev = U.to_device(x, dtype)
        got = api.build_tree(dev, k, n, d)
        torch.cuda.synchronize()
        U.assert_tree_equal(got, want, n)
        U.assert_tree_invariants(got, n, d)
        st = api.TreeStream(B, V, k, n, d, api.OT_BF16 if dtype == "bf16" else api.OT_F32)
        F = 1
        for t in range(d):
            st.expand(dev[:, t, :F])
            F = min(n, k * F)
        got = st.finalize()
        torch.cuda.synchronize()
        U.assert_tree_equal(got, want, n)
        done += 1
    assert done >= 40


def test_tree_attention_sweep():
    import torch
    from paper_2406_17276_amd import api
    g = np.random.default_rng(202)
    for it in range(40):
        dtype, D = str(g.choice(["f32", "bf16"])), int(g.choice([64, 128]))
        Hkv, grp = int(g.choice([1, 2, 3, 8])), int(g.choice([1, 2, 4, 8]))
        Hq, B = Hkv * grp, int(g.integers(1, 4))
        n = int(g.choice([1, 5, 16, 31, 32, 33, 50, 60, 64, 65, 100, 128, 200, 256]))
        Lmax = int(g.choice([0, 1, 17, 63, 64, 65, 200, 500, 1100, 2500]))
        if B * Hq * n * (Lmax + n) * D > 2e8:
            Lmax = 200
        draw = lambda *shape: wl.store(g.standard_normal(shape).astype(np.float32), dtype)
        Q, Kt, Vt = draw(B, Hq, n, D), draw(B, Hkv, n, D), draw(B, Hkv, n, D)
        Kp, Vp = draw(B, Hkv, max(Lmax, 1), D), draw(B, Hkv, max(Lmax, 1), D)
        plen = g.integers(0, Lmax + 1, size=B).astype(np.int32)
        shape = str(g.choice(["random", "chain", "star"]))
        mask = np.stack([ot_oracle.ancestor_mask(wl.random_tree_parents(n, 1000 * it + b, shape)) for b in range(B)])
        print(f"case {it}: {dtype} B={B} Hq={Hq} Hkv={Hkv} D={D} Lmax={Lmax} plen={plen.tolist()} n={n} {shape}", flush=True)
        out = api.tree_verify_attention(U.to_device(Q, dtype), U.to_device(Kp, dtype), U.to_device(Vp, dtype),
                                        U.to_device(Kt, dtype), U.to_device(Vt, dtype), torch.from_numpy(plen).cuda(),
                                        U.mask_to_device(mask))
        torch.cuda.synchronize()
        want = ta_oracle.tree_verify_attention(wl.to_f64(Q, dtype), wl.to_f64(Kp, dtype), wl.to_f64(Vp, dtype),
                                               wl.to_f64(Kt, dtype), wl.to_f64(Vt, dtype), plen, mask, None)
        assert np.abs(U.from_device_f64(out) - want).max() < (2e-2 if dtype == "bf16" else 1e-5)


def test_verification_sweep():
    """Chain trees that carry the expected ground truth, so the produced tokens are the draws / arg-maxima of all
    rows; uniform numbers keep a margin of 1e-5 to the boundaries of the oracle's CDF."""
    import torch
    from paper_2406_17276_amd import api
    g = np.random.default_rng(303)
    for it in range(30):
        dtype = str(g.choice(["f32", "bf16"]))
        V = int(g.choice([2, 3, 7, 64, 255, 256, 257, 511, 513, 1000, 2049, 4097, 9000, 40000]))
        n, B = int(g.choice([1, 2, 9, 33, 64, 100])), int(g.integers(1, 3))
        T, scale = float(g.choice([0.05, 0.3, 1.0, 2.5])), float(g.choice([0.5, 2.0, 6.0]))
        mfrac = float(g.choice([0.0, 0.0, 0.3, 0.9]))
        n = min(n, max(1, int(2e6 // (B * V)) - 1))
        x = (g.standard_normal((B, n + 1, V)) * scale).astype(np.float32)
        if mfrac > 0:
            m = g.random((B, n + 1, V)) < mfrac
            m[:, :, g.integers(V)] = False                          # at least one finite logit per row
            x[m] = -np.inf
        st = wl.store(x, dtype)
        t64 = wl.to_f64(st, dtype)
        u = np.zeros((B, n + 1), dtype=np.float32)
        for b in range(B):
            for r in range(n + 1):
                for _ in range(200):
                    cand = np.float32(g.random())
                    if cand < 1.0 and vf.sample_margin(t64[b, r], T, float(cand)) > 1e-5:
                        u[b, r] = cand
                        break
        draws = [[vf.sample_truth(t64[b, r], T, float(u[b, r])) for r in range(n + 1)] for b in range(B)]
        tops = [[int(np.argmax(t64[b, r])) for r in range(n + 1)] for b in range(B)]
        print(f"case {it}: {dtype} V={V} n={n} B={B} T={T} scale={scale} masked={mfrac}", flush=True)
        dev = U.to_device(st, dtype)
        for kind, truth in (("sample", draws), ("greedy", tops)):
            tree = api.alloc_tree(B, n)
            tree.token.copy_(torch.tensor([t[:n] for t in truth], dtype=torch.int32))
            tree.parent.copy_(torch.arange(-1, n - 1, dtype=torch.int32).repeat(B, 1))
            tree.n_out.fill_(n)
            if kind == "sample":
                alen, _, atok = api.verify_sample(dev, torch.from_numpy(u).cuda(), T, tree)
            else:
                alen, _, atok = api.verify_greedy(dev, tree)
            torch.cuda.synchronize()
            assert alen.cpu().tolist() == [n + 1] * B, kind
            np.testing.assert_array_equal(atok.cpu().numpy(), np.array(truth), err_msg=kind)
