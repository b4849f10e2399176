"""A whole decoding step (tree build, tree attention, greedy verification, cache append) recorded into a HIP
graph and replayed with fresh input contents: every replay must reproduce the eager calls bit for bit
(needs an MI355X).  The entry points allocate nothing and clear their counters with kernels, which is what
makes them recordable."""
import numpy as np
import pytest

import workloads as wl
from tests import _util as U

pytestmark = pytest.mark.gpu


def test_graph_replays_of_a_decoding_step_equal_the_eager_calls():
    import ctypes as C
    import torch
    from paper_2406_17276_amd import api
    B, V, k, n, d, Hq, Hkv, D, cap, dtype = 2, 4000, 6, 40, 6, 8, 2, 128, 700, "bf16"
    g = np.random.default_rng(21)
    fresh = lambda *shape, s=1.0: U.to_device(wl.store((g.standard_normal(shape) * s).astype(np.float32), dtype), dtype)

    # static buffers of the recorded step
    draft, target = fresh(B, d, n, V, s=3.0), fresh(B, n + 1, V, s=4.0)
    Q, Kt, Vt = fresh(B, Hq, n, D), fresh(B, Hkv, n, D), fresh(B, Hkv, n, D)
    Kp, Vp = fresh(B, Hkv, cap, D), fresh(B, Hkv, cap, D)
    plen0 = torch.tensor([611, 540], dtype=torch.int32, device="cuda")
    plen = plen0.clone()
    tree, O = api.alloc_tree(B, n), torch.empty_like(Q)
    bws = torch.empty(api.build_workspace_bytes(api.build_params(draft, k, n, d)), dtype=torch.uint8, device="cuda")
    ap = api.attn_params(Q, Kp, Vp, Kt, Vt)
    aws = api.attn_workspace(ap, Q.device)
    vws = torch.empty(int(api.lib().ot_verify_workspace_bytes(C.byref(api.VerifyParams(
        B, V, n, api.OT_BF16, target.stride(0), target.stride(1))))), dtype=torch.uint8, device="cuda")

    def step():
        api.build_tree(draft, k, n, d, out=tree, workspace=bws)
        api.tree_verify_attention(Q, Kp, Vp, Kt, Vt, plen, tree.mask, out=O, workspace=aws)
        alen, anode, atok = api.verify_greedy(target, tree, workspace=vws)
        new_len = api.kv_append(Kp, Vp, Kt, Vt, plen, alen, anode)
        return alen, anode, atok, new_len

    step()                                                          # warm-up outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            g_out = step()
    torch.cuda.synchronize()

    snapshot = lambda outs: [t.clone() for t in (tree.token, tree.parent, tree.depth, tree.score, tree.mask, tree.n_out,
                                                 tree.expect, O, Kp, Vp, *outs)]
    for replay in range(4):
        print("replay", replay, flush=True)
        # fresh contents in the same buffers; the cache rows the append wrote are restored as well
        for buf, s in ((draft, 3.0), (target, 4.0), (Q, 1.0), (Kt, 1.0), (Vt, 1.0), (Kp, 1.0), (Vp, 1.0)):
            buf.copy_(fresh(*buf.shape, s=s))
        kp0, vp0 = Kp.clone(), Vp.clone()
        plen.copy_(plen0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = snapshot(g_out)
        # the program's own eager work between the replays: the same step, same inputs
        Kp.copy_(kp0); Vp.copy_(vp0)
        for t in (tree.token, tree.parent, tree.depth, tree.n_out):
            t.fill_(-7)
        O.zero_()
        eager = step()
        torch.cuda.synchronize()
        want = snapshot(eager)
        for i, (a, b) in enumerate(zip(got, want)):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"replay {replay}: output {i} differs"
        assert int(want[5].min()) > 0                                # n_out: trees were built
