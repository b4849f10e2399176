"""Parity of ot_build_tree / ot_tree_expand / ot_tree_finalize with the fp64 oracle (needs an MI355X).

Tree structure (tokens, parents, depths, masks, n_out) must be bit-exact; log p^ within 1e-5 absolute
and E within 1e-6 relative (fp32 exp-sum with fp64 combination, error budget ~1e-7 per row).
Inputs are regenerated with the next seed until every selection cut has a cross-parent gap > 1e-5."""
import numpy as np
import pytest

from oracle import opt_tree as ot_oracle
import workloads as wl
from tests import _util as U

pytestmark = pytest.mark.gpu


def _run(logits_stored, dtype, k, n, depth):
    from paper_2406_17276_amd import api
    import torch
    dev = U.to_device(logits_stored, dtype)
    tree = api.build_tree(dev, k, n, depth)
    torch.cuda.synchronize()
    return tree


@pytest.mark.parametrize("name", ["tiny", "7b", "13b"])
def test_full_config_single_sequence(name):
    w = wl.WORKLOADS[name]
    seed, logits, want = U.gapped_logits(w, 0)
    print(f"{name}: seed {seed}, min gap {min(t['min_gap'] for t in want):.3e}", flush=True)
    got = _run(logits, w.dtype, w.k, w.n, w.depth)
    U.assert_tree_equal(got, want, w.n)


def test_70b_shape_batched_subset():
    # full per-sequence shape (V=32000, d=10, k=8, n=60), 4 of the 16 sequences: the oracle stays in seconds
    w = wl.WORKLOADS["70b"]
    seed, logits, want = U.gapped_logits(w, 0, seqs=[0, 5, 10, 15])
    got = _run(logits, w.dtype, w.k, w.n, w.depth)
    U.assert_tree_equal(got, want, w.n)


def test_70b_full_batch_as_the_bench_launches_it():
    # all 16 sequences in one launch; sequences 0, 5, 10, 15 against the oracle, the invariants on every one
    w = wl.WORKLOADS["70b"]
    seed, _, want = U.gapped_logits(w, 0, seqs=[0, 5, 10, 15])
    logits = wl.make_logits(w, seed)
    got = _run(logits, w.dtype, w.k, w.n, w.depth)
    U.assert_tree_invariants(got, w.n, w.depth)
    import torch
    from paper_2406_17276_amd import api
    sub = api.alloc_tree(4, w.n)
    idx = torch.tensor([0, 5, 10, 15], device="cuda")
    for name in ("token", "parent", "depth", "score", "mask", "n_out", "expect"):
        getattr(sub, name).copy_(getattr(got, name)[idx])
    U.assert_tree_equal(sub, want, w.n)


@pytest.mark.timeout(900)
def test_large_budget_shape_full_depth_against_the_oracle():
    # The Large workload's own configuration for one sequence: vocabulary 128256 (four scan parts), k = 16, n = 256,
    # all 20 drafting steps, logits 5 N(0,1) with planted peaks.  The oracle needs about a minute for the 4625 rows.
    w = wl.WORKLOADS["large"]
    print("large, full depth: drawing the logits and running the oracle", flush=True)
    seed, logits, want = U.gapped_logits(w, 0, seqs=[0])
    print(f"large, full depth: seed {seed}, min gap {want[0]['min_gap']:.3g}; GPU build", flush=True)
    got = _run(logits, w.dtype, w.k, w.n, w.depth)
    assert want[0]["n_out"] == w.n
    U.assert_tree_equal(got, want, w.n)
    U.assert_tree_invariants(got, w.n, w.depth)


def test_large_budget_shape_full_depth_invariants():
    # n = 256, k = 16, 20 drafting steps, vocabulary 128256 (four scan parts): two more sequences, drawn on the
    # device, under the invariants of Algorithm 1's output (the oracle comparison at this size is the test above)
    import torch
    from paper_2406_17276_amd import api
    w = wl.WORKLOADS["large"]
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    x = torch.empty((2, w.depth, w.n, w.vocab), dtype=torch.bfloat16, device="cuda")
    for t in range(w.depth):                                          # step by step: keeps the fp32 temporary small
        x[:, t] = (torch.randn((2, w.n, w.vocab), generator=g, device="cuda") * 3.0).to(torch.bfloat16)
    got = api.build_tree(x, w.k, w.n, w.depth)
    torch.cuda.synchronize()
    assert int(got.n_out.min()) == w.n
    U.assert_tree_invariants(got, w.n, w.depth)


def test_large_budget_shape_reduced_depth():
    # n=256 (4 mask words, 4 wavefronts), k=16, vocab 128256 split over 4 scan parts; 1 sequence, and
    # 6 instead of 20 drafting steps so that the oracle finishes in ~20 s
    import dataclasses
    w = dataclasses.replace(wl.WORKLOADS["large"], depth=6)
    seed, logits, want = U.gapped_logits(w, 0, seqs=[0])
    got = _run(logits, w.dtype, w.k, w.n, w.depth)
    U.assert_tree_equal(got, want, w.n)


def _random_case(V, k, n, d, B, dtype, seed, scale=3.0):
    g = np.random.default_rng(seed)
    for s in range(seed, seed + 16):
        x = (g.standard_normal((B, d, n, V)) * scale).astype(np.float32)
        stored = wl.store(x, dtype)
        want = U.oracle_trees(stored, dtype, k, n, d)
        if min(t["min_gap"] for t in want) > U.GAP:
            return stored, want
    raise RuntimeError("no gapped input")


@pytest.mark.parametrize("V,k,n,d,B,dtype", [
    (1000, 4, 16, 4, 3, "f32"),        # Tiny shape, batched
    (1001, 3, 7, 5, 2, "f32"),         # vocab not a multiple of the vector width -> scalar loads
    (777, 5, 33, 3, 2, "bf16"),
    (50, 16, 64, 3, 1, "f32"),         # k = 16, tiny vocab (most scan groups empty)
    (9000, 10, 50, 6, 2, "bf16"),      # 1024-thread scan with a ragged tail
    (40000, 6, 20, 4, 2, "bf16"),      # two scan parts + merge
    (70001, 2, 100, 9, 1, "f32"),      # three parts, unaligned vocab, 2 waves of selection
    (300, 1, 8, 5, 2, "f32"),          # k = 1: a chain, pool smaller than n
    (300, 4, 1, 3, 2, "f32"),          # n = 1
    (300, 2, 200, 4, 1, "f32"),        # n larger than the pool (2+4+8+16)
    (2048, 12, 130, 3, 2, "bf16"),     # 3 waves
    (512, 8, 256, 32, 1, "f32"),       # maximum n and depth
    (200, 16, 64, 26, 2, "f32"),       # one wavefront, but the row table exceeds LDS: general path
    (3000, 10, 64, 20, 1, "bf16"),     # one wavefront, deep tree, row table in LDS
    (400, 8, 60, 10, 16, "f32"),       # a batch of 70B-shaped trees
    (300, 16, 40, 2, 2, "f32"),        # depth 2: first cut at the second step
    (300, 3, 64, 7, 3, "f32"),         # frontier grows 1, 3, 9, 27, 64
    (300, 4, 64, 8, 50, "f32"),        # 17050 rows: more work items than workgroups (grid-stride scan)
    (262144, 16, 6, 2, 1, "bf16"),     # maximum vocabulary: eight scan parts per row, maximum k
])
def test_random_shapes_and_edges(V, k, n, d, B, dtype):
    stored, want = _random_case(V, k, n, d, B, dtype, seed=V + k + n)
    got = _run(stored, dtype, k, n, d)
    U.assert_tree_equal(got, want, n)


def test_constant_rows_exercise_every_tie_rule():
    # all logits equal: top-k ties by token id (candidate-list overflow path), layer cuts tie by
    # (parent slot, rank), the final cut ties by (depth, slot)
    for V, k, n, d, dtype in [(4096, 3, 10, 3, "f32"), (33000, 4, 9, 2, "bf16"), (64, 2, 5, 4, "f32")]:
        stored = wl.store(np.zeros((1, d, n, V), dtype=np.float32), dtype)
        want = U.oracle_trees(stored, dtype, k, n, d)
        got = _run(stored, dtype, k, n, d)
        U.assert_tree_equal(got, want, n)


def test_quantised_rows_with_many_exact_ties():
    g = np.random.default_rng(5)
    V, k, n, d = 5000, 8, 24, 4
    x = g.integers(-6, 7, size=(2, d, n, V)).astype(np.float32)      # 13 distinct values: huge tie groups
    x += (g.standard_normal((2, d, n, 1)) * 0.37).astype(np.float32)  # rows differ, ties inside rows stay
    stored = wl.store(x, "f32")
    want = U.oracle_trees(stored, "f32", k, n, d)
    assert min(t["min_gap"] for t in want) > U.GAP
    got = _run(stored, "f32", k, n, d)
    U.assert_tree_equal(got, want, n)


def test_strided_logits_view():
    import torch
    from paper_2406_17276_amd import api
    V, k, n, d, B = 1000, 4, 16, 4, 2
    stored, want = _random_case(V, k, n, d, B, "f32", seed=99)
    big = torch.zeros((B, d + 1, n + 3, V + 24), dtype=torch.float32, device="cuda")
    view = big[:, :d, :n, 8:8 + V]          # 16-byte aligned start, padded strides
    view.copy_(U.to_device(stored, "f32"))
    got = api.build_tree(view, k, n, d)
    torch.cuda.synchronize()
    U.assert_tree_equal(got, want, n)
    view2 = big[:, :d, :n, 3:3 + V]         # misaligned start: scalar-load path
    view2.copy_(U.to_device(stored, "f32"))
    got = api.build_tree(view2, k, n, d)
    torch.cuda.synchronize()
    U.assert_tree_equal(got, want, n)


def test_streaming_matches_oracle_layer_by_layer():
    """Drive expand() the way a decoder would: the rows of step t+1 depend on the frontier of step t."""
    import torch
    from paper_2406_17276_amd import api
    V, k, n, d, B = 3000, 5, 40, 6, 2

    def row_for(b, path):
        h = np.random.SeedSequence([1234, b, len(path)] + [int(p) + 1 for p in path])
        return (np.random.default_rng(h).standard_normal(V) * 3.0).astype(np.float32)

    builders = [ot_oracle.TreeBuilder(k, n) for _ in range(B)]
    paths = [[()] for _ in range(B)]
    stream = api.TreeStream(B, V, k, n, d, api.OT_F32)
    for t in range(d):
        F = len(paths[0])
        rows = np.zeros((B, n, V), dtype=np.float32)
        for b in range(B):
            for j, p in enumerate(paths[b]):
                rows[b, j] = row_for(b, p)
        ftok, fpar = stream.expand(torch.from_numpy(rows).cuda())
        torch.cuda.synchronize()
        ftok, fpar = ftok.cpu().numpy(), fpar.cpu().numpy()
        fcnt = stream.frontier_count.cpu().numpy()
        for b in range(B):
            tok, par = builders[b].expand(rows[b, :F].astype(np.float64))
            Fn = len(tok)
            assert fcnt[b] == Fn                       # rows the draft model owes for the next step
            np.testing.assert_array_equal(ftok[b, :Fn], tok)
            np.testing.assert_array_equal(fpar[b, :Fn], par)
            paths[b] = [paths[b][int(pj)] + (int(tk),) for tk, pj in zip(tok, par)]
    want = [bld.finalize() for bld in builders]
    assert min(wnt["min_gap"] for wnt in want) > U.GAP
    got = stream.finalize()
    torch.cuda.synchronize()
    U.assert_tree_equal(got, want, n)


def test_expected_length_grows_with_depth():
    # Thm. 3.2 on the GPU path: E of the depth-t tree is non-decreasing in t
    w = wl.WORKLOADS["tiny"]
    logits = wl.make_logits(w, 3)
    prev = 0.0
    for d in range(1, w.depth + 1):
        got = _run(logits, w.dtype, w.k, w.n, d)
        e = float(got.expect.cpu()[0])
        assert e >= prev - 1e-12
        prev = e


def test_repeated_calls_are_bit_identical():
    import torch
    w = wl.WORKLOADS["7b"]
    logits = wl.make_logits(w, 1)
    a = _run(logits, w.dtype, w.k, w.n, w.depth)
    for _ in range(3):
        b = _run(logits, w.dtype, w.k, w.n, w.depth)
        for f in ("token", "parent", "depth", "mask", "score", "expect"):
            assert torch.equal(getattr(a, f), getattr(b, f)), f


def test_adaptive_depth_matches_oracle():
    """Algorithm 1's loop through ot_tree_expand / ot_tree_esub / ot_tree_finalize: E_sub after every step,
    the go-on decision and the final tree of every sequence, for sequences that stop at different depths."""
    import torch
    from paper_2406_17276_amd import api
    V, k, n, dmax, B = 2000, 6, 30, 8, 5
    g = np.random.default_rng(77)
    # sequences differ in how peaked their rows are, hence in how fast E_sub saturates
    scales = np.array([0.5, 1.5, 3.0, 5.0, 8.0])
    delta = 0.01
    for attempt in range(8):
        x = (g.standard_normal((B, dmax, n, V)) * scales[:, None, None, None]).astype(np.float32)
        full = [ot_oracle.build_tree_adaptive(x[b].astype(np.float64), k, n, dmax, -1.0) for b in range(B)]
        gains = np.array([np.diff([0.0] + f["e_sub_trace"]) for f in full])
        margin = np.abs(gains - delta).min()              # no decision within rounding distance of delta
        want = [ot_oracle.build_tree_adaptive(x[b].astype(np.float64), k, n, dmax, delta) for b in range(B)]
        if margin > 1e-5 and min(w["min_gap"] for w in want) > U.GAP and len({w["steps"] for w in want}) >= 3:
            break
    else:
        raise RuntimeError("no suitable input")
    print("steps per sequence:", [w["steps"] for w in want], "delta", delta, flush=True)
    stream = api.TreeStream(B, V, k, n, dmax, api.OT_F32)
    dev = torch.from_numpy(x).cuda()
    active = [True] * B
    for t in range(dmax):
        stream.expand(dev[:, t])
        fcnt = stream.frontier_count.cpu().numpy()
        e_sub, go = stream.e_sub(delta)
        torch.cuda.synchronize()
        e_sub, go = e_sub.cpu().numpy(), go.cpu().numpy()
        for b in range(B):
            assert fcnt[b] == (min(n, k ** (t + 1)) if active[b] else 0)      # a stopped sequence asks for no rows
            if active[b]:
                assert e_sub[b] == pytest.approx(want[b]["e_sub_trace"][t], rel=1e-6)      # fp32 exp-sums behind every lse
                expect_go = t + 1 < want[b]["steps"] or (want[b]["steps"] == dmax and t + 1 == dmax and
                                                         np.diff([0.0] + want[b]["e_sub_trace"])[-1] > delta)
                assert bool(go[b]) == expect_go
                active[b] = bool(go[b])
            else:
                assert go[b] == 0
                assert e_sub[b] == pytest.approx(want[b]["e_sub_trace"][-1], rel=1e-6)    # frozen tree
        if not any(active):
            break
    got = stream.finalize()
    torch.cuda.synchronize()
    U.assert_tree_equal(got, want, n)


@pytest.mark.parametrize("V,k,n,d,B", [(1500, 4, 40, 7, 3),       # 280 pool indices: five mask words
                                       (600, 6, 100, 9, 2),       # 900 pool indices, two wavefronts per sequence
                                       (400, 16, 256, 20, 1)])    # the Large drafting shape: 5120 pool indices
def test_frontier_masks_of_the_drafting_phase_match_oracle(V, k, n, d, B):
    """ot_tree_frontier_mask after every expand: the incrementally kept ancestor masks over pool indices."""
    import torch
    from paper_2406_17276_amd import api
    for seed in range(5, 25):                              # inputs whose every cut has a gap the fp32 sums cannot flip
        g = np.random.default_rng(seed)
        x = (g.standard_normal((B, d, n, V)) * 3.0).astype(np.float32)
        want, builders = [], [ot_oracle.TreeBuilder(k, n) for _ in range(B)]
        for t in range(d):
            for b in range(B):
                F = builders[b].frontier_score.shape[0]
                builders[b].expand(x[b, t, :F].astype(np.float64))
            want.append([ot_oracle.frontier_masks(bld.layers, n, d) for bld in builders])
        if min(min(bld.cut_gaps) for bld in builders) > U.GAP:
            break
    else:
        raise RuntimeError("no gapped input")
    stream = api.TreeStream(B, V, k, n, d, api.OT_F32)
    dev = torch.from_numpy(x).cuda()
    for t in range(d):
        stream.expand(dev[:, t])
        m = stream.frontier_mask()
        torch.cuda.synchronize()
        m = m.cpu().numpy().view(np.uint64)
        for b in range(B):
            np.testing.assert_array_equal(m[b], want[t][b], err_msg=f"step {t}, sequence {b}")


@pytest.mark.parametrize("V,k,n,dmax,B,dtype,delta", [
    (2000, 6, 30, 8, 5, "f32", 0.01),
    (32000, 10, 50, 10, 2, "bf16", 0.02),      # 7B shape
    (500, 4, 64, 12, 3, "f32", 0.003),
    (900, 4, 100, 7, 4, "f32", 0.004),         # n > 64: the step-by-step form inside the call
    (3000, 16, 256, 5, 3, "bf16", 0.02),       # the widest frontier and k
    (70000, 3, 70, 6, 2, "f32", 0.01),         # rows of three scan parts
    (200, 16, 64, 26, 2, "f32", 0.002),        # one wavefront wide, but the row table exceeds LDS: step by step as well
])
def test_one_shot_adaptive_build_matches_oracle(V, k, n, dmax, B, dtype, delta):
    """ot_build_tree_adaptive: the stopping rule of Algorithm 1 applied inside the kernel."""
    import torch
    from paper_2406_17276_amd import api
    g = np.random.default_rng(V + n)
    scales = np.linspace(0.6, 7.0, B)
    for attempt in range(8):
        x = wl.store((g.standard_normal((B, dmax, n, V)) * scales[:, None, None, None]).astype(np.float32), dtype)
        x64 = wl.to_f64(x, dtype)
        full = [ot_oracle.build_tree_adaptive(x64[b], k, n, dmax, -1.0) for b in range(B)]
        gains = np.concatenate([np.diff([0.0] + f["e_sub_trace"]) for f in full])
        want = [ot_oracle.build_tree_adaptive(x64[b], k, n, dmax, delta) for b in range(B)]
        if np.abs(gains - delta).min() > 1e-5 and min(w["min_gap"] for w in want) > U.GAP:
            break
    else:
        raise RuntimeError("no suitable input")
    print("steps per sequence:", [w["steps"] for w in want], flush=True)
    got, steps, e_sub = api.build_tree_adaptive(U.to_device(x, dtype), k, n, dmax, delta)
    torch.cuda.synchronize()
    assert list(steps.cpu().numpy()) == [w["steps"] for w in want]
    np.testing.assert_allclose(e_sub.cpu().numpy(), [w["e_sub_trace"][-1] for w in want], rtol=1e-6)
    U.assert_tree_equal(got, want, n)


def test_one_shot_adaptive_build_with_a_threshold_nothing_passes_stops_after_one_step_at_any_width():
    import torch
    from paper_2406_17276_amd import api
    g = np.random.default_rng(5)
    x = g.standard_normal((2, 3, 100, 64)).astype(np.float32)
    got, steps, e_sub = api.build_tree_adaptive(torch.from_numpy(x).cuda(), 2, 100, 3, 10.0)
    torch.cuda.synchronize()
    assert list(steps.cpu().numpy()) == [1, 1]
    want = [ot_oracle.build_tree_adaptive(x[b].astype(np.float64), 2, 100, 3, 10.0) for b in range(2)]
    U.assert_tree_equal(got, want, 100)
