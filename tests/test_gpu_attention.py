"""Parity of ot_tree_verify_attention with the fp64 oracle (needs an MI355X).
Bars: max-abs 1e-5 for f32 inputs, 2e-2 for bf16 inputs, against fp64 on the stored (rounded) inputs."""
import numpy as np
import pytest

from oracle import opt_tree as ot_oracle
from oracle import tree_attention as ta_oracle
import workloads as wl
from tests import _util as U

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-5, "bf16": 2e-2}


def _gpu_attention(x, mask, dtype, scale=0.0):
    import torch
    from paper_2406_17276_amd import api
    dev = {k: U.to_device(v, dtype) for k, v in x.items() if k != "prefix_len"}
    plen = torch.from_numpy(x["prefix_len"].astype(np.int32)).cuda()
    kp, vp = dev["K_prefix"], dev["V_prefix"]
    out = api.tree_verify_attention(dev["Q"], kp, vp, dev["K_tree"], dev["V_tree"], plen, U.mask_to_device(mask),
                                    softmax_scale=scale)
    torch.cuda.synchronize()
    return U.from_device_f64(out)


def _oracle_attention(x, mask, dtype, scale=None):
    f = {k: wl.to_f64(v, dtype) for k, v in x.items() if k != "prefix_len"}
    return ta_oracle.tree_verify_attention(f["Q"], f["K_prefix"], f["V_prefix"], f["K_tree"], f["V_tree"],
                                           x["prefix_len"], mask, scale)


def _shape(dtype, B, Hq, Hkv, D, L, n, ragged=0.0, name="t"):
    return wl.Workload(name, B, 8, 1, 1, n, dtype, "normal", 1.0, Hq, Hkv, D, L, ragged=ragged)


def _random_masks(B, n, seed, shape="random"):
    return np.stack([ot_oracle.ancestor_mask(wl.random_tree_parents(n, seed + b, shape)) for b in range(B)])


@pytest.mark.parametrize("name", ["tiny", "7b"])
def test_full_config_with_the_tree_built_by_the_oracle(name):
    w = wl.WORKLOADS[name]
    logits = wl.make_logits(w, 0)
    tree = U.oracle_trees(logits, w.dtype, w.k, w.n, w.depth)[0]
    mask = tree["mask"][None]
    x = wl.make_attention_inputs(w, 0)
    got = _gpu_attention(x, mask, w.dtype)
    want = _oracle_attention(x, mask, w.dtype)
    assert np.abs(got - want).max() < TOL[w.dtype]


def test_13b_shape_sampled_heads():
    # full shape on the GPU; the oracle checks 6 of the 40 heads
    w = wl.WORKLOADS["13b"]
    x = wl.make_attention_inputs(w, 1)
    mask = _random_masks(1, w.n, 7)
    got = _gpu_attention(x, mask, w.dtype)
    heads = [0, 7, 13, 22, 31, 39]
    sub = {k: (v[:, heads] if k != "prefix_len" else v) for k, v in x.items()}
    want = _oracle_attention(sub, mask, w.dtype)
    assert np.abs(got[:, heads] - want).max() < TOL[w.dtype]


def test_70b_shape_gqa_ragged_sampled():
    # GQA 64/8 heads, ragged prefixes around 4096, n=60; 3 sequences on the GPU, oracle on 2 KV groups of each
    w = wl.WORKLOADS["70b"]
    seqs = [0, 7, 12]
    x = wl.make_attention_inputs(w, 2, seqs=seqs)
    mask = _random_masks(len(seqs), w.n, 11)
    got = _gpu_attention(x, mask, w.dtype)
    g = w.q_heads // w.kv_heads
    for kvh in (1, 6):
        qh = list(range(kvh * g, kvh * g + g))
        sub = dict(Q=x["Q"][:, qh], K_prefix=x["K_prefix"][:, [kvh]], V_prefix=x["V_prefix"][:, [kvh]],
                   K_tree=x["K_tree"][:, [kvh]], V_tree=x["V_tree"][:, [kvh]], prefix_len=x["prefix_len"])
        want = _oracle_attention(sub, mask, w.dtype)
        assert np.abs(got[:, qh] - want).max() < TOL[w.dtype]


def test_large_budget_shape_one_kv_group():
    # n = 256 (4 mask words), 32/8 heads, prefix 8192: 1 sequence on the GPU, oracle on one KV group
    w = wl.WORKLOADS["large"]
    x = wl.make_attention_inputs(w, 3, seqs=[0])
    mask = _random_masks(1, w.n, 5)
    got = _gpu_attention(x, mask, w.dtype)
    qh = [8, 9, 10, 11]
    sub = dict(Q=x["Q"][:, qh], K_prefix=x["K_prefix"][:, [2]], V_prefix=x["V_prefix"][:, [2]],
               K_tree=x["K_tree"][:, [2]], V_tree=x["V_tree"][:, [2]], prefix_len=x["prefix_len"])
    want = _oracle_attention(sub, mask, w.dtype)
    assert np.abs(got[:, qh] - want).max() < TOL[w.dtype]


def _stored(t):
    """Device bf16 tensor -> host array of bf16 bit patterns (the stored form the oracle helpers take)."""
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("name,groups", [
    ("70b", [(0, 0), (3, 5), (9, 2), (15, 7)]),        # 16 sequences, GQA 64/8, ragged prefixes around 4096, n = 60
    ("large", [(0, 3), (31, 6)]),                      # 32 sequences, 32/8 heads, prefix 8192, n = 256
])
def test_full_batch_as_the_bench_launches_it_sampled_groups(name, groups):
    """The whole batch in one launch, inputs drawn on the device; the oracle recomputes sampled (sequence, KV head)
    groups from the slices it needs."""
    import torch
    from paper_2406_17276_amd import api
    w = wl.WORKLOADS[name]
    B, g = w.batch, w.q_heads // w.kv_heads
    gen = torch.Generator(device="cuda"); gen.manual_seed(17)
    draw = lambda *shape: torch.randn(shape, generator=gen, device="cuda").to(torch.bfloat16)
    Lmax = w.max_prefix()
    Q = draw(B, w.q_heads, w.n, w.head_dim)
    Kp, Vp = draw(B, w.kv_heads, Lmax, w.head_dim), draw(B, w.kv_heads, Lmax, w.head_dim)
    Kt, Vt = draw(B, w.kv_heads, w.n, w.head_dim), draw(B, w.kv_heads, w.n, w.head_dim)
    plen = wl.prefix_lengths(w, 4).astype(np.int32)
    mask = _random_masks(B, w.n, 23)
    out = api.tree_verify_attention(Q, Kp, Vp, Kt, Vt, torch.from_numpy(plen).cuda(), U.mask_to_device(mask))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out.float()).all())
    for b, kvh in groups:
        qh = slice(kvh * g, kvh * g + g)
        sub = dict(Q=_stored(Q[b:b + 1, qh]), K_prefix=_stored(Kp[b:b + 1, kvh:kvh + 1]),
                   V_prefix=_stored(Vp[b:b + 1, kvh:kvh + 1]), K_tree=_stored(Kt[b:b + 1, kvh:kvh + 1]),
                   V_tree=_stored(Vt[b:b + 1, kvh:kvh + 1]), prefix_len=plen[b:b + 1])
        want = _oracle_attention(sub, mask[b:b + 1], "bf16")
        got = U.from_device_f64(out[b:b + 1, qh])
        print(f"{name}: sequence {b}, KV head {kvh}: max-abs err {np.abs(got - want).max():.2e}", flush=True)
        assert np.abs(got - want).max() < TOL["bf16"]


@pytest.mark.parametrize("B,Hq,Hkv,D,n,lengths", [
    (33, 16, 8, 128, 40, "ragged"),        # 128-row blocks, 264 workgroups: one more round than the chip holds at once
    (64, 8, 4, 128, 70, "ragged"),         # 256-row blocks, 256 workgroups, the largest batch that is ranked
    (40, 16, 8, 64, 33, "ties"),           # head_dim 64; many equal lengths, some zero, some beyond the buffer
    (65, 8, 4, 128, 70, "ragged"),         # one sequence too many for the ranking: the order of the sequences
])
def test_batches_that_take_their_jobs_longest_first(B, Hq, Hkv, D, n, lengths):
    """Batches that fill the chip with one key range per (sequence, KV head): every workgroup ranks the sequences by
    prefix length on the device and takes its job in that order.  Whatever the order, every (sequence, KV head) must
    come out exactly once: all outputs are finite and non-zero, and sampled sequences (the longest, the shortest, ties,
    clamped ones) agree with the oracle."""
    import torch
    from paper_2406_17276_amd import api
    Lmax, g = 320, Hq // Hkv
    rng = np.random.default_rng(B * 1000 + n)
    if lengths == "ragged":
        plen = rng.integers(1, Lmax + 1, size=B).astype(np.int32)
        plen[0], plen[B // 2], plen[B - 1] = Lmax, 1, Lmax // 2
    else:
        plen = rng.choice(np.array([0, 64, 64, 128, 200, 200, 200, Lmax], dtype=np.int32), size=B)
        plen[1], plen[2] = Lmax + 500, -7                     # clamped to Lmax and to 0 on the device
    eff = np.clip(plen, 0, Lmax)
    gen = torch.Generator(device="cuda"); gen.manual_seed(B + n)
    draw = lambda *shape: torch.randn(shape, generator=gen, device="cuda").to(torch.bfloat16)
    Q = draw(B, Hq, n, D)
    Kp, Vp = draw(B, Hkv, Lmax, D), draw(B, Hkv, Lmax, D)
    Kt, Vt = draw(B, Hkv, n, D), draw(B, Hkv, n, D)
    mask = _random_masks(B, n, 31)
    out = api.tree_verify_attention(Q, Kp, Vp, Kt, Vt, torch.from_numpy(plen).cuda(), U.mask_to_device(mask))
    torch.cuda.synchronize()
    of = out.float()
    assert bool(torch.isfinite(of).all())
    assert bool((of.abs().amax(dim=(2, 3)) > 0).all())          # no (sequence, head) was left out
    order = np.argsort(-eff, kind="stable")
    picks = sorted({int(order[0]), int(order[1]), int(order[B // 2]), int(order[-1]), 1, 2, B - 1})
    for b in picks:
        for kvh in (0, Hkv - 1):
            qh = slice(kvh * g, kvh * g + g)
            sub = dict(Q=_stored(Q[b:b + 1, qh]), K_prefix=_stored(Kp[b:b + 1, kvh:kvh + 1]),
                       V_prefix=_stored(Vp[b:b + 1, kvh:kvh + 1]), K_tree=_stored(Kt[b:b + 1, kvh:kvh + 1]),
                       V_tree=_stored(Vt[b:b + 1, kvh:kvh + 1]), prefix_len=eff[b:b + 1])
            want = _oracle_attention(sub, mask[b:b + 1], "bf16")
            got = U.from_device_f64(out[b:b + 1, qh])
            assert np.abs(got - want).max() < TOL["bf16"], (b, kvh, int(plen[b]))


@pytest.mark.parametrize("dtype,B,Hq,Hkv,D,L,n,ragged,shape", [
    ("f32", 2, 4, 4, 64, 128, 16, 0.0, "random"),
    ("f32", 2, 6, 2, 128, 77, 37, 0.3, "random"),      # GQA, ragged, n not a multiple of 16
    ("f32", 1, 2, 2, 64, 0, 20, 0.0, "random"),        # empty prefix
    ("f32", 1, 2, 1, 64, 300, 130, 0.0, "chain"),      # three mask words, chain = causal
    ("bf16", 2, 4, 4, 128, 200, 50, 0.2, "random"),
    ("bf16", 1, 8, 2, 128, 1000, 60, 0.0, "random"),   # packed GQA rows span several 64-row blocks
    ("bf16", 2, 4, 2, 64, 129, 33, 0.5, "random"),     # head_dim 64, ragged tails
    ("bf16", 1, 2, 2, 128, 0, 70, 0.0, "star"),        # empty prefix, two tree tiles
    ("bf16", 1, 4, 1, 128, 64, 256, 0.0, "random"),    # maximum n
    ("bf16", 1, 1, 1, 128, 5000, 1, 0.0, "random"),    # a single node
    ("bf16", 2, 4, 4, 64, 300, 40, 0.3, "random"),     # head_dim 64, 64-row workgroups, several splits
    ("bf16", 3, 2, 2, 128, 2000, 20, 0.9, "random"),   # very ragged: short sequences leave splits empty
    ("bf16", 1, 16, 1, 128, 700, 30, 0.0, "random"),   # 128-row workgroups, several splits, ragged last row block
])
def test_shapes_and_edges(dtype, B, Hq, Hkv, D, L, n, ragged, shape):
    w = _shape(dtype, B, Hq, Hkv, D, L, n, ragged)
    x = wl.make_attention_inputs(w, 4)
    mask = _random_masks(B, n, 3, shape)
    got = _gpu_attention(x, mask, dtype)
    want = _oracle_attention(x, mask, dtype)
    assert np.abs(got - want).max() < TOL[dtype]


def test_softmax_scale_override_and_unnormalised_inputs():
    w = _shape("f32", 1, 2, 2, 64, 90, 12)
    x = wl.make_attention_inputs(w, 6)
    x["Q"] = (x["Q"] * 4.0).astype(np.float32)          # large logits: exercises the running max
    mask = _random_masks(1, 12, 1)
    got = _gpu_attention(x, mask, "f32", scale=0.05)
    want = _oracle_attention(x, mask, "f32", scale=0.05)
    assert np.abs(got - want).max() < 1e-5


def test_strided_kv_cache_views():
    import torch
    from paper_2406_17276_amd import api
    w = _shape("bf16", 2, 4, 2, 128, 150, 24)
    x = wl.make_attention_inputs(w, 8)
    mask = _random_masks(2, 24, 2)
    want = _oracle_attention(x, mask, "bf16")
    dev = {k: U.to_device(v, "bf16") for k, v in x.items() if k != "prefix_len"}
    Lmax = dev["K_prefix"].shape[2]
    cache_k = torch.zeros((2, 2, Lmax + 40, 128 + 64), dtype=torch.bfloat16, device="cuda")
    cache_v = torch.zeros_like(cache_k)
    kview, vview = cache_k[:, :, 8:8 + Lmax, 64:], cache_v[:, :, 8:8 + Lmax, 64:]
    kview.copy_(dev["K_prefix"]); vview.copy_(dev["V_prefix"])
    plen = torch.from_numpy(x["prefix_len"]).cuda()
    out = api.tree_verify_attention(dev["Q"], kview, vview, dev["K_tree"], dev["V_tree"], plen, U.mask_to_device(mask))
    torch.cuda.synchronize()
    assert np.abs(U.from_device_f64(out) - want).max() < 2e-2


def test_prefix_length_is_clamped_on_device():
    w = _shape("f32", 1, 2, 2, 64, 40, 8)
    x = wl.make_attention_inputs(w, 9)
    mask = _random_masks(1, 8, 4)
    want = _oracle_attention(x, mask, "f32")
    y = dict(x); y["prefix_len"] = np.array([10_000], dtype=np.int32)
    got = _gpu_attention(y, mask, "f32")
    assert np.abs(got - want).max() < 1e-5


@pytest.mark.parametrize("dtype,D,L,n", [("f32", 64, 40, 8), ("bf16", 128, 300, 20)])
def test_clamped_prefix_length_is_reported_in_the_workspace_status_word(dtype, D, L, n):
    """A length outside [0, max_prefix] is clamped and sets bit 0 of the workspace's status word, which stays set
    until the workspace is prepared again; in-range lengths leave it clear."""
    import torch
    from paper_2406_17276_amd import api
    w = _shape(dtype, 3, 4, 2, D, L, n)
    x = wl.make_attention_inputs(w, 21)
    mask = _random_masks(3, n, 5)
    dev = {k: U.to_device(v, dtype) for k, v in x.items() if k != "prefix_len"}
    p = api.attn_params(dev["Q"], dev["K_prefix"], dev["V_prefix"], dev["K_tree"], dev["V_tree"])
    ws = api.attn_workspace(p, "cuda")
    call = lambda plen: api.tree_verify_attention(dev["Q"], dev["K_prefix"], dev["V_prefix"], dev["K_tree"], dev["V_tree"],
                                                  torch.tensor(plen, dtype=torch.int32, device="cuda"),
                                                  U.mask_to_device(mask), workspace=ws)
    good = call([L, L // 2, 0])
    assert api.attn_status(ws) == 0
    want = _oracle_attention(dict(x, prefix_len=np.array([L, L // 2, 0], dtype=np.int32)), mask, dtype)
    assert np.abs(U.from_device_f64(good) - want).max() < TOL[dtype]
    over = call([L, L + 1, 0])                                   # sequence 1 too long: clamped to L, flagged
    assert api.attn_status(ws) & api.OT_ATTN_STATUS_PREFIX_CLAMPED
    want = _oracle_attention(dict(x, prefix_len=np.array([L, L, 0], dtype=np.int32)), mask, dtype)
    assert np.abs(U.from_device_f64(over) - want).max() < TOL[dtype]
    call([L, L // 2, 0])
    assert api.attn_status(ws) & api.OT_ATTN_STATUS_PREFIX_CLAMPED        # sticky
    api._check(api.lib().ot_attn_workspace_prepare(ws.data_ptr(), ws.numel(), api._stream()), "prepare")
    call([L, -3, 0])                                             # negative: clamped to 0, flagged
    assert api.attn_status(ws) & api.OT_ATTN_STATUS_PREFIX_CLAMPED


def test_one_workspace_serves_consecutive_calls():
    """The split merge keeps ticket counters in the workspace and must leave them zero: the same prepared
    workspace is used for three calls in a row, the last one on a smaller problem."""
    import torch
    from paper_2406_17276_amd import api
    big = _shape("bf16", 1, 4, 4, 128, 900, 50)
    small = _shape("bf16", 1, 2, 2, 128, 260, 17)
    ws = None
    for w, seed in [(big, 11), (big, 12), (small, 13)]:
        x = wl.make_attention_inputs(w, seed)
        mask = _random_masks(w.batch, w.n, seed)
        dev = {k: U.to_device(v, "bf16") for k, v in x.items() if k != "prefix_len"}
        plen = torch.from_numpy(x["prefix_len"].astype(np.int32)).cuda()
        p = api.attn_params(dev["Q"], dev["K_prefix"], dev["V_prefix"], dev["K_tree"], dev["V_tree"])
        if ws is None:
            ws = api.attn_workspace(p, "cuda")
        assert api.attn_workspace_bytes(p) <= ws.numel()
        out = api.tree_verify_attention(dev["Q"], dev["K_prefix"], dev["V_prefix"], dev["K_tree"], dev["V_tree"],
                                        plen, U.mask_to_device(mask), workspace=ws)
        torch.cuda.synchronize()
        want = _oracle_attention(x, mask, "bf16")
        assert np.abs(U.from_device_f64(out) - want).max() < 2e-2
        assert int(ws[:4096].view(torch.int32).abs().sum().item()) == 0


@pytest.mark.parametrize("dtype,B,Hq,Hkv,D,L,k,n,d,upto", [
    ("f32", 2, 4, 2, 64, 90, 3, 12, 5, 4),          # 60 pool rows, one mask word
    ("f32", 1, 4, 2, 64, 50, 10, 50, 12, 12),        # f32 beyond eight mask words: 600 pool keys
    ("f32", 1, 2, 2, 128, 33, 16, 256, 7, 7),        # f32, the largest frontier: 1792 pool keys, 28 words
    ("bf16", 1, 8, 8, 128, 700, 10, 50, 10, 10),     # 7B-shaped drafting step: 50 queries, 500 pool keys, 8 words
    ("bf16", 2, 8, 2, 128, 300, 6, 40, 8, 6),        # packed GQA rows (128-row workgroups), 320 pool keys
    ("bf16", 1, 4, 4, 64, 0, 4, 64, 8, 3),           # no prefix, 512 pool keys of which 3 layers are filled
    ("bf16", 1, 4, 4, 128, 2048, 10, 64, 12, 12),    # the 13B drafting shape (four of its heads): 768 pool keys
    ("bf16", 2, 16, 2, 128, 700, 8, 60, 10, 10),     # the 70B drafting shape (two of its KV heads): 600 pool keys
    ("bf16", 1, 8, 2, 128, 512, 16, 256, 20, 20),    # the Large drafting shape (two of its KV heads): 5120 pool keys
])
def test_drafting_phase_attention_frontier_against_pool(dtype, B, Hq, Hkv, D, L, k, n, d, upto):
    """n frontier queries against the prefix and the K/V of all pool nodes (n_keys = depth * n), with the
    frontier masks of the drafting phase."""
    import torch
    from paper_2406_17276_amd import api
    g = np.random.default_rng(n + d)
    masks = []
    for b in range(B):
        bld = ot_oracle.TreeBuilder(k, n)
        for t in range(upto):
            bld.expand(g.standard_normal((bld.frontier_score.shape[0], 200)) * 2.0)
        masks.append(ot_oracle.frontier_masks(bld.layers, n, d))
    mask = np.stack(masks)
    w = _shape(dtype, B, Hq, Hkv, D, L, n, 0.2 if L else 0.0)
    x = wl.make_attention_inputs(w, 21)
    nk = d * n
    x["K_tree"] = wl.store(g.standard_normal((B, Hkv, nk, D)).astype(np.float32), dtype)
    x["V_tree"] = wl.store(g.standard_normal((B, Hkv, nk, D)).astype(np.float32), dtype)
    got = _gpu_attention(x, mask, dtype)
    want = _oracle_attention(x, mask, dtype)
    assert np.abs(got - want).max() < TOL[dtype]
    assert np.abs(want).max() > 0.01


def test_repeated_launches_are_bit_identical():
    """Split-heavy shape, 300 launches on one prepared workspace: the merge inside the kernel adds the splits
    in a fixed order, so every launch must reproduce the first bit for bit, and the ticket counters end at zero."""
    import torch
    from paper_2406_17276_amd import api
    w = _shape("bf16", 1, 8, 8, 128, 1000, 50)
    x = wl.make_attention_inputs(w, 31)
    mask = _random_masks(1, 50, 9)
    dev = {k: U.to_device(v, "bf16") for k, v in x.items() if k != "prefix_len"}
    plen = torch.from_numpy(x["prefix_len"].astype(np.int32)).cuda()
    pa = api.PreparedAttention(dev["Q"], dev["K_prefix"], dev["V_prefix"], dev["K_tree"], dev["V_tree"], plen,
                               U.mask_to_device(mask))
    st = torch.cuda.current_stream().cuda_stream
    pa(st)
    torch.cuda.synchronize()
    first = pa.out.clone()
    assert np.abs(U.from_device_f64(first) - _oracle_attention(x, mask, "bf16")).max() < 2e-2
    for it in range(300):
        pa(st)
        if it % 50 == 49:
            torch.cuda.synchronize()
            assert torch.equal(pa.out, first)
    assert int(pa.ws[:4096].view(torch.int32).abs().sum().item()) == 0


@pytest.mark.parametrize("Hq,Hkv,n", [(8, 2, 25), (16, 2, 40), (4, 4, 70)])      # 100, 320 and 70 packed rows per KV head
def test_scores_that_jump_between_tiles(Hq, Hkv, n):
    """The 128- and 256-row variants keep a row's softmax reference fixed while scores stay within a slack of it and
    move it up otherwise: key bands whose scores differ by factors of up to 400 (beyond what 2^x can hold in fp32
    relative to the first band) force that path again and again, in the middle of a split."""
    w = _shape("bf16", 2, Hq, Hkv, 128, 1000, n)
    x = wl.make_attention_inputs(w, 31)
    kp = wl.bf16_bits_to_f32(x["K_prefix"]).copy()
    for lo, f in [(0, 0.1), (200, 1.0), (400, 8.0), (600, 0.5), (800, 40.0), (930, 3.0)]:
        kp[:, :, lo:] = wl.bf16_bits_to_f32(x["K_prefix"])[:, :, lo:] * f
    x["K_prefix"] = wl.store(kp, "bf16")
    mask = _random_masks(2, n, 8)
    got = _gpu_attention(x, mask, "bf16")
    want = _oracle_attention(x, mask, "bf16")
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() < TOL["bf16"]
