#!/usr/bin/env python3
"""Benchmark of the OPT-Tree decoding-step hot path on one MI355X.

One step = one ot_build_tree (row scan + tree selection) followed by one
ot_tree_verify_attention (K/V streaming + split merge) on one batch of the
synthetic workload, the attention mask being the one the tree builder just
wrote.  Inputs are resident in HBM before the timed region; consecutive steps
use different copies from a ring larger than the chip's caches, so the logits
and the K/V cache are streamed from HBM every step.

Prints ONE JSON line: steps/s; `roofline` = the roofline-bound kernel that takes
longest in a step (at the 7B shape the K/V-streaming attention kernel, HBM-bound;
the tree-selection kernel is longer still but bound by latency, not by a roof),
`roofline_scan` = the logits row scan; both with the HBM traffic measured by
rocprofv3 counters (read from the committed summary under profiles/), and against
a plain streaming read of the same bytes with the same cold-buffer ring; a compact
leg at the 70B-shaped GQA batch, where the attention is MFMA-bound; and the CPU
oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published


def measured_traffic(workload: str):
    """HBM bytes per launch of the scan and the attention kernel as rocprofv3 measured them (--pmc FETCH_SIZE and
    WRITE_SIZE, scaled by the same counters' readings for a plain 256 MiB copy): the figures of the committed summary
    profiles/bench_<workload>_hbm_traffic_pmc.txt (lines `traffic <kernel> <bytes>`), or None."""
    path = os.path.join(ROOT, "profiles", f"bench_{workload}_hbm_traffic_pmc.txt")
    out = {}
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic":
                out[f[1]] = float(f[2])
    except OSError:
        return {}, None
    return out, os.path.relpath(path, ROOT)


class Hip:
    """The few HIP event calls the benchmark needs, straight from the runtime."""

    def __init__(self):
        self.lib = C.CDLL("libamdhip64.so")
        self.lib.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.lib.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        self.lib.hipEventSynchronize.argtypes = [C.c_void_p]
        self.lib.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]

    def event(self):
        e = C.c_void_p()
        assert self.lib.hipEventCreate(C.byref(e)) == 0
        return e

    def record(self, e, stream):
        assert self.lib.hipEventRecord(e, C.c_void_p(stream)) == 0

    def elapsed_ms(self, a, b) -> float:
        ms = C.c_float()
        assert self.lib.hipEventSynchronize(b) == 0
        rc = self.lib.hipEventElapsedTime(C.byref(ms), a, b)
        assert rc == 0, rc
        return float(ms.value)


def device_logits(w, seed: int, slot: int):
    """Ring copy `slot` of the workload's logits, drawn on the device with the workload's recipe."""
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(seed * 1000003 + slot)
    F = w.frontier()
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    out = torch.zeros((w.batch, w.depth, w.n, w.vocab), dtype=dt, device="cuda")
    for t in range(w.depth):
        z = torch.randn((w.batch, F[t], w.vocab), generator=g, device="cuda", dtype=torch.float32)
        if w.logit_kind == "zipf":
            rank = torch.argsort(torch.rand((w.batch, F[t], w.vocab), generator=g, device="cuda"), dim=-1).float() + 1.0
            x = -1.1 * torch.log(rank) + 0.5 * z
        else:
            x = z * w.logit_scale
            if w.logit_kind == "peak":
                idx = torch.randint(0, w.vocab, (w.batch, F[t], 1), generator=g, device="cuda")
                x.scatter_add_(2, idx, torch.full_like(idx, w.peak, dtype=torch.float32))
        out[:, t, :F[t]] = x.to(dt)
    return out


def device_attention(w, seed: int, slot: int, plen):
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(seed * 7919 + slot + 17)
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    Lmax = max(1, w.max_prefix())
    mk = lambda *s: torch.randn(s, generator=g, device="cuda", dtype=torch.float32).to(dt)
    return dict(Q=mk(w.batch, w.q_heads, w.n, w.head_dim), K_prefix=mk(w.batch, w.kv_heads, Lmax, w.head_dim),
                V_prefix=mk(w.batch, w.kv_heads, Lmax, w.head_dim), K_tree=mk(w.batch, w.kv_heads, w.n, w.head_dim),
                V_tree=mk(w.batch, w.kv_heads, w.n, w.head_dim), prefix_len=plen)


def gqa_leg(name: str, steps: int, hip, stream):
    """A compact run of another workload inside the default line: the batched GQA shape whose attention is
    MFMA-bound.  Inputs are drawn on the device (two ring copies), sequence 0's tree and one (sequence, KV head)
    group of the attention are checked against the oracle, then `steps` steps are timed with the kernels' own
    begin/end events."""
    import torch
    from oracle import opt_tree as ot_oracle, tree_attention as ta_oracle
    import workloads as wl
    from paper_2406_17276_amd import api
    from tests import _util as U
    w = wl.WORKLOADS[name]
    plen_h = wl.prefix_lengths(w, 0)
    plen_d = torch.from_numpy(plen_h).cuda()
    bits = lambda t: t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    builds, attns = [], []
    for slot in range(2):
        lg = device_logits(w, 0, slot)
        at = device_attention(w, 0, slot, plen_d)
        pb = api.PreparedBuild(lg, w.k, w.n, w.depth)
        builds.append(pb)
        attns.append(api.PreparedAttention(at["Q"], at["K_prefix"], at["V_prefix"], at["K_tree"], at["V_tree"], plen_d,
                                           pb.out.mask))
    builds[0](stream); attns[0](stream)
    torch.cuda.synchronize()
    # parity: the tree of sequence 0 (if its cut gaps allow a bit-exact comparison) and the attention of one group
    want = ot_oracle.build_tree(U.LazyF64(bits(builds[0].logits[0]), w.dtype), w.k, w.n, w.depth)
    tree_checked = bool(want["min_gap"] > U.GAP)
    if tree_checked:
        sub = api.alloc_tree(1, w.n)
        for f in ("token", "parent", "depth", "score", "mask", "n_out", "expect"):
            getattr(sub, f).copy_(getattr(builds[0].out, f)[:1])
        U.assert_tree_equal(sub, [want], w.n)
    g = w.q_heads // w.kv_heads
    Q, Kp, Vp, Kt, Vt = attns[0].keep[:5]
    f64 = lambda t: wl.to_f64(bits(t), w.dtype)
    mask_h = builds[0].out.mask[:1].cpu().numpy().view(np.uint64)
    ref = ta_oracle.tree_verify_attention(f64(Q[:1, :g]), f64(Kp[:1, :1]), f64(Vp[:1, :1]), f64(Kt[:1, :1]), f64(Vt[:1, :1]),
                                          plen_h[:1], mask_h)
    err = float(np.abs(U.from_device_f64(attns[0].out[:1, :g]) - ref).max())
    assert err < 2e-2, f"attention parity {err}"
    for i in range(4):
        builds[i % 2](stream); attns[i % 2](stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        builds[i % 2](stream); attns[i % 2](stream)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    ev = [[hip.event() for _ in range(4)] for _ in range(steps)]
    for i in range(steps):
        builds[i % 2].timed(stream, ev[i][0], ev[i][1])
        attns[i % 2].timed(stream, ev[i][2], ev[i][3])
    torch.cuda.synchronize()
    scan_us = float(np.mean([hip.elapsed_ms(e[0], e[1]) for e in ev])) * 1e3
    attn_us = float(np.mean([hip.elapsed_ms(e[2], e[3]) for e in ev])) * 1e3
    S_tot = int(sum(int(l) + w.n for l in plen_h))
    flops = 4.0 * w.n * S_tot * w.head_dim * w.q_heads
    logit_bytes = w.batch * w.rows_per_seq() * w.vocab * w.elem_bytes()
    tf = flops / (attn_us * 1e-6) / 1e12
    gbs = logit_bytes / (scan_us * 1e-6) / 1e9
    traffic, traffic_src = measured_traffic(name)
    return {"workload": f"{w.name}: batch {w.batch}, vocab {w.vocab}, depth {w.depth}, top-k {w.k}, n {w.n}; attention "
                        f"{w.q_heads}q/{w.kv_heads}kv heads, head_dim {w.head_dim}, prefix {w.prefix} +-{int(w.ragged * 100)}%",
            "steps": steps, "ms_per_step": ms, "steps_per_s": 1e3 / ms, "ring_copies": 2, "inputs": "drawn on the device",
            "parity_checked": {"tree_sequence_0": tree_checked, "attention_group_0_max_abs_err": err},
            "roofline": {"kernel": "attn_mfma_kernel", "bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS,
                         "unit": "TFLOP/s", "frac": tf / MFMA_BF16_PEAK_TFLOPS, "algorithmic_flops": flops,
                         "avg_kernel_us": attn_us, "traffic": traffic.get("attn_mfma_kernel"),
                         "traffic_source": traffic_src},
            "roofline_scan": {"kernel": "row_scan_kernel", "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS,
                              "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "algorithmic_bytes": logit_bytes,
                              "avg_kernel_us": scan_us, "traffic": traffic.get("row_scan_kernel"),
                              "traffic_source": traffic_src}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="7b", choices=["tiny", "7b", "13b", "70b", "large"])
    ap.add_argument("--mode", default="stream", choices=["stream", "graph"])
    ap.add_argument("--ring", type=int, default=0, help="input copies cycled through (0: enough for 768 MB)")
    ap.add_argument("--no-events", action="store_true", help="do not time individual kernels in the timed region")
    ap.add_argument("--skip-parity", action="store_true",
                    help="draw every input on the device and skip the oracle check and the CPU baseline (for shapes "
                         "whose oracle run takes hours, e.g. --workload large; the line then says parity_checked: false)")
    ap.add_argument("--main-only", action="store_true", help="skip the adaptive-depth and greedy-verification legs")
    ap.add_argument("--no-gqa-leg", action="store_true", help="skip the compact 70B-shaped GQA leg of the default run")
    ap.add_argument("--cpu-steps", type=int, default=16, help="oracle steps timed for cpu_baseline (0 = skip)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference dispatch for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from oracle import tree_attention as ta_oracle
    import workloads as wl
    from paper_2406_17276_amd import api
    from tests import _util as U

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = wl.WORKLOADS[args.workload]
    hip = Hip()
    stream = torch.cuda.current_stream().cuda_stream

    # ---- slot 0: the seeded host-generated workload, checked against the oracle -------------
    t_cpu0 = time.perf_counter()
    if args.skip_parity:
        seed, logits_h, want, attn_h = 0, None, None, None
        plen_h = wl.prefix_lengths(w, seed)
    else:
        seed, logits_h, want = U.gapped_logits(w, 0)
        attn_h = wl.make_attention_inputs(w, seed)
        plen_h = attn_h["prefix_len"]
    logit_bytes = w.batch * w.rows_per_seq() * w.vocab * w.elem_bytes()
    S_tot = int(sum(int(l) + w.n for l in plen_h))
    kv_bytes = 2 * w.kv_heads * S_tot * w.head_dim * w.elem_bytes()
    qo_bytes = 2 * w.batch * w.q_heads * w.n * w.head_dim * w.elem_bytes()
    attn_flops = 4.0 * w.n * S_tot * w.head_dim * w.q_heads
    per_slot = logit_bytes + 2 * w.kv_heads * w.batch * (w.max_prefix() + w.n) * w.head_dim * w.elem_bytes() + qo_bytes
    ring = args.ring or max(2, min(64, int(768e6 // per_slot) + 1))

    builds, attns = [], []
    plen_d = torch.from_numpy(plen_h).cuda()
    for slot in range(ring):
        if slot == 0 and not args.skip_parity:
            lg = U.to_device(logits_h, w.dtype)
            at = {k: U.to_device(v, w.dtype) for k, v in attn_h.items() if k != "prefix_len"}
        else:
            lg = device_logits(w, seed, slot)
            at = device_attention(w, seed, slot, plen_d)
        pb = api.PreparedBuild(lg, w.k, w.n, w.depth)
        pa = api.PreparedAttention(at["Q"], at["K_prefix"], at["V_prefix"], at["K_tree"], at["V_tree"], plen_d,
                                   pb.out.mask)
        builds.append(pb)
        attns.append(pa)
    torch.cuda.synchronize()

    # parity of slot 0 in the launch configuration that is timed
    builds[0](stream)
    attns[0](stream)
    torch.cuda.synchronize()
    if not args.skip_parity:
        U.assert_tree_equal(builds[0].out, want, w.n)
        f64 = {k: wl.to_f64(v, w.dtype) for k, v in attn_h.items() if k != "prefix_len"}
        chk_heads = list(range(0, w.q_heads, max(1, w.q_heads // 4)))[:4] if w.q_heads > 8 else list(range(w.q_heads))
        g = w.q_heads // w.kv_heads
        kvh = sorted({h // g for h in chk_heads})
        qh = [h for h in range(w.q_heads) if h // g in kvh]
        mask_h = np.stack([t["mask"] for t in want])
        ref = ta_oracle.tree_verify_attention(f64["Q"][:, qh], f64["K_prefix"][:, kvh], f64["V_prefix"][:, kvh],
                                              f64["K_tree"][:, kvh], f64["V_tree"][:, kvh], plen_h, mask_h)
        err = float(np.abs(U.from_device_f64(attns[0].out)[:, qh] - ref).max())
        tol = 2e-2 if w.dtype == "bf16" else 1e-5
        assert err < tol, f"attention parity {err}"

    if args.calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        dst.copy_(src)           # reads 256 MiB and writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # ---- warm-up ---------------------------------------------------------------------------
    for i in range(args.warmup):
        builds[i % ring](stream)
        attns[i % ring](stream)
    torch.cuda.synchronize()

    K = args.steps
    use_events = (not args.no_events) and args.mode == "stream"
    ev = [[hip.event() for _ in range(4)] for _ in range(K)] if use_events else None

    graph = None
    if args.mode == "graph":
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            cs = side.cuda_stream
            with torch.cuda.graph(graph, stream=side):
                for i in range(K):
                    builds[i % ring](cs)
                    attns[i % ring](cs)
        torch.cuda.synchronize()

    # ---- timed region: exactly K steps, plain entry points ----------------------------------------
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if graph is not None:
        graph.replay()
    else:
        for i in range(K):
            builds[i % ring](stream)
            attns[i % ring](stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / K

    # ---- the same K steps once more through the *_timed entry points: per-kernel durations from HIP events
    # recorded around the kernels themselves.  Kept out of the timed region above because the event
    # bookkeeping lengthens a step by several microseconds.
    scan_ms = attn_ms = ms_per_step_events = None
    if use_events:
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for i in range(K):
            e = ev[i]
            builds[i % ring].timed(stream, e[0], e[1])
            attns[i % ring].timed(stream, e[2], e[3])
        torch.cuda.synchronize()
        ms_per_step_events = (time.perf_counter() - t1) * 1e3 / K
        scan_all = np.array([hip.elapsed_ms(e[0], e[1]) for e in ev])
        attn_all = np.array([hip.elapsed_ms(e[2], e[3]) for e in ev])
        scan_ms, attn_ms = float(scan_all.mean()), float(attn_all.mean())

    # ---- warm variant: the same K steps on ring slot 0 only (inputs stay in the Infinity Cache / L2) --------
    ms_per_step_warm = None
    if graph is None and not args.main_only:
        for i in range(min(20, args.warmup)):
            builds[0](stream); attns[0](stream)
        torch.cuda.synchronize()
        tw = time.perf_counter()
        for i in range(K):
            builds[0](stream)
            attns[0](stream)
        torch.cuda.synchronize()
        ms_per_step_warm = (time.perf_counter() - tw) * 1e3 / K

    # ---- yardsticks: what this GPU reaches on a plain 1 GiB streaming read and on a register-only MFMA loop ---
    yard = None
    if not args.main_only:
        L = api.lib()
        big = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        big.random_(0, 255)
        sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
        for _ in range(2):
            api._check(L.ot_yardstick_stream_read(big.data_ptr(), big.numel(), sink.data_ptr(), stream), "yardstick")
        torch.cuda.synchronize()
        ty = time.perf_counter()
        for _ in range(10):
            api._check(L.ot_yardstick_stream_read(big.data_ptr(), big.numel(), sink.data_ptr(), stream), "yardstick")
        torch.cuda.synchronize()
        read_gbs = 10 * big.numel() / (time.perf_counter() - ty) / 1e9
        del big
        iters = 4000
        api._check(L.ot_yardstick_mfma_loop(iters, sink.data_ptr(), stream), "yardstick")
        torch.cuda.synchronize()
        ty = time.perf_counter()
        for _ in range(3):
            api._check(L.ot_yardstick_mfma_loop(iters, sink.data_ptr(), stream), "yardstick")
        torch.cuda.synchronize()
        mfma_tf = 3 * 2048 * 4 * 4 * iters * 32768.0 / (time.perf_counter() - ty) / 1e12
        # the same plain read at the kernels' own sizes, over the same ring of cold copies: what a launch of this
        # size can reach at all (ramp-up and tail of a microsecond-scale launch included), timed by HIP events
        def small_read(tensors, nbytes, workgroups):
            flat = [t.reshape(-1).view(torch.uint8)[:nbytes // 16 * 16] for t in tensors]
            sink2 = torch.zeros(workgroups, dtype=torch.int32, device="cuda")
            evs = [(hip.event(), hip.event()) for _ in range(3 * len(flat))]
            call = lambda f, e0, e1: api._check(L.ot_yardstick_stream_read_timed(
                f.data_ptr(), f.numel(), workgroups, sink2.data_ptr(), stream, e0, e1), "yardstick")
            for f in flat:
                call(f, None, None)
            torch.cuda.synchronize()
            for i, (e0, e1) in enumerate(evs):
                call(flat[i % len(flat)], e0, e1)
            torch.cuda.synchronize()
            us = float(np.median([hip.elapsed_ms(a_, b_) for a_, b_ in evs])) * 1e3
            return {"bytes": int(flat[0].numel()), "workgroups_of_256": workgroups, "us": us,
                    "GBs": flat[0].numel() / (us * 1e-6) / 1e9}
        # the scan's launch holds one 1024-thread workgroup per row part, the attention's one 256-thread workgroup per
        # (KV head, key split): the reads are launched with as many threads
        same_scan = (small_read([b_.logits for b_ in builds], logit_bytes, 4 * w.batch * w.rows_per_seq())
                     if builds[0].logits.is_contiguous() else None)
        same_attn = small_read([a_.keep[1] for a_ in attns], kv_bytes // 2, 256)
        yard = {"hbm_read_GBs": read_gbs, "mfma_bf16_TFLOPs": mfma_tf,
                "hbm_read_scan_sized": same_scan, "hbm_read_half_kv_sized": same_attn,
                "what": "ot_yardstick_stream_read over 1 GiB (wall clock) and over buffers of the scan's and of half the "
                        "attention's bytes from the same cold ring (the launch's own begin/end events, median); "
                        "ot_yardstick_mfma_loop (v_mfma_f32_32x32x16_bf16, register operands)"}

    result = {
        "metric": "tree-build+verify-attention steps/sec", "value": K / dt, "unit": "steps/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: batch {w.batch}, vocab {w.vocab}, depth {w.depth}, top-k {w.k}, n {w.n}; "
                               f"attention {w.q_heads}q/{w.kv_heads}kv heads, head_dim {w.head_dim}, prefix {w.prefix}",
                   "mode": args.mode, "ring_copies": ring, "seed": seed, "parity_checked": not args.skip_parity,
                   "kernel_events": "second pass of the same steps" if use_events else None,
                   "ms_per_step_with_events": ms_per_step_events, "ms_per_step_warm_inputs": ms_per_step_warm},
    }
    if scan_ms is not None:
        traffic, traffic_src = measured_traffic(w.name)
        gbs = logit_bytes / (scan_ms * 1e-3) / 1e9
        scan_roof = {"kernel": "row_scan_kernel", "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                     "traffic": traffic.get("row_scan_kernel"), "traffic_source": traffic_src,
                     "algorithmic_bytes": logit_bytes, "avg_kernel_us": scan_ms * 1e3,
                     "kernel_us_p10_p50_p90": [float(v) * 1e3 for v in np.percentile(scan_all, [10, 50, 90])]}
        agbs = (kv_bytes + qo_bytes) / (attn_ms * 1e-3) / 1e9
        attn_kernel = "attn_mfma_kernel" if w.dtype == "bf16" else "attn_f32_kernel"
        attn_tf = attn_flops / (attn_ms * 1e-3) / 1e12
        g_rows = (w.q_heads // w.kv_heads) * w.n
        mfma_bound = w.dtype == "bf16" and g_rows * 1.0 > 310          # FLOP per K/V byte ~ g n against the ~310 ridge
        attn_roof = {"kernel": attn_kernel, "avg_kernel_us": attn_ms * 1e3,
                     "kernel_us_p10_p50_p90": [float(v) * 1e3 for v in np.percentile(attn_all, [10, 50, 90])],
                     "algorithmic_bytes": kv_bytes + qo_bytes, "algorithmic_flops": attn_flops,
                     "traffic": traffic.get(attn_kernel), "traffic_source": traffic_src,
                     "hbm_GBs": agbs, "hbm_frac_of_peak": agbs / HBM_PEAK_GBS,
                     "mfma_tflops": attn_tf, "mfma_frac_of_peak": attn_tf / MFMA_BF16_PEAK_TFLOPS}
        if mfma_bound:
            attn_roof.update({"bound": "mfma", "achieved": attn_tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                              "frac": attn_tf / MFMA_BF16_PEAK_TFLOPS})
        else:
            attn_roof.update({"bound": "hbm", "achieved": agbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": agbs / HBM_PEAK_GBS})
        if yard:
            scan_roof["frac_of_measured_read"] = gbs / yard["hbm_read_GBs"]
            if yard.get("hbm_read_scan_sized"):
                scan_roof["frac_of_same_size_read"] = yard["hbm_read_scan_sized"]["us"] / (scan_ms * 1e3)
            attn_roof["hbm_frac_of_measured_read"] = agbs / yard["hbm_read_GBs"]
            attn_roof["mfma_frac_of_measured"] = attn_tf / yard["mfma_bf16_TFLOPs"]
        # `roofline`: of the kernels a roof bounds, the one that takes longest in a step
        if attn_ms >= scan_ms:
            result["roofline"], result["roofline_scan"] = attn_roof, scan_roof
        else:
            result["roofline"], result["roofline_attention"] = scan_roof, attn_roof
        result["config"]["longest_kernel_note"] = (
            "the tree-selection kernel (one wavefront per sequence, a chain of dependent selections) is not bound by a "
            "memory or arithmetic roof; its time is ms_per_step minus the two kernels above")
    if yard:
        result["yardsticks"] = yard

    def graph_us(fn, reps=40):
        """GPU time per call of fn(i) with the host out of the way: reps calls replayed from one HIP graph."""
        try:
            side = torch.cuda.Stream()
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(gr, stream=side):
                    for i in range(reps):
                        fn(i)
            torch.cuda.synchronize()
            gr.replay()
            torch.cuda.synchronize()
            t0g = time.perf_counter()
            gr.replay()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0g) * 1e6 / reps
        except Exception:                                       # a measurement aid: never in the way of the line
            return None

    # ---- adaptive depth (Algorithm 1's loop) through the streaming entry points, outside the timed region:
    # begin, then per drafting step expand + E_sub query, then finalize; delta = -1 never stops early, so the
    # figure is the cost of a full-depth loop without the host reading the go-on flags in between.
    if args.mode == "stream" and not args.main_only:
        dcode = api.OT_BF16 if w.dtype == "bf16" else api.OT_F32
        ts = api.TreeStream(w.batch, w.vocab, w.k, w.n, w.depth, dcode)
        reps = 20
        def adaptive_loop(lg):
            api._check(api.lib().ot_tree_begin(C.byref(ts.p), ts.ws.data_ptr(), ts.ws.numel(), api._stream()), "ot_tree_begin")
            ts.step = 0
            for t in range(w.depth):
                ts.expand(lg[:, t])
                ts.e_sub(-1.0)
            return ts.finalize()
        adaptive_loop(builds[0].logits)
        torch.cuda.synchronize()
        ta = time.perf_counter()
        for i in range(reps):
            adaptive_loop(builds[i % ring].logits)
        torch.cuda.synchronize()
        us_loop = (time.perf_counter() - ta) * 1e6 / reps
        ws_ad = torch.empty(api.build_workspace_bytes(builds[0].p), dtype=torch.uint8, device="cuda")
        out_ad = api.alloc_tree(w.batch, w.n)
        one_shot_us = None
        try:
            api.build_tree_adaptive(builds[0].logits, w.k, w.n, w.depth, -1.0, out=out_ad, workspace=ws_ad)
            torch.cuda.synchronize()
            ta = time.perf_counter()
            for i in range(100):
                api.build_tree_adaptive(builds[i % ring].logits, w.k, w.n, w.depth, -1.0, out=out_ad, workspace=ws_ad)
            torch.cuda.synchronize()
            one_shot_us = (time.perf_counter() - ta) * 1e4
        except api.OptTreeError:
            pass                                  # shape off the single-wavefront path
        loop_graph_us = graph_us(lambda i: adaptive_loop(builds[i % ring].logits), reps=8)
        result["adaptive_depth"] = {"one_shot_us_per_tree": one_shot_us, "us_per_tree": us_loop,
                                    "us_per_tree_graph_replay": loop_graph_us, "us_per_drafting_step": us_loop / w.depth, "steps": w.depth,
                                    "delta": -1.0, "calls_per_step": "ot_tree_expand + ot_tree_esub"}

    # ---- greedy verification + K/V append of the same shape, outside the timed region: target rows for the root
    # and the n nodes, the tree slot 0 built, the attention call's caches
    if args.mode == "stream" and not args.main_only:
        gt = torch.Generator(device="cuda"); gt.manual_seed(seed + 999)
        tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        targets = [(torch.randn((w.batch, w.n + 1, w.vocab), generator=gt, device="cuda") * 4.0).to(tdt) for _ in range(4)]
        tree0 = builds[0].out
        kp, vp, kt, vt = (attns[0].keep[i] for i in (1, 2, 3, 4))
        vws = torch.empty(int(api.lib().ot_verify_workspace_bytes(C.byref(api.VerifyParams(
            w.batch, w.vocab, w.n, api.OT_BF16 if w.dtype == "bf16" else api.OT_F32, targets[0].stride(0),
            targets[0].stride(1))))), dtype=torch.uint8, device="cuda")
        def verify_once(i):
            alen, anode, _ = api.verify_greedy(targets[i % 4], tree0, workspace=vws)
            api.kv_append(kp, vp, kt, vt, plen_d, alen, anode)
        verify_once(0)
        torch.cuda.synchronize()
        tv = time.perf_counter()
        for i in range(100):
            verify_once(i)
        torch.cuda.synchronize()
        result["greedy_verify"] = {"us_per_call_pair": (time.perf_counter() - tv) * 1e4,
                                   "us_per_call_pair_graph_replay": graph_us(verify_once),
                                   "calls": "ot_verify_greedy + ot_kv_append",
                                   "target_rows": w.batch * (w.n + 1), "target_bytes": w.batch * (w.n + 1) * w.vocab * w.elem_bytes()}

        # the same with the ground truth drawn at temperature 1 (uniform numbers resident on the device)
        us_d = torch.rand((w.batch, w.n + 1), generator=gt, device="cuda")
        sws = torch.empty(int(api.lib().ot_verify_sample_workspace_bytes(C.byref(api.VerifyParams(
            w.batch, w.vocab, w.n, api.OT_BF16 if w.dtype == "bf16" else api.OT_F32, targets[0].stride(0),
            targets[0].stride(1))))), dtype=torch.uint8, device="cuda")
        def sample_once(i):
            alen, anode, _ = api.verify_sample(targets[i % 4], us_d, 1.0, tree0, workspace=sws)
            api.kv_append(kp, vp, kt, vt, plen_d, alen, anode)
        sample_once(0)
        torch.cuda.synchronize()
        tv = time.perf_counter()
        for i in range(100):
            sample_once(i)
        torch.cuda.synchronize()
        result["sampled_verify"] = {"us_per_call_pair": (time.perf_counter() - tv) * 1e4,
                                    "us_per_call_pair_graph_replay": graph_us(sample_once),
                                    "calls": "ot_verify_sample + ot_kv_append", "temperature": 1.0,
                                    "target_rows": w.batch * (w.n + 1)}

    # ---- drafting-phase attention of the same shape, outside the timed region: the n frontier tokens against the
    # prefix and the K/V of all depth*n pool nodes (the draft model's attention of the last drafting step)
    if args.mode == "stream" and not args.main_only and w.dtype == "bf16":
        gd = torch.Generator(device="cuda"); gd.manual_seed(seed + 555)
        nk = w.depth * w.n
        ktp = torch.randn((w.batch, w.kv_heads, nk, w.head_dim), generator=gd, device="cuda").to(torch.bfloat16)
        vtp = torch.randn((w.batch, w.kv_heads, nk, w.head_dim), generator=gd, device="cuda").to(torch.bfloat16)
        ts2 = api.TreeStream(w.batch, w.vocab, w.k, w.n, w.depth, api.OT_BF16)
        for t in range(w.depth):
            ts2.expand(builds[0].logits[:, t])
        fmask = ts2.frontier_mask()
        q0 = attns[0].keep[0]
        pd = api.PreparedAttention(q0, attns[0].keep[1], attns[0].keep[2], ktp, vtp, plen_d, fmask)
        for _ in range(5):
            pd(stream)
        torch.cuda.synchronize()
        td = time.perf_counter()
        for _ in range(200):
            pd(stream)
        torch.cuda.synchronize()
        result["draft_phase_attention"] = {"us_per_call": (time.perf_counter() - td) * 1e6 / 200, "queries": w.n,
                                           "tree_keys": nk, "prefix": w.prefix, "note": "warm inputs"}

    # ---- the tree build on fp32 logits of the same shape (the stored dtype of the bf16 workloads is a reading of
    # the paper, which never states it): second line for the scan, outside the timed region
    if args.mode == "stream" and not args.main_only and w.dtype == "bf16" and w.batch * w.rows_per_seq() * w.vocab < (1 << 28):
        pbs = [api.PreparedBuild(builds[i].logits.float(), w.k, w.n, w.depth) for i in range(min(ring, 6))]
        for pb in pbs:
            pb(stream)
        torch.cuda.synchronize()
        ev32 = [[hip.event(), hip.event()] for _ in range(60)]
        t32 = time.perf_counter()
        for i in range(60):
            pbs[i % len(pbs)].timed(stream, ev32[i][0], ev32[i][1])
        torch.cuda.synchronize()
        us32 = (time.perf_counter() - t32) * 1e6 / 60
        scan32 = float(np.mean([hip.elapsed_ms(a_, b_) for a_, b_ in ev32])) * 1e3
        result["fp32_logits"] = {"build_tree_us": us32, "row_scan_kernel_us": scan32,
                                 "row_scan_GBs": 2 * logit_bytes / (scan32 * 1e-6) / 1e9,
                                 "frac_of_hbm_peak": 2 * logit_bytes / (scan32 * 1e-6) / 1e9 / HBM_PEAK_GBS}
        del pbs

    # ---- the batched GQA shape, where the attention is bound by the matrix pipe, as a compact leg of the default run
    if args.mode == "stream" and not args.main_only and not args.no_gqa_leg and w.name == "7b":
        del builds[1:], attns[1:]
        torch.cuda.empty_cache()
        result["gqa_70b"] = gqa_leg("70b", 30, hip, stream)
        if yard:
            result["gqa_70b"]["roofline"]["frac_of_measured_mfma"] = result["gqa_70b"]["roofline"]["achieved"] / yard["mfma_bf16_TFLOPs"]
            result["gqa_70b"]["roofline_scan"]["frac_of_measured_read"] = result["gqa_70b"]["roofline_scan"]["achieved"] / yard["hbm_read_GBs"]

    # ---- CPU oracle on a bounded sample of the same workload ----------------------------------
    if args.cpu_steps > 0 and not args.skip_parity:
        from threadpoolctl import threadpool_limits
        cpu_dt = 0.0
        with threadpool_limits(limits=1):
            for s in range(args.cpu_steps):
                lg = wl.make_logits(w, seed + 100 + s) if s else logits_h      # generation is not timed
                tc = time.perf_counter()
                trees = U.oracle_trees(lg, w.dtype, w.k, w.n, w.depth)
                m = np.stack([t["mask"] for t in trees])
                ta_oracle.tree_verify_attention(f64["Q"], f64["K_prefix"], f64["V_prefix"], f64["K_tree"],
                                                f64["V_tree"], plen_h, m)
                cpu_dt += time.perf_counter() - tc
        result["cpu_baseline"] = {"value": args.cpu_steps / cpu_dt, "unit": "steps/s", "cores": 1,
                                  "host_cores": os.cpu_count(), "kind": "oracle",
                                  "sample": f"{args.cpu_steps} full steps of the same workload (fp64 NumPy oracle: "
                                            "tree build + tree attention; inputs pre-generated; 1 thread)"}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
