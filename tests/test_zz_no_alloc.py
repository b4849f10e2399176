"""ot_tree_verify_attention_noalloc (the entry point for callers that cannot allocate: its workspace is a
library-owned device array) against ot_tree_verify_attention, through the C ABI: two calls in a row on the
shared array, the second on a smaller input, then a batch that needs no split partials."""
import ctypes as C

import numpy as np
import pytest

from oracle import opt_tree as ot_oracle
from oracle import tree_attention as ta_oracle
import workloads as wl
from tests import _util as U

pytestmark = pytest.mark.gpu


def _case(dtype, B, Hq, Hkv, D, L, n, seed, ragged=0.0):
    w = wl.Workload("t", B, 8, 1, 1, n, dtype, "normal", 1.0, Hq, Hkv, D, L, ragged=ragged)
    x = wl.make_attention_inputs(w, seed)
    mask = np.stack([ot_oracle.ancestor_mask(wl.random_tree_parents(n, seed + b)) for b in range(B)])
    return x, mask


def test_no_allocation_entry_point_matches_the_workspace_one():
    import torch
    from paper_2406_17276_amd import api
    cases = [("bf16", 1, 8, 8, 128, 1000, 50, 3, 0.0),          # split partials and tickets in the shared array
             ("bf16", 1, 4, 2, 128, 300, 20, 4, 0.0),           # smaller input on the same array, right after
             ("bf16", 1, 16, 4, 128, 500, 60, 5, 0.0),          # 128-row variant with key splits
             ("bf16", 40, 16, 4, 128, 200, 60, 7, 0.25),        # ragged batch that fills the chip without splits
             ("f32", 2, 4, 4, 64, 200, 16, 6, 0.0)]             # fp32 kernels + combine
    for dtype, B, Hq, Hkv, D, L, n, seed, ragged in cases:
        print("no-alloc case", dtype, B, Hq, Hkv, D, L, n, flush=True)
        x, mask = _case(dtype, B, Hq, Hkv, D, L, n, seed, ragged)
        dev = {k: U.to_device(v, dtype) for k, v in x.items() if k != "prefix_len"}
        plen = torch.from_numpy(x["prefix_len"].astype(np.int32)).cuda()
        md = U.mask_to_device(mask)
        ref = api.tree_verify_attention(dev["Q"], dev["K_prefix"], dev["V_prefix"], dev["K_tree"], dev["V_tree"], plen, md)
        out = torch.full_like(dev["Q"], float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        api.tree_verify_attention_noalloc(dev["Q"], dev["K_prefix"], dev["V_prefix"], dev["K_tree"], dev["V_tree"],
                                          plen, md, out)
        assert torch.cuda.memory_allocated() == before           # nothing came from torch's allocator either
        torch.cuda.synchronize()
        tol = 2e-2 if dtype == "bf16" else 1e-5
        f = {k: wl.to_f64(v, dtype) for k, v in x.items() if k != "prefix_len"}
        want = ta_oracle.tree_verify_attention(f["Q"], f["K_prefix"], f["V_prefix"], f["K_tree"], f["V_tree"],
                                               x["prefix_len"], mask)
        assert np.abs(U.from_device_f64(out) - want).max() < tol
        assert torch.equal(out, ref), "same kernels, same plan: the two entry points agree bit for bit"
