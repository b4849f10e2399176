"""The C-ABI library loads, exports every symbol the header declares, and rejects bad arguments on the
host before touching the GPU (no compute is launched by this file)."""
import ctypes as C
import os
import re

import pytest

from paper_2406_17276_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "opttree.h")).read()
    return re.findall(r"OT_API\s+[\w\s\*]+?\b(ot_\w+)\s*\(", text)


def test_header_declares_the_expected_entry_points():
    names = declared_symbols()
    for must in ["ot_build_tree", "ot_tree_verify_attention", "ot_tree_begin", "ot_tree_expand",
                 "ot_tree_finalize", "ot_build_workspace_bytes", "ot_attn_workspace_bytes"]:
        assert must in names


def test_library_exports_every_declared_symbol():
    L = api.lib()
    for name in declared_symbols():
        assert hasattr(L, name), name
    assert L.ot_version() >= 100
    assert L.ot_status_string(0) == b"ok"
    assert L.ot_status_string(-3) == b"workspace too small"


def _bp(**kw):
    d = dict(batch=1, vocab=1000, depth=4, k=4, n=16, logits_dtype=0, stride_seq=64000, stride_depth=16000, stride_row=1000)
    d.update(kw)
    return api.BuildParams(**d)


def test_build_workspace_query_and_limits():
    assert api.build_workspace_bytes(_bp()) > 0
    for bad in [dict(k=0), dict(n=0), dict(depth=0), dict(batch=0), dict(k=1001), dict(logits_dtype=7),
                dict(k=17), dict(n=257), dict(depth=33), dict(vocab=300000)]:
        assert api.build_workspace_bytes(_bp(**bad)) == 0, bad


def test_build_tree_rejects_bad_arguments_without_launching():
    L = api.lib()
    fake = C.c_void_p(0x1000)          # never dereferenced: validation fails first
    out = api.TreeOut(*([0x1000] * 7))
    p = _bp()
    need = api.build_workspace_bytes(p)
    assert L.ot_build_tree(None, fake, fake, need, C.byref(out), None) == -1
    assert L.ot_build_tree(C.byref(p), None, fake, need, C.byref(out), None) == -1
    assert L.ot_build_tree(C.byref(p), fake, None, need, C.byref(out), None) == -1
    assert L.ot_build_tree(C.byref(p), fake, fake, need, None, None) == -1
    assert L.ot_build_tree(C.byref(p), fake, fake, need - 1, C.byref(out), None) == -3
    assert L.ot_build_tree(C.byref(p), fake, C.c_void_p(0x1004), need, C.byref(out), None) == -1     # misaligned
    assert L.ot_build_tree(C.byref(_bp(stride_row=999)), fake, fake, need, C.byref(out), None) == -1
    assert L.ot_build_tree(C.byref(_bp(k=17)), fake, fake, need, C.byref(out), None) == -2
    bad_out = api.TreeOut(0x1000, 0, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000)
    assert L.ot_build_tree(C.byref(p), fake, fake, need, C.byref(bad_out), None) == -1
    assert L.ot_tree_expand(C.byref(p), 4, fake, 0, 1000, fake, need, fake, fake, fake, None) == -1    # step out of range
    assert L.ot_tree_expand(C.byref(p), 0, fake, 0, 1000, fake, need, fake, None, fake, None) == -1
    assert L.ot_tree_expand(C.byref(p), 0, fake, 0, 1000, fake, need, fake, fake, C.c_void_p(0x1002), None) == -1   # misaligned count
    assert L.ot_tree_expand(C.byref(p), 0, fake, 0, 999, fake, need, fake, fake, None, None) == -1     # row stride < vocab
    assert L.ot_tree_finalize(C.byref(p), 0, fake, need, C.byref(out), None) == -1


def _ap(**kw):
    s = (C.c_int64 * 3)
    d = dict(batch=1, q_heads=4, kv_heads=4, head_dim=64, n=16, max_prefix=128, dtype=0, softmax_scale=0.0,
             q_strides=s(4096, 1024, 64), kp_strides=s(32768, 8192, 64), vp_strides=s(32768, 8192, 64),
             kt_strides=s(4096, 1024, 64), vt_strides=s(4096, 1024, 64), o_strides=s(4096, 1024, 64))
    d.update(kw)
    return api.AttnParams(**d)


def test_attention_rejects_bad_arguments_without_launching():
    L = api.lib()
    s = (C.c_int64 * 3)
    assert api.attn_workspace_bytes(_ap()) > 0
    assert api.attn_workspace_bytes(_ap(q_heads=6, kv_heads=4)) == 0
    assert api.attn_workspace_bytes(_ap(head_dim=96)) == 0
    assert api.attn_workspace_bytes(_ap(n=0)) == 0
    assert api.attn_workspace_bytes(_ap(n=257)) == 0
    assert api.attn_workspace_bytes(_ap(n_keys=8193)) == 0
    assert api.attn_workspace_bytes(_ap(n_keys=-1)) == 0
    assert api.attn_workspace_bytes(_ap(n_keys=300)) > 0
    assert api.attn_workspace_bytes(_ap(q_strides=s(4096, 1024, 62))) == 0
    f = C.c_void_p(0x1000)
    p = _ap()
    need = api.attn_workspace_bytes(p)
    args = [f] * 9
    bad = list(args); bad[0] = None
    assert L.ot_tree_verify_attention(C.byref(p), *bad, need, None) == -1
    bad = list(args); bad[1] = None                                                  # K_prefix NULL with max_prefix > 0
    assert L.ot_tree_verify_attention(C.byref(p), *bad, need, None) == -1
    bad = list(args); bad[0] = C.c_void_p(0x1008)
    assert L.ot_tree_verify_attention(C.byref(p), *bad, need, None) == -1
    assert L.ot_tree_verify_attention(C.byref(p), *args, need - 1, None) == -3
    assert L.ot_tree_verify_attention(C.byref(_ap(head_dim=96)), *args, need, None) == -2
    assert need > 4096                                                               # room for the ticket counters
    assert L.ot_attn_workspace_prepare(None, need, None) == -1
    assert L.ot_attn_workspace_prepare(C.c_void_p(0x1008), need, None) == -1
    assert L.ot_attn_workspace_prepare(f, 100, None) == -3


def test_fp8_cache_attention_rejects_bad_arguments_without_launching():
    L = api.lib()
    s = (C.c_int64 * 3)
    f = C.c_void_p(0x1000)
    ok = _ap(dtype=1)                                      # bf16 Q and O; all K/V strides are multiples of 16 bytes
    need = api.attn_workspace_bytes(ok)
    call = lambda p, a, ws=need: L.ot_tree_verify_attention_fp8kv(C.byref(p), *a, ws, None)
    args = [f] * 11                                        # Q, Kp, Vp, Kt, Vt, k_scale, v_scale, prefix_len, mask, O, workspace
    assert call(_ap(dtype=0), args) == -1                  # f32 Q/O
    assert call(_ap(dtype=1, kp_strides=s(32768, 8192, 72)), args) == -1     # 72 bytes: fine for bf16 rows, not for byte rows
    bad = list(args); bad[5] = None
    assert call(ok, bad) == -1                             # k_scale NULL
    bad = list(args); bad[6] = C.c_void_p(0x1002)
    assert call(ok, bad) == -1                             # v_scale misaligned
    assert call(ok, args, need - 1) == -3
    assert call(_ap(dtype=1, head_dim=96), args) == -2


def test_no_allocation_entry_point_validates_before_touching_the_gpu():
    L = api.lib()
    f = C.c_void_p(0x1000)
    assert L.ot_tree_verify_attention_noalloc(None, *([f] * 8), None) == -1
    assert L.ot_tree_verify_attention_noalloc(C.byref(_ap(head_dim=96)), *([f] * 8), None) == -2
    # one sequence, 64 query heads on 8 KV heads, a long prefix: many key splits of 512 packed rows each, whose
    # partial results exceed the library's scratch array
    s = (C.c_int64 * 3)
    big = _ap(q_heads=64, kv_heads=8, head_dim=128, n=64, max_prefix=4096, dtype=1,
              q_strides=s(524288, 8192, 128), o_strides=s(524288, 8192, 128),
              kt_strides=s(65536, 8192, 128), vt_strides=s(65536, 8192, 128),
              kp_strides=s(4194304, 524288, 128), vp_strides=s(4194304, 524288, 128))
    assert api.attn_workspace_bytes(big) > (8 << 20)
    assert L.ot_tree_verify_attention_noalloc(C.byref(big), *([f] * 8), None) == -5
    assert L.ot_status_string(-5).startswith(b"needs more scratch")


def test_binding_rejects_tensors_smaller_than_the_frontier():
    """The C ABI sees pointers, not extents: the binding refuses a logits tensor whose slot dimension is smaller
    than the widest frontier F_t = min(n, k F_{t-1}) the library would read."""
    import torch
    ok = torch.zeros((1, 3, 16, 64), dtype=torch.float32)
    assert api.build_params(ok, 4, 16, 3).n == 16
    assert api.frontier_sizes(4, 16, 3) == [1, 4, 16, 16]
    with pytest.raises(ValueError):
        api.build_params(torch.zeros((1, 3, 15, 64)), 4, 16, 4)          # depth 4 needs 4 steps and 16 slots
    with pytest.raises(ValueError):
        api.build_params(torch.zeros((1, 4, 15, 64)), 4, 16, 4)          # step 2 and 3 read 16 rows
    assert api.build_params(torch.zeros((1, 2, 4, 64)), 4, 16, 2).depth == 2   # steps 0 and 1 read 1 and 4 rows
    ts = api.TreeStream.__new__(api.TreeStream)
    ts.p = api.BuildParams(2, 64, 3, 4, 16, api.OT_F32, 0, 0, 64)
    ts.step = 2
    with pytest.raises(ValueError):
        ts.expand(torch.zeros((2, 15, 64)))                               # step 2 reads 16 rows
    with pytest.raises(ValueError):
        ts.expand(torch.zeros((1, 16, 64)))                               # batch too small
    ts.step = 3
    with pytest.raises(ValueError):
        ts.expand(torch.zeros((2, 16, 64)))                               # all steps fed


def test_binding_fails_loudly_when_library_is_missing(monkeypatch):
    monkeypatch.setattr(api, "_lib", None)
    monkeypatch.setattr(api, "_LIB_PATH", "/nonexistent/libopttree.so")
    with pytest.raises(FileNotFoundError):
        api.lib()


def test_esub_rejects_bad_arguments_without_launching():
    L = api.lib()
    p = _bp()
    need = api.build_workspace_bytes(p)
    f = C.c_void_p(0x1000)
    assert L.ot_tree_esub(C.byref(p), 0, 0.1, f, need, f, f, None) == -1            # no step done yet
    assert L.ot_tree_esub(C.byref(p), p.depth + 1, 0.1, f, need, f, f, None) == -1
    assert L.ot_tree_esub(C.byref(p), 1, float("nan"), f, need, f, f, None) == -1
    assert L.ot_tree_esub(C.byref(p), 1, 0.1, f, need, None, f, None) == -1
    assert L.ot_tree_esub(C.byref(p), 1, 0.1, f, need, f, C.c_void_p(0x1002), None) == -1
    assert L.ot_tree_esub(C.byref(p), 1, 0.1, f, need - 1, f, f, None) == -3


def test_one_shot_adaptive_build_rejects_bad_arguments_without_launching():
    L = api.lib()
    p = _bp()
    need = api.build_workspace_bytes(p)
    f = C.c_void_p(0x1000)
    out = api.TreeOut(*([0x1000] * 7))
    call = lambda p, delta, logits, ws, nb, steps, es: L.ot_build_tree_adaptive(
        C.byref(p), C.c_double(delta), logits, ws, nb, C.byref(out), steps, es, None)
    assert call(p, float("nan"), f, f, need, f, f) == -1
    assert call(p, 0.1, None, f, need, f, f) == -1
    assert call(p, 0.1, f, f, need, None, f) == -1
    assert call(p, 0.1, f, f, need, f, C.c_void_p(0x1004)) == -1        # e_sub is double[batch]
    assert call(p, 0.1, f, f, need - 1, f, f) == -3
    # (n beyond one wavefront is served step by step: the same argument checks apply before anything is launched)
    assert call(_bp(n=100), 0.1, f, f, api.build_workspace_bytes(_bp(n=100)) - 1, f, f) == -3


def test_verify_rejects_bad_arguments_without_launching():
    L = api.lib()
    vp = lambda **kw: api.VerifyParams(**{**dict(batch=2, vocab=1000, n=16, logits_dtype=api.OT_F32, stride_seq=17000,
                                                  stride_row=1000), **kw})
    p = vp()
    need = L.ot_verify_workspace_bytes(C.byref(p))
    assert need > 0
    assert L.ot_verify_workspace_bytes(C.byref(vp(n=0))) == 0
    assert L.ot_verify_workspace_bytes(C.byref(vp(n=257))) == 0
    assert L.ot_verify_workspace_bytes(C.byref(vp(stride_row=999))) == 0
    f = C.c_void_p(0x1000)
    args = [f] * 4
    assert L.ot_verify_greedy(C.byref(p), None, f, f, f, f, need, f, f, f, None) == -1
    assert L.ot_verify_greedy(C.byref(p), f, f, f, f, f, need - 1, f, f, f, None) == -3
    assert L.ot_verify_greedy(C.byref(p), f, f, f, f, C.c_void_p(0x1008), need, f, f, f, None) == -1
    assert L.ot_verify_greedy(C.byref(vp(logits_dtype=7)), f, f, f, f, f, need, f, f, f, None) == -1
    # random-sampling verification
    need_s = L.ot_verify_sample_workspace_bytes(C.byref(p))
    assert need_s > 0
    assert L.ot_verify_sample_workspace_bytes(C.byref(vp(n=0))) == 0
    assert L.ot_verify_sample_workspace_bytes(C.byref(vp(vocab=200000, stride_row=200000))) == 0    # > 512 f32 segments
    smp = lambda p, T, logits, u, ws, nb: L.ot_verify_sample(C.byref(p), C.c_float(T), logits, u, f, f, f, ws, nb,
                                                             f, f, f, None)
    assert smp(p, 0.0, f, f, f, need_s) == -1                       # temperature must be positive
    assert smp(p, -1.0, f, f, f, need_s) == -1
    assert smp(p, float("nan"), f, f, f, need_s) == -1
    assert smp(p, float("inf"), f, f, f, need_s) == -1
    assert smp(p, 1.0, None, f, f, need_s) == -1
    assert smp(p, 1.0, f, None, f, need_s) == -1
    assert smp(p, 1.0, f, C.c_void_p(0x1002), f, need_s) == -1
    assert smp(p, 1.0, f, f, f, need_s - 1) == -3
    assert smp(vp(vocab=200000, stride_row=200000), 1.0, f, f, f, 1 << 30) == -2
    assert smp(vp(batch=4000), 1.0, f, f, f, 1 << 30) == -2         # batch * (n + 1) beyond one grid dimension
    ap = _ap()
    assert L.ot_kv_append(C.byref(ap), None, f, f, f, f, f, f, f, None) == -1
    assert L.ot_kv_append(C.byref(ap), C.c_void_p(0x1004), f, f, f, f, f, f, f, None) == -1
    assert L.ot_kv_append(C.byref(_ap(max_prefix=0)), f, f, f, f, f, f, f, f, None) == -1
    # the two length arrays must not overlap (other workgroups still read the old length when the new one lands)
    g2 = C.c_void_p(0x2000)
    assert L.ot_kv_append(C.byref(_ap(batch=4)), f, f, f, f, g2, f, f, g2, None) == -1
    assert L.ot_kv_append(C.byref(_ap(batch=4)), f, f, f, f, g2, f, f, C.c_void_p(0x2008), None) == -1


def test_yardsticks_reject_bad_arguments_without_launching():
    L = api.lib()
    f = C.c_void_p(0x1000)
    assert L.ot_yardstick_stream_read(None, 1 << 20, f, None) == -1
    assert L.ot_yardstick_stream_read(C.c_void_p(0x1008), 1 << 20, f, None) == -1
    assert L.ot_yardstick_stream_read(f, 8, f, None) == -1
    assert L.ot_yardstick_stream_read_timed(None, 1 << 20, 64, f, None, None, None) == -1
    assert L.ot_yardstick_stream_read_timed(f, 1 << 20, 0, f, None, None, None) == -1
    assert L.ot_yardstick_mfma_loop(0, f, None) == -1
    assert L.ot_yardstick_mfma_loop(10, None, None) == -1


def test_frontier_mask_rejects_bad_arguments_without_launching():
    L = api.lib()
    L.ot_tree_frontier_mask.restype = C.c_int
    p = _bp()
    need = api.build_workspace_bytes(p)
    f = C.c_void_p(0x1000)
    assert L.ot_tree_frontier_mask(C.byref(p), 0, f, need, f, None) == -1
    assert L.ot_tree_frontier_mask(C.byref(p), 1, f, need, None, None) == -1
    assert L.ot_tree_frontier_mask(C.byref(p), 1, f, need - 1, f, None) == -3
