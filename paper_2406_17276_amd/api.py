"""ctypes binding of libopttree.so: argument marshalling only.

Function names mirror include/opttree.h.  PyTorch is used for device memory
(tensors in, tensors out) and for the current HIP stream; every step of the
path runs in the library's kernels.  There is no CPU fallback: if the library
is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

OT_F32, OT_BF16 = 0, 1
OT_MAX_NODES, OT_MAX_TOPK, OT_MAX_DEPTH = 256, 16, 32

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libopttree.so")
_lib = None


class OptTreeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().ot_status_string(status).decode()
        if status == -4:
            msg += f" (hipError {lib().ot_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{status}]")


class BuildParams(C.Structure):
    _fields_ = [("batch", C.c_int32), ("vocab", C.c_int32), ("depth", C.c_int32), ("k", C.c_int32),
                ("n", C.c_int32), ("logits_dtype", C.c_int32),
                ("stride_seq", C.c_int64), ("stride_depth", C.c_int64), ("stride_row", C.c_int64)]


class TreeOut(C.Structure):
    _fields_ = [("token", C.c_void_p), ("parent", C.c_void_p), ("depth", C.c_void_p), ("score", C.c_void_p),
                ("mask", C.c_void_p), ("n_out", C.c_void_p), ("expect", C.c_void_p)]


class AttnParams(C.Structure):
    _fields_ = [("batch", C.c_int32), ("q_heads", C.c_int32), ("kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("n", C.c_int32), ("max_prefix", C.c_int32), ("dtype", C.c_int32), ("softmax_scale", C.c_float),
                ("q_strides", C.c_int64 * 3), ("kp_strides", C.c_int64 * 3), ("vp_strides", C.c_int64 * 3),
                ("kt_strides", C.c_int64 * 3), ("vt_strides", C.c_int64 * 3), ("o_strides", C.c_int64 * 3),
                ("n_keys", C.c_int32)]


class VerifyParams(C.Structure):
    _fields_ = [("batch", C.c_int32), ("vocab", C.c_int32), ("n", C.c_int32), ("logits_dtype", C.c_int32),
                ("stride_seq", C.c_int64), ("stride_row", C.c_int64)]


def lib():
    """Open libopttree.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2406_17276_amd.build` "
                "(there is no fallback path)")
        L = C.CDLL(_LIB_PATH)
        L.ot_version.restype = C.c_int
        L.ot_status_string.restype = C.c_char_p
        L.ot_status_string.argtypes = [C.c_int]
        L.ot_last_hip_error.restype = C.c_int
        L.ot_build_workspace_bytes.restype = C.c_size_t
        L.ot_build_workspace_bytes.argtypes = [C.POINTER(BuildParams)]
        L.ot_build_tree.restype = C.c_int
        L.ot_build_tree.argtypes = [C.POINTER(BuildParams), C.c_void_p, C.c_void_p, C.c_size_t,
                                    C.POINTER(TreeOut), C.c_void_p]
        L.ot_build_tree_timed.restype = C.c_int
        L.ot_build_tree_timed.argtypes = [C.POINTER(BuildParams), C.c_void_p, C.c_void_p, C.c_size_t,
                                          C.POINTER(TreeOut), C.c_void_p, C.c_void_p, C.c_void_p]
        L.ot_build_tree_adaptive.restype = C.c_int
        L.ot_build_tree_adaptive.argtypes = [C.POINTER(BuildParams), C.c_double, C.c_void_p, C.c_void_p, C.c_size_t,
                                             C.POINTER(TreeOut), C.c_void_p, C.c_void_p, C.c_void_p]
        L.ot_tree_begin.restype = C.c_int
        L.ot_tree_begin.argtypes = [C.POINTER(BuildParams), C.c_void_p, C.c_size_t, C.c_void_p]
        L.ot_tree_expand.restype = C.c_int
        L.ot_tree_expand.argtypes = [C.POINTER(BuildParams), C.c_int32, C.c_void_p, C.c_int64, C.c_int64,
                                     C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.ot_tree_finalize.restype = C.c_int
        L.ot_tree_finalize.argtypes = [C.POINTER(BuildParams), C.c_int32, C.c_void_p, C.c_size_t,
                                       C.POINTER(TreeOut), C.c_void_p]
        L.ot_tree_frontier_mask.restype = C.c_int
        L.ot_tree_frontier_mask.argtypes = [C.POINTER(BuildParams), C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p,
                                            C.c_void_p]
        L.ot_tree_esub.restype = C.c_int
        L.ot_tree_esub.argtypes = [C.POINTER(BuildParams), C.c_int32, C.c_double, C.c_void_p, C.c_size_t,
                                   C.c_void_p, C.c_void_p, C.c_void_p]
        L.ot_verify_workspace_bytes.restype = C.c_size_t
        L.ot_verify_workspace_bytes.argtypes = [C.POINTER(VerifyParams)]
        L.ot_verify_sample_workspace_bytes.restype = C.c_size_t
        L.ot_verify_sample_workspace_bytes.argtypes = [C.POINTER(VerifyParams)]
        L.ot_verify_sample.restype = C.c_int
        L.ot_verify_sample.argtypes = ([C.POINTER(VerifyParams), C.c_float] + [C.c_void_p] * 6 + [C.c_size_t] +
                                       [C.c_void_p] * 4)
        L.ot_verify_greedy.restype = C.c_int
        L.ot_verify_greedy.argtypes = [C.POINTER(VerifyParams)] + [C.c_void_p] * 5 + [C.c_size_t] + [C.c_void_p] * 4
        L.ot_kv_append.restype = C.c_int
        L.ot_kv_append.argtypes = [C.POINTER(AttnParams)] + [C.c_void_p] * 9
        L.ot_yardstick_stream_read.restype = C.c_int
        L.ot_yardstick_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.ot_yardstick_stream_read_timed.restype = C.c_int
        L.ot_yardstick_stream_read_timed.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                                     C.c_void_p]
        L.ot_yardstick_mfma_loop.restype = C.c_int
        L.ot_yardstick_mfma_loop.argtypes = [C.c_int32, C.c_void_p, C.c_void_p]
        L.ot_attn_workspace_bytes.restype = C.c_size_t
        L.ot_attn_workspace_bytes.argtypes = [C.POINTER(AttnParams)]
        L.ot_attn_workspace_prepare.restype = C.c_int
        L.ot_attn_workspace_prepare.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p]
        L.ot_tree_verify_attention.restype = C.c_int
        L.ot_tree_verify_attention.argtypes = [C.POINTER(AttnParams)] + [C.c_void_p] * 9 + [C.c_size_t, C.c_void_p]
        L.ot_tree_verify_attention_noalloc.restype = C.c_int
        L.ot_tree_verify_attention_noalloc.argtypes = [C.POINTER(AttnParams)] + [C.c_void_p] * 9
        L.ot_tree_verify_attention_fp8kv.restype = C.c_int
        L.ot_tree_verify_attention_fp8kv.argtypes = [C.POINTER(AttnParams)] + [C.c_void_p] * 11 + [C.c_size_t, C.c_void_p]
        L.ot_tree_verify_attention_timed.restype = C.c_int
        L.ot_tree_verify_attention_timed.argtypes = ([C.POINTER(AttnParams)] + [C.c_void_p] * 9 +
                                                     [C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p])
        _lib = L
    return _lib


def _check(status: int, where: str):
    if status != 0:
        raise OptTreeError(status, where)


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return OT_F32
    if t.dtype == torch.bfloat16:
        return OT_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


@dataclass
class Tree:
    token: "object"     # int32 [B, n]
    parent: "object"    # int32 [B, n]
    depth: "object"     # int32 [B, n]
    score: "object"     # float32 [B, n]
    mask: "object"      # int64 [B, n, W] (bit pattern of the uint64 words)
    n_out: "object"     # int32 [B]
    expect: "object"    # float64 [B]

    def c_struct(self) -> TreeOut:
        return TreeOut(self.token.data_ptr(), self.parent.data_ptr(), self.depth.data_ptr(), self.score.data_ptr(),
                       self.mask.data_ptr(), self.n_out.data_ptr(), self.expect.data_ptr())


def alloc_tree(batch: int, n: int, device="cuda") -> Tree:
    import torch
    W = (n + 63) // 64
    return Tree(token=torch.empty((batch, n), dtype=torch.int32, device=device),
                parent=torch.empty((batch, n), dtype=torch.int32, device=device),
                depth=torch.empty((batch, n), dtype=torch.int32, device=device),
                score=torch.empty((batch, n), dtype=torch.float32, device=device),
                mask=torch.empty((batch, n, W), dtype=torch.int64, device=device),
                n_out=torch.empty((batch,), dtype=torch.int32, device=device),
                expect=torch.empty((batch,), dtype=torch.float64, device=device))


def frontier_sizes(k: int, n: int, depth: int):
    """Rows the library reads per drafting step: F_0 = 1, F_{t+1} = min(n, k F_t) (ot_build_tree's input
    contract).  Used only to check tensor extents, which the C ABI cannot see."""
    F = [1]
    for _ in range(depth):
        F.append(min(n, k * F[-1]))
    return F


def build_params(logits, k: int, n: int, depth: int) -> BuildParams:
    """logits: [B, depth, n, V] (any strides with a contiguous last dimension)."""
    if logits.dim() != 4 or logits.stride(3) != 1:
        raise ValueError("logits must be [B, depth, n, V] with a contiguous last dimension")
    B, d, nn, V = logits.shape
    need = max(frontier_sizes(k, n, depth)[:depth]) if depth >= 1 and k >= 1 and n >= 1 else 1
    if d < depth or nn < need:
        raise ValueError(f"logits tensor [{B}, {d}, {nn}, {V}] smaller than (depth {depth}, widest frontier {need})")
    return BuildParams(B, V, depth, k, n, _dtype_code(logits), logits.stride(0), logits.stride(1), logits.stride(2))


def build_workspace_bytes(p: BuildParams) -> int:
    return int(lib().ot_build_workspace_bytes(C.byref(p)))


def build_tree(logits, k: int, n: int, depth: int, out: Tree | None = None, workspace=None) -> Tree:
    """ot_build_tree: one-shot draft-tree construction on the current stream."""
    import torch
    p = build_params(logits, k, n, depth)
    need = build_workspace_bytes(p)
    if need == 0:
        _check(lib().ot_build_tree(C.byref(p), logits.data_ptr(), None, 0, None, None), "ot_build_tree")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=logits.device)
    if out is None:
        out = alloc_tree(p.batch, n, logits.device)
    o = out.c_struct()
    _check(lib().ot_build_tree(C.byref(p), logits.data_ptr(), workspace.data_ptr(), workspace.numel(),
                               C.byref(o), _stream()), "ot_build_tree")
    return out


def build_tree_adaptive(logits, k: int, n: int, depth: int, delta: float, out: Tree | None = None, workspace=None):
    """ot_build_tree_adaptive on the current stream; returns (tree, steps_used int32 [B], e_sub float64 [B])."""
    import torch
    p = build_params(logits, k, n, depth)
    if out is None:
        out = alloc_tree(p.batch, n, logits.device)
    need = build_workspace_bytes(p)
    if need == 0:
        raise OptTreeError(-2, "ot_build_workspace_bytes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=logits.device)
    steps = torch.empty(p.batch, dtype=torch.int32, device=logits.device)
    e_sub = torch.empty(p.batch, dtype=torch.float64, device=logits.device)
    o = out.c_struct()
    _check(lib().ot_build_tree_adaptive(C.byref(p), float(delta), logits.data_ptr(), workspace.data_ptr(),
                                        workspace.numel(), C.byref(o), steps.data_ptr(), e_sub.data_ptr(), _stream()),
           "ot_build_tree_adaptive")
    return out, steps, e_sub


class TreeStream:
    """ot_tree_begin / ot_tree_expand / ot_tree_finalize for one batch of trees."""

    def __init__(self, batch: int, vocab: int, k: int, n: int, depth: int, dtype_code: int, device="cuda"):
        import torch
        self.p = BuildParams(batch, vocab, depth, k, n, dtype_code, 0, 0, vocab)
        need = build_workspace_bytes(self.p)
        if need == 0:
            _check(lib().ot_tree_begin(C.byref(self.p), None, 0, None), "ot_tree_begin")
        self.ws = torch.empty(need, dtype=torch.uint8, device=device)
        self.frontier_token = torch.full((batch, n), -1, dtype=torch.int32, device=device)
        self.frontier_parent = torch.full((batch, n), -1, dtype=torch.int32, device=device)
        self.frontier_count = torch.zeros((batch,), dtype=torch.int32, device=device)
        self.step = 0
        _check(lib().ot_tree_begin(C.byref(self.p), self.ws.data_ptr(), self.ws.numel(), _stream()), "ot_tree_begin")

    def expand(self, rows):
        """rows: [B, >=F_t, V]; returns (tokens, parent_slots) views of the next frontier [B, n]."""
        if rows.dim() != 3 or rows.stride(2) != 1:
            raise ValueError("rows must be [B, F, V] with a contiguous last dimension")
        if self.step >= self.p.depth:
            raise ValueError(f"all {self.p.depth} drafting steps have been fed")
        need = frontier_sizes(self.p.k, self.p.n, self.p.depth)[self.step]
        if rows.shape[0] < self.p.batch or rows.shape[1] < need or rows.shape[2] < self.p.vocab:
            raise ValueError(f"rows {tuple(rows.shape)} smaller than [batch {self.p.batch}, F_{self.step} = {need}, "
                             f"vocab {self.p.vocab}]")
        _check(lib().ot_tree_expand(C.byref(self.p), self.step, rows.data_ptr(), rows.stride(0), rows.stride(1),
                                    self.ws.data_ptr(), self.ws.numel(), self.frontier_token.data_ptr(),
                                    self.frontier_parent.data_ptr(), self.frontier_count.data_ptr(), _stream()),
               "ot_tree_expand")
        self.step += 1
        return self.frontier_token, self.frontier_parent

    def frontier_mask(self):
        """ot_tree_frontier_mask after the latest expand: int64 [B, n, W] (bit pattern of the uint64 words),
        W = ceil(depth * n / 64), over pool indices step * n + slot."""
        import torch
        W = (self.p.depth * self.p.n + 63) // 64
        m = torch.empty((self.p.batch, self.p.n, W), dtype=torch.int64, device=self.ws.device)
        _check(lib().ot_tree_frontier_mask(C.byref(self.p), self.step, self.ws.data_ptr(), self.ws.numel(),
                                           m.data_ptr(), _stream()), "ot_tree_frontier_mask")
        return m

    def e_sub(self, delta: float):
        """ot_tree_esub after the latest expand: (E_sub per sequence, go-on flag per sequence), device tensors."""
        import torch
        if not hasattr(self, "_esub"):
            self._esub = torch.empty(self.p.batch, dtype=torch.float64, device=self.ws.device)
            self._go = torch.empty(self.p.batch, dtype=torch.int32, device=self.ws.device)
        _check(lib().ot_tree_esub(C.byref(self.p), self.step, float(delta), self.ws.data_ptr(), self.ws.numel(),
                                  self._esub.data_ptr(), self._go.data_ptr(), _stream()), "ot_tree_esub")
        return self._esub, self._go

    def finalize(self, out: Tree | None = None) -> Tree:
        if out is None:
            out = alloc_tree(self.p.batch, self.p.n, self.ws.device)
        o = out.c_struct()
        _check(lib().ot_tree_finalize(C.byref(self.p), self.step, self.ws.data_ptr(), self.ws.numel(),
                                      C.byref(o), _stream()), "ot_tree_finalize")
        return out


def attn_params(Q, K_prefix, V_prefix, K_tree, V_tree, max_prefix=None, softmax_scale: float = 0.0) -> AttnParams:
    B, Hq, n, D = Q.shape
    Hkv = K_tree.shape[1]
    if max_prefix is None:
        max_prefix = 0 if K_prefix is None else K_prefix.shape[2]

    def st(t):
        if t is None:
            return (C.c_int64 * 3)(0, 0, D)
        if t.stride(3) != 1:
            raise ValueError("last dimension must be contiguous")
        return (C.c_int64 * 3)(t.stride(0), t.stride(1), t.stride(2))

    n_keys = K_tree.shape[2]
    return AttnParams(B, Hq, Hkv, D, n, max_prefix, _dtype_code(Q), float(softmax_scale),
                      st(Q), st(K_prefix), st(V_prefix), st(K_tree), st(V_tree), st(Q), 0 if n_keys == n else n_keys)


def attn_workspace_bytes(p: AttnParams) -> int:
    return int(lib().ot_attn_workspace_bytes(C.byref(p)))


def attn_workspace(p: AttnParams, device):
    """A workspace for ot_tree_verify_attention, already prepared (ot_attn_workspace_prepare on the
    current stream): its ticket counters are zero, and every completed call leaves them zero."""
    import torch
    need = attn_workspace_bytes(p)
    if need == 0:
        raise OptTreeError(-2, "ot_attn_workspace_bytes")
    ws = torch.empty(need, dtype=torch.uint8, device=device)
    _check(lib().ot_attn_workspace_prepare(ws.data_ptr(), ws.numel(), _stream()), "ot_attn_workspace_prepare")
    torch.cuda.current_stream().synchronize()      # the workspace may be used on any stream afterwards
    return ws


OT_ATTN_STATUS_OFFSET = 4092
OT_ATTN_STATUS_PREFIX_CLAMPED = 1


def attn_status(workspace) -> int:
    """The status word the attention calls keep in their workspace (bit 0: a prefix length was clamped).
    Reads device memory: synchronises the current stream."""
    import torch
    return int(workspace[OT_ATTN_STATUS_OFFSET:OT_ATTN_STATUS_OFFSET + 4].view(torch.int32).item())


def tree_verify_attention(Q, K_prefix, V_prefix, K_tree, V_tree, prefix_len, mask, out=None, workspace=None,
                          softmax_scale: float = 0.0):
    """ot_tree_verify_attention on the current stream.  Q [B,Hq,n,D]; K/V_prefix [B,Hkv,Lmax,D] (or None);
    K/V_tree [B,Hkv,n,D]; prefix_len int32 [B]; mask int64 [B,n,W].  A caller-supplied workspace must be a
    prepared one (attn_workspace)."""
    import torch
    p = attn_params(Q, K_prefix, V_prefix, K_tree, V_tree, softmax_scale=softmax_scale)
    if out is None:
        out = torch.empty_like(Q)
    p.o_strides = (C.c_int64 * 3)(out.stride(0), out.stride(1), out.stride(2))
    if workspace is None:
        workspace = attn_workspace(p, Q.device)
    ptr = lambda t: None if t is None else t.data_ptr()
    _check(lib().ot_tree_verify_attention(
        C.byref(p), ptr(Q), ptr(K_prefix), ptr(V_prefix), ptr(K_tree), ptr(V_tree), ptr(prefix_len), ptr(mask),
        ptr(out), ptr(workspace), 0 if workspace is None else workspace.numel(), _stream()),
        "ot_tree_verify_attention")
    return out


def tree_verify_attention_noalloc(Q, K_prefix, V_prefix, K_tree, V_tree, prefix_len, mask, out, softmax_scale=0.0):
    """ot_tree_verify_attention_noalloc on the current stream: as tree_verify_attention, with the library's own
    scratch array as workspace; `out` is supplied by the caller (nothing is allocated)."""
    p = attn_params(Q, K_prefix, V_prefix, K_tree, V_tree, softmax_scale=softmax_scale)
    p.o_strides = (C.c_int64 * 3)(out.stride(0), out.stride(1), out.stride(2))
    ptr = lambda t: None if t is None else t.data_ptr()
    _check(lib().ot_tree_verify_attention_noalloc(
        C.byref(p), ptr(Q), ptr(K_prefix), ptr(V_prefix), ptr(K_tree), ptr(V_tree), ptr(prefix_len), ptr(mask),
        ptr(out), _stream()), "ot_tree_verify_attention_noalloc")
    return out


def tree_verify_attention_fp8kv(Q, K_prefix, V_prefix, K_tree, V_tree, k_scale, v_scale, prefix_len, mask, out=None,
                                workspace=None, softmax_scale: float = 0.0):
    """ot_tree_verify_attention_fp8kv on the current stream.  Q bf16 [B,Hq,n,D]; K/V uint8 tensors of FP8 E4M3 bytes
    [B,Hkv,rows,D]; k_scale, v_scale float32 [B,Hkv]."""
    import torch
    for t in (K_prefix, V_prefix, K_tree, V_tree):
        if t is not None and t.dtype != torch.uint8:
            raise TypeError("the 8-bit cache is passed as uint8 tensors")
    for t in (k_scale, v_scale):
        if t.dtype != torch.float32 or not t.is_contiguous() or tuple(t.shape) != (Q.shape[0], K_tree.shape[1]):
            raise ValueError("scales must be contiguous float32 [B, Hkv]")
    p = attn_params(Q, K_prefix, V_prefix, K_tree, V_tree, softmax_scale=softmax_scale)
    if out is None:
        out = torch.empty_like(Q)
    p.o_strides = (C.c_int64 * 3)(out.stride(0), out.stride(1), out.stride(2))
    if workspace is None:
        workspace = attn_workspace(p, Q.device)
    ptr = lambda t: None if t is None else t.data_ptr()
    _check(lib().ot_tree_verify_attention_fp8kv(
        C.byref(p), ptr(Q), ptr(K_prefix), ptr(V_prefix), ptr(K_tree), ptr(V_tree), ptr(k_scale), ptr(v_scale),
        ptr(prefix_len), ptr(mask), ptr(out), ptr(workspace), workspace.numel(), _stream()),
        "ot_tree_verify_attention_fp8kv")
    return out


def verify_greedy(target_logits, tree: "Tree", workspace=None):
    """ot_verify_greedy on the current stream.  target_logits [B, n + 1, V] (row 0 = the root position);
    returns (accept_len [B], accept_node [B, n], accept_token [B, n + 1]) as int32 device tensors."""
    import torch
    if target_logits.dim() != 3 or target_logits.stride(2) != 1:
        raise ValueError("target_logits must be [B, n + 1, V] with a contiguous last dimension")
    B, rows, V = target_logits.shape
    n = rows - 1
    p = VerifyParams(B, V, n, _dtype_code(target_logits), target_logits.stride(0), target_logits.stride(1))
    need = int(lib().ot_verify_workspace_bytes(C.byref(p)))
    if need == 0:
        raise OptTreeError(-2, "ot_verify_workspace_bytes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=target_logits.device)
    dev = target_logits.device
    accept_len = torch.empty(B, dtype=torch.int32, device=dev)
    accept_node = torch.empty((B, n), dtype=torch.int32, device=dev)
    accept_token = torch.empty((B, n + 1), dtype=torch.int32, device=dev)
    _check(lib().ot_verify_greedy(C.byref(p), target_logits.data_ptr(), tree.token.data_ptr(), tree.parent.data_ptr(),
                                  tree.n_out.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                  accept_len.data_ptr(), accept_node.data_ptr(), accept_token.data_ptr(), _stream()),
           "ot_verify_greedy")
    return accept_len, accept_node, accept_token


def verify_sample(target_logits, u, temperature, tree: "Tree", workspace=None):
    """ot_verify_sample on the current stream.  target_logits [B, n + 1, V]; u float32 [B, n + 1] uniform
    numbers in [0, 1), one per target row; returns (accept_len, accept_node, accept_token) as in
    verify_greedy."""
    import torch
    if target_logits.dim() != 3 or target_logits.stride(2) != 1:
        raise ValueError("target_logits must be [B, n + 1, V] with a contiguous last dimension")
    B, rows, V = target_logits.shape
    n = rows - 1
    if u.dtype != torch.float32 or tuple(u.shape) != (B, rows) or not u.is_contiguous():
        raise ValueError("u must be a contiguous float32 tensor [B, n + 1]")
    p = VerifyParams(B, V, n, _dtype_code(target_logits), target_logits.stride(0), target_logits.stride(1))
    need = int(lib().ot_verify_sample_workspace_bytes(C.byref(p)))
    if need == 0:
        raise OptTreeError(-2, "ot_verify_sample_workspace_bytes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=target_logits.device)
    dev = target_logits.device
    accept_len = torch.empty(B, dtype=torch.int32, device=dev)
    accept_node = torch.empty((B, n), dtype=torch.int32, device=dev)
    accept_token = torch.empty((B, n + 1), dtype=torch.int32, device=dev)
    _check(lib().ot_verify_sample(C.byref(p), C.c_float(temperature), target_logits.data_ptr(), u.data_ptr(),
                                  tree.token.data_ptr(), tree.parent.data_ptr(), tree.n_out.data_ptr(),
                                  workspace.data_ptr(), workspace.numel(), accept_len.data_ptr(),
                                  accept_node.data_ptr(), accept_token.data_ptr(), _stream()), "ot_verify_sample")
    return accept_len, accept_node, accept_token


def kv_append(K_prefix, V_prefix, K_tree, V_tree, prefix_len, accept_len, accept_node):
    """ot_kv_append on the current stream: the accepted nodes' K/V rows are appended to the prefix cache in
    place; returns the new prefix lengths (int32 [B])."""
    import torch
    B, Hkv, n, D = K_tree.shape
    p = attn_params(K_tree, K_prefix, V_prefix, K_tree, V_tree)
    new_len = torch.empty(B, dtype=torch.int32, device=K_tree.device)
    _check(lib().ot_kv_append(C.byref(p), K_prefix.data_ptr(), V_prefix.data_ptr(), K_tree.data_ptr(),
                              V_tree.data_ptr(), prefix_len.data_ptr(), accept_len.data_ptr(),
                              accept_node.data_ptr(), new_len.data_ptr(), _stream()), "ot_kv_append")
    return new_len


# ---------------------------------------------------------------------------
# Prepared calls: everything marshalled once, so that a hot loop (or a HIP graph capture) pays one
# foreign call per library call.  Used by bench.py.
# ---------------------------------------------------------------------------
class PreparedBuild:
    def __init__(self, logits, k: int, n: int, depth: int):
        import torch
        self.logits = logits
        self.p = build_params(logits, k, n, depth)
        need = build_workspace_bytes(self.p)
        if need == 0:
            raise OptTreeError(-2, "ot_build_workspace_bytes")
        self.ws = torch.empty(need, dtype=torch.uint8, device=logits.device)
        self.out = alloc_tree(self.p.batch, n, logits.device)
        self.o = self.out.c_struct()
        self._args = (C.byref(self.p), logits.data_ptr(), self.ws.data_ptr(), self.ws.numel(), C.byref(self.o))

    def __call__(self, stream: int):
        st = lib().ot_build_tree(*self._args, stream)
        if st:
            raise OptTreeError(st, "ot_build_tree")

    def timed(self, stream: int, ev0, ev1):
        st = lib().ot_build_tree_timed(*self._args, stream, ev0, ev1)
        if st:
            raise OptTreeError(st, "ot_build_tree_timed")


class PreparedAttention:
    def __init__(self, Q, K_prefix, V_prefix, K_tree, V_tree, prefix_len, mask, softmax_scale: float = 0.0):
        import torch
        self.keep = (Q, K_prefix, V_prefix, K_tree, V_tree, prefix_len, mask)
        self.p = attn_params(Q, K_prefix, V_prefix, K_tree, V_tree, softmax_scale=softmax_scale)
        self.out = torch.empty_like(Q)
        self.ws = attn_workspace(self.p, Q.device)
        ptr = lambda t: None if t is None else t.data_ptr()
        self._args = (C.byref(self.p), ptr(Q), ptr(K_prefix), ptr(V_prefix), ptr(K_tree), ptr(V_tree),
                      ptr(prefix_len), ptr(mask), ptr(self.out), self.ws.data_ptr(), self.ws.numel())

    def __call__(self, stream: int):
        st = lib().ot_tree_verify_attention(*self._args, stream)
        if st:
            raise OptTreeError(st, "ot_tree_verify_attention")

    def timed(self, stream: int, ev0, ev1):
        st = lib().ot_tree_verify_attention_timed(*self._args, stream, ev0, ev1)
        if st:
            raise OptTreeError(st, "ot_tree_verify_attention_timed")
