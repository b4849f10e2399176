"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle.

This module holds data plumbing only -- shapes, random draws, dtype rounding --
and none of the method's arithmetic.  The paper (arxiv 2406.17276) evaluates on
MT-Bench / GSM8K with trained draft and target models; neither is available, so
the draft model's per-node logits rows and the target model's Q/K/V are drawn
at random with the geometry of the models the paper uses (Sec. 4.1: LLaMA-2
7B/13B/70B, node budgets 25-60) plus one larger-budget shape (Sec. 4.3,
tree-size scaling).

Every logits row is drawn from its own Philox stream keyed by
(seed, sequence, depth, slot); bf16 tensors are carried on the host as uint16
bit patterns (NumPy has no bf16) and are rounded to nearest-even exactly once.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


# --------------------------------------------------------------------------
# dtype plumbing
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def e4m3_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of FP8 E4M3 bytes (the OCP 8-bit format: 1 sign, 4 exponent bits with bias 7, 3 mantissa bits,
    no infinities, S.1111.111 = NaN, largest finite value 448) to float32."""
    b = np.asarray(b, dtype=np.uint8).astype(np.int32)
    sign = np.where(b & 0x80, -1.0, 1.0)
    e, m = (b >> 3) & 15, b & 7
    mag = np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))
    mag = np.where((e == 15) & (m == 7), np.nan, mag)
    return (sign * mag).astype(np.float32)


def f32_to_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to FP8 E4M3 (nearest, ties to even; magnitudes beyond 448 saturate to 448): the byte whose
    decoded value is nearest, found by search in the sorted table of the 127 non-negative finite codes."""
    x = np.asarray(x, dtype=np.float32).astype(np.float64)
    table = e4m3_bits_to_f32(np.arange(0x7F, dtype=np.uint8)).astype(np.float64)      # codes 0..0x7e, increasing
    a = np.minimum(np.abs(x), 448.0)
    hi = np.clip(np.searchsorted(table, a, side="left"), 1, 0x7E)
    lo = hi - 1
    dlo, dhi = a - table[lo], table[hi] - a
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (hi % 2 == 0))                             # tie: the even code
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    return np.where(np.signbit(x), code | 0x80, code).astype(np.uint8)


def to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 view of a stored tensor ('f32' array, 'bf16' bit patterns or 'e4m3' bytes)."""
    if dtype == "bf16":
        return bf16_bits_to_f32(a).astype(np.float64)
    if dtype == "e4m3":
        return e4m3_bits_to_f32(a).astype(np.float64)
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def store(x32: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float32 array to the stored dtype (bf16 -> uint16 bits, e4m3 -> bytes)."""
    if dtype == "bf16":
        return f32_to_bf16_bits(x32)
    if dtype == "e4m3":
        return f32_to_e4m3_bits(x32)
    return np.ascontiguousarray(x32, dtype=np.float32)


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    vocab: int
    depth: int
    k: int
    n: int
    dtype: str               # "f32" | "bf16"  (logits and attention tensors)
    logit_kind: str          # "normal" | "peak" | "zipf"
    logit_scale: float
    q_heads: int
    kv_heads: int
    head_dim: int
    prefix: int              # nominal prefix length
    ragged: float = 0.0      # +- fraction of seeded raggedness of prefix lengths
    peak: float = 6.0
    extra: dict = field(default_factory=dict)

    def frontier(self):
        F = [1]
        for _ in range(self.depth):
            F.append(min(self.n, self.k * F[-1]))
        return F

    def rows_per_seq(self):
        return sum(self.frontier()[: self.depth])

    def max_prefix(self):
        return int(round(self.prefix * (1.0 + self.ragged)))

    def elem_bytes(self):
        return 2 if self.dtype == "bf16" else 4


WORKLOADS = {
    "tiny": Workload("tiny", 1, 1000, 4, 4, 16, "f32", "normal", 3.0, 4, 4, 64, 128),
    "7b": Workload("7b", 1, 32000, 10, 10, 50, "bf16", "peak", 4.0, 32, 32, 128, 1024),
    "13b": Workload("13b", 1, 32000, 12, 10, 64, "bf16", "zipf", 1.0, 40, 40, 128, 2048),
    "70b": Workload("70b", 16, 32000, 10, 8, 60, "bf16", "normal", 4.0, 64, 8, 128, 4096, ragged=0.25),
    "large": Workload("large", 32, 128256, 20, 16, 256, "bf16", "peak", 5.0, 32, 8, 128, 8192),
}


def _rng(seed: int, *key: int) -> np.random.Generator:
    k = 0
    for v in key:
        k = (k << 20) | (int(v) & 0xFFFFF)
    return np.random.Generator(np.random.Philox(key=[int(seed) & (2**64 - 1), k & (2**64 - 1)]))


def logits_row(w: Workload, seed: int, seq: int, depth: int, slot: int) -> np.ndarray:
    """One float32 logits row (before rounding to the stored dtype)."""
    g = _rng(seed, 1, seq, depth, slot)
    z = g.standard_normal(w.vocab, dtype=np.float32)
    if w.logit_kind == "normal":
        return z * np.float32(w.logit_scale)
    if w.logit_kind == "peak":
        x = z * np.float32(w.logit_scale)
        x[int(g.integers(0, w.vocab))] += np.float32(w.peak)
        return x
    if w.logit_kind == "zipf":
        rank = g.permutation(w.vocab).astype(np.float32) + np.float32(1.0)
        return (np.float32(-1.1) * np.log(rank) + np.float32(0.5) * z).astype(np.float32)
    raise ValueError(w.logit_kind)


def make_logits(w: Workload, seed: int, seqs=None) -> np.ndarray:
    """Stored logits [B, depth, n, vocab]; rows beyond the frontier size of a depth stay zero."""
    seqs = list(range(w.batch)) if seqs is None else list(seqs)
    F = w.frontier()
    np_dtype = np.uint16 if w.dtype == "bf16" else np.float32
    out = np.zeros((len(seqs), w.depth, w.n, w.vocab), dtype=np_dtype)
    for bi, b in enumerate(seqs):
        for t in range(w.depth):
            for j in range(F[t]):
                out[bi, t, j] = store(logits_row(w, seed, b, t, j), w.dtype)
    return out


def prefix_lengths(w: Workload, seed: int) -> np.ndarray:
    if w.ragged == 0.0:
        return np.full(w.batch, w.prefix, dtype=np.int32)
    u = _rng(seed, 2).uniform(-w.ragged, w.ragged, size=w.batch)
    return np.round(w.prefix * (1.0 + u)).astype(np.int32)


def make_attention_inputs(w: Workload, seed: int, seqs=None, n=None):
    """Q [B,Hq,n,D], prefix K/V [B,Hkv,Lmax,D], tree K/V [B,Hkv,n,D] in the stored dtype, prefix_len [B]."""
    seqs = list(range(w.batch)) if seqs is None else list(seqs)
    n = w.n if n is None else n
    plen = prefix_lengths(w, seed)[seqs]
    Lmax = max(1, w.max_prefix())
    B = len(seqs)

    def draw(tag, b, shape):
        return store(_rng(seed, 3, tag, b).standard_normal(shape, dtype=np.float32), w.dtype)

    Q = np.stack([draw(0, b, (w.q_heads, n, w.head_dim)) for b in seqs])
    Kp = np.stack([draw(1, b, (w.kv_heads, Lmax, w.head_dim)) for b in seqs])
    Vp = np.stack([draw(2, b, (w.kv_heads, Lmax, w.head_dim)) for b in seqs])
    Kt = np.stack([draw(3, b, (w.kv_heads, n, w.head_dim)) for b in seqs])
    Vt = np.stack([draw(4, b, (w.kv_heads, n, w.head_dim)) for b in seqs])
    assert Q.shape[0] == B
    return dict(Q=Q, K_prefix=Kp, V_prefix=Vp, K_tree=Kt, V_tree=Vt, prefix_len=plen.astype(np.int32))


def quantise_cache_e4m3(prefix_stored: np.ndarray, tree_stored: np.ndarray, dtype: str):
    """The caller-side step that writes an 8-bit cache: one scale per (sequence, KV head) = largest magnitude over
    prefix and tree rows / 448 (the format's largest value), values divided by it and rounded to E4M3 bytes.
    Inputs [B,Hkv,rows,D] in the stored dtype; returns (prefix bytes, tree bytes, float32 scales [B,Hkv])."""
    pre = to_f64(prefix_stored, dtype).astype(np.float32)
    tre = to_f64(tree_stored, dtype).astype(np.float32)
    amax = np.maximum(np.abs(pre).max(axis=(2, 3)), np.abs(tre).max(axis=(2, 3)))
    scale = (np.maximum(amax, 1e-12) / np.float32(448.0)).astype(np.float32)
    s = scale[:, :, None, None]
    return f32_to_e4m3_bits(pre / s), f32_to_e4m3_bits(tre / s), scale


def random_tree_parents(n: int, seed: int, shape: str = "random") -> np.ndarray:
    """A random forest over n nodes in parents-first order: parent[i] in [-1, i) (-1 = child of the root)."""
    g = _rng(seed, 4, n)
    parent = np.full(n, -1, dtype=np.int64)
    for i in range(n):
        if shape == "chain":
            parent[i] = i - 1
        elif shape == "star":
            parent[i] = -1
        else:
            parent[i] = int(g.integers(-1, i)) if i > 0 else -1
    return parent
