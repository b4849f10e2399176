"""Parity of ot_tree_verify_attention_fp8kv (K/V cache in FP8 E4M3 bytes, one scale per sequence and KV head) with
the fp64 oracle on the values those bytes stand for (needs an MI355X).  Bar: max-abs 2e-2 (bf16 Q, P and O), as for
the bf16 cache."""
import numpy as np
import pytest

from oracle import opt_tree as ot_oracle
from oracle import tree_attention as ta_oracle
import workloads as wl
from tests import _util as U

pytestmark = pytest.mark.gpu
TOL = 2e-2


def _masks(B, n, seed, shape="random"):
    return np.stack([ot_oracle.ancestor_mask(wl.random_tree_parents(n, seed + b, shape)) for b in range(B)])


def _inputs(B, Hq, Hkv, D, L, n, ragged, seed):
    w = wl.Workload("f8", B, 8, 1, 1, n, "bf16", "normal", 1.0, Hq, Hkv, D, L, ragged=ragged)
    x = wl.make_attention_inputs(w, seed)
    kp, kt, ks = wl.quantise_cache_e4m3(x["K_prefix"], x["K_tree"], "bf16")
    vp, vt, vs = wl.quantise_cache_e4m3(x["V_prefix"], x["V_tree"], "bf16")
    return dict(Q=x["Q"], K_prefix=kp, V_prefix=vp, K_tree=kt, V_tree=vt, k_scale=ks, v_scale=vs,
                prefix_len=x["prefix_len"])


def _gpu(x, mask, scale=0.0, views=None):
    import torch
    from paper_2406_17276_amd import api
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    kv = {k: dev(x[k]) for k in ("K_prefix", "V_prefix", "K_tree", "V_tree")}
    if views:
        kv = views(kv)
    out = api.tree_verify_attention_fp8kv(U.to_device(x["Q"], "bf16"), kv["K_prefix"], kv["V_prefix"], kv["K_tree"],
                                          kv["V_tree"], dev(x["k_scale"]), dev(x["v_scale"]),
                                          dev(x["prefix_len"].astype(np.int32)), U.mask_to_device(mask),
                                          softmax_scale=scale)
    torch.cuda.synchronize()
    return U.from_device_f64(out)


def _oracle(x, mask, scale=None, heads=None):
    q = wl.to_f64(x["Q"], "bf16")
    return ta_oracle.tree_verify_attention_fp8kv(q, x["K_prefix"], x["V_prefix"], x["K_tree"], x["V_tree"],
                                                 x["k_scale"], x["v_scale"], x["prefix_len"], mask,
                                                 wl.e4m3_bits_to_f32, scale)


@pytest.mark.parametrize("B,Hq,Hkv,D,L,n,ragged,shape", [
    (2, 4, 4, 64, 150, 20, 0.0, "random"),       # one query head per KV head, 64 wide
    (1, 8, 8, 128, 1000, 50, 0.0, "random"),     # 128 wide, several key splits
    (2, 16, 2, 128, 700, 60, 0.2, "random"),     # GQA 8:1, 480 packed rows: 128-row blocks, ragged prefixes
    (1, 8, 2, 64, 300, 40, 0.0, "chain"),        # GQA 4:1, 64 wide, a chain (every ancestor visible)
    (1, 8, 8, 64, 0, 33, 0.0, "star"),           # no prefix at all: tree keys only
    (3, 4, 2, 128, 65, 256, 0.5, "random"),      # the largest tree, short ragged prefixes (tree tiles dominate)
    (1, 2, 2, 128, 63, 1, 0.0, "random"),        # a single node
    (33, 16, 8, 128, 150, 40, 0.5, "random"),    # a batch that fills the chip: jobs taken longest first
])
def test_shapes_and_edges(B, Hq, Hkv, D, L, n, ragged, shape):
    x = _inputs(B, Hq, Hkv, D, L, n, ragged, 5)
    mask = _masks(B, n, 3, shape)
    got = _gpu(x, mask)
    want = _oracle(x, mask)
    assert np.abs(got - want).max() < TOL


def test_every_byte_code_and_uneven_scales():
    """Rows holding all 254 finite byte codes (both zeros, subnormals, +-448), scales far from 1 that differ between
    K and V and between heads, and an explicit softmax scale."""
    B, Hq, Hkv, D, L, n = 1, 4, 2, 128, 200, 24
    x = _inputs(B, Hq, Hkv, D, L, n, 0.0, 9)
    codes = np.arange(256, dtype=np.uint8)
    codes[0x7F], codes[0xFF] = 0x7E, 0xFE                      # the two NaN codes are not cache values
    for t in ("K_prefix", "V_prefix", "K_tree", "V_tree"):
        x[t][0, :, 3, :] = codes[:128]
        x[t][0, :, 4, :] = codes[128:]
        x[t][0, :, 5, :] = codes[::-1][:128]
    x["k_scale"] = np.array([[2.0 ** -9, 3.1e-3]], dtype=np.float32)
    x["v_scale"] = np.array([[0.75, 40.0]], dtype=np.float32)
    mask = _masks(B, n, 1)
    got = _gpu(x, mask, scale=0.05)
    want = _oracle(x, mask, scale=0.05)
    ref = np.abs(want).max(axis=(2, 3), keepdims=True)          # V of head group 1 is of order 40 * 448
    assert (np.abs(got - want) / np.maximum(ref, 1.0)).max() < TOL


def test_strided_cache_views():
    """K and V as the two halves of one [B,Hkv,rows,2,D] byte allocation: row stride 2*D bytes."""
    import torch
    B, Hq, Hkv, D, L, n = 2, 8, 4, 64, 130, 18
    x = _inputs(B, Hq, Hkv, D, L, n, 0.0, 2)

    def views(kv):
        pre = torch.stack([kv["K_prefix"], kv["V_prefix"]], dim=3)
        tre = torch.stack([kv["K_tree"], kv["V_tree"]], dim=3)
        return dict(K_prefix=pre[:, :, :, 0], V_prefix=pre[:, :, :, 1], K_tree=tre[:, :, :, 0], V_tree=tre[:, :, :, 1])

    mask = _masks(B, n, 8)
    assert np.abs(_gpu(x, mask, views=views) - _oracle(x, mask)).max() < TOL


def test_full_7b_and_a_70b_shaped_group():
    """The 7B verification shape whole (32 heads, prefix 1024, n = 50), and one sequence of the 70B shape (64 query
    heads on 8 KV heads, prefix near 4096, n = 60) checked on two KV groups."""
    w = wl.WORKLOADS["7b"]
    x = _inputs(1, w.q_heads, w.kv_heads, w.head_dim, w.prefix, w.n, 0.0, 4)
    mask = _masks(1, w.n, 2)
    assert np.abs(_gpu(x, mask) - _oracle(x, mask)).max() < TOL
    w = wl.WORKLOADS["70b"]
    x = _inputs(1, w.q_heads, w.kv_heads, w.head_dim, w.prefix, w.n, 0.0, 6)
    mask = _masks(1, w.n, 4)
    got = _gpu(x, mask)
    g = w.q_heads // w.kv_heads
    for kvh in (0, 5):
        qh = list(range(kvh * g, kvh * g + g))
        sub = dict(Q=x["Q"][:, qh], prefix_len=x["prefix_len"],
                   **{k: x[k][:, [kvh]] for k in ("K_prefix", "V_prefix", "K_tree", "V_tree", "k_scale", "v_scale")})
        assert np.abs(got[:, qh] - _oracle(sub, mask)).max() < TOL


def test_scales_of_one_on_bytes_that_hold_bf16_representable_values_match_the_bf16_cache_path():
    """Every E4M3 value is a bf16 value: with scales of 1 the 8-bit entry point must agree with the bf16 entry point
    fed the widened cache, to the bf16 output's rounding (the two differ only in where the scale is applied)."""
    import torch
    from paper_2406_17276_amd import api
    B, Hq, Hkv, D, L, n = 2, 8, 2, 128, 500, 30
    x = _inputs(B, Hq, Hkv, D, L, n, 0.1, 12)
    x["k_scale"][:] = 1.0
    x["v_scale"][:] = 1.0
    mask = _masks(B, n, 6)
    got8 = _gpu(x, mask)
    wide = {k: U.to_device(wl.f32_to_bf16_bits(wl.e4m3_bits_to_f32(x[k])), "bf16")
            for k in ("K_prefix", "V_prefix", "K_tree", "V_tree")}
    out = api.tree_verify_attention(U.to_device(x["Q"], "bf16"), wide["K_prefix"], wide["V_prefix"], wide["K_tree"],
                                    wide["V_tree"], torch.from_numpy(x["prefix_len"].astype(np.int32)).cuda(),
                                    U.mask_to_device(mask))
    torch.cuda.synchronize()
    got16 = U.from_device_f64(out)
    scale = np.maximum(np.abs(got16), 1.0)
    assert (np.abs(got8 - got16) / scale).max() < 2.0 ** -6
