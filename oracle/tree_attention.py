"""fp64 oracle for tree-masked verification attention.  TEST INFRASTRUCTURE ONLY.

Algorithm 2 of the paper (arxiv 2406.17276) feeds the n draft nodes to the
target model together with the attention mask that belongs to the tree: every
node attends to the whole cached prefix and, inside the tree, to itself and
its ancestors only (Sec. 1, tree-structured drafts; Sec. 3, Algorithm 2).
The paper gives no formula for attention itself; this is ordinary scaled
dot-product attention written out key by key:

    O[b,h,i,:] = sum_j w_ij V[b,h//g,j,:],
    w_i. = softmax_j( scale * Q[b,h,i,:] . K[b,h//g,j,:] )   over visible j

with visible j = {prefix rows 0..L_b-1} U {tree rows j : bit j of mask[b,i]},
g = q_heads / kv_heads (grouped-query attention: query head h reads KV head
h // g), scale = 1/sqrt(head_dim) unless given.
"""
from __future__ import annotations

import numpy as np


def mask_bit(mask_row: np.ndarray, j: int) -> bool:
    return bool((int(mask_row[j // 64]) >> (j % 64)) & 1)


def tree_verify_attention(Q, K_prefix, V_prefix, K_tree, V_tree, prefix_len, mask, scale=None):
    """Q [B,Hq,n,D]; K/V_prefix [B,Hkv,Lmax,D]; K/V_tree [B,Hkv,nk,D];
    prefix_len [B]; mask [B,n,ceil(nk/64)] uint64.  Returns O [B,Hq,n,D] float64.
    nk = n when the target verifies the tree; nk > n in the drafting phase, where the n tokens fed to the
    draft model attend to the K/V cache of everything drafted so far (Sec. 4, last paragraph)."""
    Q = np.asarray(Q, dtype=np.float64)
    K_prefix = np.asarray(K_prefix, dtype=np.float64)
    V_prefix = np.asarray(V_prefix, dtype=np.float64)
    K_tree = np.asarray(K_tree, dtype=np.float64)
    V_tree = np.asarray(V_tree, dtype=np.float64)
    B, Hq, n, D = Q.shape
    nk = K_tree.shape[2]
    Hkv = K_tree.shape[1]
    if Hq % Hkv:
        raise ValueError("q_heads must be a multiple of kv_heads")
    g = Hq // Hkv
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    O = np.zeros((B, Hq, n, D), dtype=np.float64)
    for b in range(B):
        L = int(prefix_len[b])
        for h in range(Hq):
            hk = h // g
            K = np.concatenate([K_prefix[b, hk, :L], K_tree[b, hk]], axis=0)   # [L+n, D]
            V = np.concatenate([V_prefix[b, hk, :L], V_tree[b, hk]], axis=0)
            logits = scale * (Q[b, h] @ K.T)                                   # [n, L+nk]
            for i in range(n):
                visible = np.ones(L + nk, dtype=bool)
                for j in range(nk):
                    visible[L + j] = mask_bit(mask[b, i], j)
                if not visible.any():
                    continue          # a node with no visible key (empty mask row, no prefix)
                s = np.where(visible, logits[i], -np.inf)
                w = np.exp(s - s[visible].max())
                w = np.where(visible, w, 0.0)
                O[b, h, i] = (w / w.sum()) @ V
    return O


def tree_verify_attention_fp8kv(Q, K8_prefix, V8_prefix, K8_tree, V8_tree, k_scale, v_scale, prefix_len, mask,
                                decode, scale=None):
    """The same attention over a K/V cache kept in 8 bits.  The paper states no precision for the cache; the reading
    built here: K and V (prefix and tree rows alike) are stored as FP8 E4M3 bytes with one real scale factor per
    (sequence, KV head) for K and one for V, the value a byte stands for being  scale * decode(byte);  Q and O keep
    their 16-bit type.  What is computed is the attention of the function above on exactly those values -- the
    rounding happened when the cache was written and is not part of this step.
    K8_* / V8_* uint8 [B,Hkv,rows,D]; k_scale, v_scale [B,Hkv]; decode: bytes -> real values (exact widening)."""
    ks = np.asarray(k_scale, dtype=np.float64)[:, :, None, None]
    vs = np.asarray(v_scale, dtype=np.float64)[:, :, None, None]
    wide = lambda a: np.asarray(decode(a), dtype=np.float64)
    return tree_verify_attention(Q, ks * wide(K8_prefix), vs * wide(V8_prefix), ks * wide(K8_tree), vs * wide(V8_tree),
                                 prefix_len, mask, scale)
