"""fp64 / exact oracle for the verification of a draft tree (greedy and random sampling).  TEST INFRASTRUCTURE ONLY.

Preliminaries, "Speculative Decoding", and Algorithm 2 of the paper (arxiv 2406.17276): with greedy
sampling the ground truth at a position is the target model's most probable token there; among the
branches of the draft tree that start at the root, the longest one that agrees with the ground truth is
accepted, and the target's token after the last accepted node comes for free, so A tokens are produced
where A - 1 is the number of accepted draft nodes.  The accepted nodes' K/V rows then join the cache.

Plain Python loops and NumPy indexing only; the most probable token of a row is numpy.argmax (first
maximum = smallest token id among equal logits, the same tie rule as in the tree builder).

Random sampling (Sec. 4, "Performance on Non-greedy Settings"): the paper states only that the acceptable
tokens change and gives no rule.  The reading taken here: the ground truth at a position is a token DRAWN
from the target's distribution softmax(logits / temperature) there, and everything else (longest agreeing
root branch, the free token, the cache append) stays as in the greedy case.  The draw is the inverse CDF
in token-id order of a uniform number u in [0, 1) that the caller supplies per position, so the function is
deterministic; since every produced token is an exact draw from the target's distribution at its position,
the output is distributed as plain sampling from the target, whatever the tree.
"""
from __future__ import annotations

import numpy as np


def greedy_verify(target_logits: np.ndarray, token: np.ndarray, parent: np.ndarray, n_out: int):
    """target_logits[0] is the target's row at the root position (the last token of the input), row 1 + i
    its row at tree node i.  token / parent as produced by the tree builder (parent -1 = child of the
    root).  Returns (A, accepted node indices [A - 1], produced tokens [A])."""
    n_out = int(n_out)
    cur = -1                                    # the root
    nodes, produced = [], []
    while True:
        g = int(np.argmax(target_logits[cur + 1]))      # ground truth after `cur`
        produced.append(g)
        nxt = [i for i in range(n_out) if int(parent[i]) == cur and int(token[i]) == g]
        if not nxt:
            break                               # no branch continues with the ground truth
        if len(nxt) != 1:
            raise AssertionError("two children of one node carry the same token")
        cur = nxt[0]
        nodes.append(cur)
    return len(produced), nodes, produced


def sample_truth(row: np.ndarray, temperature: float, u: float) -> int:
    """Inverse-CDF draw from softmax(row / temperature): the smallest token v whose cumulative probability
    q_0 + ... + q_v exceeds u.  -inf logits have probability 0 and are never drawn."""
    if not temperature > 0:
        raise ValueError("temperature must be positive")
    z = np.asarray(row, dtype=np.float64) / float(temperature)
    e = np.exp(z - z.max())                     # unnormalised probabilities, the largest is 1
    c = np.cumsum(e)
    target = float(u) * c[-1]
    for v in range(len(c)):
        if c[v] > target:
            return v
    return int(np.nonzero(e > 0)[0][-1])        # only reachable through rounding when u is next to 1


def sample_margin(row: np.ndarray, temperature: float, u: float) -> float:
    """Distance from u to the nearest boundary of the inverse CDF of softmax(row / temperature) (boundaries
    at 0 and 1 excluded): a draw with a margin above an implementation's rounding error is the same token in
    every correct implementation."""
    z = np.asarray(row, dtype=np.float64) / float(temperature)
    e = np.exp(z - z.max())
    cdf = np.cumsum(e)[:-1] / e.sum()
    return float(np.abs(cdf - float(u)).min()) if len(cdf) else 1.0


def sampled_verify(target_logits: np.ndarray, temperature: float, u: np.ndarray, token: np.ndarray,
                   parent: np.ndarray, n_out: int):
    """greedy_verify with the ground truth after position `cur` drawn by sample_truth(target_logits[cur + 1],
    temperature, u[cur + 1]).  Returns (A, accepted node indices [A - 1], produced tokens [A])."""
    n_out = int(n_out)
    cur = -1
    nodes, produced = [], []
    while True:
        g = sample_truth(target_logits[cur + 1], temperature, u[cur + 1])
        produced.append(g)
        nxt = [i for i in range(n_out) if int(parent[i]) == cur and int(token[i]) == g]
        if not nxt:
            break
        if len(nxt) != 1:
            raise AssertionError("two children of one node carry the same token")
        cur = nxt[0]
        nodes.append(cur)
    return len(produced), nodes, produced


def kv_append(K_prefix, V_prefix, K_tree, V_tree, prefix_len, nodes):
    """Append the accepted nodes' K/V rows to the cache of one sequence (arrays [heads][rows][D]); rows that
    would not fit in the allocated prefix are dropped.  Returns the new prefix length."""
    L = int(prefix_len)
    cap = K_prefix.shape[1]
    for j, i in enumerate(nodes):
        if L + j >= cap:
            return cap
        K_prefix[:, L + j, :] = K_tree[:, i, :]
        V_prefix[:, L + j, :] = V_tree[:, i, :]
    return L + len(nodes)
