"""fp64 oracle for OPT-Tree draft-tree construction.  TEST INFRASTRUCTURE ONLY.

Follows Sec. 3 of the paper (arxiv 2406.17276) step by step, in log space:

  * a node's children are the k most probable next tokens of its own
    next-token distribution p_d = softmax(logits row)        (Sec. 3, text after Eq. 2)
  * a node's path probability p^ is the product of p_d over the node and its
    ancestors, the root excluded                              (Eq. 2 and the note on the root)
  * each drafting step keeps the n candidates with largest p^ among the
    children of the last layer                                (Algorithm 1, "topk")
  * after d steps the n nodes with largest p^ in the whole tree form T_opt;
    by Thm. 3.1 they are closed under "parent of"             (Algorithm 1, last line + proof)
  * E(A) = sum of p^ over the chosen nodes                    (Eq. 3)
  * nodes of one layer share one position index               (Fig. 1 caption)
  * the tree attention mask lets a node see itself and its ancestors (Algorithm 2)

Readings where the paper is silent (ties, slot order, k < n) are the ones
listed in the design notes; they are spelled out at the point of use below.

No blocking, fusion or reordering: one Python loop per frontier node, NumPy
only for the per-row reductions and the stable sort.
"""
from __future__ import annotations

import numpy as np

NEG_INF = float("-inf")


def row_logsumexp(x: np.ndarray) -> float:
    """log sum_v exp(x_v) of one logits row, i.e. the normaliser of p_d (softmax)."""
    x = np.asarray(x, dtype=np.float64)
    m = x.max()
    return float(m + np.log(np.exp(x - m).sum()))


def row_top_k(x: np.ndarray, k: int) -> np.ndarray:
    """Token ids of the k largest logits; equal logits -> smaller token id first.

    A stable ascending sort of -x keeps equal keys in index order, which is
    exactly that tie rule.
    """
    x = np.asarray(x, dtype=np.float64)
    order = np.argsort(-x, kind="stable")
    return order[:k].astype(np.int64)


class TreeBuilder:
    """Layer-by-layer construction (the loop of Algorithm 1 with a fixed depth).

    expand(rows) is one drafting step: rows[j] is the logits row the draft
    model produced for frontier slot j (layer 0 = the root alone).  It returns
    the next frontier as (tokens, parent_slots).  finalize() is the last line
    of Algorithm 1 plus the bookkeeping the verifier needs.
    """

    def __init__(self, k: int, n: int):
        if k < 1 or n < 1:
            raise ValueError("k and n must be positive")
        self.k = int(k)
        self.n = int(n)
        # log p^ of the current frontier; the root contributes nothing to any product
        self.frontier_score = np.zeros(1, dtype=np.float64)
        self.layers = []          # per layer: dict(token, parent_slot, score) arrays
        self.cut_gaps = []        # diagnostic: smallest cross-parent score gap at each cut
        self.row_lse = []         # diagnostic: lse of every scanned row, per layer
        self.row_topk = []        # diagnostic: top-k tokens of every scanned row, per layer

    # -- one drafting step -------------------------------------------------
    def expand(self, rows: np.ndarray):
        rows = np.asarray(rows, dtype=np.float64)
        F = self.frontier_score.shape[0]
        if rows.ndim != 2 or rows.shape[0] < F:
            raise ValueError("need one logits row per frontier slot")
        V = rows.shape[1]
        k = min(self.k, V)
        cand = []                 # (score, parent slot j, rank r, token)
        lses, tops = [], []
        for j in range(F):
            x = rows[j]
            lse = row_logsumexp(x)
            top = row_top_k(x, k)
            lses.append(lse)
            tops.append(top)
            for r in range(k):
                v = int(top[r])
                # Eq. 2 in log space: log p^(child) = log p^(parent) + log p_d(token)
                cand.append((float(self.frontier_score[j] + (x[v] - lse)), j, r, v))
        self.row_lse.append(np.array(lses))
        self.row_topk.append(np.array(tops))
        keep = min(self.n, len(cand))
        # largest p^ first; equal p^ -> smaller parent slot, then smaller rank
        ranked = sorted(range(len(cand)), key=lambda c: (-cand[c][0], cand[c][1], cand[c][2]))
        kept, dropped = ranked[:keep], ranked[keep:]
        self.cut_gaps.append(_cross_parent_gap(
            [(cand[c][0], cand[c][1]) for c in kept],
            [(cand[c][0], cand[c][1]) for c in dropped]))
        # slot order inside the new layer is structural: (parent slot, rank)
        kept_sorted = sorted(kept, key=lambda c: (cand[c][1], cand[c][2]))
        layer = dict(
            token=np.array([cand[c][3] for c in kept_sorted], dtype=np.int64),
            parent_slot=np.array([cand[c][1] for c in kept_sorted], dtype=np.int64),
            score=np.array([cand[c][0] for c in kept_sorted], dtype=np.float64),
        )
        self.layers.append(layer)
        self.frontier_score = layer["score"]
        return layer["token"].copy(), layer["parent_slot"].copy()

    # -- E_sub(T, n): the best E over root-containing n-node subtrees of the
    #    tree drafted so far = sum of the n largest p^ (Sec. 3, before Alg. 1)
    def e_sub(self) -> float:
        if not self.layers:
            return 0.0
        s = np.sort(np.concatenate([l["score"] for l in self.layers]))[::-1]
        return float(np.exp(s[: self.n]).sum())

    # -- last line of Algorithm 1 + mask / positions -----------------------
    def finalize(self):
        n = self.n
        pool = []                 # (score, depth, slot)
        for t, layer in enumerate(self.layers, start=1):
            for s in range(layer["score"].shape[0]):
                pool.append((float(layer["score"][s]), t, s))
        n_out = min(n, len(pool))
        # largest p^ first; equal p^ -> shallower node, then smaller slot
        ranked = sorted(pool, key=lambda e: (-e[0], e[1], e[2]))
        chosen = ranked[:n_out]
        rest = ranked[n_out:]
        final_gap = self._final_gap(chosen, rest)
        # output order: depth ascending, slot ascending => parents precede children
        chosen_sorted = sorted(chosen, key=lambda e: (e[1], e[2]))
        index_of = {(t, s): i for i, (_, t, s) in enumerate(chosen_sorted)}
        W = (n + 63) // 64
        token = np.full(n, -1, dtype=np.int64)
        parent = np.full(n, -1, dtype=np.int64)
        depth = np.zeros(n, dtype=np.int64)
        score = np.full(n, NEG_INF, dtype=np.float64)
        mask = np.zeros((n, W), dtype=np.uint64)
        for i, (sc, t, s) in enumerate(chosen_sorted):
            layer = self.layers[t - 1]
            token[i] = layer["token"][s]
            depth[i] = t          # position id = position of the root + depth
            score[i] = sc
            if t == 1:
                parent[i] = -1    # child of the root
            else:
                key = (t - 1, int(layer["parent_slot"][s]))
                if key not in index_of:
                    raise AssertionError("selected node whose parent is not selected (Thm. 3.1 violated)")
                parent[i] = index_of[key]
                mask[i] = mask[parent[i]]
            mask[i, i // 64] |= np.uint64(1) << np.uint64(i % 64)
        expect = float(np.exp(score[:n_out]).sum())       # Eq. 3
        return dict(token=token, parent=parent, depth=depth, score=score, mask=mask,
                    n_out=n_out, expect=expect,
                    min_gap=min([final_gap] + self.cut_gaps) if self.cut_gaps else final_gap)

    def _final_gap(self, chosen, rest) -> float:
        """Diagnostic only: smallest score difference between a chosen and a
        rejected node that are neither siblings nor ancestor/descendant."""
        if not chosen or not rest:
            return float("inf")

        def chain(t, s):
            out = []
            while t >= 1:
                out.append((t, s))
                s = int(self.layers[t - 1]["parent_slot"][s])
                t -= 1
            return out

        best = float("inf")
        lo = sorted(chosen, key=lambda e: e[0])[:32]
        hi = sorted(rest, key=lambda e: -e[0])[:32]
        for (sa, ta, a) in lo:
            ca = chain(ta, a)
            for (sb, tb, b) in hi:
                cb = chain(tb, b)
                if (ta, a) in cb or (tb, b) in ca:
                    continue      # ancestor/descendant: ordered by construction
                if ta == tb and len(ca) > 1 and len(cb) > 1 and ca[1] == cb[1]:
                    continue      # siblings: ordered by their raw logits
                if ta == tb == 1:
                    continue      # both children of the root: siblings
                best = min(best, sa - sb)
        return best


def _cross_parent_gap(kept, dropped) -> float:
    """Diagnostic only: min over (kept a, dropped b) with different parents of score(a)-score(b)."""
    if not kept or not dropped:
        return float("inf")
    ks = np.array([s for s, _ in kept]); kp = np.array([p for _, p in kept])
    ds = np.array([s for s, _ in dropped]); dp = np.array([p for _, p in dropped])
    diff = ks[:, None] - ds[None, :]
    diff = np.where(kp[:, None] != dp[None, :], diff, np.inf)
    return float(diff.min())


def ancestor_mask(parent: np.ndarray) -> np.ndarray:
    """Tree attention mask of Algorithm 2 from parent indices given parents-first:
    bit j of row i is set iff j is i or an ancestor of i (the root, -1, is not a tree row)."""
    parent = np.asarray(parent, dtype=np.int64)
    n = parent.shape[0]
    W = (n + 63) // 64
    mask = np.zeros((n, W), dtype=np.uint64)
    for i in range(n):
        p = int(parent[i])
        if p >= i:
            raise ValueError("parents must precede children")
        if p >= 0:
            mask[i] = mask[p]
        mask[i, i // 64] |= np.uint64(1) << np.uint64(i % 64)
    return mask


def frontier_sizes(k: int, n: int, depth: int):
    """F_0 = 1 (the root), F_t = min(n, k * F_{t-1}): rows scanned at drafting step t."""
    F = [1]
    for _ in range(depth):
        F.append(min(n, k * F[-1]))
    return F


def build_tree(logits: np.ndarray, k: int, n: int, depth: int):
    """One-shot form: logits[t, j, :] is the row for slot j of layer t (t = 0 is the root).

    Only the first F_t rows of depth t are read.  Returns finalize()'s dict plus
    the per-layer frontiers ('layers').
    """
    b = TreeBuilder(k, n)
    for t in range(depth):
        F = b.frontier_score.shape[0]
        b.expand(np.asarray(logits[t, :F, :], dtype=np.float64))
    out = b.finalize()
    out["layers"] = b.layers
    out["row_lse"] = b.row_lse
    out["row_topk"] = b.row_topk
    return out


def build_tree_adaptive(logits: np.ndarray, k: int, n: int, max_depth: int, delta: float):
    """Algorithm 1 with its stopping rule: after the first drafting step, another step is drafted while the
    depth is below max_depth and E_sub(T, n) - E > delta, with E <- E_sub(T, n) before the step (E starts
    at 0).  logits[t, j, :] as in build_tree.  Returns finalize()'s dict plus 'steps' (layers drafted) and
    'e_sub_trace' (E_sub after every step)."""
    b = TreeBuilder(k, n)
    E = 0.0
    b.expand(np.asarray(logits[0, :1, :], dtype=np.float64))
    trace = [b.e_sub()]
    while len(b.layers) < max_depth and b.e_sub() - E > delta:
        E = b.e_sub()
        F = b.frontier_score.shape[0]
        b.expand(np.asarray(logits[len(b.layers), :F, :], dtype=np.float64))
        trace.append(b.e_sub())
    out = b.finalize()
    out["layers"] = b.layers
    out["steps"] = len(b.layers)
    out["e_sub_trace"] = trace
    return out


def frontier_masks(layers, n: int, depth: int) -> np.ndarray:
    """Tree attention mask of the drafting phase (Algorithm 2's mask, for the draft model's forward of the next
    drafting step): row s belongs to the node in slot s of the last layer and has bit j set iff pool node j is
    that node or one of its ancestors.  Pool index of (layer made by step t, slot s) = t * n + s.
    Returns uint64 [n, ceil(depth * n / 64)]; rows past the frontier are zero."""
    W = (depth * n + 63) // 64
    out = np.zeros((n, W), dtype=np.uint64)
    last = len(layers) - 1
    for s in range(layers[last]["token"].shape[0]):
        t, slot = last, s
        while t >= 0:                       # walk up to the root
            j = t * n + slot
            out[s, j // 64] |= np.uint64(1) << np.uint64(j % 64)
            slot = int(layers[t]["parent_slot"][slot])
            t -= 1
    return out
