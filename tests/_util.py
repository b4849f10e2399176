"""Helpers shared by the GPU parity tests: host arrays <-> device tensors, oracle drivers."""
import numpy as np

from oracle import opt_tree as ot_oracle
import workloads as wl

GAP = 1e-5          # minimum cross-parent score gap (log p^) required of generated inputs


def to_device(a: np.ndarray, dtype: str):
    import torch
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def from_device_f64(t) -> np.ndarray:
    import torch
    return t.detach().to(torch.float64).cpu().numpy()


def mask_to_device(mask_u64: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(mask_u64).view(np.int64)).cuda()


def oracle_trees(logits_stored: np.ndarray, dtype: str, k: int, n: int, depth: int):
    """Run the fp64 oracle on every sequence of stored logits [B, depth, n, V]."""
    out = []
    for b in range(logits_stored.shape[0]):
        out.append(ot_oracle.build_tree(LazyF64(logits_stored[b], dtype), k, n, depth))
    return out


class LazyF64:
    """Indexable view that widens stored logits to float64 one step at a time (saves host memory)."""

    def __init__(self, stored, dtype):
        self.stored, self.dtype = stored, dtype

    def __getitem__(self, idx):
        return wl.to_f64(self.stored[idx], self.dtype)


def gapped_logits(w: wl.Workload, seed0: int = 0, seqs=None, max_tries: int = 8):
    """Logits of workload w whose every selection cut has a cross-parent gap > GAP (seed bumped until so)."""
    for seed in range(seed0, seed0 + max_tries):
        logits = wl.make_logits(w, seed, seqs)
        trees = oracle_trees(logits, w.dtype, w.k, w.n, w.depth)
        if min(t["min_gap"] for t in trees) > GAP:
            return seed, logits, trees
    raise RuntimeError("no seed with the required score gap")


def assert_tree_equal(got, want_list, n, score_atol=1e-5):
    """got: api.Tree on device; want_list: oracle dicts per sequence.  Structure must be bit-exact."""
    tok = got.token.cpu().numpy(); par = got.parent.cpu().numpy(); dep = got.depth.cpu().numpy()
    sc = got.score.cpu().numpy().astype(np.float64); msk = got.mask.cpu().numpy().view(np.uint64)
    nout = got.n_out.cpu().numpy(); ex = got.expect.cpu().numpy()
    for b, want in enumerate(want_list):
        assert nout[b] == want["n_out"], f"seq {b}: n_out"
        np.testing.assert_array_equal(tok[b], want["token"], err_msg=f"seq {b}: token")
        np.testing.assert_array_equal(par[b], want["parent"], err_msg=f"seq {b}: parent")
        np.testing.assert_array_equal(dep[b], want["depth"], err_msg=f"seq {b}: depth")
        np.testing.assert_array_equal(msk[b], want["mask"], err_msg=f"seq {b}: mask")
        m = want["n_out"]
        np.testing.assert_allclose(sc[b, :m], want["score"][:m], rtol=0, atol=score_atol, err_msg=f"seq {b}: score")
        assert np.all(np.isneginf(sc[b, m:]))
        np.testing.assert_allclose(ex[b], want["expect"], rtol=1e-6, err_msg=f"seq {b}: E")


def assert_tree_invariants(got, n, depth):
    """What holds for every tree of Algorithm 1 whatever the input (used where the oracle cannot follow, at full
    sizes): nodes in (depth, slot) order with parents first, depth = parent's + 1, p^ never grows along a branch
    (Thm. 3.1), siblings carry distinct tokens, mask = parent's mask + own bit, E = sum of p^ (Eq. 3)."""
    tok = got.token.cpu().numpy(); par = got.parent.cpu().numpy(); dep = got.depth.cpu().numpy()
    sc = got.score.cpu().numpy().astype(np.float64); nout = got.n_out.cpu().numpy(); ex = got.expect.cpu().numpy()
    msk = got.mask.cpu().numpy().view(np.uint64).reshape(tok.shape[0], n, -1)
    for b in range(tok.shape[0]):
        m = int(nout[b])
        assert 1 <= m <= n
        assert np.all(np.diff(dep[b, :m]) >= 0) and dep[b, 0] == 1 and dep[b, m - 1] <= depth
        seen = set()
        for i in range(m):
            p = int(par[b, i])
            assert -1 <= p < i, (b, i, p)
            assert dep[b, i] == (1 if p < 0 else dep[b, p] + 1)
            assert p < 0 or sc[b, i] <= sc[b, p] + 1e-6
            assert sc[b, i] <= 1e-6
            assert (p, int(tok[b, i])) not in seen, "two children of one node carry the same token"
            seen.add((p, int(tok[b, i])))
            want = np.zeros(msk.shape[2], dtype=np.uint64) if p < 0 else msk[b, p].copy()
            want[i // 64] |= np.uint64(1) << np.uint64(i % 64)
            np.testing.assert_array_equal(msk[b, i], want)
        assert np.all(par[b, m:] == -1) and np.all(tok[b, m:] == -1) and not msk[b, m:].any()
        np.testing.assert_allclose(ex[b], np.exp(sc[b, :m]).sum(), rtol=5e-6)      # score is stored as float32
