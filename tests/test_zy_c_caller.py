"""The library driven from plain C (tests/abi_client.c: gcc, include/opttree.h and the HIP runtime; no PyTorch, no
Python in the process): one decoding step's tree build and tree attention, compared with the oracle (needs an
MI355X).  The program is compiled by the package's build step (a third of a second of gcc; compiled here if it
is not there).  Collected late on purpose: it starts another process on the GPU."""
import os
import subprocess

import numpy as np
import pytest

from oracle import tree_attention as ta_oracle
import workloads as wl
from tests import _util as U

pytestmark = pytest.mark.gpu
EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "abi_client")


@pytest.mark.parametrize("dtype,V,k,n,d,Hq,Hkv,D,Lmax", [("bf16", 4000, 6, 40, 5, 8, 2, 128, 300),
                                                        ("f32", 700, 4, 20, 4, 2, 2, 64, 90)])
def test_plain_c_caller_matches_oracle(tmp_path, dtype, V, k, n, d, Hq, Hkv, D, Lmax):
    if not os.path.exists(EXE):
        from paper_2406_17276_amd import build
        build.build_abi_client()
    B = 2
    g = np.random.default_rng(V + n)
    for _ in range(8):
        logits = wl.store((g.standard_normal((B, d, n, V)) * 3.0).astype(np.float32), dtype)
        trees = U.oracle_trees(logits, dtype, k, n, d)
        if min(t["min_gap"] for t in trees) > U.GAP:
            break
    else:
        raise RuntimeError("no draft logits with the required score gap")
    draw = lambda *shape: wl.store(g.standard_normal(shape).astype(np.float32), dtype)
    Q, Kp, Vp = draw(B, Hq, n, D), draw(B, Hkv, Lmax, D), draw(B, Hkv, Lmax, D)
    Kt, Vt = draw(B, Hkv, n, D), draw(B, Hkv, n, D)
    plen = np.array([Lmax - 17, Lmax // 2], dtype=np.int32)
    fin, fout = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(fin, "wb") as f:
        f.write(np.array([B, V, d, k, n, 1 if dtype == "bf16" else 0, Hq, Hkv, D, Lmax], dtype=np.int32).tobytes())
        for a in (plen, logits, Q, Kp, Vp, Kt, Vt):
            f.write(np.ascontiguousarray(a).tobytes())
    r = subprocess.run([EXE, str(fin), str(fout)], capture_output=True, text=True, timeout=100)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0

    W = (n + 63) // 64
    raw = open(fout, "rb").read()
    off = 0
    def take(np_dtype, *shape):
        nonlocal off
        cnt = int(np.prod(shape))
        a = np.frombuffer(raw, dtype=np_dtype, count=cnt, offset=off).reshape(shape)
        off += cnt * np.dtype(np_dtype).itemsize
        return a
    tok, par, dep = take(np.int32, B, n), take(np.int32, B, n), take(np.int32, B, n)
    score, mask = take(np.float32, B, n), take(np.uint64, B, n, W)
    n_out, expect = take(np.int32, B), take(np.float64, B)
    O = take(np.uint16 if dtype == "bf16" else np.float32, B, Hq, n, D)
    assert off == len(raw)
    for b, want in enumerate(trees):
        assert n_out[b] == want["n_out"]
        np.testing.assert_array_equal(tok[b], want["token"])
        np.testing.assert_array_equal(par[b], want["parent"])
        np.testing.assert_array_equal(dep[b], want["depth"])
        np.testing.assert_array_equal(mask[b], want["mask"].reshape(n, W))
        m = want["n_out"]
        np.testing.assert_allclose(score[b, :m], want["score"][:m], rtol=0, atol=1e-5)
        np.testing.assert_allclose(expect[b], want["expect"], rtol=1e-6)
    want_O = ta_oracle.tree_verify_attention(wl.to_f64(Q, dtype), wl.to_f64(Kp, dtype), wl.to_f64(Vp, dtype),
                                             wl.to_f64(Kt, dtype), wl.to_f64(Vt, dtype), plen,
                                             np.stack([t["mask"] for t in trees]), None)
    assert np.abs(wl.to_f64(O, dtype) - want_O).max() < (2e-2 if dtype == "bf16" else 1e-5)
