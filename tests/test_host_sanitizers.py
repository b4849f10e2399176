"""The library's host code under AddressSanitizer + UndefinedBehaviorSanitizer, without a GPU.

Builds the HIP sources once more with the sanitizers on the host side only (device code is compiled but never runs
here) and runs tests/host_sanitize.c against it: ~75 000 calls that cover argument validation, workspace sizing and
carving, the attention launch plan and the frontier tables over grids of shapes.  Every call must return the expected
status before anything is launched, and neither sanitizer may report."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
from paper_2406_17276_amd import build as B  # noqa: E402

SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]


@pytest.mark.timeout(900)
def test_host_paths_are_clean_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clang = os.path.join(os.environ.get("ROCM_PATH", "/opt/rocm"), "lib", "llvm", "bin", "clang")
    if not (os.path.exists(hipcc) and os.path.exists(clang)):
        pytest.skip("no ROCm compiler")
    procs, objs = [], []
    for src in B.SOURCES:
        obj = str(tmp_path / src.replace(".hip", ".o"))
        objs.append(obj)
        # device code is not what is tested: unoptimised where the source allows it (the attention kernel's inline
        # assembly needs the optimiser to prove its scalar operands uniform)
        dev = [] if src == "tree_attn.hip" else ["-Xarch_device", "-O0"]
        flags = [f for f in B.FLAGS if f != "-O3"] + ["-O1", "-Xarch_device", "-O3"] + dev + SAN
        procs.append(subprocess.Popen([hipcc] + flags + B.EXTRA_FLAGS.get(src, []) + ["-c", os.path.join(B.CSRC, src), "-o", obj],
                                      stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))
    for pr in procs:
        out, _ = pr.communicate()
        assert pr.returncode == 0, out[-3000:]
    lib = str(tmp_path / "libopttree_san.so")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address,undefined", "-o", lib] + objs, check=True)
    exe = str(tmp_path / "host_sanitize")
    rocm_lib = os.path.join(os.environ.get("ROCM_PATH", "/opt/rocm"), "lib")
    subprocess.run([clang, "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer",
                    "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "host_sanitize.c"),
                    "-o", exe, "-L" + str(tmp_path), "-lopttree_san", "-L" + rocm_lib, "-lamdhip64",
                    "-Wl,-rpath," + str(tmp_path), "-Wl,-rpath," + rocm_lib], check=True)
    env = dict(os.environ)
    # (the link-order check is about preloaded libraries of the environment, not about this program)
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    out = run.stdout
    assert "runtime error" not in out, out[-4000:]
    assert "AddressSanitizer" not in out, out[-4000:]
    assert run.returncode == 0 and out.strip().splitlines()[-1].startswith("ok "), out[-4000:]
    shutil.rmtree(tmp_path, ignore_errors=True)
