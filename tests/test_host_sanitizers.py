"""The host side of the C ABI (argument and state checks, workspace layout, the partitioner) under
AddressSanitizer and UndefinedBehaviorSanitizer.  lp_api.cpp and partition.cpp are compiled a second time with
the sanitizers on their host code (device code is not affected), linked with the kernels' ordinary objects and
with tests/host_sanitize/driver.c, and the driver runs every validation path; no device is touched.  Needs hipcc
(the cross-compiling container and the GPU machine both have it); skipped where it is missing."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANG = "/opt/rocm/lib/llvm/bin/clang"
CSRC = os.path.join(ROOT, "paper_2108_06629_amd", "csrc")
KERNEL_OBJECTS = ["gemm_bf16.o", "gemm_skinny.o", "gemm_f32.o", "elementwise.o", "conv_bf16.o", "conv_thin.o"]
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "not a recognized feature" not in l)
    assert r.returncode == 0, "%s\n%s" % (" ".join(cmd), err[-3000:])
    return r


@pytest.mark.timeout(600)
def test_host_paths_under_address_and_undefined_sanitizers(tmp_path):
    build = os.path.join(ROOT, "_build")
    if not (os.path.exists(HIPCC) and os.path.exists(CLANG)):
        pytest.skip("no hipcc / clang here")
    if not all(os.path.exists(os.path.join(build, o)) for o in KERNEL_OBJECTS):
        pytest.skip("the kernels' objects are not in _build (run __graft_entry__.build() first)")
    objs = []
    for src in ("lp_api.cpp", "partition.cpp"):
        obj = str(tmp_path / (src + ".o"))
        host_san = [a for f in SAN for a in ("-Xarch_host", f)]
        run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-I", os.path.join(ROOT, "include")] + host_san + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    drv = str(tmp_path / "driver.o")
    run([CLANG, "-O1", "-g"] + SAN + ["-I", os.path.join(ROOT, "include"), "-c", os.path.join(ROOT, "tests", "host_sanitize", "driver.c"), "-o", drv])
    exe = str(tmp_path / "driver")
    run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-o", exe, drv] + objs + [os.path.join(build, o) for o in KERNEL_OBJECTS])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and "sanitize ok" in r.stdout, (r.returncode, r.stdout[-2000:], r.stderr[-4000:])
