"""The library's host code (argument validation, size queries, the Case II prune / re-root of
Sec. 3.2) rebuilt with the host compiler's address and undefined-behaviour sanitizers and driven by
`tests/sanitize/abi_host_paths.cpp` with seeded valid and invalid arguments.  CPU only: every call
of the driver returns before anything would be enqueued on a GPU.  The kernels' objects are linked
as built (device code is not instrumented)."""
import os
import shutil
import subprocess

import pytest

from paper_2601_23180_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True, cwd=ROOT)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    assert r.returncode == 0, " ".join(cmd) + "\n" + err
    return r


@pytest.mark.skipif(shutil.which(B.HIPCC) is None, reason="no hipcc")
def test_host_paths_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    host_srcs = ("api.cpp", "ternary.cpp")
    kernel_objs = [os.path.join(B.BUILD, os.path.splitext(s)[0] + ".o") for s in B.SOURCES if s not in host_srcs]
    if not all(os.path.exists(o) for o in kernel_objs):
        B.build(verbose=False)
    drv_o, exe = str(tmp_path / "driver.o"), str(tmp_path / "driver")
    host_objs = [str(tmp_path / (os.path.splitext(s)[0] + "_san.o")) for s in host_srcs]
    host_san = [x for f in SAN for x in ("-Xarch_host", f)]      # the host pass only
    flags = [f for f in B.FLAGS if f != "-O3"]
    for src, obj in zip(host_srcs, host_objs):
        _run([B.HIPCC, "-O1", "-g", *flags, *host_san, "-c", os.path.join(B.CSRC, src), "-o", obj])
    _run([B.HIPCC, "-O1", "-g", "-std=c++17", "-I", os.path.join(ROOT, "include"), *SAN, "-x", "c++", "-c",
          os.path.join(ROOT, "tests", "sanitize", "abi_host_paths.cpp"), "-o", drv_o])
    _run([B.HIPCC, "--offload-arch=gfx950", *SAN, "-fno-gpu-sanitize", "-o", exe, drv_o, *host_objs, *kernel_objs])
    for obj in host_objs:
        syms = subprocess.run(["nm", obj], capture_output=True, text=True).stdout
        assert "__asan_" in syms and "__ubsan_" in syms      # the instrumentation is really there
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300,
                       env={**os.environ, "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=0"})
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert r.stdout.startswith("ok ")
