"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer, without a GPU: the library is built a
second time with the sanitizers on the host pass only (device code is compiled as usual and never runs here), and
tests/host_sanitize_driver.c walks every host-side query, the schedule dumps into exactly-sized buffers and the argument
checks through a context made by tl_ctx_create_host.  The build is kept under _build/ and reused while the sources are
unchanged (a fresh one takes about a minute)."""
import hashlib
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2503_20313_amd", "csrc")
HIPCC = "/opt/rocm/bin/hipcc"
CLANG = "/opt/rocm/llvm/bin/clang"


def source_digest():
    h = hashlib.sha256()
    files = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC)) + [os.path.join(ROOT, "include", "tilelink_mi355.h"),
                                                                         os.path.join(ROOT, "tests", "host_sanitize_driver.c")]
    for f in files:
        h.update(f.encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANG)), reason="needs the ROCm compilers")
def test_host_code_is_clean_under_asan_and_ubsan():
    out = os.path.join(ROOT, "_build", "asan")
    tag = os.path.join(out, "digest")
    digest = source_digest()
    lib, drv = os.path.join(out, "libtilelink_mi355_asan.so"), os.path.join(out, "host_sanitize_driver")
    if not (os.path.exists(tag) and open(tag).read() == digest and os.path.exists(lib) and os.path.exists(drv)):
        shutil.rmtree(out, ignore_errors=True)
        os.makedirs(out)
        srcs = [os.path.join(CSRC, f) for f in ("tl_dense.hip", "tl_moe.hip", "tl_attention.hip")]
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-shared", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
                        "-packed-fp32-ops", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-o", lib] + srcs,
                       check=True, capture_output=True, timeout=900)
        subprocess.run([CLANG, "-fsanitize=address,undefined", "-g", "-I", os.path.join(ROOT, "include"),
                        os.path.join(ROOT, "tests", "host_sanitize_driver.c"), "-o", drv, "-L", out, "-ltilelink_mi355_asan",
                        f"-Wl,-rpath,{out}", "-Wl,-rpath,/opt/rocm/lib"], check=True, capture_output=True, timeout=300)
        open(tag, "w").write(digest)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:halt_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([drv], capture_output=True, text=True, timeout=600, env=env)
    text = r.stdout + r.stderr
    assert r.returncode == 0, text[-3000:]
    assert "host_sanitize_driver ok" in r.stdout
    assert "AddressSanitizer" not in text and "runtime error" not in text and "LeakSanitizer" not in text, text[-3000:]
