"""AddressSanitizer + UndefinedBehaviorSanitizer on the CPU side (the only place sanitizers can run): the oracle, and
the host half of the C ABI (argument checks, planning, scratch sizing).  Both are exercised from small programs of
their own (tests/sanitize/), linked with the sanitizer runtime, so that the Python process needs no preloading.  No
GPU is touched: every ABI call in the driver fails validation or has nothing to do."""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-g", "-O1"]


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-3000:]}\n{r.stderr[-3000:]}"
    return r.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_asan_and_ubsan(tmp_path):
    src = os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c")
    san, plain = str(tmp_path / "oracle_san"), str(tmp_path / "oracle_plain")
    _run(["gcc", "-std=c11", *SAN, "-static-libasan", src, "-lm", "-o", san])
    _run(["gcc", "-std=c11", "-O2", src, "-lm", "-o", plain])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    out_san = _run([san], env=env)
    out_plain = _run([plain])
    assert out_san == out_plain                     # same bits with and without the instrumentation
    assert out_san.strip().endswith("status 0") and len(out_san.splitlines()) > 90


HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc")
def test_abi_host_code_under_asan_and_ubsan(tmp_path):
    """The library rebuilt with its host code instrumented (device code as usual), linked with the driver."""
    csrc = os.path.join(ROOT, "paper_2509_21354_amd", "csrc")
    host_san = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"):
        host_san += ["-Xarch_host", f]
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", *host_san]
    srcs = sorted(glob.glob(os.path.join(csrc, "*.hip")))
    procs = []
    for s in srcs:
        o = str(tmp_path / (os.path.basename(s)[:-4] + ".o"))
        procs.append((s, o, subprocess.Popen([HIPCC, *flags, "-c", s, "-o", o], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)))
    objs = []
    for s, o, p in procs:
        out, err = p.communicate()
        assert p.returncode == 0, f"{s}\n{err[-3000:]}"
        objs.append(o)
    drv = os.path.join(ROOT, "tests", "sanitize", "abi_driver.cpp")
    exe = str(tmp_path / "abi_san")
    _run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", *host_san, "-x", "hip", drv, "-x", "none", *objs,
          "-fsanitize=address", "-fsanitize=undefined", "-static-libsan", "-o", exe])
    # (leak detection off: the HIP runtime keeps allocations of its own until exit)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1")
    out = _run([exe], env=env)
    assert "abi driver: 0 unexpected" in out
