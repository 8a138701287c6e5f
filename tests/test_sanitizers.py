"""CPU-side code under AddressSanitizer and UndefinedBehaviorSanitizer: the oracle (oracle/ws_oracle.c) running
its closed-form pins, and the C-ABI front end's host validation (csrc/api.hip) against stub launchers.  Both are
host-only builds made here; nothing touches a GPU.  (GPU-side sanitizers are not available for gfx950 kernels on
this pool; the kernels' guards are bounds checks on the host plus index clamping in the kernels.)"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
# (a library preloaded into every process of the host may sit in front of the sanitizer runtime: tolerated)
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")


def run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines() if "not a recognized feature" not in l)
    return r.returncode, out


def test_oracle_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_pins")
    rc, out = run(["gcc", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
                   "-fno-sanitize-recover=all", "-o", exe, os.path.join(SAN, "oracle_pins_driver.c"),
                   os.path.join(ROOT, "oracle", "ws_oracle.c"), "-lm"])
    assert rc == 0, out
    rc, out = run([exe], env=ENV)
    assert rc == 0 and "all checks passed" in out, out


def test_abi_validation_under_address_and_undefined_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clang = "/opt/rocm/bin/amdclang"
    if not (os.path.exists(hipcc) and os.path.exists(clang)):
        pytest.skip("no hipcc on this host")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=all"]
    common = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17"] + san
    objs = []
    for src in (os.path.join(ROOT, "paper_2601_01298_amd", "csrc", "api.hip"), os.path.join(SAN, "api_stubs.cpp")):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        rc, out = run(common + ["-x", "hip", "-c", src, "-o", obj])
        assert rc == 0, out
        objs.append(obj)
    drv = str(tmp_path / "api_driver.o")
    rc, out = run([clang, "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-c",
                   os.path.join(SAN, "api_driver.c"), "-o", drv])
    assert rc == 0, out
    exe = str(tmp_path / "api_checks")
    rc, out = run([hipcc, "--offload-arch=gfx950", "-fsanitize=address,undefined"] + objs + [drv, "-o", exe])
    assert rc == 0, out
    rc, out = run([exe], env=dict(ENV, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0"))     # the HIP runtime's own start-up allocations
    assert rc == 0 and "all checks passed" in out, out
