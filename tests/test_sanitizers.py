"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU-side code, run on the host (no GPU):
the oracle (oracle/lpg_oracle.c) under tests/sanitize/oracle_driver.c, and the library's host side
(csrc/lpg_api.cpp: descriptor validation, view and stride arithmetic, the host index function, the chain's
link check and dry pass) under tests/sanitize/host_driver.cpp.  Device code cannot be sanitized here; the
host driver only makes calls that fail validation or are dry passes, so nothing is launched."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines() if "packed-fp32-ops" not in l)
    return r.returncode, out


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    rc, out = _run(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan",
                    "-ffp-contract=off", "-std=c11", "-o", exe, os.path.join(SAN, "oracle_driver.c"),
                    os.path.join(ROOT, "oracle", "lpg_oracle.c"), "-lm"])
    assert rc == 0, out
    rc, out = _run([exe], env=ENV, timeout=300)
    assert rc == 0 and "clean" in out, out
    assert "runtime error" not in out and "AddressSanitizer" not in out, out


def test_host_side_of_the_library_is_clean_under_asan_and_ubsan(tmp_path):
    hipcc = "/opt/rocm/bin/hipcc"
    clang = "/opt/rocm/lib/llvm/bin/clang++"
    lib_dir = os.path.join(ROOT, "paper_2604_04599_amd")
    if not (os.path.exists(hipcc) and os.path.exists(clang)):
        pytest.skip("no ROCm toolchain")
    if not os.path.exists(os.path.join(lib_dir, "liblpg.so")):
        pytest.skip("liblpg.so not built (the launchers the host side links against come from it)")
    obj, exe = str(tmp_path / "lpg_api_san.o"), str(tmp_path / "host_san")
    rc, out = _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                    "-packed-fp32-ops", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                    "-Xarch_host", "-fno-sanitize-recover=undefined", "-x", "hip", "-c",
                    os.path.join(lib_dir, "csrc", "lpg_api.cpp"), "-o", obj])
    assert rc == 0, out
    rc, out = _run([clang, "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-fno-sanitize-recover=undefined",
                    "-I", os.path.join(ROOT, "include"), os.path.join(SAN, "host_driver.cpp"), obj, "-L", lib_dir, "-llpg",
                    "-L/opt/rocm/lib", "-lamdhip64", f"-Wl,-rpath,{lib_dir}", "-Wl,-rpath,/opt/rocm/lib", "-o", exe])
    assert rc == 0, out
    rc, out = _run([exe], env=ENV, timeout=300)
    assert rc == 0 and "clean" in out, out
    assert "runtime error" not in out and "AddressSanitizer" not in out, out
