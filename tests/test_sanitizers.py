"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU needed, none used):
  * the CPU oracle's C routines, driven by tests/sanitize/oracle_driver.c over small and degenerate geometries;
  * the host side of the C ABI (csrc/api.hip: validation, state machine, error texts, context life cycle), driven by
    tests/sanitize/api_driver.cpp.  Only the host pass of api.hip is instrumented (`-Xarch_host -fsanitize=...`);
    the other translation units are taken as built, since their host parts are launch stubs.
A sanitizer report aborts the driver with a non-zero status."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0", UBSAN_OPTIONS="halt_on_error=1")


def run(cmd, **kw):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert p.returncode == 0, " ".join(cmd) + "\n" + p.stdout[-4000:]
    return p.stdout


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    run(["gcc", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
         "-fopenmp", "-o", exe, os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "ddcca_oracle.c"),
         "-lm"])
    out = run([exe], env=ENV)
    assert "oracle sanitize ok" in out and "runtime error" not in out


def test_api_host_side_under_asan_ubsan(tmp_path):
    from paper_2209_13027_amd import build
    hipcc = build._hipcc()
    clangxx = "/opt/rocm/lib/llvm/bin/clang++"
    if shutil.which(hipcc) is None or not os.path.exists(clangxx):
        pytest.skip("no ROCm compiler")
    build_dir = os.path.join(build.HERE, "_build")
    others = [os.path.join(build_dir, s.replace(".hip", ".o")) for s in build.SOURCES if s != "api.hip"]
    if not all(os.path.exists(o) for o in others):
        build.build_library()
    api_o, drv_o, exe = str(tmp_path / "api_san.o"), str(tmp_path / "api_driver.o"), str(tmp_path / "api_san")
    host_san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
                "-fno-sanitize-recover=all"]
    run([hipcc, *[f for f in build.FLAGS if f != "-O3"], "-O1", "-g", *host_san, "-c",
         os.path.join(build.CSRC, "api.hip"), "-o", api_o])
    run([clangxx, "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-c",
         os.path.join(SAN, "api_driver.cpp"), "-o", drv_o])
    run([hipcc, "--offload-arch=gfx950", "--hip-link", "-fsanitize=address,undefined", "-fno-gpu-sanitize", "-o", exe,
         drv_o, api_o, *others])
    out = run([exe], env=ENV)
    assert "api sanitize ok" in out and "runtime error" not in out
