"""Host-side AddressSanitizer / UndefinedBehaviorSanitizer runs (no GPU code is instrumented or run):
the CPU oracle end to end, and the host-only parts of libadacomp (table validation, plan and size
arithmetic, early error returns)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=0",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)


def test_oracle_under_asan_ubsan(tmp_path):
    exe = tmp_path / "driver_oracle"
    subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-ffp-contract=off", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-static-libasan", "-I" + os.path.join(ROOT, "oracle"),
                    "-o", str(exe), os.path.join(SAN, "driver_oracle.c"), os.path.join(ROOT, "oracle", "adacomp_oracle.c"),
                    "-lm"], check=True)
    res = subprocess.run([str(exe)], capture_output=True, text=True, env=ENV, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "driver ok" in res.stdout
    print(res.stdout.strip())


def test_library_host_code_under_asan_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which("hipcc")):
        pytest.skip("no hipcc")
    exe = tmp_path / "driver_api"
    csrc = os.path.join(ROOT, "paper_1712_02679_amd", "csrc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-ffp-contract=off",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all",
           "-I" + os.path.join(ROOT, "include"), "-I" + csrc, "-o", str(exe), os.path.join(SAN, "driver_api.cpp"),
           os.path.join(csrc, "adacomp_api.hip"), os.path.join(csrc, "adacomp_kernels.hip")]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    res = subprocess.run([str(exe)], capture_output=True, text=True, env=ENV, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "driver ok" in res.stdout
    print(res.stdout.strip())
