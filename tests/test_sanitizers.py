"""Host-side sanitizer builds (AddressSanitizer + UndefinedBehaviorSanitizer, CPU only): the C oracle under a
driver that runs small layers of every kind through every entry point, and the C ABI's host code (argument
validation, workspace arithmetic, closed forms) linked with launch stubs that enqueue nothing."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="2")


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-Wall", "-Wextra"]
                   + SAN + ["-o", exe, os.path.join(HERE, "native", "oracle_sanitize_main.c"), "-lm"], check=True)
    r = subprocess.run([exe], env=ENV, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "oracle_sanitize: ok" in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])


def test_abi_host_code_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc")
    exe = str(tmp_path / "abi_args")
    host_san = [a for f in SAN for a in ("-Xarch_host", f)]
    csrc = os.path.join(ROOT, "paper_2505_19645_amd", "csrc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-x", "hip", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops"] + host_san + [os.path.join(HERE, "native", "abi_args_main.cpp"),
                                             os.path.join(csrc, "moesd_api.cpp"), os.path.join(csrc, "closed_forms.cpp"),
                                             "-o", exe]
    b = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert b.returncode == 0, b.stderr[-4000:]
    r = subprocess.run([exe], env=ENV, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "abi_args: ok" in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])
