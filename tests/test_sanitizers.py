"""AddressSanitizer + UndefinedBehaviorSanitizer pass over the two host-only native pieces: the
fp64 oracle (oracle/pbkv_oracle.c) and the policy core (csrc/policy.cpp).  Each is compiled with
its driver under tests/sanitize/ into a sanitized executable of its own (no instrumented library
is loaded into Python) and run once; any report aborts the driver."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


def _run(cmd, exe, tmp_path):
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, cwd=tmp_path)
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert "clean" in r.stdout


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-std=c11", *SAN, "-fopenmp", os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
          os.path.join(ROOT, "oracle", "pbkv_oracle.c"), "-o", exe, "-lm"], exe, tmp_path)


def test_policy_core_under_sanitizers(tmp_path):
    rocm_inc = "/opt/rocm/include"
    if not os.path.exists(os.path.join(rocm_inc, "hip", "hip_runtime.h")) or not shutil.which("g++"):
        pytest.skip("needs the HIP headers (declarations only) and g++")
    exe = str(tmp_path / "policy_san")
    _run(["g++", "-std=c++17", *SAN, "-w", "-D__HIP_PLATFORM_AMD__", "-I" + rocm_inc,
          "-I" + os.path.join(ROOT, "paper_2605_06472_amd", "csrc"),
          os.path.join(ROOT, "tests", "sanitize", "policy_driver.cpp"),
          os.path.join(ROOT, "paper_2605_06472_amd", "csrc", "policy.cpp"), "-o", exe], exe, tmp_path)
