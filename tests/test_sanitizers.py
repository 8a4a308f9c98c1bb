"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU oracle and of the host side of the C-ABI.

Both run on the CPU: the oracle is plain C; the C-ABI's host code (validation, gather plans, launch planning,
workspace layout) is built from csrc/tr_api.hip with stand-ins for the kernel launchers, which also check the
argument blocks a kernel would receive (tests/san/).  No kernel is launched, with or without a GPU in the machine.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "san")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    assert res.returncode == 0, "%s\nexit status %d\n%s\n%s" % (" ".join(cmd), res.returncode, res.stdout[-4000:], err[-8000:])
    return res.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not found")
def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-Wall",
          "-o", exe, os.path.join(SAN, "oracle_san.c"), os.path.join(ROOT, "oracle", "turborag_oracle.c"), "-lm"])
    out = _run([exe])
    assert "oracle sanitizer run ok" in out


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_host_side_of_the_c_abi_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "host_abi_san")
    # each -fsanitize= sits directly behind -Xarch_host: only the host pass is instrumented
    _run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
          "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-o", exe, os.path.join(SAN, "host_abi_san.cpp"), os.path.join(ROOT, "paper_2410_07590_amd", "csrc", "tr_api.hip")])
    out = _run([exe, "300"])
    assert "host abi sanitizer run ok: 300 request mixes" in out
