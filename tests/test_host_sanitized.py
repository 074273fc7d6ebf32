"""The host side of the C ABI (argument checks, policy, bucket bookkeeping: recover_host.cpp) built for the CPU
with AddressSanitizer and UBSan and driven by 240,000 random calls, many of them invalid, on host-only contexts
(tests/host/fuzz.cpp).  The kernel launchers are replaced by stand-ins that abort (tests/host/stubs.cpp): a
host-only context must never reach one.  No GPU code is compiled or sanitized.  CPU only."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(ROOT, "paper_2605_11215_amd", "csrc")


def test_host_logic_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    exe = str(tmp_path / "host_fuzz")
    # host compilation only; the sanitizers instrument host code, nothing is built for the GPU
    flags = "--cuda-host-only -fno-gpu-sanitize -O1 -g -std=c++17 -fsanitize=address -fsanitize=undefined -fno-sanitize-recover=undefined"
    subprocess.run([hipcc] + flags.split() + ["-I", os.path.join(ROOT, "include"), "-I", CSRC,
                                              os.path.join(HERE, "host", "fuzz.cpp"), os.path.join(HERE, "host", "stubs.cpp"),
                                              os.path.join(CSRC, "recover_host.cpp"), "-o", exe], check=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    assert "fuzz ok: 240000 calls" in r.stdout
