"""The library's host logic under the address and undefined-behaviour sanitizers (host code only; the device code
is compiled as usual and never runs): tests/host_stress.cpp drives the bookkeeping-only pool, the layer
scheduler, the chunk book and the controller with random call sequences and checks their invariants after every
call.  Runs without a GPU."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
from paper_2411_09317_amd import build as BUILD  # noqa: E402


@pytest.mark.timeout(600)
def test_host_logic_is_clean_under_asan_and_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        hipcc = shutil.which("hipcc")
    if not hipcc:
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "host_stress")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-ffp-contract=off",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           f"-I{os.path.join(ROOT, 'include')}", f"-I{BUILD.CSRC}"]
    for src in [os.path.join(BUILD.CSRC, s) for s in BUILD.SOURCES] + [os.path.join(ROOT, "tests", "host_stress.cpp")]:
        cmd += ["-x", "hip", src]
    cmd += ["-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:protect_shadow_gap=0")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=500)
    assert r.returncode == 0 and "host stress ok" in r.stdout, (r.stdout[-1500:] + r.stderr[-3000:])
