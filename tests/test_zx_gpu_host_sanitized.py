"""The host code of the GPU paths under the address and undefined-behaviour sanitizers (host side only):
tests/gpu_host_check.cpp, built by __graft_entry__.build() from the library's own sources, runs pie_step in every
monitoring mode and swap path with residency changes in between, the per-layer calls by hand, the layer pool and
the elastic pool on the GPU, and the sanitizers watch the host code meanwhile.  Collected after the parity tests."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
EXE = os.path.join(HERE, "gpu_host_check")


def test_host_code_of_the_gpu_paths_is_clean_under_asan_and_ubsan():
    if not os.path.exists(EXE):                                      # normally built beforehand
        sys.path.insert(0, ROOT)
        from paper_2411_09317_amd import build as b
        cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
               "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-value",
               "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
               "-Xarch_host", "-fno-sanitize-recover=undefined",
               "-I" + os.path.join(ROOT, "include"), "-I" + b.CSRC]
        for src in [os.path.join(b.CSRC, s) for s in b.SOURCES] + [os.path.join(HERE, "gpu_host_check.cpp")]:
            cmd += ["-x", "hip", src]
        subprocess.run(cmd + ["-o", EXE], check=True, capture_output=True)
    # the HIP runtime maps memory where the sanitizer would otherwise keep a guard gap; leaks are the runtime's own
    env = dict(os.environ, ASAN_OPTIONS="protect_shadow_gap=0:detect_leaks=0")
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=100, env=env)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "gpu host check ok" in r.stdout
