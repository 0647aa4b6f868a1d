"""The C boundary from plain C: tests/c_abi_check.c (built by __graft_entry__.build() with gcc) allocates its own
device and pinned memory, decodes forty tokens through pie_step with two of the sequence's three blocks in the
host pool, and checks the last output against the attention definition written out in C."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
EXE = os.path.join(HERE, "c_abi_check")


def test_decode_through_the_c_abi_without_python():
    if not os.path.exists(EXE):                                      # normally built beforehand; one second of gcc
        subprocess.run(["gcc", "-std=c11", "-O1", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                        "-I" + os.path.join(ROOT, "include"), os.path.join(HERE, "c_abi_check.c"), "-o", EXE,
                        "-L" + os.path.join(ROOT, "paper_2411_09317_amd"), "-lpie", "-L/opt/rocm/lib", "-lamdhip64",
                        "-lm", "-Wl,-rpath,$ORIGIN/../paper_2411_09317_amd", "-Wl,-rpath,/opt/rocm/lib"], check=True)
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.stdout, r.stderr)
    assert "c abi ok" in r.stdout
