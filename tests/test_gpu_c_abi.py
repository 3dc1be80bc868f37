"""The C boundary used from a plain host program (no Python, no torch in the process): built with
hipcc against include/qadam.h and libqadam_hip.so, linked with the C oracle, run as a subprocess.
__graft_entry__.build() compiles it beforehand (tests/c_abi_parity.bin); the test compiles it itself
only when that binary is missing or older than its source."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "c_abi_parity.cpp")
EXE = os.path.join(ROOT, "tests", "c_abi_parity.bin")


def build_c_abi_parity(exe=EXE):
    from paper_2004_14180_amd import binding
    from oracle import qadam_oracle
    qadam_oracle.build()
    pkg = os.path.dirname(binding.library_path())
    odir = os.path.join(ROOT, "oracle")
    cmd = ["/opt/rocm/bin/hipcc", "-O1", "-std=c++17", "-ffp-contract=off",
           "-I", os.path.join(ROOT, "include"), "-I", odir, SRC,
           "-L", pkg, "-lqadam_hip", "-Wl,-rpath," + pkg,
           "-L", odir, "-loracle_qadam", "-Wl,-rpath," + odir, "-lm", "-o", exe]
    subprocess.check_call(cmd)
    return exe


@pytest.mark.gpu
def test_c_program_matches_the_oracle():
    if not os.path.exists(EXE) or os.path.getmtime(EXE) < os.path.getmtime(SRC):
        build_c_abi_parity()
    out = subprocess.run([EXE], capture_output=True, text=True, timeout=300)
    print(out.stdout, out.stderr, flush=True)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-2000:]
    assert out.stdout.count("all outputs equal the oracle's") == 4
