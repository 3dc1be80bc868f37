"""Compile the gfx950 shared library (``libqadam_hip.so``) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqadam_hip.so")
SOURCES = ["qadam_kernels.hip", "qadam_api.cpp"]

# -ffp-contract=off: one rounding per operation, so integer codes are reproducible bit for bit.
# The target-feature switch keeps the gfx950 pass from forming packed-fp32 instructions (v_pk_add_f32,
# v_pk_mul_f32, v_pk_fma_f32): with it the device assembly of qadam_kernels.hip holds none of them, without
# it several hundred (tests/test_library_boundary.py checks this).  -Xclang options reach both passes of
# hipcc, and the HOST (x86-64) pass does not know the feature: it prints "'-packed-fp32-ops' is not a
# recognized feature for this target (ignoring feature)" once per function it compiles.  That warning is
# the host pass's and is harmless; the device pass honours the switch silently.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # The kernels take their arguments as one struct with per-worker pointer arrays that are indexed at run
    # time.  The compiler reads such a struct straight from the kernel-argument segment only if a use scan of
    # bounded length succeeds (default 300 uses); the fused kernel, with its tile loop instantiated for each
    # layer kind, has more, and past the bound the whole 1.2 KB struct is copied to per-lane scratch memory
    # at kernel entry.  tests/test_library_boundary.py checks that no kernel has a scratch segment.
    "-mllvm", "-instcombine-max-copied-from-constant-users=4000",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


PROBE_SRC = os.path.join(CSRC, "qadam_probe.hip")
PROBE = os.path.join(HERE, "qadam_probe.bin")


def build_probe(verbose: bool = True) -> str:
    """The stand-alone memory-system probes (measurement aid, not part of the library)."""
    tmp = PROBE + ".tmp%d" % os.getpid()
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-o", tmp, PROBE_SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, PROBE)
    return PROBE


def device_assembly(source: str = "qadam_kernels.hip", packed_fp32_off: bool = True) -> str:
    """gfx950 assembly text of one of this package's own sources (for checks of what the compiler emitted)."""
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    if not packed_fp32_off:
        flags = [f for f in flags if f not in ("-Xclang", "-target-feature", "-packed-fp32-ops")]
    cmd = [hipcc(), *flags, "--cuda-device-only", "-S", "-I", os.path.join(HERE, "..", "include"), "-o", "-",
           os.path.join(CSRC, source)]
    return subprocess.run(cmd, check=True, capture_output=True, text=True).stdout


def device_resource_usage(source: str = "qadam_kernels.hip") -> dict:
    """Registers, scratch and LDS of every kernel of one of this package's sources, as the compiler reports
    them for the library's flags: {demangled-ish kernel name: {"vgprs", "sgprs", "scratch_bytes", "lds_bytes",
    "waves_per_simd"}}."""
    import re
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    cmd = [hipcc(), *flags, "--cuda-device-only", "-c", "-Rpass-analysis=kernel-resource-usage",
           "-I", os.path.join(HERE, "..", "include"), "-o", os.devnull, os.path.join(CSRC, source)]
    text = subprocess.run(cmd, check=True, capture_output=True, text=True).stderr
    out, cur = {}, None
    keys = {"VGPRs": "vgprs", "TotalSGPRs": "sgprs", "ScratchSize [bytes/lane]": "scratch_bytes",
            "LDS Size [bytes/block]": "lds_bytes", "Occupancy [waves/SIMD]": "waves_per_simd"}
    for line in text.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z \[\]/]+): (\d+)", line)
        if m and cur is not None and m.group(1).strip() in keys:
            cur[keys[m.group(1).strip()]] = int(m.group(2))
    return out


def build_library(verbose: bool = True) -> str:
    srcs = []
    for s in SOURCES:
        path = os.path.join(CSRC, s)
        srcs += (["-x", "hip", path] if s.endswith(".cpp") else [path])
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc(), *HIPCC_FLAGS, "-I", os.path.join(HERE, "..", "include"), "-o", tmp, *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build_library()
    build_probe()
    sys.exit(0)
