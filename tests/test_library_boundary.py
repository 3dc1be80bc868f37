"""CPU-only checks of the C boundary: the shared library loads, exports every function that
include/qadam.h declares, and rejects bad arguments before touching the GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "qadam.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qadam_[a-z_0-9]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    from paper_2004_14180_amd import binding
    if not os.path.exists(binding.library_path()):
        from paper_2004_14180_amd.build import build_library
        build_library(verbose=False)
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert len(names) >= 12 and "qadam_step_fused" in names
    for n in names:
        assert hasattr(lib, n), n
    from paper_2004_14180_amd.binding import EXPORTS
    assert sorted(EXPORTS) == names


def test_bad_configs_are_rejected_on_the_host(lib):
    """Argument validation happens before any HIP call, so it can be exercised without a GPU."""
    from paper_2004_14180_amd.binding import _Config
    segs = (C.c_int64 * 3)(0, 10, 20)
    h = C.c_void_p()

    def init(cfg, segs=segs, L=2, N=2):
        return lib.qadam_init(C.byref(h), C.byref(cfg), segs, L, N)

    good = dict(struct_size=C.sizeof(_Config), k_g=2, k_x=6, rounding=0, weight_ef=1, adam_flavor=0,
                beta1=0.9, eps=1e-8, seed=0)
    for bad in [dict(struct_size=4), dict(k_g=-2), dict(k_g=7), dict(k_x=15), dict(k_x=-2), dict(rounding=2),
                dict(weight_ef=3), dict(beta1=1.0), dict(eps=-1.0)]:
        cfg = _Config(**{**good, **bad})
        assert init(cfg) == -1, bad
        assert lib.qadam_last_error()
    cfg = _Config(**good)
    assert init(cfg, N=0) == -1
    assert init(cfg, N=33) == -3
    assert init(cfg, segs=(C.c_int64 * 3)(1, 10, 20)) == -1
    assert init(cfg, segs=(C.c_int64 * 3)(0, 30, 20)) == -1
    # sizes beyond one launch (one workgroup per 4096-element tile, fewer than 2^24 tiles) and beyond 2^40
    assert init(cfg, segs=(C.c_int64 * 2)(0, 1 << 36), L=1) == -3
    assert init(cfg, segs=(C.c_int64 * 2)(0, (1 << 40) + 1), L=1) == -3
    assert lib.qadam_destroy(None) == 0
    assert lib.qadam_grad_code_bytes(None) == 0


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2004_14180_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libqadam_hip.so")
    with pytest.raises(ImportError):
        binding.load_library()


def test_device_code_holds_no_packed_fp32_instructions():
    """The library is built with the packed-fp32 feature switched off for the gfx950 pass (the host pass
    only warns that it does not know the feature).  Check the effect where it matters: the device
    assembly of the kernels has no packed fp32 add / mul / fma."""
    from paper_2004_14180_amd.build import device_assembly
    asm = device_assembly("qadam_kernels.hip")
    assert "k_fused" in asm and "gfx950" in asm
    packed = re.findall(r"\bv_pk_(?:add|mul|fma)_f32\b", asm)
    assert not packed, "%d packed fp32 instructions in the device code" % len(packed)


def test_kernels_keep_their_arguments_out_of_scratch_and_the_main_pass_its_occupancy():
    """What the compiler reports for the library's kernels under the library's flags.  No kernel may have a
    per-lane scratch segment to speak of: the kernels take one argument struct with pointer arrays indexed
    at run time, and when the compiler cannot prove it can read that struct in place it copies all of it
    (1.2 KB for the fused kernel) to scratch at kernel entry and reads every pointer back from there, silently.
    The fused main pass in the benchmark's configuration (nearest rounding, four workers' loads in flight,
    variant S) must also stay within 96 vector registers, i.e. five wavefronts per SIMD."""
    from paper_2004_14180_amd.build import device_resource_usage
    usage = device_resource_usage("qadam_kernels.hip")
    assert len(usage) >= 30, "kernel list not parsed"
    for name, u in usage.items():
        assert u["scratch_bytes"] <= 64, "%s: %d bytes of scratch per lane" % (name, u["scratch_bytes"])
    main = [u for name, u in usage.items() if "k_fusedILi0ELi4ELb0" in name]
    assert len(main) == 1
    assert main[0]["scratch_bytes"] == 0 and main[0]["vgprs"] <= 96 and main[0]["waves_per_simd"] >= 5, main[0]
