"""Python binding of the C boundary (``include/qadam.h``): argument marshalling only.

Every step of the optimizer runs in the HIP kernels of ``libqadam_hip.so``.  The library must have
been built (``python paper_2004_14180_amd/build.py``); loading fails loudly otherwise -- there is no
CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libqadam_hip.so")

QADAM_OK, QADAM_EINVAL, QADAM_EALIGN, QADAM_ERANGE, QADAM_EHIP = 0, -1, -2, -3, -4
QADAM_MAX_WORKERS = 32
QADAM_IDENTITY = -1          # k_g or k_x: that quantizer is the identity
QADAM_STATUS_NONFINITE_SCALE = 1
QADAM_STATUS_ERR_BOUND_VIOLATED = 2

EXPORTS = [
    "qadam_init", "qadam_destroy", "qadam_grad_code_bytes", "qadam_weight_code_bytes",
    "qadam_num_params", "qadam_worker_quantize", "qadam_server_step", "qadam_weight_quantize",
    "qadam_step_fused", "qadam_worker_step_w", "qadam_server_apply_w", "qadam_step_fused_w", "qadam_weight_dequantize",
    "qadam_weight_dequantize_f16", "qadam_layer_sumsq", "qadam_trust_error_buffers",
    "qadam_get_status", "qadam_last_error", "qadam_profile_enable", "qadam_profile_read",
    "qadam_quantize_segment_noalloc", "qadam_arena_layout",
]


class QAdamError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("qadam error %d: %s" % (code, msg))
        self.code = code


class _Config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("k_g", C.c_int32), ("k_x", C.c_int32),
                ("rounding", C.c_int32), ("weight_ef", C.c_int32), ("adam_flavor", C.c_int32),
                ("beta1", C.c_float), ("eps", C.c_float), ("seed", C.c_uint64)]


class _Profile(C.Structure):
    _fields_ = [("scale_pass_ms", C.c_float), ("main_pass_ms", C.c_float)]


class _Arena(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("x", "m", "v", "werr", "wcodes")] + \
               [(n, C.c_size_t * QADAM_MAX_WORKERS) for n in ("grads", "errs", "codes", "scales", "mw", "vw")] + \
               [("bytes_needed", C.c_size_t)]


class _Status(C.Structure):
    _fields_ = [("flags", C.c_uint32), ("reserved", C.c_uint32)]


@dataclass
class QAdamConfig:
    k_g: int = 2
    k_x: int = 6
    rounding: int = 0
    weight_ef: int = 1
    adam_flavor: int = 0
    beta1: float = 0.9
    eps: float = 1e-8
    seed: int = 0


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """dlopen the HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            "%s is missing: build it with `python paper_2004_14180_amd/build.py` "
            "(hipcc, --offload-arch=gfx950). There is no fallback path." % _LIB_PATH)
    # torch first: it ships its own HIP runtime under the same soname as the system's, and the
    # process must end up with ONE runtime shared by torch (device memory, streams) and this library.
    # Loaded the other way round, the library's HIP calls fail with "no ROCm-capable device".
    import torch  # noqa: F401
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    lib.qadam_init.argtypes = [C.POINTER(vp), C.POINTER(_Config), C.POINTER(i64), i32, i32]
    lib.qadam_destroy.argtypes = [vp]
    lib.qadam_grad_code_bytes.argtypes = [vp]
    lib.qadam_grad_code_bytes.restype = C.c_size_t
    lib.qadam_weight_code_bytes.argtypes = [vp]
    lib.qadam_weight_code_bytes.restype = C.c_size_t
    lib.qadam_num_params.argtypes = [vp]
    lib.qadam_num_params.restype = i64
    lib.qadam_worker_quantize.argtypes = [vp, i32, i64, vp, vp, vp, vp, vp]
    lib.qadam_server_step.argtypes = [vp, i64, f32, f32, C.POINTER(vp), C.POINTER(vp), vp, vp, vp, vp]
    lib.qadam_weight_quantize.argtypes = [vp, i64, vp, vp, vp, vp]
    lib.qadam_step_fused.argtypes = [vp, i64, f32, f32, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                                     C.POINTER(vp), vp, vp, vp, vp, vp, vp]
    lib.qadam_worker_step_w.argtypes = [vp, i32, i64, f32, f32, vp, vp, vp, vp, vp, vp, vp]
    lib.qadam_step_fused_w.argtypes = [vp, i64, f32, f32, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                                       C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), vp, vp, vp, vp]
    lib.qadam_server_apply_w.argtypes = [vp, i64, C.POINTER(vp), C.POINTER(vp), vp, vp]
    lib.qadam_weight_dequantize.argtypes = [vp, vp, vp, vp]
    lib.qadam_weight_dequantize_f16.argtypes = [vp, vp, vp, vp]
    lib.qadam_layer_sumsq.argtypes = [vp, vp, vp, vp, vp]
    lib.qadam_trust_error_buffers.argtypes = [vp, i32]
    lib.qadam_get_status.argtypes = [vp, C.POINTER(_Status), i32, vp]
    lib.qadam_last_error.restype = C.c_char_p
    lib.qadam_profile_enable.argtypes = [vp, i32]
    lib.qadam_profile_read.argtypes = [vp, C.POINTER(_Profile)]
    lib.qadam_quantize_segment_noalloc.argtypes = [i32, i64, vp, vp, vp, vp, vp]
    lib.qadam_arena_layout.argtypes = [vp, C.c_size_t, i32, C.POINTER(_Arena)]
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    """Device address of a torch tensor (or None)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return t.data_ptr()


def _ptr_array(ts: Optional[Sequence]):
    if ts is None:
        return None
    arr = (C.c_void_p * len(ts))()
    for i, t in enumerate(ts):
        arr[i] = _ptr(t)
    return arr


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


QADAM_NOALLOC_MAX_ELEMS = 1 << 28


def quantize_segment_noalloc(k_g, n, grad, err, codes, scale, stream=None):
    """qadam_quantize_segment_noalloc: one segment, no handle, no allocation (see include/qadam.h)."""
    lib = load_library()
    rc = lib.qadam_quantize_segment_noalloc(int(k_g), int(n), _ptr(grad), _ptr(err), _ptr(codes), _ptr(scale),
                                            _stream(stream))
    if rc != QADAM_OK:
        raise QAdamError(rc, (lib.qadam_last_error() or b"").decode())


class QAdam:
    """One handle = one flat parameter vector with its layer segments and N logical workers.

    Methods carry the names of the C entry points and take torch device tensors; they enqueue on
    the given (default: current) stream and do not synchronise.
    """

    def __init__(self, cfg: QAdamConfig, seg_offsets: Sequence[int], num_workers: int):
        self._lib = load_library()
        self.cfg = cfg
        self.num_workers = int(num_workers)
        self.seg_offsets = [int(s) for s in seg_offsets]
        self.num_segments = len(self.seg_offsets) - 1
        c = _Config(C.sizeof(_Config), cfg.k_g, cfg.k_x, cfg.rounding, cfg.weight_ef, cfg.adam_flavor,
                    cfg.beta1, cfg.eps, cfg.seed)
        segs = (C.c_int64 * len(self.seg_offsets))(*self.seg_offsets)
        h = C.c_void_p()
        self._h = None
        self._check(self._lib.qadam_init(C.byref(h), C.byref(c), segs, self.num_segments, self.num_workers))
        self._h = h

    def _check(self, rc: int):
        if rc != QADAM_OK:
            raise QAdamError(rc, (self._lib.qadam_last_error() or b"").decode())

    def close(self):
        if self._h is not None:
            self._lib.qadam_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # sizes -------------------------------------------------------------------------------------
    @property
    def num_params(self) -> int:
        return int(self._lib.qadam_num_params(self._h))

    def grad_code_bytes(self) -> int:
        return int(self._lib.qadam_grad_code_bytes(self._h))

    def weight_code_bytes(self) -> int:
        return int(self._lib.qadam_weight_code_bytes(self._h))

    # argument checks ---------------------------------------------------------------------------
    # The kernels write P-sized streams through the raw addresses they are given, so a buffer of the
    # wrong type, size or device would be an out-of-bounds device access: refuse it here.
    def _buf(self, t, name, numel, kind="f32", optional=False):
        """Device address of tensor `t` after checking device, layout, element type and size."""
        import torch
        if t is None:
            if optional:
                return None
            raise ValueError("%s is required" % name)
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("%s: expected a contiguous device tensor" % name)
        if t.device.index != torch.cuda.current_device():
            raise ValueError("%s lives on %s, the current device is %d" % (name, t.device, torch.cuda.current_device()))
        if kind == "f32":
            if t.dtype != torch.float32:
                raise ValueError("%s: expected float32, got %s" % (name, t.dtype))
            have = t.numel()
        elif kind == "f16":
            if t.dtype != torch.float16:
                raise ValueError("%s: expected float16, got %s" % (name, t.dtype))
            have = t.numel()
        elif kind == "f64":
            if t.dtype != torch.float64:
                raise ValueError("%s: expected float64, got %s" % (name, t.dtype))
            have = t.numel()
        else:                                   # "bytes": any integer type, size counted in bytes
            if t.dtype.is_floating_point or t.dtype.is_complex:
                raise ValueError("%s: expected an integer tensor, got %s" % (name, t.dtype))
            have = t.numel() * t.element_size()
        if have < numel:
            raise ValueError("%s holds %d %s, the call needs %d" % (name, have, "bytes" if kind == "bytes" else "elements", numel))
        return t.data_ptr()

    def _bufs(self, ts, name, numel, kind="f32", optional=False):
        if ts is None:
            if optional:
                return None
            raise ValueError("%s is required" % name)
        if len(ts) != self.num_workers:
            raise ValueError("%s: expected %d tensors (one per worker), got %d" % (name, self.num_workers, len(ts)))
        arr = (C.c_void_p * len(ts))()
        for i, t in enumerate(ts):
            arr[i] = self._buf(t, "%s[%d]" % (name, i), numel, kind)
        return arr

    # the calls ---------------------------------------------------------------------------------
    def worker_quantize(self, worker, step, grad, err, codes, scales, stream=None):
        P, L = self.num_params, self.num_segments
        self._check(self._lib.qadam_worker_quantize(
            self._h, worker, step, self._buf(grad, "grad", P), self._buf(err, "err", P),
            self._buf(codes, "codes", self.grad_code_bytes(), "bytes"), self._buf(scales, "scales", L),
            _stream(stream)))

    def server_step(self, step, lr, beta2, codes, scales, x, m, v, stream=None):
        P, L = self.num_params, self.num_segments
        self._check(self._lib.qadam_server_step(
            self._h, step, lr, beta2, self._bufs(codes, "codes", self.grad_code_bytes(), "bytes"),
            self._bufs(scales, "scales", L), self._buf(x, "x", P), self._buf(m, "m", P), self._buf(v, "v", P),
            _stream(stream)))

    def weight_quantize(self, step, x, werr, wcodes, stream=None):
        P = self.num_params
        self._check(self._lib.qadam_weight_quantize(
            self._h, step, self._buf(x, "x", P), self._buf(werr, "werr", P, optional=self.cfg.weight_ef == 0),
            self._buf(wcodes, "wcodes", self.weight_code_bytes(), "bytes"), _stream(stream)))

    def _server_side(self, werr, wcodes):
        idx = self.cfg.k_x == QADAM_IDENTITY
        P = self.num_params
        if idx:                                     # Q_x = id: no weight codes, no residual
            return None, None
        return (self._buf(werr, "werr", P, optional=self.cfg.weight_ef == 0),
                self._buf(wcodes, "wcodes", self.weight_code_bytes(), "bytes"))

    def step_fused(self, step, lr, beta2, grads, errs, codes, scales, x, m, v, werr, wcodes, stream=None):
        P, L = self.num_params, self.num_segments
        idg = self.cfg.k_g == QADAM_IDENTITY
        pw, pc = self._server_side(werr, wcodes)
        self._check(self._lib.qadam_step_fused(
            self._h, step, lr, beta2, self._bufs(grads, "grads", P),
            None if idg else self._bufs(errs, "errs", P),          # Q_g = id: errs, codes, scales are not used
            None if idg else self._bufs(codes, "codes", self.grad_code_bytes(), "bytes"),
            None if idg else self._bufs(scales, "scales", L), self._buf(x, "x", P), self._buf(m, "m", P),
            self._buf(v, "v", P), pw, pc, _stream(stream)))

    def worker_step_w(self, worker, step, lr, beta2, grad, mw, vw, err, codes, scales, stream=None):
        P, L = self.num_params, self.num_segments
        self._check(self._lib.qadam_worker_step_w(
            self._h, worker, step, lr, beta2, self._buf(grad, "grad", P), self._buf(mw, "mw", P),
            self._buf(vw, "vw", P), self._buf(err, "err", P),
            self._buf(codes, "codes", self.grad_code_bytes(), "bytes"), self._buf(scales, "scales", L),
            _stream(stream)))

    def step_fused_w(self, step, lr, beta2, grads, mw, vw, errs, codes, scales, x, werr, wcodes, stream=None):
        P, L = self.num_params, self.num_segments
        idg = self.cfg.k_g == QADAM_IDENTITY
        pw, pc = self._server_side(werr, wcodes)
        self._check(self._lib.qadam_step_fused_w(
            self._h, step, lr, beta2, self._bufs(grads, "grads", P), self._bufs(mw, "mw", P),
            self._bufs(vw, "vw", P), self._bufs(errs, "errs", P),
            None if idg else self._bufs(codes, "codes", self.grad_code_bytes(), "bytes"),
            None if idg else self._bufs(scales, "scales", L), self._buf(x, "x", P), pw, pc, _stream(stream)))

    def server_apply_w(self, step, codes, scales, x, stream=None):
        P, L = self.num_params, self.num_segments
        self._check(self._lib.qadam_server_apply_w(
            self._h, step, self._bufs(codes, "codes", self.grad_code_bytes(), "bytes"),
            self._bufs(scales, "scales", L), self._buf(x, "x", P), _stream(stream)))

    def weight_dequantize(self, wcodes, xhat, stream=None):
        self._check(self._lib.qadam_weight_dequantize(
            self._h, self._buf(wcodes, "wcodes", self.weight_code_bytes(), "bytes"),
            self._buf(xhat, "xhat", self.num_params), _stream(stream)))

    def weight_dequantize_f16(self, wcodes, xhat_half, stream=None):
        self._check(self._lib.qadam_weight_dequantize_f16(
            self._h, self._buf(wcodes, "wcodes", self.weight_code_bytes(), "bytes"),
            self._buf(xhat_half, "xhat_half", self.num_params, "f16"), _stream(stream)))

    def layer_sumsq(self, a, b, out, stream=None):
        """out[l] = sum over layer l of (a + b)^2 in fp64 (b may be None)."""
        P = self.num_params
        self._check(self._lib.qadam_layer_sumsq(self._h, self._buf(a, "a", P), self._buf(b, "b", P, optional=True),
                                                self._buf(out, "out", self.num_segments, "f64"), _stream(stream)))

    def arena_layout(self, arena_bytes, with_worker_moments=False):
        """qadam_arena_layout: dict of byte offsets (lists per worker) inside one caller-allocated block;
        `bytes_needed` is the smallest block that fits.  Host arithmetic only."""
        a = _Arena()
        rc = self._lib.qadam_arena_layout(self._h, int(arena_bytes), int(bool(with_worker_moments)), C.byref(a))
        if rc == QADAM_ERANGE:
            raise QAdamError(rc, "the block of %d bytes is smaller than the %d bytes the buffers need"
                             % (arena_bytes, a.bytes_needed))
        self._check(rc)
        N = self.num_workers
        out = {n: int(getattr(a, n)) for n in ("x", "m", "v", "werr", "wcodes", "bytes_needed")}
        for n in ("grads", "errs", "codes", "scales"):
            out[n] = [int(getattr(a, n)[i]) for i in range(N)]
        if with_worker_moments:
            for n in ("mw", "vw"):
                out[n] = [int(getattr(a, n)[i]) for i in range(N)]
        return out

    def trust_error_buffers(self, on=1):
        """Opt in to the filtered scale pass (see include/qadam.h for the contract):
        0 off, 1 where it pays, 2 always, 3 full pass plus a check of the contract (status bit 2)."""
        self._check(self._lib.qadam_trust_error_buffers(self._h, int(on)))

    def profile_enable(self, on=True):
        self._check(self._lib.qadam_profile_enable(self._h, int(on)))

    def profile_read(self):
        """(scale_pass_ms, main_pass_ms) of the last qadam_step_fused call; waits for it."""
        pr = _Profile()
        self._check(self._lib.qadam_profile_read(self._h, C.byref(pr)))
        return float(pr.scale_pass_ms), float(pr.main_pass_ms)

    def get_status(self, clear=False, stream=None) -> int:
        st = _Status()
        self._check(self._lib.qadam_get_status(self._h, C.byref(st), int(clear), _stream(stream)))
        return int(st.flags)
