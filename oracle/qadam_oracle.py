"""ctypes front end of the CPU oracle (``qadam_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
``cpu_baseline`` leg of the benchmark; never by the product path.  This file
only marshals numpy arrays into the C functions -- all arithmetic of the method
lives in the C source, which cites the passages of arXiv 2004.14180 it follows.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qadam_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_qadam.so")

CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a second or two)."""
    stale = (not os.path.exists(_LIB)) or any(
        os.path.getmtime(os.path.join(_HERE, f)) > os.path.getmtime(_LIB)
        for f in ("qadam_oracle.c", "qadam_oracle.h"))
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def build_selftest() -> str:
    """Compile the memory-safety driver (sanitize_selftest.c) plainly, as a does-it-build check; the
    sanitizer run itself is tests/test_oracle_sanitizers.py."""
    exe = os.path.join(_HERE, "sanitize_selftest.bin")
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-ffp-contract=off", "-o", exe,
                           os.path.join(_HERE, "sanitize_selftest.c"), _SRC, "-lm"])
    return exe


class _Cfg(C.Structure):
    _fields_ = [("k_g", C.c_int32), ("k_x", C.c_int32), ("rounding", C.c_int32),
                ("weight_ef", C.c_int32), ("adam_flavor", C.c_int32),
                ("identity_g", C.c_int32), ("identity_x", C.c_int32),
                ("beta1", C.c_float), ("eps", C.c_float), ("seed", C.c_uint64)]


@dataclass
class OracleConfig:
    k_g: int = 2
    k_x: int = 6
    rounding: int = 0
    weight_ef: int = 1
    adam_flavor: int = 0
    identity_g: int = 0
    identity_x: int = 0
    beta1: float = 0.9
    eps: float = 1e-8
    seed: int = 0

    def c(self) -> _Cfg:
        return _Cfg(self.k_g, self.k_x, self.rounding, self.weight_ef, self.adam_flavor,
                    self.identity_g, self.identity_x, self.beta1, self.eps, self.seed)


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oq_uniform24.restype = C.c_float
        _lib.oq_uniform24.argtypes = [C.c_uint64, C.c_int64, C.c_int64, C.c_int32, C.c_int32]
        _lib.oq_grad_code_bits.restype = C.c_int32
        _lib.oq_grad_code_words_segment.restype = C.c_int64
        _lib.oq_grad_code_words_segment.argtypes = [C.c_int32, C.c_int64]
        _lib.oq_grad_code_words.restype = C.c_int64
        _lib.oq_weight_code_bytes_per_elem.restype = C.c_int32
        _lib.oq_qg_decode.restype = C.c_float
        _lib.oq_qg_decode.argtypes = [C.c_int32, C.c_float, C.c_uint8]
    return _lib


def _p(a, ty=C.c_void_p):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ty)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _ptr_array(arrs):
    if arrs is None:
        return None
    arr = (C.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        arr[i] = a.ctypes.data if a is not None else None
    return arr


def _segs(seg_off):
    s = np.ascontiguousarray(seg_off, dtype=np.int64)
    assert s[0] == 0 and np.all(np.diff(s) >= 0)
    return s


# ----------------------------------------------------------------------------
def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    out = (C.c_uint32 * 4)()
    lib().oq_philox4x32_10(c, k, out)
    return [int(v) for v in out]


def uniform24(seed, j, step, worker, stream):
    return float(lib().oq_uniform24(seed, j, step, worker, stream))


def grad_code_bits(k_g):
    return int(lib().oq_grad_code_bits(C.c_int32(k_g)))


def grad_code_words(k_g, seg_off):
    s = _segs(seg_off)
    return int(lib().oq_grad_code_words(C.c_int32(k_g), _p(s), C.c_int32(len(s) - 1)))


def weight_code_dtype(k_x):
    return np.int8 if lib().oq_weight_code_bytes_per_elem(C.c_int32(k_x)) == 1 else np.int16


def qg_layer(cfg: OracleConfig, p, j0=0, step=1, worker=0):
    """Q_g on one layer: returns (status, s, code[n] uint8, q[n], tie[n])."""
    p = _f32(p)
    n = p.size
    s = C.c_float(0)
    code = np.zeros(n, np.uint8)
    q = np.zeros(n, np.float32)
    tie = np.zeros(n, np.uint8)
    cc = cfg.c()
    st = lib().oq_qg_layer(C.byref(cc), _p(p), C.c_int64(n), C.c_int64(j0), C.c_int64(step),
                           C.c_int32(worker), C.byref(s), _p(code), _p(q), _p(tie))
    return st, np.float32(s.value), code, q, tie


def qg_decode(k_g, s, code):
    return np.array([lib().oq_qg_decode(k_g, float(s), int(c)) for c in np.asarray(code).ravel()],
                    dtype=np.float32)


def worker_quantize_window(cfg, grad, err, s, j0=0, step=1, worker=0):
    """Worker side on a window with the layer scale given; err updated in place.
    Returns (code, tie, q)."""
    grad = _f32(grad)
    assert err.dtype == np.float32 and err.flags["C_CONTIGUOUS"]
    n = grad.size
    code = np.zeros(n, np.uint8)
    tie = np.zeros(n, np.uint8)
    q = np.zeros(n, np.float32)
    cc = cfg.c()
    lib().oq_worker_quantize_window(C.byref(cc), C.c_int64(n), C.c_int64(j0), C.c_int32(worker),
                                    C.c_int64(step), C.c_float(float(s)), _p(grad), _p(err),
                                    _p(code), _p(tie), _p(q))
    return code, tie, q


def qx(cfg: OracleConfig, y, j0=0, step=1):
    """Q_x element-wise: returns (j[n] int32, xhat[n], tie[n])."""
    y = _f32(y)
    n = y.size
    j = np.zeros(n, np.int32)
    xh = np.zeros(n, np.float32)
    tie = np.zeros(n, np.uint8)
    cc = cfg.c()
    lib().oq_qx(C.byref(cc), _p(y), C.c_int64(n), C.c_int64(j0), C.c_int64(step), _p(j), _p(xh), _p(tie))
    return j, xh, tie


def pack_codes(bits, code):
    code = np.ascontiguousarray(code, dtype=np.uint8)
    n = code.size
    groups = (n + 31) // 32
    words = np.zeros((groups * bits + 3) // 4 * 4, np.uint32)
    lib().oq_pack_codes(C.c_int32(bits), _p(code), C.c_int64(n), _p(words))
    return words


def unpack_codes(bits, words, n):
    words = np.ascontiguousarray(words, dtype=np.uint32)
    code = np.zeros(n, np.uint8)
    lib().oq_unpack_codes(C.c_int32(bits), _p(words), C.c_int64(n), _p(code))
    return code


def unpack_all(k_g, seg_off, words):
    """Per-element codes of a whole packed vector (all segments)."""
    s = _segs(seg_off)
    bits = grad_code_bits(k_g)
    out = np.zeros(int(s[-1]), np.uint8)
    woff = 0
    for l in range(len(s) - 1):
        n = int(s[l + 1] - s[l])
        nw = int(lib().oq_grad_code_words_segment(k_g, n))
        out[s[l]:s[l + 1]] = unpack_codes(bits, words[woff:woff + nw], n)
        woff += nw
    return out


def adam_update(cfg, lr, beta2, step, g, m, v):
    """In-place m, v; returns the step u."""
    g = _f32(g)
    u = np.zeros_like(g)
    cc = cfg.c()
    lib().oq_adam_update(C.byref(cc), C.c_float(lr), C.c_float(beta2), C.c_int64(step),
                         _p(g), _p(m), _p(v), _p(u), C.c_int64(g.size))
    return u


def worker_quantize(cfg, seg_off, worker, step, grad, err, index_base=0,
                    want_tie=True, want_q=False):
    """err updated in place.  Returns dict(status, words, codes, scales, tie, q)."""
    s = _segs(seg_off)
    L = len(s) - 1
    P = int(s[-1])
    grad = _f32(grad)
    assert err.dtype == np.float32 and err.size == P and grad.size == P
    words = np.zeros(grad_code_words(cfg.k_g, s), np.uint32)
    codes = np.zeros(P, np.uint8)
    scales = np.zeros(L, np.float32)
    tie = np.zeros(P, np.uint8) if want_tie else None
    q = np.zeros(P, np.float32) if want_q else None
    cc = cfg.c()
    st = lib().oq_worker_quantize(C.byref(cc), _p(s), C.c_int32(L), C.c_int64(index_base),
                                  C.c_int32(worker), C.c_int64(step), _p(grad), _p(err),
                                  _p(words), _p(codes), _p(scales), _p(tie), _p(q))
    return dict(status=st, words=words, codes=codes, scales=scales, tie=tie, q=q)


def server_step(cfg, seg_off, step, lr, beta2, words, scales, x, m, v):
    s = _segs(seg_off)
    N = len(words)
    cc = cfg.c()
    lib().oq_server_step(C.byref(cc), _p(s), C.c_int32(len(s) - 1), C.c_int32(N), C.c_int64(step),
                         C.c_float(lr), C.c_float(beta2), _ptr_array(words), _ptr_array(scales),
                         _p(x), _p(m), _p(v))


def weight_quantize(cfg, step, x, werr, index_base=0, want_tie=True):
    """werr (may be None when weight_ef == 0) updated in place.
    Returns dict(wcodes, xhat, tie)."""
    P = x.size
    wcodes = np.zeros(P, weight_code_dtype(cfg.k_x))
    xhat = np.zeros(P, np.float32)
    tie = np.zeros(P, np.uint8) if want_tie else None
    cc = cfg.c()
    lib().oq_weight_quantize(C.byref(cc), C.c_int64(P), C.c_int64(index_base), C.c_int64(step),
                             _p(x), _p(werr), _p(wcodes), _p(xhat), _p(tie))
    return dict(wcodes=wcodes, xhat=xhat, tie=tie)


def _step_common(cfg, seg_off, N, want_tie):
    s = _segs(seg_off)
    L = len(s) - 1
    P = int(s[-1])
    nw = grad_code_words(cfg.k_g, s)
    words = [np.zeros(nw, np.uint32) for _ in range(N)]
    scales = [np.zeros(L, np.float32) for _ in range(N)]
    wcodes = np.zeros(P, weight_code_dtype(cfg.k_x))
    tie_g = [np.zeros(P, np.uint8) for _ in range(N)] if want_tie else None
    tie_x = np.zeros(P, np.uint8) if want_tie else None
    return s, L, P, words, scales, wcodes, tie_g, tie_x


def step_s(cfg, seg_off, step, lr, beta2, grads, errs, x, m, v, werr,
           index_base=0, want_tie=True):
    """One step of variant S; errs, x, m, v, werr updated in place."""
    N = len(grads)
    s, L, P, words, scales, wcodes, tie_g, tie_x = _step_common(cfg, seg_off, N, want_tie)
    grads = [_f32(g) for g in grads]
    cc = cfg.c()
    st = lib().oq_step_s(C.byref(cc), _p(s), C.c_int32(L), C.c_int32(N), C.c_int64(index_base),
                         C.c_int64(step), C.c_float(lr), C.c_float(beta2),
                         _ptr_array(grads), _ptr_array(errs), _ptr_array(words), _ptr_array(scales),
                         _p(x), _p(m), _p(v), _p(werr), _p(wcodes),
                         _ptr_array(tie_g), _p(tie_x))
    return dict(status=st, words=words, scales=scales, wcodes=wcodes, tie_g=tie_g, tie_x=tie_x)


def step_s_window(cfg, j0, step, lr, beta2, scales, grads, errs, x, m, v, werr, want_tie=True):
    """Variant S on a window of one layer, scales[i] = the workers' layer scales.
    Returns dict(status, codes (per element, per worker), wcodes, tie_g, tie_x)."""
    N = len(grads)
    n = x.size
    grads = [_f32(g) for g in grads]
    s = np.ascontiguousarray(scales, dtype=np.float32)
    codes = [np.zeros(n, np.uint8) for _ in range(N)]
    wcodes = np.zeros(n, weight_code_dtype(cfg.k_x))
    tie_g = [np.zeros(n, np.uint8) for _ in range(N)] if want_tie else None
    tie_x = np.zeros(n, np.uint8) if want_tie else None
    cc = cfg.c()
    st = lib().oq_step_s_window(C.byref(cc), C.c_int64(n), C.c_int64(j0), C.c_int32(N), C.c_int64(step),
                                C.c_float(lr), C.c_float(beta2), _p(s), _ptr_array(grads),
                                _ptr_array(errs), _p(x), _p(m), _p(v), _p(werr), _ptr_array(codes),
                                _p(wcodes), _ptr_array(tie_g), _p(tie_x))
    return dict(status=st, codes=codes, wcodes=wcodes, tie_g=tie_g, tie_x=tie_x)


def step_w(cfg, seg_off, step, lr, beta2, grads, errs, mw, vw, x, werr,
           index_base=0, want_tie=True):
    """One step of variant W (Algorithms 2-3); errs, mw, vw, x, werr in place."""
    N = len(grads)
    s, L, P, words, scales, wcodes, tie_g, tie_x = _step_common(cfg, seg_off, N, want_tie)
    grads = [_f32(g) for g in grads]
    cc = cfg.c()
    st = lib().oq_step_w(C.byref(cc), _p(s), C.c_int32(L), C.c_int32(N), C.c_int64(index_base),
                         C.c_int64(step), C.c_float(lr), C.c_float(beta2),
                         _ptr_array(grads), _ptr_array(errs), _ptr_array(mw), _ptr_array(vw),
                         _ptr_array(words), _ptr_array(scales),
                         _p(x), _p(werr), _p(wcodes), _ptr_array(tie_g), _p(tie_x))
    return dict(status=st, words=words, scales=scales, wcodes=wcodes, tie_g=tie_g, tie_x=tie_x)
