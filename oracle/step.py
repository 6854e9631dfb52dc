"""TEST INFRASTRUCTURE.  numpy-facing wrapper around ``step.c``.

Argument marshalling only: every arithmetic step of the oracle is in the C
file.  Arrays are host numpy arrays; bf16 data travels as ``uint16`` bit
patterns.
"""
import ctypes as C
import os
import sys

import numpy as np

from . import build as _build

_lib = None


class Scalars(C.Structure):
    _fields_ = [(k, C.c_float) for k in
                ("gs", "cc", "b1", "omb1", "b2", "omb2", "ep", "step", "isb2", "lw")]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


def lib():
    global _lib
    if _lib is None:
        path = os.environ.get("PS_ORACLE_LIB_UNDER_TEST")
        if path:
            # tests/test_oracle_mutants.py points this at a deliberately broken build to
            # show that the pins notice; nothing else sets it
            print("oracle: loading %s instead of the built oracle" % path, file=sys.stderr)
        else:
            path = _build.LIB
            if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
                _build.build()
        L = C.CDLL(path)
        pp = C.POINTER(C.c_void_p)
        L.oracle_widen_bf16.restype = C.c_float
        L.oracle_widen_bf16.argtypes = [C.c_uint16]
        L.oracle_bf16_rne.restype = C.c_uint16
        L.oracle_bf16_rne.argtypes = [C.c_float]
        L.oracle_bf16_rne_array.restype = None
        L.oracle_bf16_rne_array.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64]
        L.oracle_widen_f16.restype = C.c_float
        L.oracle_widen_f16.argtypes = [C.c_uint16]
        L.oracle_f16_rne.restype = C.c_uint16
        L.oracle_f16_rne.argtypes = [C.c_float]
        L.oracle_f16_rne_array.restype = None
        L.oracle_f16_rne_array.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64]
        L.oracle_derive_scalars.restype = None
        L.oracle_derive_scalars.argtypes = [C.c_double] * 5 + [C.c_uint64, C.c_uint32,
                                                               C.c_double, C.c_double,
                                                               C.POINTER(Scalars)]
        L.oracle_reduce_sum.restype = None
        L.oracle_reduce_sum.argtypes = [pp, C.c_uint32, C.c_int, C.c_void_p,
                                        C.c_uint64, C.c_uint64]
        L.oracle_accumulate.restype = None
        L.oracle_accumulate.argtypes = [pp, C.c_uint32, C.c_int, C.c_void_p, C.c_int,
                                        C.c_uint64, C.c_uint64]
        L.oracle_diff_sumsq.restype = None
        L.oracle_diff_sumsq.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_uint64, C.c_uint64,
                                        C.POINTER(C.c_double)]
        L.oracle_checksum.restype = C.c_uint64
        L.oracle_checksum.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64]
        L.oracle_mean_sumsq.restype = C.c_double
        L.oracle_mean_sumsq.argtypes = [pp, C.c_uint32, C.c_int, C.c_float, C.c_void_p,
                                        C.c_uint64, C.c_uint64]
        L.oracle_clip_coef.restype = C.c_double
        L.oracle_clip_coef.argtypes = [C.c_double] * 3
        L.oracle_step_f32.restype = None
        L.oracle_step_f32.argtypes = [pp, C.c_uint32, C.c_int, C.POINTER(Scalars),
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                      C.c_uint64, C.c_uint64]
        L.oracle_step_f64.restype = None
        L.oracle_step_f64.argtypes = ([pp, C.c_uint32, C.c_int] + [C.c_double] * 5 +
                                      [C.c_uint64, C.c_double, C.c_double] +
                                      [C.c_void_p] * 6 + [C.c_uint64, C.c_uint64])
        _lib = L
    return _lib


def _contrib_ptrs(grads):
    """grads: list of equally long 1-D arrays, all uint16 (bf16 bits), all float32 or all
    float16.  Returns (pointer array, count, dtype code 0/1/2, length)."""
    if not grads:
        raise ValueError("need at least one contribution")
    dt = grads[0].dtype
    codes = {np.dtype(np.uint16): 0, np.dtype(np.float32): 1, np.dtype(np.float16): 2}
    if dt not in codes:
        raise TypeError("contributions must be uint16 (bf16 bits), float32 or float16")
    n = grads[0].shape[0]
    for g in grads:
        if g.dtype != dt or g.ndim != 1 or g.shape[0] != n or not g.flags.c_contiguous:
            raise ValueError("contributions must share dtype/length and be contiguous")
    arr = (C.c_void_p * len(grads))(*[g.ctypes.data for g in grads])
    return arr, len(grads), codes[dt], n


def _check(a, dtype, n):
    if a.dtype != np.dtype(dtype) or a.ndim != 1 or a.shape[0] != n or not a.flags.c_contiguous:
        raise ValueError("bad array: want contiguous %s[%d]" % (np.dtype(dtype), n))


def derive_scalars(lr, beta1, beta2, eps, weight_decay, t, n_devices,
                   grad_scale=0.0, clip_coef=0.0):
    s = Scalars()
    lib().oracle_derive_scalars(lr, beta1, beta2, eps, weight_decay, int(t), int(n_devices),
                                float(grad_scale), float(clip_coef), C.byref(s))
    return s


def widen_bf16(bits):
    return lib().oracle_widen_bf16(int(bits))


def bf16_rne(x):
    return lib().oracle_bf16_rne(float(np.float32(x)))


def bf16_rne_bits(u32):
    """Cast arbitrary binary32 bit patterns (uint32 array) -> uint16 array."""
    u32 = np.ascontiguousarray(u32, dtype=np.uint32)
    out = np.empty(u32.shape[0], dtype=np.uint16)
    lib().oracle_bf16_rne_array(u32.ctypes.data, out.ctypes.data, u32.shape[0])
    return out


def widen_f16(bits):
    return lib().oracle_widen_f16(int(bits))


def f16_rne_bits(u32):
    """Cast arbitrary binary32 bit patterns (uint32 array) -> binary16 bit patterns (uint16)."""
    u32 = np.ascontiguousarray(u32, dtype=np.uint32)
    out = np.empty(u32.shape[0], dtype=np.uint16)
    lib().oracle_f16_rne_array(u32.ctypes.data, out.ctypes.data, u32.shape[0])
    return out


def reduce_sum(grads, lo=0, hi=None):
    ptrs, n_c, dtype, n = _contrib_ptrs(grads)
    hi = n if hi is None else hi
    acc = np.zeros(n, dtype=np.float32)
    lib().oracle_reduce_sum(ptrs, n_c, dtype, acc.ctypes.data, lo, hi)
    return acc


def accumulate(grads, accum, overwrite, lo=0, hi=None):
    """accum[lo:hi] (+)= fixed-order sum of one micro-batch's contributions, in place."""
    ptrs, n_c, dtype, n = _contrib_ptrs(grads)
    hi = n if hi is None else hi
    _check(accum, np.float32, n)
    lib().oracle_accumulate(ptrs, n_c, dtype, accum.ctypes.data, int(bool(overwrite)), lo, hi)


def mean_sumsq(grads, gs, lo=0, hi=None, want_mean=True):
    ptrs, n_c, dtype, n = _contrib_ptrs(grads)
    hi = n if hi is None else hi
    gm = np.zeros(n, dtype=np.float32) if want_mean else None
    ss = lib().oracle_mean_sumsq(ptrs, n_c, dtype, float(np.float32(gs)),
                                 gm.ctypes.data if want_mean else None, lo, hi)
    return gm, ss


def clip_coef(sumsq_local, sumsq_others, max_norm):
    return lib().oracle_clip_coef(sumsq_local, sumsq_others, max_norm)


def step_f32(grads, scalars, theta, m, v, p, lo=0, hi=None):
    """In-place binary32 step on [lo, hi) of the full-length arrays.  p is uint16 (receives
    bf16 bit patterns) or float16 (receives the binary16 image)."""
    ptrs, n_c, dtype, n = _contrib_ptrs(grads)
    hi = n if hi is None else hi
    for a in (theta, m, v):
        _check(a, np.float32, n)
    p_f16 = p.dtype == np.dtype(np.float16)
    _check(p, np.float16 if p_f16 else np.uint16, n)
    if not (0 <= lo <= hi <= n):
        raise ValueError("bad range")
    lib().oracle_step_f32(ptrs, n_c, dtype, C.byref(scalars), theta.ctypes.data,
                          m.ctypes.data, v.ctypes.data, p.ctypes.data, int(p_f16), lo, hi)


def step_f64(grads, lr, beta1, beta2, eps, weight_decay, t, theta, m, v,
             grad_scale=0.0, clip_coef=0.0, lo=0, hi=None):
    """Binary64 pass; returns (theta', m', v') as float64 arrays (zeros outside [lo,hi))."""
    ptrs, n_c, dtype, n = _contrib_ptrs(grads)
    hi = n if hi is None else hi
    for a in (theta, m, v):
        _check(a, np.float32, n)
    to, mo, vo = (np.zeros(n, dtype=np.float64) for _ in range(3))
    lib().oracle_step_f64(ptrs, n_c, dtype, lr, beta1, beta2, eps, weight_decay, int(t),
                          float(grad_scale), float(clip_coef), theta.ctypes.data,
                          m.ctypes.data, v.ctypes.data, to.ctypes.data, mo.ctypes.data,
                          vo.ctypes.data, lo, hi)
    return to, mo, vo


def diff_sumsq(a, b, lo=0, hi=None):
    """(sum (a-b)^2, sum a^2) over [lo, hi), sequential binary64."""
    ptrs, _, dtype, n = _contrib_ptrs([a, b])
    hi = n if hi is None else hi
    out = (C.c_double * 2)()
    lib().oracle_diff_sumsq(a.ctypes.data, b.ctypes.data, dtype, lo, hi, out)
    return out[0], out[1]


def checksum(buf, first_index=0):
    """Checksum of a contiguous array whose byte length is a multiple of 8."""
    raw = np.ascontiguousarray(buf).view(np.uint8)
    if raw.shape[0] % 8:
        raise ValueError("byte length must be a multiple of 8")
    return lib().oracle_checksum(raw.ctypes.data, raw.shape[0] // 8, int(first_index))
