"""ctypes front end of the CPU oracle (co2_oracle.cpp) -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the bench's CPU-baseline leg may import this
module.  It compiles co2_oracle.cpp with g++ (-O2 -ffp-contract=off) into
libco2_oracle.so next to the source and marshals numpy arrays; every bit of
arithmetic happens in the C++ loops.  It imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "co2_oracle.cpp")
_LIB = os.path.join(_HERE, "libco2_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle shared library; returns its path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math",
               "-fPIC", "-shared", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_ENTRY_POINTS = ("co2_oracle_sqnorms", "co2_oracle_outer_step_f32", "co2_oracle_outer_step_f64",
                 "co2_oracle_outer_step_variant_f32", "co2_oracle_outer_step_f16",
                 "co2_oracle_outer_step_bf16", "co2_oracle_adamw_f32", "co2_oracle_adamw_f64")


def _open(path):
    lib = C.CDLL(path)
    for name in _ENTRY_POINTS:
        getattr(lib, name).restype = C.c_int
    lib.co2_oracle_f32_to_bf16.restype = C.c_uint16
    lib.co2_oracle_f32_to_bf16.argtypes = [C.c_float]
    lib.co2_oracle_bf16_to_f32.restype = C.c_float
    lib.co2_oracle_bf16_to_f32.argtypes = [C.c_uint16]
    lib.co2_oracle_f32_to_f16.restype = C.c_uint16
    lib.co2_oracle_f32_to_f16.argtypes = [C.c_float]
    lib.co2_oracle_f16_to_f32.restype = C.c_float
    lib.co2_oracle_f16_to_f32.argtypes = [C.c_uint16]
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _open(build())
    return _lib


class use_library:
    """Context manager for tests of the pins themselves: route every call of this
    module to another build of the oracle source (e.g. one with a planted mistake)."""

    def __init__(self, path):
        self.path = path

    def __enter__(self):
        global _lib
        self.saved = _lib
        _lib = _open(self.path)
        return self

    def __exit__(self, *exc):
        global _lib
        _lib = self.saved
        return False


def compile_source(src_path: str, out_path: str) -> str:
    """Compile an oracle source file (the real one or a mutated copy) with the real flags."""
    subprocess.run(["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC",
                    "-shared", "-o", out_path, src_path], check=True)
    return out_path


def _ptr(a, dtype):
    if a is None:
        return None
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags.c_contiguous, (
        f"need contiguous {dtype} array")
    return a.ctypes.data_as(C.c_void_p)


def _table(n, seg_off):
    t = np.ascontiguousarray(np.asarray(seg_off, dtype=np.int64))
    assert t.ndim == 1 and t.size >= 2
    return t, t.size - 1


def _ptr_array(arrs, dtype):
    ptrs = (C.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        ptrs[i] = _ptr(a, dtype).value
    return ptrs


def sqnorms(buf, seg_off, phi: float = 0.0):
    """Per-segment sums of squares (fp64); phi > 0 clips coordinate-wise first."""
    lib = _load()
    t, S = _table(buf.size, seg_off)
    out = np.empty(S, dtype=np.float64)
    rc = lib.co2_oracle_sqnorms(C.c_int64(buf.size), C.c_int32(S), _ptr(t, np.int64),
                                _ptr(buf, np.float32), C.c_float(phi), _ptr(out, np.float64))
    if rc:
        raise ValueError("co2_oracle_sqnorms rejected its arguments")
    return out


def outer_step_f32(*, seg_off, alpha, beta, phi, c, tau, step, x, a, m, deltas,
                   a_out=None, first_step_norm=None):
    """One outer update, in place on x (may be None), m, and a (or into a_out).

    Returns dict(dout, lam, M2, T, nclipped)."""
    lib = _load()
    n = a.size
    t, S = _table(n, seg_off)
    if a_out is None:
        a_out = a
    dout = np.empty(n, dtype=np.float32) if x is not None else None
    lam = np.empty(S, dtype=np.float32)
    M2 = np.empty(S, dtype=np.float64)
    T = np.empty(S, dtype=np.float64)
    ncl = C.c_int64(0)
    K = len(deltas) if deltas is not None else 1
    dptr = _ptr_array(deltas, np.float32) if deltas is not None else None
    rc = lib.co2_oracle_outer_step_f32(
        C.c_int64(n), C.c_int32(S), _ptr(t, np.int64), C.c_int32(K),
        C.c_float(alpha), C.c_float(beta), C.c_float(phi), C.c_float(c),
        C.c_int32(tau), C.c_int64(step),
        _ptr(x, np.float32), _ptr(a, np.float32), _ptr(a_out, np.float32),
        _ptr(m, np.float32), dptr, _ptr(dout, np.float32),
        _ptr(first_step_norm, np.float32), _ptr(lam, np.float32),
        _ptr(M2, np.float64), _ptr(T, np.float64), C.byref(ncl))
    if rc:
        raise ValueError("co2_oracle_outer_step_f32 rejected its arguments")
    return dict(dout=dout, lam=lam, M2=M2, T=T, nclipped=ncl.value)


def outer_step_f64(*, seg_off, alpha, beta, phi, c, tau, step, x, a, m, deltas,
                   a_out=None, first_step_norm=None):
    """All-fp64 evaluation of the same update; arrays are float64, in place."""
    lib = _load()
    n = a.size
    t, S = _table(n, seg_off)
    if a_out is None:
        a_out = a
    dout = np.empty(n, dtype=np.float64) if x is not None else None
    lam = np.empty(S, dtype=np.float64)
    K = len(deltas) if deltas is not None else 1
    dptr = _ptr_array(deltas, np.float64) if deltas is not None else None
    rc = lib.co2_oracle_outer_step_f64(
        C.c_int64(n), C.c_int32(S), _ptr(t, np.int64), C.c_int32(K),
        C.c_double(alpha), C.c_double(beta), C.c_double(phi), C.c_double(c),
        C.c_int32(tau), C.c_int64(step),
        _ptr(x, np.float64), _ptr(a, np.float64), _ptr(a_out, np.float64),
        _ptr(m, np.float64), dptr, _ptr(dout, np.float64),
        _ptr(first_step_norm, np.float64), _ptr(lam, np.float64))
    if rc:
        raise ValueError("co2_oracle_outer_step_f64 rejected its arguments")
    return dict(dout=dout, lam=lam)


def outer_step_variant_f32(*, seg_off, alpha, beta, phi, c, tau, step, x, a, m, deltas,
                           nonstale=False, norm_clip=False, pull_rho=1.0, a_out=None,
                           first_step_norm=None):
    """The outer update with the variant switches of co2_oracle_outer_step_variant_f32
    (current-round mean, norm-rescale clip, anchor pull); in place like outer_step_f32.
    With `nonstale`, deltas[0] is not read and may be None.
    Returns dict(dout, lam, scale, nclipped)."""
    lib = _load()
    n = a.size
    t, S = _table(n, seg_off)
    if a_out is None:
        a_out = a
    dout = np.empty(n, dtype=np.float32) if x is not None else None
    lam = np.empty(S, dtype=np.float32)
    scale = np.empty(S, dtype=np.float32)
    ncl = C.c_int64(0)
    K = len(deltas) if deltas is not None else 1
    dptr = None
    if deltas is not None:
        dptr = (C.c_void_p * K)()
        for i, arr in enumerate(deltas):
            dptr[i] = None if arr is None else _ptr(arr, np.float32).value
    rc = lib.co2_oracle_outer_step_variant_f32(
        C.c_int64(n), C.c_int32(S), _ptr(t, np.int64), C.c_int32(K),
        C.c_float(alpha), C.c_float(beta), C.c_float(phi), C.c_float(c),
        C.c_int32(tau), C.c_int64(step), C.c_int32(int(nonstale)), C.c_int32(int(norm_clip)),
        C.c_float(pull_rho),
        _ptr(x, np.float32), _ptr(a, np.float32), _ptr(a_out, np.float32),
        _ptr(m, np.float32), dptr, _ptr(dout, np.float32),
        _ptr(first_step_norm, np.float32), _ptr(lam, np.float32), _ptr(scale, np.float32),
        C.byref(ncl))
    if rc:
        raise ValueError("co2_oracle_outer_step_variant_f32 rejected its arguments")
    return dict(dout=dout, lam=lam, scale=scale, nclipped=ncl.value)


def f32_to_bf16(values):
    """fp32 array -> bf16 bit patterns (uint16), element by element through the C loop."""
    lib = _load()
    v = np.asarray(values, dtype=np.float32).ravel()
    return np.array([lib.co2_oracle_f32_to_bf16(C.c_float(f)) for f in v], dtype=np.uint16)


def bf16_to_f32(bits):
    lib = _load()
    b = np.asarray(bits, dtype=np.uint16).ravel()
    return np.array([lib.co2_oracle_bf16_to_f32(int(x)) for x in b], dtype=np.float32)


def f32_to_f16(values):
    """fp32 array -> IEEE binary16 bit patterns (uint16), element by element through the C loop."""
    lib = _load()
    v = np.asarray(values, dtype=np.float32).ravel()
    return np.array([lib.co2_oracle_f32_to_f16(C.c_float(f)) for f in v], dtype=np.uint16)


def f16_to_f32(bits):
    lib = _load()
    b = np.asarray(bits, dtype=np.uint16).ravel()
    return np.array([lib.co2_oracle_f16_to_f32(int(x)) for x in b], dtype=np.float32)


def outer_step_f16(**kw):
    """Outer update with binary16 pseudo-gradient buffers (uint16 bit patterns).
    Returns dict(dout (uint16), lam, nclipped)."""
    return outer_step_bf16(_entry="co2_oracle_outer_step_f16", **kw)


def outer_step_bf16(*, seg_off, alpha, beta, phi, c, tau, step, x, a, m, deltas,
                    a_out=None, first_step_norm=None, _entry="co2_oracle_outer_step_bf16"):
    """Outer update with bf16 pseudo-gradient buffers (uint16 bit patterns).
    Returns dict(dout (uint16), lam, nclipped)."""
    lib = _load()
    n = a.size
    t, S = _table(n, seg_off)
    if a_out is None:
        a_out = a
    dout = np.empty(n, dtype=np.uint16) if x is not None else None
    lam = np.empty(S, dtype=np.float32)
    ncl = C.c_int64(0)
    K = len(deltas) if deltas is not None else 1
    dptr = _ptr_array(deltas, np.uint16) if deltas is not None else None
    rc = getattr(lib, _entry)(
        C.c_int64(n), C.c_int32(S), _ptr(t, np.int64), C.c_int32(K),
        C.c_float(alpha), C.c_float(beta), C.c_float(phi), C.c_float(c),
        C.c_int32(tau), C.c_int64(step),
        _ptr(x, np.float32), _ptr(a, np.float32), _ptr(a_out, np.float32),
        _ptr(m, np.float32), dptr, _ptr(dout, np.uint16),
        _ptr(first_step_norm, np.float32), _ptr(lam, np.float32), C.byref(ncl))
    if rc:
        raise ValueError(f"{_entry} rejected its arguments")
    return dict(dout=dout, lam=lam, nclipped=ncl.value)


def adamw_f32(*, p_in, p_out, grad_bf16, exp_avg, exp_avg_sq, lr, beta1, beta2,
              eps, weight_decay, k, anchor=None, seg_off=None, want_step_sq=False):
    """Fused AdamW local update; returns dict(dout, step_sq)."""
    lib = _load()
    n = p_in.size
    dout = np.empty(n, dtype=np.float32) if anchor is not None else None
    S, t, step_sq = 0, None, None
    if want_step_sq:
        t, S = _table(n, seg_off)
        step_sq = np.empty(S, dtype=np.float64)
    rc = lib.co2_oracle_adamw_f32(
        C.c_int64(n), _ptr(p_in, np.float32), _ptr(p_out, np.float32),
        _ptr(grad_bf16, np.uint16), _ptr(exp_avg, np.float32),
        _ptr(exp_avg_sq, np.float32), C.c_float(lr), C.c_float(beta1),
        C.c_float(beta2), C.c_float(eps), C.c_float(weight_decay), C.c_int64(k),
        _ptr(anchor, np.float32), _ptr(dout, np.float32), C.c_int32(S),
        _ptr(t, np.int64), _ptr(step_sq, np.float64))
    if rc:
        raise ValueError("co2_oracle_adamw_f32 rejected its arguments")
    return dict(dout=dout, step_sq=step_sq)


def adamw_f64(*, p, grad, exp_avg, exp_avg_sq, lr, beta1, beta2, eps, weight_decay, k):
    lib = _load()
    rc = lib.co2_oracle_adamw_f64(
        C.c_int64(p.size), _ptr(p, np.float64), _ptr(grad, np.float64),
        _ptr(exp_avg, np.float64), _ptr(exp_avg_sq, np.float64), C.c_double(lr),
        C.c_double(beta1), C.c_double(beta2), C.c_double(eps),
        C.c_double(weight_decay), C.c_int64(k))
    if rc:
        raise ValueError("co2_oracle_adamw_f64 rejected its arguments")
