"""ctypes binding of libco2.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

from . import build as _build

CO2_OK, CO2_EINVAL, CO2_EWORKSPACE, CO2_EHIP, CO2_ESCRATCH = 0, -1, -2, -3, -4
CO2_STATIC_SCRATCH_BYTES = 32 << 20
CO2_MAX_K = 16
CO2_MAX_NORM_BUFS = 32
CO2_FLAG_NONE = 0
CO2_FLAG_CARRIED_NORMS = 1
CO2_FLAG_CURRENT_ROUND = 2
CO2_FLAG_ANCHOR_PULL = 4
CO2_FLAG_NORM_CLIP = 8
CO2_MAX_BUFFER_SET = 64


class Co2Params(C.Structure):
    """Mirror of struct co2_params (include/co2.h)."""
    _fields_ = [
        ("n", C.c_int64), ("S", C.c_int32), ("K", C.c_int32),
        ("seg_off", C.c_void_p), ("seg_off_dev", C.c_void_p),
        ("alpha", C.c_float), ("beta", C.c_float), ("clip_phi", C.c_float),
        ("penalty_c", C.c_float), ("tau", C.c_int32), ("flags", C.c_uint32),
        ("step", C.c_int64), ("ev_sweep_begin", C.c_void_p), ("ev_sweep_end", C.c_void_p),
        ("clipped_out", C.c_void_p), ("pull_rho", C.c_float), ("sweep_waves_per_cu", C.c_int32),
    ]


class Co2Error(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code})")


_lib = None


def lib_path() -> str:
    return _build.LIB_PATH


def lib() -> C.CDLL:
    """The loaded libco2.so; built first if no library is there.  Raises if the
    HIP library cannot be produced or loaded -- there is no other code path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB_PATH):
            _build.build_lib()
        L = C.CDLL(_build.LIB_PATH)
        L.co2_workspace_bytes.restype = C.c_size_t
        L.co2_workspace_bytes.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        L.co2_strerror.restype = C.c_char_p
        L.co2_strerror.argtypes = [C.c_int]
        L.co2_last_hip_error.restype = C.c_int
        L.co2_last_hip_error.argtypes = []
        L.co2_outer_step.restype = C.c_int
        L.co2_outer_step.argtypes = [C.POINTER(Co2Params)] + [C.c_void_p] * 9 + [C.c_size_t, C.c_void_p]
        L.co2_outer_step_static.restype = C.c_int
        L.co2_outer_step_static.argtypes = [C.POINTER(Co2Params)] + [C.c_void_p] * 8 + [C.c_void_p]
        L.co2_outer_step_bf16.restype = C.c_int
        L.co2_outer_step_bf16.argtypes = L.co2_outer_step.argtypes
        L.co2_outer_step_f16.restype = C.c_int
        L.co2_outer_step_f16.argtypes = L.co2_outer_step.argtypes
        L.co2_pseudo_grad_norms.restype = C.c_int
        L.co2_pseudo_grad_norms.argtypes = [C.POINTER(Co2Params), C.c_void_p, C.c_int32, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.co2_inner_adamw.restype = C.c_int
        L.co2_inner_adamw.argtypes = ([C.c_int64] + [C.c_void_p] * 5 + [C.c_float] * 5 + [C.c_int64]
                                      + [C.c_void_p] * 4 + [C.c_int32, C.c_void_p, C.c_void_p,
                                                            C.c_size_t, C.c_void_p])
        L.co2_sqrt_to_f32.restype = C.c_int
        L.co2_sqrt_to_f32.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        L.co2_copy_f32.restype = C.c_int
        L.co2_copy_f32.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.co2_buffer_set_create.restype = C.c_int
        L.co2_buffer_set_create.argtypes = [C.c_int32, C.POINTER(C.c_size_t), C.c_size_t,
                                            C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]
        L.co2_buffer_set_destroy.restype = C.c_int
        L.co2_buffer_set_destroy.argtypes = [C.c_void_p]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().co2_strerror(int(code)).decode()


def workspace_bytes(n: int, S: int, K: int) -> int:
    return int(lib().co2_workspace_bytes(n, S, K))


class SegmentTable:
    """S+1 offsets, once on the host (validated by every call) and once on the device."""

    def __init__(self, seg_off: Sequence[int], device: Optional[torch.device] = None):
        self.host = np.ascontiguousarray(np.asarray(seg_off, dtype=np.int64))
        assert self.host.ndim == 1 and self.host.size >= 2
        self.S = int(self.host.size - 1)
        self.n = int(self.host[-1])
        self.dev = None
        if device is not None:
            self.dev = torch.from_numpy(self.host).to(device)

    @property
    def host_ptr(self) -> int:
        return self.host.ctypes.data

    @property
    def dev_ptr(self) -> Optional[int]:
        return None if self.dev is None else self.dev.data_ptr()


class HipEvent:
    """A hipEvent_t created through the HIP runtime (timing of the sweep kernel on
    whatever stream the library launches it on)."""
    _hip = None

    @classmethod
    def _rt(cls):
        if cls._hip is None:
            cls._hip = C.CDLL("libamdhip64.so")
            cls._hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
            cls._hip.hipEventDestroy.argtypes = [C.c_void_p]
            cls._hip.hipEventSynchronize.argtypes = [C.c_void_p]
            cls._hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
            cls._hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        return cls._hip

    def __init__(self):
        self.handle = C.c_void_p()
        rc = self._rt().hipEventCreate(C.byref(self.handle))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed: {rc}")

    def record(self, stream: int = 0):
        rc = self._rt().hipEventRecord(self.handle, C.c_void_p(stream))
        if rc != 0:
            raise RuntimeError(f"hipEventRecord failed: {rc}")

    def synchronize(self):
        rc = self._rt().hipEventSynchronize(self.handle)
        if rc != 0:
            raise RuntimeError(f"hipEventSynchronize failed: {rc}")

    def elapsed_ms(self, end: "HipEvent") -> float:
        ms = C.c_float()
        rc = self._rt().hipEventElapsedTime(C.byref(ms), self.handle, end.handle)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)

    def __del__(self):
        try:
            if self.handle:
                self._rt().hipEventDestroy(self.handle)
        except Exception:
            pass


class _DeviceSpan:
    """A raw device address range presented through __cuda_array_interface__ so that
    torch can view it as a uint8 tensor; keeps the owning BufferSet alive."""

    def __init__(self, ptr: int, nbytes: int, owner):
        self.owner = owner
        self.__cuda_array_interface__ = {"shape": (nbytes,), "typestr": "|u1", "data": (ptr, False),
                                         "version": 2, "strides": None}


class BufferSet:
    """co2_buffer_set: device buffers whose physical memory is obtained piece-major
    (include/co2.h).  `views` are uint8 torch tensors over the buffers; they, and
    anything derived from them, must not be used after close()."""

    def __init__(self, sizes: Sequence[int], piece_bytes: int = 0, device=None):
        count = len(sizes)
        arr = (C.c_size_t * count)(*[int(b) for b in sizes])
        ptrs = (C.c_void_p * count)()
        self._set = C.c_void_p()
        self.sizes = [int(b) for b in sizes]
        dev = torch.device("cuda:0" if device is None else device)
        with torch.cuda.device(dev):
            rc = lib().co2_buffer_set_create(count, arr, int(piece_bytes), ptrs, C.byref(self._set))
        if rc != CO2_OK:
            self._set = None
            raise Co2Error(rc, f"co2_buffer_set_create (hip error {lib().co2_last_hip_error()})")
        self.ptrs = [int(p) for p in ptrs]
        self.device = dev
        self.views = [torch.as_tensor(_DeviceSpan(p, b, self), device=dev)
                      for p, b in zip(self.ptrs, self.sizes)]

    def close(self):
        """Frees the memory.  The caller has synchronised and dropped every use of the views."""
        if self._set:
            self.views = []
            rc = lib().co2_buffer_set_destroy(self._set)
            self._set = None
            if rc != CO2_OK:
                raise Co2Error(rc, "co2_buffer_set_destroy")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _dp(t: Optional[torch.Tensor], dtype=None) -> Optional[int]:
    """Device pointer of a contiguous tensor (None passes NULL)."""
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors passed to libco2 must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(rc: int, where: str, check: bool) -> int:
    if check and rc != CO2_OK:
        raise Co2Error(rc, where)
    return rc


def make_params(table: SegmentTable, K: int, alpha: float, beta: float, clip_phi: float,
                penalty_c: float, tau: int, step: int, flags: int = 0,
                ev_begin: Optional[HipEvent] = None, ev_end: Optional[HipEvent] = None,
                clipped_out: Optional[torch.Tensor] = None, pull_rho: float = 1.0,
                sweep_waves_per_cu: int = 0) -> Co2Params:
    return Co2Params(pull_rho=pull_rho, sweep_waves_per_cu=sweep_waves_per_cu,
                     n=table.n, S=table.S, K=K, seg_off=table.host_ptr, seg_off_dev=table.dev_ptr,
                     alpha=alpha, beta=beta, clip_phi=clip_phi, penalty_c=penalty_c, tau=tau,
                     flags=flags, step=step,
                     ev_sweep_begin=ev_begin.handle if ev_begin else None,
                     ev_sweep_end=ev_end.handle if ev_end else None,
                     clipped_out=_dp(clipped_out, torch.int64))


def co2_outer_step(p: Co2Params, params, anchor, anchor_out, momentum, deltas, delta_out,
                   first_step_norm, lambda_out, workspace, stream=None, check: bool = True) -> int:
    """int co2_outer_step(...) -- see include/co2.h.  Tensors are torch CUDA tensors."""
    f32 = torch.float32
    dptrs = None
    if deltas is not None:
        if len(deltas) != p.K:
            raise ValueError(f"{len(deltas)} delta buffers for K={p.K}")
        dptrs = (C.c_void_p * len(deltas))(*[_dp(d, f32) for d in deltas])   # an entry may be None
    rc = lib().co2_outer_step(
        C.byref(p), _dp(params, f32), _dp(anchor, f32), _dp(anchor_out, f32), _dp(momentum, f32),
        dptrs, _dp(delta_out, f32), _dp(first_step_norm, f32), _dp(lambda_out, f32),
        _dp(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
        _stream(stream))
    return _check(rc, "co2_outer_step", check)


def co2_outer_step_static(p: Co2Params, params, anchor, anchor_out, momentum, deltas, delta_out,
                          first_step_norm, lambda_out, stream=None, check: bool = True) -> int:
    """int co2_outer_step_static(...) -- see include/co2.h: co2_outer_step without a
    workspace argument (the library's own per-GPU scratch array is used)."""
    f32 = torch.float32
    dptrs = None
    if deltas is not None:
        if len(deltas) != p.K:
            raise ValueError(f"{len(deltas)} delta buffers for K={p.K}")
        dptrs = (C.c_void_p * len(deltas))(*[_dp(d, f32) for d in deltas])
    rc = lib().co2_outer_step_static(
        C.byref(p), _dp(params, f32), _dp(anchor, f32), _dp(anchor_out, f32), _dp(momentum, f32),
        dptrs, _dp(delta_out, f32), _dp(first_step_norm, f32), _dp(lambda_out, f32),
        _stream(stream))
    return _check(rc, "co2_outer_step_static", check)


def _bf16_ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if t.dtype not in (torch.bfloat16, torch.uint16, torch.int16):
        raise ValueError("expected a tensor of bf16 values / bit patterns")
    return _dp(t)


def co2_outer_step_bf16(p: Co2Params, params, anchor, anchor_out, momentum, deltas_bf16,
                        delta_out_bf16, first_step_norm, lambda_out, workspace, stream=None,
                        check: bool = True) -> int:
    """int co2_outer_step_bf16(...) -- see include/co2.h.  Delta tensors are torch.bfloat16."""
    f32 = torch.float32
    dptrs = None
    if deltas_bf16 is not None:
        if len(deltas_bf16) != p.K:
            raise ValueError(f"{len(deltas_bf16)} delta buffers for K={p.K}")
        dptrs = (C.c_void_p * len(deltas_bf16))(*[_bf16_ptr(d) for d in deltas_bf16])
    rc = lib().co2_outer_step_bf16(
        C.byref(p), _dp(params, f32), _dp(anchor, f32), _dp(anchor_out, f32), _dp(momentum, f32),
        dptrs, _bf16_ptr(delta_out_bf16), _dp(first_step_norm, f32), _dp(lambda_out, f32),
        _dp(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
        _stream(stream))
    return _check(rc, "co2_outer_step_bf16", check)


def _f16_ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if t.dtype not in (torch.float16, torch.uint16, torch.int16):
        raise ValueError("expected a tensor of fp16 values / bit patterns")
    return _dp(t)


def co2_outer_step_f16(p: Co2Params, params, anchor, anchor_out, momentum, deltas_f16,
                       delta_out_f16, first_step_norm, lambda_out, workspace, stream=None,
                       check: bool = True) -> int:
    """int co2_outer_step_f16(...) -- see include/co2.h.  Delta tensors are torch.float16."""
    f32 = torch.float32
    dptrs = None
    if deltas_f16 is not None:
        if len(deltas_f16) != p.K:
            raise ValueError(f"{len(deltas_f16)} delta buffers for K={p.K}")
        dptrs = (C.c_void_p * len(deltas_f16))(*[_f16_ptr(d) for d in deltas_f16])
    rc = lib().co2_outer_step_f16(
        C.byref(p), _dp(params, f32), _dp(anchor, f32), _dp(anchor_out, f32), _dp(momentum, f32),
        dptrs, _f16_ptr(delta_out_f16), _dp(first_step_norm, f32), _dp(lambda_out, f32),
        _dp(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
        _stream(stream))
    return _check(rc, "co2_outer_step_f16", check)


def co2_pseudo_grad_norms(p: Co2Params, bufs, momentum, sqnorm_out, workspace, stream=None,
                          check: bool = True) -> int:
    f32 = torch.float32
    bufs = list(bufs or [])
    bptrs = (C.c_void_p * max(1, len(bufs)))(*[_dp(b, f32) for b in bufs]) if bufs else None
    rc = lib().co2_pseudo_grad_norms(
        C.byref(p), bptrs, len(bufs), _dp(momentum, f32), _dp(sqnorm_out, torch.float64),
        _dp(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
        _stream(stream))
    return _check(rc, "co2_pseudo_grad_norms", check)


def co2_inner_adamw(n, p_in, p_out, grad_bf16, exp_avg, exp_avg_sq, lr, beta1, beta2, eps,
                    weight_decay, adam_step, anchor=None, delta_out=None,
                    table: Optional[SegmentTable] = None, step_sq_out=None, workspace=None,
                    stream=None, check: bool = True) -> int:
    f32 = torch.float32
    if grad_bf16 is not None and grad_bf16.dtype not in (torch.bfloat16, torch.uint16, torch.int16):
        raise ValueError("grad_bf16 must hold bf16 bit patterns")
    rc = lib().co2_inner_adamw(
        n, _dp(p_in, f32), _dp(p_out, f32), _dp(grad_bf16), _dp(exp_avg, f32), _dp(exp_avg_sq, f32),
        lr, beta1, beta2, eps, weight_decay, adam_step, _dp(anchor, f32), _dp(delta_out, f32),
        table.host_ptr if table else None, table.dev_ptr if table else None,
        table.S if table else 0, _dp(step_sq_out, torch.float64), _dp(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream))
    return _check(rc, "co2_inner_adamw", check)


def co2_sqrt_to_f32(sq, out, S, stream=None, check: bool = True) -> int:
    rc = lib().co2_sqrt_to_f32(_dp(sq, torch.float64), _dp(out, torch.float32), S, _stream(stream))
    return _check(rc, "co2_sqrt_to_f32", check)


def co2_copy_f32(src, dst, n, stream=None, check: bool = True) -> int:
    rc = lib().co2_copy_f32(_dp(src, torch.float32), _dp(dst, torch.float32), n, _stream(stream))
    return _check(rc, "co2_copy_f32", check)
