"""ctypes binding of libswift_undo.so: argument marshalling only.

Every function has the name and the meaning of the C entry point in include/swift_undo.h; all
arithmetic runs in the HIP kernels behind it.  torch is used for device memory and streams.  There
is no CPU fallback: if the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libswift_undo.so")

SWIFT_OK, SWIFT_EINVAL, SWIFT_ENOTINVERTIBLE, SWIFT_EHIP = 0, -1, -2, -3
SWIFT_SGDM, SWIFT_ADAM, SWIFT_ADAMW, SWIFT_LAMB, SWIFT_SGD = 0, 1, 2, 3, 4
SWIFT_F32, SWIFT_BF16 = 0, 1
SWIFT_CLAMP_V = 1
KINDS = {"sgdm": SWIFT_SGDM, "adam": SWIFT_ADAM, "adamw": SWIFT_ADAMW, "lamb": SWIFT_LAMB, "sgd": SWIFT_SGD}

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2302_06173_amd.build` "
        "(there is no fallback path)")
_lib = ctypes.CDLL(LIB_PATH)


class SwiftHparams(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("grad_dtype", ctypes.c_int32), ("step", ctypes.c_int64),
                ("lr", ctypes.c_double), ("weight_decay", ctypes.c_double), ("momentum", ctypes.c_double),
                ("dampening", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double), ("flags", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class SwiftTensorList(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("param", ctypes.POINTER(ctypes.c_void_p)),
                ("grad", ctypes.POINTER(ctypes.c_void_p)), ("m", ctypes.POINTER(ctypes.c_void_p)),
                ("v", ctypes.POINTER(ctypes.c_void_p)), ("numel", ctypes.POINTER(ctypes.c_int64)),
                ("param_bf16", ctypes.POINTER(ctypes.c_void_p))]


_P = ctypes.c_void_p
for _name in ("swift_opt_step", "swift_opt_undo", "swift_opt_step_dmask", "swift_opt_undo_dmask",
              "swift_opt_undo_dmask_noalloc"):
    getattr(_lib, _name).argtypes = [ctypes.POINTER(SwiftTensorList), ctypes.POINTER(SwiftHparams), _P, _P]
    getattr(_lib, _name).restype = ctypes.c_int
for _name in ("swift_lamb_step", "swift_lamb_undo", "swift_opt_step_digest", "swift_opt_undo_digest"):
    getattr(_lib, _name).argtypes = [ctypes.POINTER(SwiftTensorList), ctypes.POINTER(SwiftHparams), _P, _P, _P]
    getattr(_lib, _name).restype = ctypes.c_int
_lib.swift_state_digest.argtypes = [ctypes.c_int64, ctypes.POINTER(_P), ctypes.POINTER(ctypes.c_int64),
                                    ctypes.c_int64, _P, _P]
_lib.swift_state_digest.restype = ctypes.c_int
_lib.swift_digest_count.argtypes = [ctypes.c_int64, ctypes.POINTER(ctypes.c_int64), ctypes.c_int64]
_lib.swift_digest_count.restype = ctypes.c_int64
_lib.swift_mask_from_digests.argtypes = [ctypes.c_int64, ctypes.c_int64, _P, _P, _P, _P]
_lib.swift_mask_from_digests.restype = ctypes.c_int
_lib.swift_stream_copy.argtypes = [_P, _P, ctypes.c_int64, _P]
_lib.swift_stream_copy.restype = ctypes.c_int
_lib.swift_tracker_create.argtypes = [ctypes.c_int64, ctypes.POINTER(_P)]
_lib.swift_tracker_begin.argtypes = [_P, ctypes.c_int64]
_lib.swift_tracker_step.argtypes = [_P, ctypes.POINTER(SwiftTensorList), ctypes.POINTER(ctypes.c_int64),
                                    ctypes.POINTER(SwiftHparams), _P, _P]
_lib.swift_tracker_marks.argtypes = [_P, _P]
_lib.swift_tracker_undo.argtypes = [_P, ctypes.POINTER(SwiftTensorList), ctypes.POINTER(SwiftHparams), _P]
_lib.swift_tracker_destroy.argtypes = [_P]
for _name in ("create", "begin", "step", "marks", "undo", "destroy"):
    getattr(_lib, "swift_tracker_" + _name).restype = ctypes.c_int
_lib.swift_cache_stats.argtypes = [ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]
_lib.swift_cache_stats.restype = ctypes.c_int
_lib.swift_cache_trim.argtypes = [ctypes.c_int64]
_lib.swift_cache_trim.restype = ctypes.c_int
_lib.swift_shutdown.argtypes = []
_lib.swift_shutdown.restype = ctypes.c_int
_lib.swift_last_error.argtypes = []
_lib.swift_last_error.restype = ctypes.c_char_p

EXPORTS = ("swift_opt_step", "swift_opt_undo", "swift_opt_step_dmask", "swift_opt_undo_dmask",
           "swift_opt_undo_dmask_noalloc", "swift_cache_stats", "swift_cache_trim", "swift_arena_layout",
           "swift_lamb_step", "swift_lamb_undo", "swift_opt_step_digest", "swift_opt_undo_digest",
           "swift_tracker_create", "swift_tracker_begin", "swift_tracker_step", "swift_tracker_marks",
           "swift_tracker_undo", "swift_tracker_destroy",
           "swift_state_digest", "swift_digest_count", "swift_mask_from_digests", "swift_stream_copy",
           "swift_logging_groups", "swift_shutdown", "swift_last_error")


class SwiftError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"swift error {code}: {message}")
        self.code = code
        self.message = message


def swift_last_error() -> str:
    return (_lib.swift_last_error() or b"").decode()


def _check(rc: int) -> None:
    if rc != SWIFT_OK:
        raise SwiftError(rc, swift_last_error())


# torch's current stream as a raw handle without building a Stream object (a third of a per-group launch's host
# time otherwise); the private accessor is what torch's own compiled-kernel launchers use
_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def current_stream_handle() -> Optional[int]:
    """hipStream_t of torch's current stream on the current device (None = the default stream)."""
    if _raw_stream is not None:
        return _raw_stream(torch.cuda.current_device()) or None
    return torch.cuda.current_stream().cuda_stream or None


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        return current_stream_handle()
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def hparams(kind, step: int, lr: float, weight_decay: float = 0.0, momentum: float = 0.0,
            dampening: float = 0.0, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
            grad_bf16: bool = False, clamp_v: bool = False) -> SwiftHparams:
    k = KINDS[kind] if isinstance(kind, str) else int(kind)
    return SwiftHparams(k, SWIFT_BF16 if grad_bf16 else SWIFT_F32, int(step), float(lr), float(weight_decay),
                        float(momentum), float(dampening), float(beta1), float(beta2), float(eps),
                        SWIFT_CLAMP_V if clamp_v else 0, 0)


def _ptr_array(tensors: Sequence[torch.Tensor]):
    arr = (ctypes.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = t.data_ptr() if t.numel() else None
    return arr


class TensorList:
    """Marshalled swift_tensor_list; keeps the tensors and the host arrays alive."""

    def __init__(self, param: Sequence[torch.Tensor], grad: Sequence[torch.Tensor],
                 m: Optional[Sequence[torch.Tensor]] = None, v: Optional[Sequence[torch.Tensor]] = None,
                 param_bf16: Optional[Sequence[torch.Tensor]] = None):
        """m is None for plain SGD (no optimizer state), v for plain SGD and SGD with momentum."""
        n = len(param)
        if len(grad) != n or (m is not None and len(m) != n) or (v is not None and len(v) != n) or \
                (param_bf16 is not None and len(param_bf16) != n):
            raise ValueError("tensor lists differ in length")
        if param_bf16 is not None:
            for i, t in enumerate(param_bf16):
                if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous() or t.numel() != param[i].numel():
                    raise ValueError(f"tensor {i}: param_bf16 must be a contiguous CUDA bfloat16 tensor of the same size")
        self.grad_bf16 = n > 0 and grad[0].dtype == torch.bfloat16
        for i in range(n):
            group = [param[i], grad[i]] + ([m[i]] if m is not None else []) + ([v[i]] if v is not None else [])
            for t in group:
                if not t.is_cuda or not t.is_contiguous():
                    raise ValueError(f"tensor {i}: need contiguous CUDA tensors")
                if t.numel() != param[i].numel():
                    raise ValueError(f"tensor {i}: numel differs between param, grad and moments")
            if param[i].dtype != torch.float32 or (m is not None and m[i].dtype != torch.float32) or \
                    (v is not None and v[i].dtype != torch.float32):
                raise ValueError(f"tensor {i}: param, m and v must be float32")
            if grad[i].dtype != (torch.bfloat16 if self.grad_bf16 else torch.float32):
                raise ValueError(f"tensor {i}: gradients must all be float32 or all bfloat16")
        self._keep = (list(param), list(grad), None if m is None else list(m), None if v is None else list(v),
                      None if param_bf16 is None else list(param_bf16))
        self._xb = None if param_bf16 is None else _ptr_array(param_bf16)
        self._param, self._grad = _ptr_array(param), _ptr_array(grad)
        self._m = None if m is None else _ptr_array(m)
        self._v = None if v is None else _ptr_array(v)
        self._numel = (ctypes.c_int64 * n)(*[t.numel() for t in param])
        self.n = n
        self.c = SwiftTensorList(
            n, ctypes.cast(self._param, ctypes.POINTER(_P)), ctypes.cast(self._grad, ctypes.POINTER(_P)),
            ctypes.cast(self._m, ctypes.POINTER(_P)) if self._m is not None else None,
            ctypes.cast(self._v, ctypes.POINTER(_P)) if self._v is not None else None,
            ctypes.cast(self._numel, ctypes.POINTER(ctypes.c_int64)),
            ctypes.cast(self._xb, ctypes.POINTER(_P)) if self._xb is not None else None)


def _host_mask(mask, n: int):
    if mask is None:
        return None, None
    if len(mask) != n:
        raise ValueError("mask length differs from the tensor count")
    buf = (ctypes.c_uint8 * max(n, 1))(*[1 if b else 0 for b in mask])
    return buf, ctypes.cast(buf, _P)


def swift_opt_step(tl: TensorList, hp: SwiftHparams, host_mask=None, stream=None) -> None:
    keep, p = _host_mask(host_mask, tl.n)
    _check(_lib.swift_opt_step(ctypes.byref(tl.c), ctypes.byref(hp), p, _stream_handle(stream)))


def swift_opt_undo(tl: TensorList, hp: SwiftHparams, host_mask=None, stream=None) -> None:
    keep, p = _host_mask(host_mask, tl.n)
    _check(_lib.swift_opt_undo(ctypes.byref(tl.c), ctypes.byref(hp), p, _stream_handle(stream)))


def _dmask_ptr(device_mask: torch.Tensor, n: int) -> int:
    if device_mask.dtype != torch.uint8 or not device_mask.is_cuda or not device_mask.is_contiguous() \
            or device_mask.numel() != n:
        raise ValueError("device mask must be a contiguous CUDA uint8 tensor with one byte per tensor")
    return device_mask.data_ptr()


def swift_opt_step_dmask(tl: TensorList, hp: SwiftHparams, device_mask: torch.Tensor, stream=None) -> None:
    _check(_lib.swift_opt_step_dmask(ctypes.byref(tl.c), ctypes.byref(hp), _dmask_ptr(device_mask, tl.n),
                                     _stream_handle(stream)))


def swift_opt_undo_dmask(tl: TensorList, hp: SwiftHparams, device_mask: torch.Tensor, stream=None) -> None:
    _check(_lib.swift_opt_undo_dmask(ctypes.byref(tl.c), ctypes.byref(hp), _dmask_ptr(device_mask, tl.n),
                                     _stream_handle(stream)))


def swift_opt_undo_dmask_noalloc(tl: TensorList, hp: SwiftHparams, device_mask: torch.Tensor, stream=None) -> None:
    _check(_lib.swift_opt_undo_dmask_noalloc(ctypes.byref(tl.c), ctypes.byref(hp), _dmask_ptr(device_mask, tl.n),
                                             _stream_handle(stream)))


def _norms_ptr(norms: torch.Tensor, n: int) -> int:
    if norms.dtype != torch.float64 or not norms.is_cuda or not norms.is_contiguous() or norms.numel() != 2 * n:
        raise ValueError("norms must be a contiguous CUDA float64 tensor with two entries per tensor")
    return norms.data_ptr()


def swift_lamb_step(tl: TensorList, hp: SwiftHparams, norms: Optional[torch.Tensor] = None, host_mask=None,
                    stream=None) -> torch.Tensor:
    """LAMB step; returns the float64 CUDA tensor of saved norms (||x_t||, ||u|| per tensor)."""
    if norms is None:
        norms = torch.zeros(2 * tl.n, dtype=torch.float64, device="cuda")
    keep, p = _host_mask(host_mask, tl.n)
    _check(_lib.swift_lamb_step(ctypes.byref(tl.c), ctypes.byref(hp), p, _norms_ptr(norms, tl.n) if tl.n else None,
                                _stream_handle(stream)))
    return norms


def swift_lamb_undo(tl: TensorList, hp: SwiftHparams, norms: torch.Tensor, host_mask=None, stream=None) -> None:
    keep, p = _host_mask(host_mask, tl.n)
    _check(_lib.swift_lamb_undo(ctypes.byref(tl.c), ctypes.byref(hp), p, _norms_ptr(norms, tl.n) if tl.n else None,
                                _stream_handle(stream)))


def _fused(fn, tl: TensorList, hp: SwiftHparams, digests, host_mask, stream) -> torch.Tensor:
    n_groups = {SWIFT_SGD: 1, SWIFT_SGDM: 2}.get(hp.kind, 3)
    if digests is None:
        digests = torch.zeros(n_groups * tl.n, dtype=torch.int64, device="cuda")
    elif digests.dtype != torch.int64 or not digests.is_cuda or not digests.is_contiguous() \
            or digests.numel() != n_groups * tl.n:
        raise ValueError(f"digests must be a contiguous CUDA int64 tensor of {n_groups * tl.n} elements")
    keep, p = _host_mask(host_mask, tl.n)
    _check(fn(ctypes.byref(tl.c), ctypes.byref(hp), p, digests.data_ptr() if tl.n else None, _stream_handle(stream)))
    return digests


def swift_opt_step_digest(tl: TensorList, hp: SwiftHparams, digests: Optional[torch.Tensor] = None, host_mask=None,
                          stream=None) -> torch.Tensor:
    """Step, and the per-tensor digests (theta.., m.., v..) of the state it leaves (int64 CUDA tensor)."""
    return _fused(_lib.swift_opt_step_digest, tl, hp, digests, host_mask, stream)


def swift_opt_undo_digest(tl: TensorList, hp: SwiftHparams, digests: Optional[torch.Tensor] = None, host_mask=None,
                          stream=None) -> torch.Tensor:
    """Undo, and the per-tensor digests of the state it leaves."""
    return _fused(_lib.swift_opt_undo_digest, tl, hp, digests, host_mask, stream)


class BufferList:
    """Marshalled (buf, numel) arrays for swift_state_digest; keeps tensors and arrays alive."""

    def __init__(self, bufs: Sequence[torch.Tensor]):
        for i, t in enumerate(bufs):
            if not t.is_cuda or not t.is_contiguous() or t.element_size() != 4:
                raise ValueError(f"buffer {i}: need contiguous CUDA tensors with 4-byte elements")
        self._keep = list(bufs)
        self.n = len(bufs)
        self._ptrs = _ptr_array(bufs)
        self._numel = (ctypes.c_int64 * max(self.n, 1))(*[t.numel() for t in bufs])
        self.ptrs = ctypes.cast(self._ptrs, ctypes.POINTER(_P))
        self.numel = ctypes.cast(self._numel, ctypes.POINTER(ctypes.c_int64))


def swift_digest_count(numel: Sequence[int], shard_elems: int = 0) -> int:
    arr = (ctypes.c_int64 * max(len(numel), 1))(*numel)
    n = _lib.swift_digest_count(len(numel), arr, int(shard_elems))
    if n < 0:
        raise SwiftError(int(n), swift_last_error())
    return int(n)


def swift_state_digest(bufs, shard_elems: int = 0, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Returns (or fills) an int64 CUDA tensor holding the raw 64-bit digests, buffer-major."""
    bl = bufs if isinstance(bufs, BufferList) else BufferList(bufs)
    n_out = _lib.swift_digest_count(bl.n, bl.numel, int(shard_elems))
    if n_out < 0:
        raise SwiftError(int(n_out), swift_last_error())
    if out is None:
        out = torch.empty(n_out, dtype=torch.int64, device="cuda")
    elif out.dtype != torch.int64 or not out.is_cuda or not out.is_contiguous() or out.numel() != n_out:
        raise ValueError(f"out must be a contiguous CUDA int64 tensor of {n_out} elements")
    _check(_lib.swift_state_digest(bl.n, bl.ptrs, bl.numel, int(shard_elems), out.data_ptr() if n_out else None,
                                   _stream_handle(stream)))
    return out


def swift_mask_from_digests(before: torch.Tensor, after: torch.Tensor, n_tensors: int,
                            out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """uint8 CUDA mask, one byte per tensor, from two group-major int64 digest tensors."""
    if before.numel() != after.numel() or (n_tensors and before.numel() % n_tensors):
        raise ValueError("digest arrays must have n_groups * n_tensors entries each")
    for t in (before, after):
        if t.dtype != torch.int64 or not t.is_cuda or not t.is_contiguous():
            raise ValueError("digest arrays must be contiguous CUDA int64 tensors")
    n_groups = before.numel() // n_tensors if n_tensors else 1
    if out is None:
        out = torch.empty(n_tensors, dtype=torch.uint8, device="cuda")
    elif out.dtype != torch.uint8 or not out.is_cuda or out.numel() != n_tensors:
        raise ValueError("out must be a CUDA uint8 tensor with one byte per tensor")
    _check(_lib.swift_mask_from_digests(n_tensors, n_groups, before.data_ptr() if n_tensors else None,
                                        after.data_ptr() if n_tensors else None,
                                        out.data_ptr() if n_tensors else None, _stream_handle(stream)))
    return out


class Tracker:
    """swift_tracker_*: the paper's per-parameter "marked as updated" bookkeeping for one training loop."""

    def __init__(self, n_tensors: int):
        self._h = ctypes.c_void_p()
        _check(_lib.swift_tracker_create(int(n_tensors), ctypes.byref(self._h)))
        self.n = int(n_tensors)

    def begin(self, step: int) -> None:
        _check(_lib.swift_tracker_begin(self._h, int(step)))

    @staticmethod
    def ids(tensor_ids: Sequence[int]):
        """The ids of a group marshalled once (a loop that steps the same groups every iteration keeps these)."""
        return (ctypes.c_int64 * max(len(tensor_ids), 1))(*tensor_ids)

    def step(self, group: TensorList, tensor_ids, hp: SwiftHparams, grad_ready_event=None,
             stream=None) -> None:
        if len(tensor_ids) != max(group.n, 1) and len(tensor_ids) != group.n:
            raise ValueError("one id per tensor of the group")
        ids = tensor_ids if isinstance(tensor_ids, ctypes.Array) else self.ids(tensor_ids)
        ev = None
        if grad_ready_event is not None:
            ev = grad_ready_event.cuda_event if isinstance(grad_ready_event, torch.cuda.Event) else int(grad_ready_event)
        _check(_lib.swift_tracker_step(self._h, ctypes.byref(group.c), ids, ctypes.byref(hp), ev, _stream_handle(stream)))

    def marks(self) -> List[int]:
        buf = (ctypes.c_uint8 * max(self.n, 1))()
        _check(_lib.swift_tracker_marks(self._h, ctypes.cast(buf, _P)))
        return list(buf[:self.n])

    def undo(self, full: TensorList, hp: SwiftHparams, stream=None) -> None:
        _check(_lib.swift_tracker_undo(self._h, ctypes.byref(full.c), ctypes.byref(hp), _stream_handle(stream)))

    def close(self) -> None:
        if self._h:
            _check(_lib.swift_tracker_destroy(self._h))
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def swift_stream_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("stream_copy: sizes differ")
    _check(_lib.swift_stream_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream_handle(stream)))


_lib.swift_logging_groups.argtypes = [ctypes.c_int64, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                      ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_int,
                                      ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_double)]
_lib.swift_logging_groups.restype = ctypes.c_int


def swift_logging_groups(compute_time: Sequence[float], message_bytes: Sequence[float], checkpoint_interval: float,
                         bandwidth: float, storage_limit: float, parallel_recovery: bool = False):
    """Machine groups for selective logging: returns (group_of, storage, expected_recovery)."""
    n = len(compute_time)
    if len(message_bytes) != max(n - 1, 0):
        raise ValueError("need one message size per pair of adjacent machines")
    R = (ctypes.c_double * max(n, 1))(*[float(v) for v in compute_time])
    M = (ctypes.c_double * max(n - 1, 1))(*[float(v) for v in message_bytes])
    out = (ctypes.c_int32 * max(n, 1))()
    storage, recovery = ctypes.c_double(), ctypes.c_double()
    _check(_lib.swift_logging_groups(n, R, M, float(checkpoint_interval), float(bandwidth), float(storage_limit),
                                     1 if parallel_recovery else 0, out, ctypes.byref(storage), ctypes.byref(recovery)))
    return list(out[:n]), storage.value, recovery.value


_lib.swift_arena_layout.argtypes = [ctypes.c_int64, ctypes.POINTER(ctypes.c_int64), ctypes.c_int32, ctypes.c_int32,
                                    ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]
_lib.swift_arena_layout.restype = ctypes.c_int


def swift_arena_layout(numel: Sequence[int], grad_bf16: bool = False, with_v: bool = True, with_m: bool = True):
    """Byte offsets (one row [theta, g(, m(, v))] per tensor) and the total size of an arena that holds the state."""
    if with_v and not with_m:
        raise ValueError("a second moment without a first moment is no optimizer of this library")
    n, s = len(numel), 4 if with_v else (3 if with_m else 2)
    sizes = (ctypes.c_int64 * max(n, 1))(*numel)
    offs = (ctypes.c_int64 * max(n * s, 1))()
    total = ctypes.c_int64()
    _check(_lib.swift_arena_layout(n, sizes, SWIFT_BF16 if grad_bf16 else SWIFT_F32, 1 if with_v else (0 if with_m else -1), offs,
                                   ctypes.byref(total)))
    return [list(offs[i * s:(i + 1) * s]) for i in range(n)], total.value


def swift_cache_stats():
    """(number of cached lists, bytes of device memory behind them)."""
    n, b = ctypes.c_int64(), ctypes.c_int64()
    _check(_lib.swift_cache_stats(ctypes.byref(n), ctypes.byref(b)))
    return n.value, b.value


def swift_cache_trim(max_device_bytes: int = 0) -> None:
    _check(_lib.swift_cache_trim(int(max_device_bytes)))


def swift_shutdown() -> None:
    _check(_lib.swift_shutdown())
