"""Thin ctypes binding of libpipad.so: argument marshalling only.

Every step of the path (overlap extraction, normalisation, aggregation) runs in the HIP kernels of
the library; nothing here computes.  PyTorch supplies device memory and streams.  There is no CPU
fallback: if the library cannot be loaded the import of this module's functions fails loudly.

The names mirror ``include/pipad.h``:
  pipad_frame_build_overlap  -> :func:`frame_build_overlap`   (Section 4.1 / 4.3: overlap + exclusive parts)
  pipad_frame_aggregate      -> :func:`frame_aggregate`       (Section 4.2: parallel + exclusive aggregation)
  pipad_frame_common / _delta / _dinv -> :meth:`Frame.common`, :meth:`Frame.delta`, :meth:`Frame.dinv`
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple, Union

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpipad.so")
MAX_K = 32
VALIDATE = 1

_lib = None


class PipadError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libpipad: {text} (status {status})")
        self.status = status


class _Csr(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int32), ("nnz", ctypes.c_int32),
                ("rowptr", ctypes.c_void_p), ("colidx", ctypes.c_void_p)]


ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p)

# symbol -> (restype, argtypes); also the list the ABI test checks against include/pipad.h
_vp, _i32, _i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
SIGNATURES = {
    "pipad_frame_build_overlap": (ctypes.c_int, [_i32, _i32, ctypes.POINTER(_Csr), ctypes.c_uint32,
                                                 _vp, _vp, _vp, ctypes.POINTER(_vp)]),
    "pipad_frame_common": (ctypes.c_int, [_vp, ctypes.POINTER(_Csr)]),
    "pipad_frame_delta": (ctypes.c_int, [_vp, _i32, ctypes.POINTER(_Csr)]),
    "pipad_frame_dinv": (ctypes.c_int, [_vp, ctypes.POINTER(_vp), ctypes.POINTER(_i64),
                                        ctypes.POINTER(_i64)]),
    "pipad_frame_shape": (ctypes.c_int, [_vp, ctypes.POINTER(_i32), ctypes.POINTER(_i32)]),
    "pipad_frame_aggregate": (ctypes.c_int, [_vp, _i32, ctypes.POINTER(_vp), _i64,
                                             ctypes.POINTER(_vp), _i64, _vp]),
    "pipad_frame_aggregate_subset": (ctypes.c_int, [_vp, _i32, ctypes.POINTER(_i32), _i32,
                                                    ctypes.POINTER(_vp), _i64, ctypes.POINTER(_vp), _i64, _vp]),
    "pipad_frame_aggregate_static": (ctypes.c_int, [_vp, _i32, ctypes.POINTER(_vp), _i64,
                                                    ctypes.POINTER(_vp), _i64, _vp]),
    "pipad_frame_aggregate_update": (ctypes.c_int, [_vp, _i32, ctypes.POINTER(_vp), _i64, _vp, _i64,
                                                    _vp, _i32, ctypes.POINTER(_vp), _i64,
                                                    ctypes.POINTER(_vp), _i64, _vp]),
    "pipad_frame_transpose": (ctypes.c_int, [_vp, _vp, _vp, _vp, ctypes.POINTER(_vp)]),
    "pipad_frame_temporaries": (ctypes.c_int, [_vp, ctypes.POINTER(_vp), ctypes.POINTER(ctypes.c_size_t)]),
    "pipad_recommended_row_stride": (ctypes.c_int64, [_i32]),
    "pipad_frame_destroy": (None, [_vp]),
    "pipad_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "pipad_last_hip_error": (ctypes.c_char_p, []),
    "pipad_set_option": (ctypes.c_int, [ctypes.c_char_p, _i64]),
    # include/pipad_ceilings.h (measurement kernels)
    "pipad_ceiling_stream_read": (ctypes.c_int, [_vp, ctypes.c_size_t, _vp, _vp]),
    "pipad_ceiling_stream_copy": (ctypes.c_int, [_vp, _vp, ctypes.c_size_t, _vp]),
    "pipad_ceiling_gather": (ctypes.c_int, [_vp, _i64, _i32, _i64, _vp, _i64, _i32, _vp, _vp]),
    "pipad_ceiling_sink_floats": (ctypes.c_size_t, []),
    "pipad_get_option": (ctypes.c_int, [ctypes.c_char_p, ctypes.POINTER(_i64)]),
}


def load_library():
    """Loads libpipad.so (building it first only if it does not exist yet).  The environment
    variable PIPAD_LIBRARY names another build of the library to load instead (measurement builds,
    see build.py); a missing file is an error, never a fallback."""
    global _lib
    if _lib is None:
        path = os.environ.get("PIPAD_LIBRARY") or LIB_PATH
        if path == LIB_PATH and not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build()
        lib = ctypes.CDLL(path)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _check(status: int) -> None:
    if status != 0:
        lib = load_library()
        text = lib.pipad_strerror(status).decode()
        if status == -5:
            text += ": " + lib.pipad_last_hip_error().decode()
        raise PipadError(status, text)


def set_option(key: str, value: int) -> None:
    _check(load_library().pipad_set_option(key.encode(), int(value)))


def get_option(key: str) -> int:
    v = _i64(0)
    _check(load_library().pipad_get_option(key.encode(), ctypes.byref(v)))
    return int(v.value)


class _DevArray:
    """Exposes a raw device pointer through __cuda_array_interface__ (view, copied at once by the caller)."""

    def __init__(self, ptr: int, count: int, typestr: str):
        self.__cuda_array_interface__ = {"shape": (count,), "typestr": typestr,
                                         "data": (ptr, False), "version": 2}


def _copy_from_device(ptr: Optional[int], count: int, dtype: torch.dtype, device) -> torch.Tensor:
    if count == 0 or not ptr:
        return torch.empty(0, dtype=dtype, device=device)
    typestr = {torch.int32: "<i4", torch.float32: "<f4"}[dtype]
    return torch.as_tensor(_DevArray(ptr, count, typestr), device=device).clone()


def _stream_handle(stream) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


Snapshot = Tuple[torch.Tensor, torch.Tensor]  # (rowptr int32[n+1], colidx int32[nnz]) on the GPU


class Frame:
    """Owner of one ``pipad_frame_t``.  Built by :func:`frame_build_overlap`."""

    def __init__(self, handle: int, n: int, k: int, device, buffers: list, callback=None,
                 stream=None):
        self._h = handle
        self.n, self.k, self.device = n, k, device
        self._buffers = buffers  # torch tensors handed to the library through the allocator
        self._callback = callback  # the library may call it again (aggregate scratch)
        # torch's allocator hands memory out, and takes it back, in the order of the stream that
        # was current at the allocation; work on any other stream has to be waited for in close()
        self._alloc_stream = torch.cuda.current_stream(device)
        self._streams = {stream if stream is not None else self._alloc_stream}
        self._temp = None
        if callback is not None:
            # the build's temporaries can go back to the allocator as soon as the build's kernels
            # have run: remember the buffer and an event behind them
            ptr, size = _vp(), ctypes.c_size_t()
            _check(load_library().pipad_frame_temporaries(handle, ctypes.byref(ptr), ctypes.byref(size)))
            if ptr.value:
                held = [b for b in buffers if b.data_ptr() == ptr.value]
                event = torch.cuda.Event()
                event.record(next(iter(self._streams)))
                self._temp = (held, event)

    def _release_temporaries(self, wait: bool = False) -> None:
        if self._temp is not None and (wait or self._temp[1].query()):
            if wait:
                self._temp[1].synchronize()
            held = {id(b) for b in self._temp[0]}
            self._buffers[:] = [b for b in self._buffers if id(b) not in held]
            self._temp = None

    def close(self) -> None:
        if self._h:
            # work of this frame may still be running on streams other than the one its buffers
            # are ordered on
            for s in self._streams:
                if s != self._alloc_stream:
                    s.synchronize()
            load_library().pipad_frame_destroy(self._h)
            self._h = None
            self._temp = None
            # in place: the allocator callback's closure holds the same list, and ctypes callback
            # objects sit in a reference cycle that only the garbage collector breaks - rebinding
            # the attribute would keep every buffer alive until its next run
            self._buffers.clear()
            self._callback = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _view(self, t: Optional[int]) -> Tuple[torch.Tensor, torch.Tensor]:
        lib = load_library()
        v = _Csr()
        if t is None:
            _check(lib.pipad_frame_common(self._h, ctypes.byref(v)))
        else:
            _check(lib.pipad_frame_delta(self._h, t, ctypes.byref(v)))
        torch.cuda.synchronize(self.device)
        rowptr = _copy_from_device(v.rowptr, self.n + 1, torch.int32, self.device)
        col = _copy_from_device(v.colidx, v.nnz, torch.int32, self.device)
        return rowptr, col

    def common(self) -> Snapshot:
        """Copy of the overlap CSR (pipad_frame_common)."""
        return self._view(None)

    def delta(self, t: int) -> Snapshot:
        """Copy of the exclusive CSR of snapshot t (pipad_frame_delta)."""
        return self._view(t)

    def dinv(self) -> torch.Tensor:
        """Copy of D^-1/2 as a float32[k, n] tensor (pipad_frame_dinv)."""
        lib = load_library()
        ptr, ldn, lds = _vp(), _i64(), _i64()
        _check(lib.pipad_frame_dinv(self._h, ctypes.byref(ptr), ctypes.byref(ldn), ctypes.byref(lds)))
        assert ldn.value == 1 and lds.value == self.n
        torch.cuda.synchronize(self.device)
        return _copy_from_device(ptr.value, self.k * self.n, torch.float32, self.device).view(self.k, self.n)


def _make_allocator(allocator: str, device):
    """(list that keeps the handed-out tensors alive, C callback or None)."""
    buffers: list = []
    if allocator == "library":
        return buffers, None
    if allocator != "torch":
        raise ValueError("allocator must be 'torch' or 'library'")

    def _alloc(nbytes, _ctx):
        try:
            buf = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
            buffers.append(buf)
            return buf.data_ptr()
        except Exception:  # out of memory -> NULL -> PIPAD_ERR_ALLOC
            return None
    return buffers, ALLOC_FN(_alloc)


def frame_transpose(frame: Frame, allocator: str = "torch", stream=None) -> Frame:
    """pipad_frame_transpose: the frame of the transposed patterns with the same D^-1/2; aggregating
    with it applies the transposed operator (the backward pass for directed patterns)."""
    lib = load_library()
    buffers, cb = _make_allocator(allocator, frame.device)
    out = _vp()
    with torch.cuda.device(frame.device):
        status = lib.pipad_frame_transpose(frame._h, ctypes.cast(cb, _vp) if cb is not None else None,
                                           None, _stream_handle(stream), ctypes.byref(out))
    _check(status)
    return Frame(out.value, frame.n, frame.k, frame.device, buffers, cb, stream)


def frame_build_overlap(snapshots: Sequence[Snapshot], validate: bool = False,
                        allocator: str = "torch", stream=None) -> Frame:
    """pipad_frame_build_overlap: k CSR snapshots -> frame (overlap CSR + k exclusive CSRs + D^-1/2).

    ``allocator="torch"`` hands every frame buffer out of PyTorch's caching allocator through the
    C callback; ``"library"`` lets the library hipMalloc its own."""
    lib = load_library()
    k = len(snapshots)
    if k < 1:
        raise ValueError("a frame needs at least one snapshot")
    rp0 = snapshots[0][0]
    n = rp0.numel() - 1
    device = rp0.device
    arr = (_Csr * k)()
    keep = []
    for t, (rp, col) in enumerate(snapshots):
        for x in (rp, col):
            if x.dtype != torch.int32 or not x.is_cuda or not x.is_contiguous() or x.device != device:
                raise ValueError("snapshots must be contiguous int32 tensors on one GPU")
        keep.append((rp, col))
        arr[t].n = rp.numel() - 1
        arr[t].nnz = col.numel()
        arr[t].rowptr = rp.data_ptr()
        arr[t].colidx = col.data_ptr() if col.numel() else None
    buffers, cb = _make_allocator(allocator, device)
    out = _vp()
    with torch.cuda.device(device):
        status = lib.pipad_frame_build_overlap(
            n, k, arr, VALIDATE if validate else 0,
            ctypes.cast(cb, _vp) if cb is not None else None, None,
            _stream_handle(stream), ctypes.byref(out))
    _check(status)
    return Frame(out.value, n, k, device, buffers, cb, stream)


Features = Union[torch.Tensor, Sequence[torch.Tensor]]


def _operand(x: Features, n: int, k: int, name: str) -> Tuple[List[int], int, int]:
    """Returns (k device pointers, row stride in elements, F).  Accepts a list of k [n, F] matrices
    sharing one row stride, or one [n, k, F] tensor (the physically concatenated coalescent operand)."""
    if isinstance(x, torch.Tensor):
        if x.dim() != 3 or x.shape[0] != n or x.shape[1] != k:
            raise ValueError(f"{name}: a single tensor must have shape [n, k, F]")
        mats = [x[:, t, :] for t in range(k)]
    else:
        mats = list(x)
        if len(mats) != k:
            raise ValueError(f"{name}: need k = {k} matrices")
    F = mats[0].shape[1]
    ld = None
    ptrs = []
    for m in mats:
        if m.dtype != torch.float32 or not m.is_cuda or m.dim() != 2 or tuple(m.shape) != (n, F):
            raise ValueError(f"{name}: every matrix must be float32 [n, F] on the GPU")
        if F > 1 and m.stride(1) != 1:
            raise ValueError(f"{name}: feature columns must be contiguous")
        row = m.stride(0) if n > 1 else max(m.stride(0), F)
        if ld is None:
            ld = row
        elif n > 1 and row != ld:
            raise ValueError(f"{name}: all matrices must share one row stride")
        ptrs.append(m.data_ptr())
    return ptrs, int(ld), int(F)


def frame_aggregate(frame: Frame, X: Features, Y: Optional[Features] = None, stream=None,
                    static_scratch: bool = False) -> Features:
    """pipad_frame_aggregate: Y_t = D_t^-1/2 (A_t + I) D_t^-1/2 X_t for every snapshot of the frame.

    Y is allocated like X when not given.  Only enqueues work on the stream.
    ``static_scratch=True`` calls pipad_frame_aggregate_static instead (no device allocation inside
    the library; pass Y, or this wrapper allocates it before the call)."""
    lib = load_library()
    n, k = frame.n, frame.k
    xp, ldx, F = _operand(X, n, k, "X")
    if Y is None:
        if isinstance(X, torch.Tensor):
            Y = torch.empty_like(X, memory_format=torch.contiguous_format)
        else:
            Y = [torch.empty((n, F), dtype=torch.float32, device=frame.device) for _ in range(k)]
    yp, ldy, Fy = _operand(Y, n, k, "Y")
    if Fy != F:
        raise ValueError("X and Y must have the same number of feature columns")
    xa = (_vp * k)(*xp)
    ya = (_vp * k)(*yp)
    frame._release_temporaries()
    frame._streams.add(stream if stream is not None else torch.cuda.current_stream(frame.device))
    with torch.cuda.device(frame.device):
        fn = lib.pipad_frame_aggregate_static if static_scratch else lib.pipad_frame_aggregate
        _check(fn(frame._h, F, xa, ldx, ya, ldy, _stream_handle(stream)))
    return Y


def frame_aggregate_subset(frame: Frame, snapshots: Sequence[int], X: Sequence[Optional[torch.Tensor]],
                           Y: Sequence[Optional[torch.Tensor]], stream=None) -> None:
    """pipad_frame_aggregate_subset: Y[t] = D_t^-1/2 (A_t + I) D_t^-1/2 X[t] for the listed snapshots
    of the frame only (inter-frame reuse: the other Y_t are kept from the previous frame).  X and Y
    are lists of k entries; those of snapshots not listed may be None."""
    lib = load_library()
    n, k = frame.n, frame.k
    sel = [int(t) for t in snapshots]
    if not sel:
        return
    if len(X) != k or len(Y) != k:
        raise ValueError("X and Y must have k entries")
    F, ldx, ldy = None, None, None
    xa, ya = (_vp * k)(), (_vp * k)()
    for t in sel:
        for m, name in ((X[t], "X"), (Y[t], "Y")):
            if m is None or m.dtype != torch.float32 or not m.is_cuda or m.dim() != 2 or m.shape[0] != n:
                raise ValueError(f"{name}[{t}] must be a float32 [n, F] matrix on the GPU")
            if m.shape[1] > 1 and m.stride(1) != 1:
                raise ValueError("feature columns must be contiguous")
        if F is None:
            F = int(X[t].shape[1])
            ldx = int(X[t].stride(0)) if n > 1 else max(int(X[t].stride(0)), F)
            ldy = int(Y[t].stride(0)) if n > 1 else max(int(Y[t].stride(0)), F)
        if X[t].shape[1] != F or Y[t].shape[1] != F or (n > 1 and (X[t].stride(0) != ldx or Y[t].stride(0) != ldy)):
            raise ValueError("the chosen matrices must share their shape and row strides")
        xa[t], ya[t] = X[t].data_ptr(), Y[t].data_ptr()
    arr = (_i32 * len(sel))(*sel)
    frame._release_temporaries()
    frame._streams.add(stream if stream is not None else torch.cuda.current_stream(frame.device))
    with torch.cuda.device(frame.device):
        _check(lib.pipad_frame_aggregate_subset(frame._h, len(sel), arr, F, xa, ldx, ya, ldy,
                                                _stream_handle(stream)))


def frame_aggregate_update(frame: Frame, X: Features, W: torch.Tensor,
                           bias: Optional[torch.Tensor] = None, H: Optional[Features] = None,
                           A: Optional[Features] = None, stream=None) -> Features:
    """pipad_frame_aggregate_update: H_t = (D_t^-1/2 (A_t + I) D_t^-1/2 X_t) W + bias for every
    snapshot of the frame.  W is a float32 [F, Fo] device matrix (row stride >= Fo), bias a float32
    [Fo] device vector or None.  H is allocated (k matrices [n, Fo]) when not given; A, when given,
    receives the aggregation results.  Only enqueues work on the stream."""
    lib = load_library()
    n, k = frame.n, frame.k
    xp, ldx, F = _operand(X, n, k, "X")
    if W.dtype != torch.float32 or W.dim() != 2 or W.shape[0] != F or W.stride(1) != 1:
        raise ValueError("W must be a float32 [F, Fo] matrix with unit column stride")
    Fo = int(W.shape[1])
    if bias is not None and (bias.dtype != torch.float32 or bias.dim() != 1 or
                             bias.shape[0] != Fo or bias.stride(0) != 1):
        raise ValueError("bias must be a contiguous float32 vector of Fo entries")
    if H is None:
        H = [torch.empty((n, Fo), dtype=torch.float32, device=frame.device) for _ in range(k)]
    hp, ldh, Fh = _operand(H, n, k, "H")
    if Fh != Fo:
        raise ValueError("H must have Fo feature columns")
    xa = (_vp * k)(*xp)
    ha = (_vp * k)(*hp)
    aa, lda = None, F
    if A is not None:
        ap, lda, Fa = _operand(A, n, k, "A")
        if Fa != F:
            raise ValueError("A must have F feature columns")
        aa = (_vp * k)(*ap)
    frame._release_temporaries()
    frame._streams.add(stream if stream is not None else torch.cuda.current_stream(frame.device))
    with torch.cuda.device(frame.device):
        _check(lib.pipad_frame_aggregate_update(
            frame._h, F, xa, ldx, W.data_ptr(), W.stride(0) if F > 1 else max(Fo, W.stride(0)),
            bias.data_ptr() if bias is not None else None, Fo, aa, lda, ha, ldh,
            _stream_handle(stream)))
    return H
