"""Sharing device buffers and events between the service process and the users' processes on one GPU.

The paper's deployment (section 4, step 3; section 5) runs each user's private attention in a process of its own and
moves Q to it and (A_in, lse_in) back through the host (GLOO), which section 6.2 names as the dominant cost; section 5
mentions device IPC as the alternative.  This module is that alternative for HIP: the service allocates q, A_in and
lse_in once, exports them as IPC memory handles, and the users' processes map them and write their partials in place:
no byte of the message crosses the host.  What orders the two sides' streams is the caller's choice: IPC events
(SharedEvent; some HIP runtimes hand out the handles and then refuse to record such an event - the error names the
call), or a host-side handshake after each side has synchronised its own stream.

Only marshalling: HIP runtime calls through ctypes on the runtime library the process already has loaded.
"""
from __future__ import annotations

import ctypes as C
from typing import Tuple

import torch

HANDLE_BYTES = 64          # hipIpcMemHandle_t and hipIpcEventHandle_t are 64 opaque bytes
_EVENT_DISABLE_TIMING = 0x2
_EVENT_INTERPROCESS = 0x4
_IPC_LAZY_PEER = 0x1


class _Handle(C.Structure):
    """hipIpcMemHandle_t / hipIpcEventHandle_t: the open calls take it by value."""
    _fields_ = [("reserved", C.c_char * HANDLE_BYTES)]


def _handle(raw: bytes) -> _Handle:
    assert len(raw) == HANDLE_BYTES
    h = _Handle()
    C.memmove(C.byref(h), raw, HANDLE_BYTES)
    return h


def _runtime() -> C.CDLL:
    """The HIP runtime this process already uses (loading another copy by name would start a second runtime)."""
    with open("/proc/self/maps") as f:
        paths = {line.split()[-1] for line in f if "libamdhip64" in line}
    assert len(paths) == 1, f"expected one HIP runtime in the process, found {sorted(paths)}"
    hip = C.CDLL(paths.pop())
    hip.hipMalloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t]
    hip.hipFree.argtypes = [C.c_void_p]
    hip.hipIpcGetMemHandle.argtypes = [C.POINTER(_Handle), C.c_void_p]
    hip.hipIpcOpenMemHandle.argtypes = [C.POINTER(C.c_void_p), _Handle, C.c_uint]
    hip.hipIpcCloseMemHandle.argtypes = [C.c_void_p]
    hip.hipEventCreateWithFlags.argtypes = [C.POINTER(C.c_void_p), C.c_uint]
    hip.hipEventDestroy.argtypes = [C.c_void_p]
    hip.hipIpcGetEventHandle.argtypes = [C.POINTER(_Handle), C.c_void_p]
    hip.hipIpcOpenEventHandle.argtypes = [C.POINTER(C.c_void_p), _Handle]
    hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
    hip.hipStreamWaitEvent.argtypes = [C.c_void_p, C.c_void_p, C.c_uint]
    hip.hipEventSynchronize.argtypes = [C.c_void_p]
    for name in ("hipMalloc", "hipFree", "hipIpcGetMemHandle", "hipIpcOpenMemHandle", "hipIpcCloseMemHandle",
                 "hipEventCreateWithFlags", "hipEventDestroy", "hipIpcGetEventHandle", "hipIpcOpenEventHandle",
                 "hipEventRecord", "hipStreamWaitEvent", "hipEventSynchronize"):
        getattr(hip, name).restype = C.c_int
    return hip


_hip = None


def hip() -> C.CDLL:
    global _hip
    if _hip is None:
        assert torch.cuda.is_available(), "device IPC needs a GPU"
        torch.cuda.current_stream()          # the runtime is loaded and the device initialised
        _hip = _runtime()
    return _hip


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"{what} failed with hipError {rc}")


class _Raw:
    """A raw device pointer as something torch.as_tensor understands."""

    def __init__(self, ptr: int, shape: Tuple[int, ...], typestr: str):
        self.__cuda_array_interface__ = {"shape": tuple(shape), "typestr": typestr, "data": (int(ptr), False),
                                         "version": 3, "strides": None}


_TYPESTR = {torch.float32: "<f4", torch.int32: "<i4", torch.uint8: "|u1", torch.int16: "<i2"}


def _as_tensor(ptr: int, shape, dtype: torch.dtype, device) -> torch.Tensor:
    """A tensor over memory this module owns or has mapped (never freed by torch)."""
    if dtype in (torch.bfloat16, torch.float16):      # the array interface has no bf16: view 16-bit integers
        return torch.as_tensor(_Raw(ptr, shape, "<i2"), device=device).view(dtype)
    return torch.as_tensor(_Raw(ptr, shape, _TYPESTR[dtype]), device=device)


class SharedBuffer:
    """A device allocation of its own (hipMalloc, far below the 2 GiB that a shared allocation may have here) that
    other processes can map.  `tensor` views it; `handle` is what the other process passes to `open_buffer`."""

    def __init__(self, shape, dtype: torch.dtype, device="cuda:0"):
        n = 1
        for s in shape:
            n *= int(s)
        self.nbytes = max(256, n * torch.empty((), dtype=dtype).element_size())
        assert self.nbytes < (2 << 30)
        p = C.c_void_p()
        _check(hip().hipMalloc(C.byref(p), self.nbytes), "hipMalloc")
        self.ptr = p.value
        h = _Handle()
        _check(hip().hipIpcGetMemHandle(C.byref(h), self.ptr), "hipIpcGetMemHandle")
        self.handle = C.string_at(C.byref(h), HANDLE_BYTES)
        self.tensor = _as_tensor(self.ptr, tuple(shape), dtype, device)

    def free(self):
        if self.ptr:
            self.tensor = None
            _check(hip().hipFree(self.ptr), "hipFree")
            self.ptr = None


class MappedBuffer:
    """Another process's SharedBuffer, mapped into this one."""

    def __init__(self, handle: bytes, shape, dtype: torch.dtype, device="cuda:0"):
        p = C.c_void_p()
        _check(hip().hipIpcOpenMemHandle(C.byref(p), _handle(handle), _IPC_LAZY_PEER), "hipIpcOpenMemHandle")
        self.ptr = p.value
        self.tensor = _as_tensor(self.ptr, tuple(shape), dtype, device)

    def close(self):
        if self.ptr:
            self.tensor = None
            _check(hip().hipIpcCloseMemHandle(self.ptr), "hipIpcCloseMemHandle")
            self.ptr = None


class SharedEvent:
    """An event that streams of two processes can record and wait for (no timing).  Created by one process
    (`SharedEvent()`), opened by the other (`SharedEvent(handle)`).  Whether the runtime supports it has to be tried:
    the HIP runtime of ROCm 7.2 returns hipErrorInvalidValue from hipEventRecord on an interprocess event (and from the
    first hipIpcGetEventHandle call on it), in which case the two sides synchronise their streams on the host."""

    def __init__(self, handle: bytes = None):
        e = C.c_void_p()
        if handle is None:
            _check(hip().hipEventCreateWithFlags(C.byref(e), _EVENT_DISABLE_TIMING | _EVENT_INTERPROCESS),
                   "hipEventCreateWithFlags")
            h = _Handle()
            if hip().hipIpcGetEventHandle(C.byref(h), e) != 0:      # the first call on an event may fail: once more
                _check(hip().hipIpcGetEventHandle(C.byref(h), e), "hipIpcGetEventHandle")
            self.handle = C.string_at(C.byref(h), HANDLE_BYTES)
        else:
            _check(hip().hipIpcOpenEventHandle(C.byref(e), _handle(handle)), "hipIpcOpenEventHandle")
            self.handle = handle
        self.event = e

    def record(self, stream: "torch.cuda.Stream"):
        _check(hip().hipEventRecord(self.event, C.c_void_p(stream.cuda_stream)), "hipEventRecord")

    def wait(self, stream: "torch.cuda.Stream"):
        """Work enqueued on `stream` after this call runs after the event's latest record."""
        _check(hip().hipStreamWaitEvent(C.c_void_p(stream.cuda_stream), self.event, 0), "hipStreamWaitEvent")

    def synchronize(self):
        _check(hip().hipEventSynchronize(self.event), "hipEventSynchronize")
