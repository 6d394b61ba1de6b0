"""Thin ctypes binding of the C ABI in include/spd.h (argument marshalling only).

Every step of the path runs in the HIP library; there is no Python or CPU fallback.  Importing this
module without the built library raises, and so does any call without a GPU.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SPD_HIP_LIBRARY") or os.path.join(_PKG, "libspd_hip.so")

SPD_OK = 0
SPD_ERR_NULL, SPD_ERR_SHAPE, SPD_ERR_LEN, SPD_ERR_ALIGN = -1, -2, -3, -4
SPD_ERR_WORKSPACE, SPD_ERR_HIP, SPD_ERR_NOMEM = -5, -6, -7
SPD_F32, SPD_BF16, SPD_F16 = 0, 1, 2
(SPD_OPT_HEAD_PER_WAVE, SPD_OPT_TARGET_WG_PER_CU, SPD_OPT_NO_SPLIT_MAX, SPD_OPT_CHUNK_MAX, SPD_OPT_SEG_COST,
 SPD_OPT_HALF_SKEW, SPD_OPT_RESULT_ROWS, SPD_OPT_STEPS_IN_FLIGHT) = range(8)

EXPORTED_SYMBOLS = (
    "spd_create", "spd_destroy", "spd_strerror", "spd_last_hip_error",
    "spd_partial_attn_private", "spd_partial_attn_public_batched", "spd_lse_merge",
    "spd_validate_partial", "spd_build_schedule", "spd_set_kernel_timing", "spd_get_kernel_timing",
    "spd_decode_step", "spd_partial_attn_public_batched_append", "spd_get_schedule_stats",
    "spd_attention_mass_track", "spd_get_kernel_timing_samples", "spd_lse_merge_n", "spd_public_attn_merge",
    "spd_abi_version", "spd_decode_step_static", "spd_set_option", "spd_get_option",
    "spd_get_last_kernel_instance",
)

SPD_ABI_VERSION = 4      # include/spd.h's; checked against the loaded library below


class SpdError(RuntimeError):
    def __init__(self, code: int, where: str, hip: int = 0):
        self.code = code
        msg = f"{where}: {spd_strerror(code)} (code {code})"
        if hip:
            msg += f", hipError {hip}"
        super().__init__(msg)


class spd_shape(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("scale", C.c_float)]


class spd_kv_view(C.Structure):
    _fields_ = [("n_users", C.c_int32), ("lens", C.POINTER(C.c_int32)),
                ("k_ptrs", C.POINTER(C.c_void_p)), ("v_ptrs", C.POINTER(C.c_void_p)),
                ("token_stride", C.c_int64), ("head_stride", C.c_int64), ("head_strides", C.POINTER(C.c_int64)),
                ("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("block_size", C.c_int32),
                ("block_table", C.c_void_p), ("max_blocks", C.c_int32), ("block_stride", C.c_int64),
                ("k_ptrs_dev", C.c_void_p), ("v_ptrs_dev", C.c_void_p)]


class spd_work_item(C.Structure):
    _fields_ = [("user", C.c_int32), ("kv_head", C.c_int32), ("t_begin", C.c_int32), ("t_end", C.c_int32),
                ("slot", C.c_int32), ("n_chunks", C.c_int32), ("chunk", C.c_int32), ("piece", C.c_int32)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(the SPD path has no fallback)")
    lib = C.CDLL(LIB_PATH)
    if not hasattr(lib, "spd_abi_version") or lib.spd_abi_version() != SPD_ABI_VERSION:
        raise ImportError(f"{LIB_PATH} was built from another version of include/spd.h; build it again")
    vp, fp = C.c_void_p, C.c_void_p
    lib.spd_create.restype = C.c_int
    lib.spd_create.argtypes = [C.POINTER(vp), C.c_int]
    lib.spd_destroy.restype = C.c_int
    lib.spd_destroy.argtypes = [vp]
    lib.spd_strerror.restype = C.c_char_p
    lib.spd_strerror.argtypes = [C.c_int]
    lib.spd_last_hip_error.restype = C.c_int
    lib.spd_last_hip_error.argtypes = [vp]
    for name in ("spd_partial_attn_private", "spd_partial_attn_public_batched"):
        fn = getattr(lib, name)
        fn.restype = C.c_int
        fn.argtypes = [vp, C.POINTER(spd_shape), vp, C.POINTER(spd_kv_view), fp, fp, vp]
    lib.spd_lse_merge.restype = C.c_int
    lib.spd_lse_merge.argtypes = [vp, C.c_int32, C.c_int32, fp, fp, fp, fp, fp, fp, fp, vp]
    lib.spd_public_attn_merge.restype = C.c_int
    lib.spd_public_attn_merge.argtypes = [vp, C.POINTER(spd_shape), vp, C.POINTER(spd_kv_view), vp, vp, fp, fp, fp, fp,
                                          fp, fp, fp, vp]
    lib.spd_lse_merge_n.restype = C.c_int
    lib.spd_lse_merge_n.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                    fp, fp, fp, vp]
    lib.spd_attention_mass_track.restype = C.c_int
    lib.spd_attention_mass_track.argtypes = [vp, C.c_int32, fp, C.c_float, fp, fp, vp, vp]
    lib.spd_decode_step.restype = C.c_int
    lib.spd_decode_step.argtypes = [vp, C.POINTER(spd_shape), vp, C.POINTER(spd_kv_view), C.POINTER(spd_kv_view),
                                    vp, vp, fp, fp, fp, fp, fp, fp, fp, vp]
    lib.spd_decode_step_static.restype = C.c_int
    lib.spd_decode_step_static.argtypes = lib.spd_decode_step.argtypes
    lib.spd_partial_attn_public_batched_append.restype = C.c_int
    lib.spd_partial_attn_public_batched_append.argtypes = [vp, C.POINTER(spd_shape), vp, vp, vp,
                                                           C.POINTER(spd_kv_view), fp, fp, vp]
    lib.spd_get_schedule_stats.restype = C.c_int
    lib.spd_get_schedule_stats.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    lib.spd_set_kernel_timing.restype = C.c_int
    lib.spd_set_kernel_timing.argtypes = [vp, C.c_int32]
    lib.spd_get_kernel_timing.restype = C.c_int
    lib.spd_get_kernel_timing.argtypes = [vp, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_double),
                                          C.POINTER(C.c_double)]
    lib.spd_get_kernel_timing_samples.restype = C.c_int
    lib.spd_get_kernel_timing_samples.argtypes = [vp, C.c_int32, C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_int32)]
    lib.spd_get_last_kernel_instance.restype = C.c_int
    lib.spd_get_last_kernel_instance.argtypes = [vp, C.POINTER(C.c_int32)]
    lib.spd_set_option.restype = C.c_int
    lib.spd_set_option.argtypes = [vp, C.c_int32, C.c_int32]
    lib.spd_get_option.restype = C.c_int
    lib.spd_get_option.argtypes = [vp, C.c_int32, C.POINTER(C.c_int32)]
    lib.spd_validate_partial.restype = C.c_int
    lib.spd_validate_partial.argtypes = [C.POINTER(spd_shape), vp, C.POINTER(spd_kv_view), fp, fp]
    lib.spd_build_schedule.restype = C.c_int
    lib.spd_build_schedule.argtypes = [C.POINTER(spd_shape), C.c_int32, C.POINTER(C.c_int32), C.c_int32, C.c_int32,
                                       C.POINTER(spd_work_item), C.c_int64, C.POINTER(C.c_int64),
                                       C.POINTER(C.c_int32)]
    return lib


lib = _load()


def spd_strerror(code: int) -> str:
    return lib.spd_strerror(int(code)).decode()


def make_shape(dtype, n_q_heads: int, n_kv_heads: int, head_dim: int, scale: float) -> spd_shape:
    if isinstance(dtype, torch.dtype):
        dtype = {torch.float32: SPD_F32, torch.bfloat16: SPD_BF16, torch.float16: SPD_F16}[dtype]
    return spd_shape(int(dtype), int(n_q_heads), int(n_kv_heads), int(head_dim), float(scale))


class KVView:
    """Marshalled spd_kv_view; keeps the host arrays (and the tensors they point into) alive."""

    def __init__(self, lens, token_stride: int, head_stride: int, k: Optional[Sequence[torch.Tensor]] = None,
                 v: Optional[Sequence[torch.Tensor]] = None, k_pool: Optional[torch.Tensor] = None,
                 v_pool: Optional[torch.Tensor] = None, block_table: Optional[torch.Tensor] = None,
                 block_size: int = 0, block_stride: int = 0, max_blocks: Optional[int] = None,
                 head_strides=None, device_pointer_tables: bool = False):
        """device_pointer_tables (contiguous mode): also hand the per-user pointers over in device arrays, which makes
        the split schedule independent of the buffers' addresses (views of different layers then share one)."""
        self.lens = np.ascontiguousarray(lens, dtype=np.int32)
        n = int(self.lens.shape[0])
        self._keep = (k, v, k_pool, v_pool, block_table)
        st = spd_kv_view()
        st.n_users = n
        st.lens = self.lens.ctypes.data_as(C.POINTER(C.c_int32))
        st.token_stride, st.head_stride = int(token_stride), int(head_stride)
        st.block_size, st.block_stride = int(block_size), int(block_stride)
        if head_strides is not None:
            self.head_strides = np.ascontiguousarray(head_strides, dtype=np.int64)
            assert self.head_strides.shape == (n,)
            st.head_strides = self.head_strides.ctypes.data_as(C.POINTER(C.c_int64))
        if block_size == 0:
            assert k is not None and v is not None and len(k) == n == len(v)
            self._kp = (C.c_void_p * max(1, n))(*[t.data_ptr() if t.numel() else None for t in k])
            self._vp = (C.c_void_p * max(1, n))(*[t.data_ptr() if t.numel() else None for t in v])
            st.k_ptrs = C.cast(self._kp, C.POINTER(C.c_void_p))
            st.v_ptrs = C.cast(self._vp, C.POINTER(C.c_void_p))
            if device_pointer_tables and n:
                dev = k[0].device
                self._kp_dev = torch.tensor([t.data_ptr() if t.numel() else 0 for t in k], dtype=torch.int64, device=dev)
                self._vp_dev = torch.tensor([t.data_ptr() if t.numel() else 0 for t in v], dtype=torch.int64, device=dev)
                st.k_ptrs_dev, st.v_ptrs_dev = self._kp_dev.data_ptr(), self._vp_dev.data_ptr()
        else:
            st.k_pool, st.v_pool = k_pool.data_ptr(), v_pool.data_ptr()
            st.block_table = block_table.data_ptr()
            st.max_blocks = int(block_table.shape[1] if max_blocks is None else max_blocks)
        self.struct = st

    @classmethod
    def from_side(cls, side, device_pointer_tables: bool = False) -> "KVView":
        """From a workloads.KVSide (tensors already on the GPU)."""
        if side.paged:
            return cls(side.lens, side.token_stride, side.head_stride, k_pool=side.k_pool, v_pool=side.v_pool,
                       block_table=side.block_table, block_size=side.page_tokens, block_stride=side.block_stride)
        return cls(side.lens, side.token_stride, side.head_stride, k=side.k, v=side.v,
                   head_strides=getattr(side, "head_strides", None), device_pointer_tables=device_pointer_tables)


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


class Context:
    """Owns an spd_ctx on one device."""

    def __init__(self, device: int = 0):
        h = C.c_void_p()
        rc = lib.spd_create(C.byref(h), int(device))
        if rc != SPD_OK:
            raise SpdError(rc, "spd_create")
        self.handle = h
        self.device = int(device)

    def close(self):
        if self.handle:
            lib.spd_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int, where: str):
        if rc != SPD_OK:
            raise SpdError(rc, where, lib.spd_last_hip_error(self.handle) if rc == SPD_ERR_HIP else 0)

    def _partial(self, fn, name, shape: spd_shape, q: torch.Tensor, view: KVView, out, lse, stream):
        n, Hq, d = view.struct.n_users, shape.n_q_heads, shape.head_dim
        if out is None:
            out = torch.empty((n, Hq, d), device=q.device, dtype=torch.float32)
        if lse is None:
            lse = torch.empty((n, Hq), device=q.device, dtype=torch.float32)
        assert q.is_contiguous() and out.is_contiguous() and lse.is_contiguous()
        assert tuple(q.shape) == (n, Hq, d) and tuple(out.shape) == (n, Hq, d) and tuple(lse.shape) == (n, Hq)
        assert out.dtype == torch.float32 and lse.dtype == torch.float32
        rc = fn(self.handle, C.byref(shape), q.data_ptr(), C.byref(view.struct), out.data_ptr(), lse.data_ptr(),
                _stream_ptr(stream))
        self._check(rc, name)
        return out, lse

    def spd_last_kernel_name(self) -> str:
        """The partial kernel instance launched last, as a profiler prints it."""
        a = (C.c_int32 * 6)()
        self._check(lib.spd_get_last_kernel_instance(self.handle, a), "spd_get_last_kernel_instance")
        b = lambda x: "true" if x else "false"
        return f"partial_mfma_kernel<{a[0]}, {a[1]}, {b(a[2])}, {b(a[3])}, {b(a[4])}, {b(a[5])}>"

    def spd_set_option(self, option: int, value: int):
        self._check(lib.spd_set_option(self.handle, int(option), int(value)), "spd_set_option")

    def spd_get_option(self, option: int) -> int:
        v = C.c_int32(0)
        self._check(lib.spd_get_option(self.handle, int(option), C.byref(v)), "spd_get_option")
        return int(v.value)

    def spd_get_schedule_stats(self):
        """(builds, hits) of the split-schedule cache."""
        b, h = C.c_int64(0), C.c_int64(0)
        self._check(lib.spd_get_schedule_stats(self.handle, C.byref(b), C.byref(h)), "spd_get_schedule_stats")
        return int(b.value), int(h.value)

    def spd_get_kernel_timing_samples(self, entry_point: int, capacity: int = 1 << 16):
        """Durations (us) of the recorded launches of one entry point, in launch order; clears the record."""
        buf = (C.c_float * max(1, capacity))()
        n = C.c_int32(0)
        self._check(lib.spd_get_kernel_timing_samples(self.handle, int(entry_point), int(capacity), buf, C.byref(n)),
                    "spd_get_kernel_timing_samples")
        return [float(buf[i]) for i in range(min(int(n.value), capacity))]

    def spd_set_kernel_timing(self, max_launches: int):
        self._check(lib.spd_set_kernel_timing(self.handle, int(max_launches)), "spd_set_kernel_timing")

    def spd_get_kernel_timing(self, entry_point: int):
        """(n_launches, mean_us, min_us) of the partial kernel of entry point 0 (private) or 1 (public)."""
        n, mean, mn = C.c_int32(0), C.c_double(0), C.c_double(0)
        self._check(lib.spd_get_kernel_timing(self.handle, entry_point, C.byref(n), C.byref(mean), C.byref(mn)),
                    "spd_get_kernel_timing")
        return int(n.value), float(mean.value), float(mn.value)

    def spd_partial_attn_private(self, shape, q, view, out=None, lse=None, stream=None):
        return self._partial(lib.spd_partial_attn_private, "spd_partial_attn_private", shape, q, view, out, lse, stream)

    def spd_partial_attn_public_batched(self, shape, q, view, out=None, lse=None, stream=None):
        return self._partial(lib.spd_partial_attn_public_batched, "spd_partial_attn_public_batched", shape, q, view,
                             out, lse, stream)

    def spd_partial_attn_public_batched_append(self, shape, q, k_new, v_new, view, out=None, lse=None, stream=None):
        n, Hq, d = view.struct.n_users, shape.n_q_heads, shape.head_dim
        if out is None:
            out = torch.empty((n, Hq, d), device=q.device, dtype=torch.float32)
        if lse is None:
            lse = torch.empty((n, Hq), device=q.device, dtype=torch.float32)
        for t in (k_new, v_new):
            assert t.is_contiguous() and t.dtype == q.dtype and tuple(t.shape) == (n, shape.n_kv_heads, d)
        assert q.is_contiguous() and tuple(q.shape) == (n, Hq, d)
        rc = lib.spd_partial_attn_public_batched_append(self.handle, C.byref(shape), q.data_ptr(), k_new.data_ptr(),
                                                        v_new.data_ptr(), C.byref(view.struct), out.data_ptr(),
                                                        lse.data_ptr(), _stream_ptr(stream))
        self._check(rc, "spd_partial_attn_public_batched_append")
        return out, lse

    def spd_decode_step(self, shape, q, private, public, a_in, lse_in, a_out, lse_out, y, lse, w_in, stream=None,
                        k_new=None, v_new=None):
        n, Hq, d = private.struct.n_users, shape.n_q_heads, shape.head_dim
        for t in (a_in, a_out, y):
            assert t.is_contiguous() and t.dtype == torch.float32 and tuple(t.shape) == (n, Hq, d)
        for t in (lse_in, lse_out, lse, w_in):
            assert t.is_contiguous() and t.dtype == torch.float32 and tuple(t.shape) == (n, Hq)
        assert q.is_contiguous() and tuple(q.shape) == (n, Hq, d)
        for t in (k_new, v_new):
            assert t is None or (t.is_contiguous() and t.dtype == q.dtype and tuple(t.shape) == (n, shape.n_kv_heads, d))
        rc = lib.spd_decode_step(self.handle, C.byref(shape), q.data_ptr(), C.byref(private.struct),
                                 C.byref(public.struct), None if k_new is None else k_new.data_ptr(),
                                 None if v_new is None else v_new.data_ptr(),
                                 a_in.data_ptr(), lse_in.data_ptr(), a_out.data_ptr(),
                                 lse_out.data_ptr(), y.data_ptr(), lse.data_ptr(), w_in.data_ptr(), _stream_ptr(stream))
        self._check(rc, "spd_decode_step")
        return y

    def spd_decode_step_static(self, shape, q, private, public, a_in, lse_in, a_out, lse_out, y, lse, w_in, stream=None,
                               k_new=None, v_new=None):
        """spd_decode_step on the library's fixed scratch array (allocates nothing)."""
        n, Hq, d = private.struct.n_users, shape.n_q_heads, shape.head_dim
        for t in (a_in, a_out, y):
            assert t.is_contiguous() and t.dtype == torch.float32 and tuple(t.shape) == (n, Hq, d)
        for t in (lse_in, lse_out, lse, w_in):
            assert t.is_contiguous() and t.dtype == torch.float32 and tuple(t.shape) == (n, Hq)
        assert q.is_contiguous() and tuple(q.shape) == (n, Hq, d)
        for t in (k_new, v_new):
            assert t is None or (t.is_contiguous() and t.dtype == q.dtype and tuple(t.shape) == (n, shape.n_kv_heads, d))
        rc = lib.spd_decode_step_static(self.handle, C.byref(shape), q.data_ptr(), C.byref(private.struct),
                                        C.byref(public.struct), None if k_new is None else k_new.data_ptr(),
                                        None if v_new is None else v_new.data_ptr(),
                                        a_in.data_ptr(), lse_in.data_ptr(), a_out.data_ptr(),
                                        lse_out.data_ptr(), y.data_ptr(), lse.data_ptr(), w_in.data_ptr(), _stream_ptr(stream))
        self._check(rc, "spd_decode_step_static")
        return y

    def spd_attention_mass_track(self, w_in, threshold, mass_min=None, mass_sum=None, n_below=None, stream=None):
        n = w_in.numel()
        for t in (w_in, mass_min, mass_sum):
            assert t is None or (t.is_contiguous() and t.dtype == torch.float32 and t.numel() == n)
        assert n_below is None or (n_below.is_contiguous() and n_below.dtype == torch.int32 and n_below.numel() == n)
        ptr = lambda t: None if t is None else t.data_ptr()
        rc = lib.spd_attention_mass_track(self.handle, n, w_in.data_ptr(), float(threshold), ptr(mass_min), ptr(mass_sum),
                                          ptr(n_below),
                                          _stream_ptr(stream))
        self._check(rc, "spd_attention_mass_track")

    def spd_lse_merge(self, a0, lse0, a1, lse1, y=None, lse_out=None, w0_out=None, stream=None):
        n_rows = lse0.numel()
        d = a0.shape[-1]
        if y is None:
            y = torch.empty_like(a0)
        for t in (a0, a1, y, lse0, lse1):
            assert t.is_contiguous() and t.dtype == torch.float32
        assert a0.numel() == n_rows * d == a1.numel() == y.numel() and lse1.numel() == n_rows
        rc = lib.spd_lse_merge(self.handle, n_rows, d, a0.data_ptr(), lse0.data_ptr(), a1.data_ptr(), lse1.data_ptr(),
                               y.data_ptr(), None if lse_out is None else lse_out.data_ptr(),
                               None if w0_out is None else w0_out.data_ptr(), _stream_ptr(stream))
        self._check(rc, "spd_lse_merge")
        return y


    def spd_public_attn_merge(self, shape, q, public, a_in, lse_in, a_out, lse_out, y, lse, w_in, stream=None,
                              k_new=None, v_new=None):
        """The service's half of a step: public partial (+ append) and the merge with delivered private partials."""
        n, Hq, d = public.struct.n_users, shape.n_q_heads, shape.head_dim
        for t in (a_in, a_out, y):
            assert t.is_contiguous() and t.dtype == torch.float32 and tuple(t.shape) == (n, Hq, d)
        for t in (lse_in, lse_out, lse, w_in):
            assert t.is_contiguous() and t.dtype == torch.float32 and tuple(t.shape) == (n, Hq)
        assert q.is_contiguous() and tuple(q.shape) == (n, Hq, d)
        assert (k_new is None) == (v_new is None)
        for t in (k_new, v_new):
            assert t is None or (t.is_contiguous() and t.dtype == q.dtype and tuple(t.shape) == (n, shape.n_kv_heads, d))
        rc = lib.spd_public_attn_merge(self.handle, C.byref(shape), q.data_ptr(), C.byref(public.struct),
                                       None if k_new is None else k_new.data_ptr(),
                                       None if v_new is None else v_new.data_ptr(), a_in.data_ptr(), lse_in.data_ptr(),
                                       a_out.data_ptr(), lse_out.data_ptr(), y.data_ptr(), lse.data_ptr(),
                                       w_in.data_ptr(), _stream_ptr(stream))
        self._check(rc, "spd_public_attn_merge")
        return y

    def spd_lse_merge_n(self, a_parts, lse_parts, y=None, lse_out=None, w_out=None, stream=None):
        """n-way merge of partials (lists of [n_rows..., d] and [n_rows...] fp32 tensors); w_out: [n_parts, n_rows]."""
        n = len(a_parts)
        assert n == len(lse_parts) and n >= 1
        n_rows = lse_parts[0].numel()
        d = a_parts[0].shape[-1]
        if y is None:
            y = torch.empty_like(a_parts[0])
        for t in (*a_parts, *lse_parts, y):
            assert t.is_contiguous() and t.dtype == torch.float32
        assert all(a.numel() == n_rows * d for a in a_parts) and all(l.numel() == n_rows for l in lse_parts)
        assert w_out is None or (w_out.is_contiguous() and w_out.dtype == torch.float32 and w_out.numel() == n * n_rows)
        ap = (C.c_void_p * n)(*[a.data_ptr() for a in a_parts])
        lp = (C.c_void_p * n)(*[l.data_ptr() for l in lse_parts])
        rc = lib.spd_lse_merge_n(self.handle, n, n_rows, d, ap, lp, y.data_ptr(),
                                 None if lse_out is None else lse_out.data_ptr(),
                                 None if w_out is None else w_out.data_ptr(), _stream_ptr(stream))
        self._check(rc, "spd_lse_merge_n")
        return y


def spd_validate_partial(shape: spd_shape, q_ptr, view: spd_kv_view, out_ptr, lse_ptr) -> int:
    return int(lib.spd_validate_partial(C.byref(shape), q_ptr, C.byref(view), out_ptr, lse_ptr))


def spd_build_schedule(shape: spd_shape, lens, n_compute_units: int, head_per_wave=False):
    """Host-only: the split schedule for `lens`.  Returns (list of item dicts, chunk_tokens).
    head_per_wave: False / 0 the head-major mapping; True / 1 the head-per-wave mapping with the widest head groups
    (up to 8 KV heads); 2..8 the same with at most that many heads per group."""
    lens = np.ascontiguousarray(lens, dtype=np.int32)
    n = C.c_int64(0)
    chunk = C.c_int32(0)
    lp = lens.ctypes.data_as(C.POINTER(C.c_int32))
    hpw = int(head_per_wave)
    rc = lib.spd_build_schedule(C.byref(shape), len(lens), lp, n_compute_units, hpw, None, 0, C.byref(n), C.byref(chunk))
    if rc != SPD_OK:
        raise SpdError(rc, "spd_build_schedule")
    items = (spd_work_item * max(1, n.value))()
    rc = lib.spd_build_schedule(C.byref(shape), len(lens), lp, n_compute_units, hpw, items, n.value, C.byref(n),
                                C.byref(chunk))
    if rc != SPD_OK:
        raise SpdError(rc, "spd_build_schedule")
    fields = [f[0] for f in spd_work_item._fields_]
    return [{f: getattr(items[i], f) for f in fields} for i in range(n.value)], int(chunk.value)
