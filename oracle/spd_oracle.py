"""ctypes front end of the fp64 CPU oracle (oracle/spd_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg.  The product package never imports this module
and this module never imports the product package.

All arrays are host numpy arrays; bf16 data travels as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spd_oracle.c")
_LIB = os.path.join(_HERE, "libspd_oracle.so")

F32, BF16, F16 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (fp64, OpenMP over output rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _View(C.Structure):
    _fields_ = [
        ("n_users", C.c_int32), ("lens", C.POINTER(C.c_int32)),
        ("k_ptrs", C.POINTER(C.c_void_p)), ("v_ptrs", C.POINTER(C.c_void_p)),
        ("token_stride", C.c_int64), ("head_stride", C.c_int64), ("head_strides", C.POINTER(C.c_int64)),
        ("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("block_size", C.c_int32),
        ("block_table", C.POINTER(C.c_int32)), ("max_blocks", C.c_int32), ("block_stride", C.c_int64),
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        dp = C.POINTER(C.c_double)
        ip = C.POINTER(C.c_int32)
        lib.orc_attention.restype = C.c_int
        lib.orc_attention.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, C.c_int, C.c_void_p,
                                      C.c_int, C.POINTER(C.POINTER(_View)), C.c_int, ip, dp, dp]
        lib.orc_partial.restype = C.c_int
        lib.orc_partial.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, C.c_int, C.c_void_p,
                                    C.POINTER(_View), ip, ip, C.c_int, ip, dp, dp, dp]
        lib.orc_merge.restype = None
        lib.orc_merge.argtypes = [C.c_int, C.c_int, dp, dp, dp, dp, dp, dp, dp, dp, dp, dp]
        lib.orc_threads.restype = C.c_int
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().orc_threads())


class HostView:
    """One owner's cache on the host.  Keeps every array alive for the C side."""

    def __init__(self, lens, token_stride, head_stride, k: Optional[Sequence[np.ndarray]] = None,
                 v: Optional[Sequence[np.ndarray]] = None, k_pool: Optional[np.ndarray] = None,
                 v_pool: Optional[np.ndarray] = None, block_size: int = 0,
                 block_table: Optional[np.ndarray] = None, block_stride: int = 0, head_strides=None):
        self.lens = np.ascontiguousarray(lens, dtype=np.int32)
        self.n_users = int(self.lens.shape[0])
        self.k, self.v, self.k_pool, self.v_pool = k, v, k_pool, v_pool
        self.block_size = int(block_size)
        self.token_stride, self.head_stride, self.block_stride = int(token_stride), int(head_stride), int(block_stride)
        st = _View()
        st.n_users = self.n_users
        st.lens = self.lens.ctypes.data_as(C.POINTER(C.c_int32))
        st.token_stride, st.head_stride = self.token_stride, self.head_stride
        st.block_size, st.block_stride = self.block_size, self.block_stride
        self.head_strides = None
        if head_strides is not None:
            self.head_strides = np.ascontiguousarray(head_strides, dtype=np.int64)
            assert self.head_strides.shape == (self.n_users,)
            st.head_strides = self.head_strides.ctypes.data_as(C.POINTER(C.c_int64))
        if self.block_size == 0:
            assert k is not None and v is not None and len(k) == self.n_users == len(v)
            for a in list(k) + list(v):
                assert a.flags["C_CONTIGUOUS"]
            self._kp = (C.c_void_p * max(1, self.n_users))(*[a.ctypes.data for a in k])
            self._vp = (C.c_void_p * max(1, self.n_users))(*[a.ctypes.data for a in v])
            st.k_ptrs = C.cast(self._kp, C.POINTER(C.c_void_p))
            st.v_ptrs = C.cast(self._vp, C.POINTER(C.c_void_p))
        else:
            assert k_pool is not None and v_pool is not None and block_table is not None
            assert k_pool.flags["C_CONTIGUOUS"] and v_pool.flags["C_CONTIGUOUS"]
            self.block_table = np.ascontiguousarray(block_table, dtype=np.int32)
            assert self.block_table.ndim == 2 and self.block_table.shape[0] == self.n_users
            need = -(-self.lens.astype(np.int64) // self.block_size)
            assert (need <= self.block_table.shape[1]).all()
            n_blocks = k_pool.size // self.block_stride
            for u in range(self.n_users):
                used = self.block_table[u, :need[u]]
                assert used.size == 0 or (used.min() >= 0 and used.max() < n_blocks), "page id out of range"
            st.k_pool, st.v_pool = k_pool.ctypes.data, v_pool.ctypes.data
            st.block_table = self.block_table.ctypes.data_as(C.POINTER(C.c_int32))
            st.max_blocks = int(self.block_table.shape[1])
        self.struct = st


class HostWorkload:
    """Host-side copy of a workload (exact bits) in the form the oracle reads."""

    def __init__(self, dtype: int, n_q_heads: int, n_kv_heads: int, head_dim: int, scale: float,
                 q: np.ndarray, private: HostView, public: HostView):
        assert n_q_heads % n_kv_heads == 0
        self.dtype, self.Hq, self.Hkv, self.d, self.scale = dtype, n_q_heads, n_kv_heads, head_dim, float(scale)
        self.q = np.ascontiguousarray(q)
        self.U = int(self.q.shape[0])
        assert self.q.shape == (self.U, self.Hq, self.d)
        assert self.q.dtype == (np.float32 if dtype == F32 else np.uint16)
        self.private, self.public = private, public
        assert private.n_users == self.U and public.n_users == self.U


def from_workload(wl) -> HostWorkload:
    """Copy a workloads.Workload (tensors on any device) to the host, bit for bit."""
    import torch
    from workloads import host_array

    def side(s) -> HostView:
        if s.paged:
            return HostView(s.lens, s.token_stride, s.head_stride, k_pool=host_array(s.k_pool),
                            v_pool=host_array(s.v_pool), block_size=s.page_tokens,
                            block_table=s.block_table.cpu().numpy(), block_stride=s.block_stride)
        return HostView(s.lens, s.token_stride, s.head_stride, k=[host_array(t) for t in s.k],
                        v=[host_array(t) for t in s.v], head_strides=getattr(s, "head_strides", None))

    dt = {torch.float32: F32, torch.bfloat16: BF16, torch.float16: F16}[wl.dtype]
    return HostWorkload(dt, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.scale, host_array(wl.q),
                        side(wl.private), side(wl.public))


def _rows_arg(rows, U, Hq):
    if rows is None:
        return None, U * Hq, None
    r = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 2)
    assert r.size == 0 or (r[:, 0].min() >= 0 and r[:, 0].max() < U and r[:, 1].min() >= 0 and r[:, 1].max() < Hq)
    return r.ctypes.data_as(C.POINTER(C.c_int32)), int(r.shape[0]), r


def _dp(a):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def attention(hw: HostWorkload, views: Optional[List[HostView]] = None, rows=None):
    """Unsplit softmax attention over concat(private, public) (or the given views, in order).

    Returns (Y [n_rows, d] float64, lse [n_rows] float64); rows default to all (u, h) in order.
    """
    lib = _load()
    views = [hw.private, hw.public] if views is None else views
    rp, n_rows, keep = _rows_arg(rows, hw.U, hw.Hq)
    Y = np.zeros((n_rows, hw.d), dtype=np.float64)
    lse = np.zeros((n_rows,), dtype=np.float64)
    arr = (C.POINTER(_View) * len(views))(*[C.pointer(v.struct) for v in views])
    rc = lib.orc_attention(hw.U, hw.Hq, hw.Hkv, hw.d, hw.scale, hw.dtype, hw.q.ctypes.data,
                           len(views), arr, n_rows, rp, _dp(Y), _dp(lse))
    if rc != 0:
        raise MemoryError("orc_attention")
    return Y, lse


def partial(hw: HostWorkload, view: HostView, t0=None, t1=None, rows=None):
    """One owner's message over tokens [t0[u], t1[u]) of ``view`` (default: all of it).

    Returns (A [n_rows, d], m [n_rows], gamma [n_rows]) in the paper's notation.
    """
    lib = _load()
    rp, n_rows, keep = _rows_arg(rows, hw.U, hw.Hq)
    ip = C.POINTER(C.c_int32)
    a0 = None if t0 is None else np.ascontiguousarray(t0, dtype=np.int32)
    a1 = None if t1 is None else np.ascontiguousarray(t1, dtype=np.int32)
    if a0 is not None:
        assert a0.shape == (hw.U,) and (a0 >= 0).all()
    if a1 is not None:
        assert a1.shape == (hw.U,) and (a1 <= view.lens).all()
    A = np.zeros((n_rows, hw.d), dtype=np.float64)
    m = np.zeros((n_rows,), dtype=np.float64)
    g = np.zeros((n_rows,), dtype=np.float64)
    rc = lib.orc_partial(hw.U, hw.Hq, hw.Hkv, hw.d, hw.scale, hw.dtype, hw.q.ctypes.data,
                         C.byref(view.struct),
                         None if a0 is None else a0.ctypes.data_as(ip),
                         None if a1 is None else a1.ctypes.data_as(ip),
                         n_rows, rp, _dp(A), _dp(m), _dp(g))
    if rc != 0:
        raise MemoryError("orc_partial")
    return A, m, g


def merge(A_in, m_in, g_in, A_out, m_out, g_out):
    """Theorem 1 with stabilised coefficients.  Returns (Y, m, gamma, w_in)."""
    lib = _load()
    A_in = np.ascontiguousarray(A_in, dtype=np.float64)
    A_out = np.ascontiguousarray(A_out, dtype=np.float64)
    n, d = A_in.shape
    assert A_out.shape == (n, d)
    st = [np.ascontiguousarray(x, dtype=np.float64) for x in (m_in, g_in, m_out, g_out)]
    for x in st:
        assert x.shape == (n,)
    Y = np.zeros((n, d)); m = np.zeros(n); g = np.zeros(n); w = np.zeros(n)
    lib.orc_merge(n, d, _dp(A_in), _dp(st[0]), _dp(st[1]), _dp(A_out), _dp(st[2]), _dp(st[3]),
                  _dp(Y), _dp(m), _dp(g), _dp(w))
    return Y, m, g, w


def lse_of(m, gamma):
    """ln of the unshifted softmax denominator: m + ln(gamma); -inf for an empty part."""
    m = np.asarray(m, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    with np.errstate(divide="ignore", invalid="ignore"):
        out = m + np.log(gamma)
    return np.where(gamma == 0.0, -np.inf, out)


def merge_n(parts):
    """Theorem 1 for n owners of disjoint token sets (the theorem applied n - 1 times; written out once):
    with lse_i = m_i + ln gamma_i the merged output is Y = sum_i (e^{lse_i} / sum_j e^{lse_j}) A_i, the weight of
    part i being its share of the softmax denominator, and lse = ln sum_j e^{lse_j}.

    parts: sequence of (A_i [n_rows, d], lse_i [n_rows]); an empty part has lse_i = -inf and weight 0 (its A_i is
    ignored).  Returns (Y [n_rows, d], lse [n_rows], w [n_parts, n_rows]); rows whose parts are all empty give
    Y = 0, lse = -inf, w = 0.
    """
    A = [np.asarray(a, dtype=np.float64) for a, _ in parts]
    L = [np.asarray(l, dtype=np.float64) for _, l in parts]
    n_rows, d = A[0].shape
    Y = np.zeros((n_rows, d))
    lse = np.full(n_rows, -np.inf)
    W = np.zeros((len(parts), n_rows))
    for r in range(n_rows):
        top = max(float(l[r]) for l in L)          # the largest log-sum-exp: shift so that no exponential overflows
        if top == -np.inf:
            continue
        e = [np.exp(float(l[r]) - top) for l in L]
        den = sum(e)
        lse[r] = top + np.log(den)
        for i in range(len(parts)):
            W[i, r] = e[i] / den
            if e[i] != 0.0:
                Y[r] += W[i, r] * A[i][r]
    return Y, lse, W


def attention_mass_track(w_steps, threshold: float):
    """Running statistics of the private part's attention mass w_in = gamma_in / (gamma_in + gamma_out) (the weight
    of A_in in Theorem 1) over a sequence of decode steps: the quantity a user's process would watch to notice that
    generation has stopped attending to its prompt (the attention-based detection discussed in sections 2.4 and 7.1).

    w_steps: [n_steps, n_rows] masses in [0, 1].  Returns, per row: the minimum over the steps, the sum over the steps
    (mean = sum / n_steps) and the number of steps whose mass lies strictly below ``threshold``.  An empty sequence
    gives (1, 0, 0): 1 is the largest value a mass can take.
    """
    w = np.asarray(w_steps, dtype=np.float64)
    assert w.ndim == 2
    n_rows = w.shape[1]
    mn = np.ones(n_rows, dtype=np.float64)
    sm = np.zeros(n_rows, dtype=np.float64)
    below = np.zeros(n_rows, dtype=np.int64)
    for step in range(w.shape[0]):          # one decode step after the other, as the statistic is kept
        mn = np.minimum(mn, w[step])
        sm = sm + w[step]
        below = below + (w[step] < float(threshold))
    return mn, sm, below
