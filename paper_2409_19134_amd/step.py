"""One SPD decode step for one layer: private partial, public batched partial, merge (paper section 4, step 3).

Pure call sequencing over the C ABI; holds the output buffers so a step allocates nothing.
"""
from __future__ import annotations

import torch

from .binding import Context, KVView, make_shape


class DecodeStep:
    def __init__(self, ctx: Context, dtype, n_q_heads: int, n_kv_heads: int, head_dim: int, scale: float,
                 private: KVView, public: KVView, device="cuda:0"):
        self.ctx = ctx
        self.shape = make_shape(dtype, n_q_heads, n_kv_heads, head_dim, scale)
        self.private, self.public = private, public
        n = private.struct.n_users
        assert public.struct.n_users == n
        f32 = dict(device=device, dtype=torch.float32)
        self.a_in = torch.empty((n, n_q_heads, head_dim), **f32)
        self.a_out = torch.empty((n, n_q_heads, head_dim), **f32)
        self.y = torch.empty((n, n_q_heads, head_dim), **f32)
        self.lse_in = torch.empty((n, n_q_heads), **f32)
        self.lse_out = torch.empty((n, n_q_heads), **f32)
        self.lse = torch.empty((n, n_q_heads), **f32)
        self.w_in = torch.empty((n, n_q_heads), **f32)

    @classmethod
    def from_workload(cls, ctx: Context, wl, device_pointer_tables: bool = False) -> "DecodeStep":
        return cls(ctx, wl.dtype, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.scale,
                   KVView.from_side(wl.private, device_pointer_tables), KVView.from_side(wl.public, device_pointer_tables),
                   device=wl.q.device)

    def run(self, q: torch.Tensor, stream=None):
        """Enqueue the three calls on `stream` (default: torch's current stream).  No synchronisation."""
        c = self.ctx
        c.spd_partial_attn_private(self.shape, q, self.private, self.a_in, self.lse_in, stream)
        c.spd_partial_attn_public_batched(self.shape, q, self.public, self.a_out, self.lse_out, stream)
        c.spd_lse_merge(self.a_in, self.lse_in, self.a_out, self.lse_out, self.y, self.lse, self.w_in, stream)
        return self.y

    def run_two_parties(self, q: torch.Tensor, stream=None, k_new=None, v_new=None):
        """The deployment of the paper in two calls: the users' side (private partials) and the service's side
        (public partial, optional append, and the merge) - spd_public_attn_merge closes the step."""
        c = self.ctx
        c.spd_partial_attn_private(self.shape, q, self.private, self.a_in, self.lse_in, stream)
        return c.spd_public_attn_merge(self.shape, q, self.public, self.a_in, self.lse_in, self.a_out, self.lse_out,
                                       self.y, self.lse, self.w_in, stream, k_new, v_new)

    def run_fused(self, q: torch.Tensor, stream=None, k_new=None, v_new=None):
        """The same step through spd_decode_step: one launch for both owners, one closing kernel.  With k_new / v_new
        the new token is appended to the public cache in the same launch (the view's lengths already count it)."""
        return self.ctx.spd_decode_step(self.shape, q, self.private, self.public, self.a_in, self.lse_in, self.a_out,
                                        self.lse_out, self.y, self.lse, self.w_in, stream, k_new, v_new)

    def prepare(self, q: torch.Tensor, stream_ptr: int, k_new=None, v_new=None):
        """Marshal the three calls' arguments once; `run_prepared` then only makes the three C calls.
        For loops that reuse the same q buffer and stream (serving loops, benchmarks)."""
        import ctypes as C
        from .binding import lib
        n, Hq, d = self.private.struct.n_users, self.shape.n_q_heads, self.shape.head_dim
        assert q.is_contiguous() and tuple(q.shape) == (n, Hq, d)
        h, sp, st = self.ctx.handle, C.byref(self.shape), C.c_void_p(stream_ptr)
        self._keep_q = (q, k_new, v_new)
        self._calls = (
            (lib.spd_partial_attn_private, (h, sp, q.data_ptr(), C.byref(self.private.struct),
                                            self.a_in.data_ptr(), self.lse_in.data_ptr(), st)),
            (lib.spd_partial_attn_public_batched, (h, sp, q.data_ptr(), C.byref(self.public.struct),
                                                   self.a_out.data_ptr(), self.lse_out.data_ptr(), st)),
            (lib.spd_lse_merge, (h, n * Hq, d, self.a_in.data_ptr(), self.lse_in.data_ptr(), self.a_out.data_ptr(),
                                 self.lse_out.data_ptr(), self.y.data_ptr(), self.lse.data_ptr(),
                                 self.w_in.data_ptr(), st)),
        )

        self._fused = (lib.spd_decode_step, (h, sp, q.data_ptr(), C.byref(self.private.struct),
                                             C.byref(self.public.struct),
                                             None if k_new is None else k_new.data_ptr(),
                                             None if v_new is None else v_new.data_ptr(), self.a_in.data_ptr(),
                                             self.lse_in.data_ptr(), self.a_out.data_ptr(), self.lse_out.data_ptr(),
                                             self.y.data_ptr(), self.lse.data_ptr(), self.w_in.data_ptr(), st))

        self._two_parties = (
            self._calls[0],
            (lib.spd_public_attn_merge, (h, sp, q.data_ptr(), C.byref(self.public.struct),
                                         None if k_new is None else k_new.data_ptr(),
                                         None if v_new is None else v_new.data_ptr(), self.a_in.data_ptr(),
                                         self.lse_in.data_ptr(), self.a_out.data_ptr(), self.lse_out.data_ptr(),
                                         self.y.data_ptr(), self.lse.data_ptr(), self.w_in.data_ptr(), st)),
        )

    def run_prepared_two_parties(self):
        """The users' call (private partials) and the service's call (public partial and merge), arguments prepared."""
        for fn, args in self._two_parties:
            rc = fn(*args)
            if rc != 0:
                self.ctx._check(rc, fn.__name__)
        return self.y

    def run_prepared_fused(self):
        fn, args = self._fused
        rc = fn(*args)
        if rc != 0:
            self.ctx._check(rc, "spd_decode_step")
        return self.y

    def run_prepared(self, public_first: bool = False):
        """The three calls in sequence on the prepared stream; public_first swaps the two partial calls (the order
        in which the paper's service runs its own attention before it hears from the user processes)."""
        order = (1, 0, 2) if public_first else (0, 1, 2)
        for i in order:
            fn, args = self._calls[i]
            rc = fn(*args)
            if rc != 0:
                self.ctx._check(rc, fn.__name__)
        return self.y

    def run_streams(self, q: torch.Tensor, side: "torch.cuda.Stream"):
        """The two owners on two HIP streams of equal priority: the private call on torch's current stream, the public
        call on `side`, joined by events before the merge (the paper's "start the private computation as soon as Q
        exists" schedule, section 5, with streams standing in for processes).  No host synchronisation."""
        c = self.ctx
        main = torch.cuda.current_stream()
        fork = torch.cuda.Event()
        fork.record(main)          # everything already queued on main (the previous merge reads a_out) comes first
        side.wait_event(fork)
        c.spd_partial_attn_public_batched(self.shape, q, self.public, self.a_out, self.lse_out, side)
        join = torch.cuda.Event()
        join.record(side)
        c.spd_partial_attn_private(self.shape, q, self.private, self.a_in, self.lse_in, main)
        main.wait_event(join)
        c.spd_lse_merge(self.a_in, self.lse_in, self.a_out, self.lse_out, self.y, self.lse, self.w_in, main)
        return self.y
