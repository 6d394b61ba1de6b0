"""Runtime behaviour of the library on the GPU: schedule cache eviction, scratch growth, streams, several contexts."""
import numpy as np
import pytest
import torch

import workloads
from oracle import spd_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _oracle_y(wl):
    return orc.attention(orc.from_workload(wl))[0]


def _err(step, Y):
    return float(np.abs(step.y.cpu().double().numpy().reshape(Y.shape) - Y).max())


def test_more_views_than_cache_entries_and_scratch_growth(monkeypatch):
    """40 distinct views with a cache of 16 schedules per entry point, sizes going up and down: every result stays
    right, also when an evicted view comes back."""
    import paper_2409_19134_amd as spd
    monkeypatch.setenv("SPD_SCHEDULE_CACHE_ENTRIES", "16")       # read when the context is created
    ctx = spd.Context(0)
    rng = np.random.default_rng(3)
    cases = []
    for i in range(40):
        U = int(rng.integers(1, 5))
        lp = rng.integers(0, 3000 if i % 7 else 20000, size=U).tolist()
        lo = rng.integers(0, 300, size=U).tolist()
        wl = workloads.random_case(300 + i, torch.bfloat16, U, 32, 8, 128, lp, lo, device=DEV,
                                   layout=("nhd", "hnd", "hnd_exact")[i % 3], paged=(i % 5 == 0))
        cases.append((wl, spd.DecodeStep.from_workload(ctx, wl), _oracle_y(wl)))
    for rnd in range(2):
        for j, (wl, step, Y) in enumerate(cases):
            if (j + rnd) % 2:
                step.run_fused(wl.q)
            else:
                step.run(wl.q)
        torch.cuda.synchronize()      # all 40 were enqueued back to back: evictions happened with work in flight
        for wl, step, Y in cases:
            assert _err(step, Y) <= 2e-3
    ctx.close()


def test_private_and_public_calls_on_two_streams():
    """The two partial calls use separate scratch memory and may overlap on two streams; the merge waits for both."""
    import paper_2409_19134_amd as spd
    ctx = spd.Context(0)
    wl = workloads.random_case(401, torch.bfloat16, 6, 32, 8, 128, [5000, 100, 0, 900, 2500, 64], [300, 900, 5, 0, 64, 1],
                               device=DEV)
    step = spd.DecodeStep.from_workload(ctx, wl)
    Y = _oracle_y(wl)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for _ in range(5):
        ctx.spd_partial_attn_private(step.shape, wl.q, step.private, step.a_in, step.lse_in, stream=s1)
        ctx.spd_partial_attn_public_batched(step.shape, wl.q, step.public, step.a_out, step.lse_out, stream=s2)
        s1.wait_stream(s2)
        ctx.spd_lse_merge(step.a_in, step.lse_in, step.a_out, step.lse_out, step.y, step.lse, step.w_in, stream=s1)
        s2.wait_stream(s1)
    torch.cuda.synchronize()
    assert _err(step, Y) <= 2e-3
    ctx.close()


def test_step_orderings_give_the_same_result():
    """The orderings of the overlap study (private first, public first, two streams, one fused launch) are the same
    computation: identical partials bit for bit where the same kernels run (the three unfused orderings)."""
    import paper_2409_19134_amd as spd
    ctx = spd.Context(0)
    wl = workloads.random_case(402, torch.bfloat16, 5, 32, 8, 128, [3000, 100, 0, 900, 64], [300, 900, 5, 0, 1], device=DEV)
    step = spd.DecodeStep.from_workload(ctx, wl)
    Y = _oracle_y(wl)
    step.prepare(wl.q, torch.cuda.current_stream().cuda_stream)
    outs = []
    side = torch.cuda.Stream()
    for mode in ("calls", "public_first", "streams", "streams", "fused"):
        step.y.zero_()
        if mode == "calls":
            step.run_prepared()
        elif mode == "public_first":
            step.run_prepared(public_first=True)
        elif mode == "streams":
            step.run_streams(wl.q, side)
        else:
            step.run_prepared_fused()
        torch.cuda.synchronize()
        assert _err(step, Y) <= 2e-3
        outs.append(step.y.clone())
    for o in outs[1:4]:
        assert torch.equal(o, outs[0])
    ctx.close()


def test_two_contexts_and_non_default_stream():
    import paper_2409_19134_amd as spd
    a, b = spd.Context(0), spd.Context(0)
    wl = workloads.make_workload(2, DEV, len_div=8)
    Y = _oracle_y(wl)
    sa, sb = spd.DecodeStep.from_workload(a, wl), spd.DecodeStep.from_workload(b, wl)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        sa.run_fused(wl.q)          # binding picks up torch's current stream
    sb.run(wl.q)
    torch.cuda.synchronize()
    assert _err(sa, Y) <= 2e-3 and _err(sb, Y) <= 2e-3
    a.close()
    b.close()


def test_kernel_timing_counts_launches():
    import paper_2409_19134_amd as spd
    ctx = spd.Context(0)
    wl = workloads.make_workload(2, DEV, len_div=8)
    step = spd.DecodeStep.from_workload(ctx, wl)
    step.run(wl.q)
    ctx.spd_set_kernel_timing(3)
    for _ in range(5):
        step.run(wl.q)              # only the first three launches of each entry point are timed
    n0, mean0, min0 = ctx.spd_get_kernel_timing(0)
    n1, mean1, min1 = ctx.spd_get_kernel_timing(1)
    assert (n0, n1) == (3, 3) and 0 < min0 <= mean0 < 1e4 and 0 < min1 <= mean1 < 1e4
    assert ctx.spd_get_kernel_timing(0)[0] == 0      # reading clears
    ctx.spd_set_kernel_timing(4)
    for _ in range(2):
        step.run_fused(wl.q)        # the two-owner launch is booked under entry point 0
    samples = ctx.spd_get_kernel_timing_samples(0)
    assert len(samples) == 2 and all(0 < s < 1e4 for s in samples)
    assert ctx.spd_get_kernel_timing_samples(1) == [] and ctx.spd_get_kernel_timing_samples(0) == []
    for _ in range(2):
        step.run_fused(wl.q)
    assert len(ctx.spd_get_kernel_timing_samples(0, capacity=1)) == 1      # more recorded than asked for
    ctx.spd_set_kernel_timing(0)
    step.run_fused(wl.q)
    torch.cuda.synchronize()
    assert ctx.spd_get_kernel_timing(0)[0] == 0
    ctx.close()


def test_zero_users_and_decode_step_validation():
    import ctypes as C
    import paper_2409_19134_amd as spd
    ctx = spd.Context(0)
    wl = workloads.random_case(409, torch.bfloat16, 2, 32, 8, 128, [10, 20], [3, 4], device=DEV)
    step = spd.DecodeStep.from_workload(ctx, wl)
    empty = spd.KVView([], 1024, 128, k=[], v=[])
    q0 = torch.empty((0, 32, 128), device=DEV, dtype=torch.bfloat16)
    out0 = torch.empty((0, 32, 128), device=DEV)
    lse0 = torch.empty((0, 32), device=DEV)
    rc = spd.lib.spd_partial_attn_private(ctx.handle, C.byref(step.shape), None, C.byref(empty.struct), None, None, None)
    assert rc == spd.SPD_OK                          # nothing to do is not an error
    one = spd.KVView(wl.public.lens[:1], wl.public.token_stride, wl.public.head_stride, k=wl.public.k[:1], v=wl.public.v[:1])
    rc = spd.lib.spd_decode_step(ctx.handle, C.byref(step.shape), wl.q.data_ptr(), C.byref(step.private.struct),
                                 C.byref(one.struct), None, None, step.a_in.data_ptr(), step.lse_in.data_ptr(),
                                 step.a_out.data_ptr(), step.lse_out.data_ptr(), step.y.data_ptr(), step.lse.data_ptr(),
                                 step.w_in.data_ptr(), None)
    assert rc == spd.SPD_ERR_LEN                     # the two owners must describe the same users
    rc = spd.lib.spd_decode_step(ctx.handle, C.byref(step.shape), wl.q.data_ptr(), C.byref(step.private.struct),
                                 C.byref(step.public.struct), None, None, step.a_in.data_ptr(), step.lse_in.data_ptr(),
                                 step.a_out.data_ptr(), step.lse_out.data_ptr(), None, step.lse.data_ptr(),
                                 step.w_in.data_ptr(), None)
    assert rc == spd.SPD_ERR_NULL
    assert spd.lib.spd_lse_merge(ctx.handle, 4, 130, step.a_in.data_ptr(), step.lse_in.data_ptr(), step.a_out.data_ptr(),
                                 step.lse_out.data_ptr(), step.y.data_ptr(), None, None, None) == spd.SPD_ERR_SHAPE
    ctx.close()


def test_layers_share_one_schedule_per_step_in_paged_mode():
    """A model's layers share lengths and block table and own a pool each: one schedule per owner serves them all.
    Three decode steps over four layers, each step appending one token per user to every layer's public cache."""
    import copy
    import paper_2409_19134_amd as spd
    ctx = spd.Context(0)
    U, Hq, Hkv, d, n_layers, n_steps = 3, 32, 8, 128, 4, 3
    lp, lo0 = [700, 40, 2100], [30, 1, 200]
    cap = [x + n_steps for x in lo0]          # pages for the tokens that will be appended exist from the start
    base = workloads.random_case(500, torch.bfloat16, U, Hq, Hkv, d, lp, cap, device=DEV, paged=True)
    layers = []
    for i in range(n_layers):                  # same tables, another pool (other values) per layer
        w = copy.copy(base)
        w.private, w.public = copy.copy(base.private), copy.copy(base.public)
        for side in (w.private, w.public):
            g = torch.Generator(device=DEV).manual_seed(600 + i)
            side.k_pool = torch.randn(side.k_pool.shape, generator=g, device=DEV).to(torch.bfloat16)
            side.v_pool = torch.randn(side.v_pool.shape, generator=g, device=DEV).to(torch.bfloat16)
        layers.append(w)
    g = torch.Generator(device=DEV).manual_seed(7)
    builds0, _ = ctx.spd_get_schedule_stats()
    for s in range(n_steps):
        lens_now = np.asarray([x + s + 1 for x in lo0], dtype=np.int32)     # counts the token appended in this step
        outs = []
        for w in layers:
            w.public.lens = lens_now
            q = torch.randn((U, Hq, d), generator=g, device=DEV).to(torch.bfloat16)
            kn = torch.randn((U, Hkv, d), generator=g, device=DEV).to(torch.bfloat16)
            vn = torch.randn((U, Hkv, d), generator=g, device=DEV).to(torch.bfloat16)
            w.q = q
            step = spd.DecodeStep.from_workload(ctx, w)
            step.run_fused(q, k_new=kn, v_new=vn)
            outs.append(step)
        torch.cuda.synchronize()
        builds, hits = ctx.spd_get_schedule_stats()
        # both schedules are built once (step 0): the public one also serves the lengths of the following steps
        assert builds - builds0 == 2
        for w, step in zip(layers, outs):
            assert _err(step, _oracle_y(w)) <= 2e-3
    assert hits == 2 * n_layers * n_steps - 2
    ctx.close()


@pytest.mark.parametrize("layout", ["hnd", "nhd", "hnd_exact"])
def test_layers_share_one_schedule_with_device_pointer_tables(layout):
    """Contiguous per-user buffers: with the pointers also handed over in device arrays the schedule does not depend
    on the buffers' addresses, so the layers of a model (a set of buffers each, same lengths) share one per owner and
    decode step.  Without the tables every layer builds its own.  Three steps over four layers, appending a token."""
    import paper_2409_19134_amd as spd
    ctx = spd.Context(0)
    U, Hq, Hkv, d, n_layers, n_steps = 3, 32, 8, 128, 4, 3
    lp, lo0 = [700, 40, 2100], [30, 1, 200]
    cap = [x + n_steps for x in lo0]          # room for the tokens that will be appended
    layers = [workloads.random_case(520 + i, torch.bfloat16, U, Hq, Hkv, d, lp, cap, device=DEV, layout=layout)
              for i in range(n_layers)]
    g = torch.Generator(device=DEV).manual_seed(8)
    for tables in (True, False):
        builds0, hits0 = ctx.spd_get_schedule_stats()
        for s in range(n_steps):
            lens_now = np.asarray([x + s + 1 for x in lo0], dtype=np.int32)
            outs = []
            for w in layers:
                w.public.lens = lens_now
                if layout == "hnd_exact":      # the buffers keep the head stride they were allocated with
                    w.public.head_strides = np.asarray(cap, dtype=np.int64) * d
                q = torch.randn((U, Hq, d), generator=g, device=DEV).to(torch.bfloat16)
                kn = torch.randn((U, Hkv, d), generator=g, device=DEV).to(torch.bfloat16)
                vn = torch.randn((U, Hkv, d), generator=g, device=DEV).to(torch.bfloat16)
                w.q = q
                step = spd.DecodeStep.from_workload(ctx, w, device_pointer_tables=tables)
                step.run_fused(q, k_new=kn, v_new=vn)
                outs.append(step)
            torch.cuda.synchronize()
            for w, step in zip(layers, outs):
                assert _err(step, _oracle_y(w)) <= 2e-3
        builds, hits = ctx.spd_get_schedule_stats()
        if tables:   # one build per owner in all (the public one also serves the grown lengths of the later steps)
            assert builds - builds0 == 2
            assert hits - hits0 == 2 * n_layers * n_steps - 2
        else:        # one per owner and layer
            assert builds - builds0 == 2 * n_layers
    ctx.close()


def test_device_pointer_tables_three_call_path_and_fp32():
    import paper_2409_19134_amd as spd
    ctx = spd.Context(0)
    for dtype, Hq, Hkv, d in ((torch.bfloat16, 16, 4, 128), (torch.float32, 8, 2, 64)):
        wl = workloads.random_case(530, dtype, 4, Hq, Hkv, d, [3000, 0, 65, 900], [5, 700, 0, 128], device=DEV, layout="hnd")
        step = spd.DecodeStep.from_workload(ctx, wl, device_pointer_tables=True)
        step.run(wl.q)
        torch.cuda.synchronize()
        assert _err(step, _oracle_y(wl)) <= (2e-3 if dtype == torch.bfloat16 else 1e-5)
    ctx.close()


def test_attention_mass_track_against_oracle():
    """Seeded masses (some exactly on the threshold, zeros, ones) folded step by step; then the masses of real decode
    steps with KV append, against the oracle's w_in."""
    import paper_2409_19134_amd as spd
    ctx = spd.Context(0)
    n_rows, steps, thr = 1000, 9, 0.375
    g = torch.Generator().manual_seed(611)
    w = torch.rand((steps, n_rows), generator=g, dtype=torch.float32)
    w[2, ::7] = thr
    w[3, ::11] = 0.0
    w[4, ::13] = 1.0
    mn = torch.ones(n_rows, device=DEV)
    sm = torch.zeros(n_rows, device=DEV)
    below = torch.zeros(n_rows, device=DEV, dtype=torch.int32)
    wd = w.to(DEV)
    for s in range(steps):
        ctx.spd_attention_mass_track(wd[s], thr, mn, sm, below)
    only_min = torch.ones(n_rows, device=DEV)
    ctx.spd_attention_mass_track(wd[0], thr, mass_min=only_min)          # the other two statistics left out
    torch.cuda.synchronize()
    o_mn, o_sm, o_below = orc.attention_mass_track(w.double().numpy(), thr)
    assert np.array_equal(mn.cpu().double().numpy(), o_mn)               # a minimum of fp32 values is exact
    assert np.array_equal(below.cpu().numpy().astype(np.int64), o_below)
    assert np.abs(sm.cpu().double().numpy() - o_sm).max() <= steps * 6e-7
    assert torch.equal(only_min.cpu(), w[0])

    # three decode steps of a growing public cache: w_in of the step against the oracle's merge weight
    lp, lo0 = [300, 40, 0, 2000], [1, 5, 3, 0]
    U, Hq, Hkv, d = 4, 32, 8, 128
    cap = 8
    wl = workloads.random_case(612, torch.bfloat16, U, Hq, Hkv, d, lp, [l + cap for l in lo0], device=DEV, layout="hnd")
    mn = torch.ones(U * Hq, device=DEV)
    sm = torch.zeros(U * Hq, device=DEV)
    masses = []
    for s in range(3):
        wl.public.lens = np.asarray([l + s + 1 for l in lo0], dtype=np.int32)     # the step appends one token
        step = spd.DecodeStep.from_workload(ctx, wl)
        gq = torch.Generator(device=DEV).manual_seed(620 + s)
        q = torch.randn((U, Hq, d), generator=gq, device=DEV).to(torch.bfloat16)
        k_new = torch.randn((U, Hkv, d), generator=gq, device=DEV).to(torch.bfloat16)
        v_new = torch.randn((U, Hkv, d), generator=gq, device=DEV).to(torch.bfloat16)
        step.run_fused(q, k_new=k_new, v_new=v_new)
        ctx.spd_attention_mass_track(step.w_in, 0.5, mn, sm)
        torch.cuda.synchronize()
        wl.q = q                                   # the cache now holds the new rows: the oracle reads it as it is
        hw = orc.from_workload(wl)
        A0, m0, g0 = orc.partial(hw, hw.private)
        A1, m1, g1 = orc.partial(hw, hw.public)
        masses.append(orc.merge(A0, m0, g0, A1, m1, g1)[3])
        assert np.abs(step.w_in.cpu().double().numpy().reshape(-1) - masses[-1]).max() <= 2e-3
    o_mn, o_sm, _ = orc.attention_mass_track(np.stack(masses), 0.5)
    assert np.abs(mn.cpu().double().numpy() - o_mn).max() <= 2e-3
    assert np.abs(sm.cpu().double().numpy() - o_sm).max() <= 3 * 2e-3
    assert (mn.cpu().numpy().reshape(U, Hq)[2] == 0).all()               # user 2 has no private part
    ctx.close()


def test_attention_mass_track_argument_errors():
    import paper_2409_19134_amd as spd
    from paper_2409_19134_amd import binding as b
    ctx = spd.Context(0)
    w = torch.zeros(4, device=DEV)
    assert b.lib.spd_attention_mass_track(ctx.handle, -1, w.data_ptr(), 0.5, None, None, None, None) == b.SPD_ERR_LEN
    assert b.lib.spd_attention_mass_track(ctx.handle, 4, None, 0.5, None, None, None, None) == b.SPD_ERR_NULL
    assert b.lib.spd_attention_mass_track(None, 4, w.data_ptr(), 0.5, None, None, None, None) == b.SPD_ERR_NULL
    assert b.lib.spd_attention_mass_track(ctx.handle, 0, None, 0.5, None, None, None, None) == b.SPD_OK
    ctx.close()


@pytest.mark.parametrize("fused", [True, False])
def test_layers_captured_in_one_hip_graph(fused):
    """Four layers of a decode step (a set of buffers each, one shared schedule) recorded into one HIP graph after an
    eager pass has built the schedules and sized the scratch memory: a call with warm caches only launches kernels,
    so it can be captured.  Every replay - with eager work of the library and fresh inputs in between - must give
    the bits of the eager run on the same inputs."""
    import paper_2409_19134_amd as spd
    ctx = spd.Context(0)
    U, Hq, Hkv, d, n_layers = 3, 32, 8, 128, 4
    layers = [workloads.random_case(540 + i, torch.bfloat16, U, Hq, Hkv, d, [700, 40, 2100], [30, 0, 200], device=DEV,
                                    layout="hnd") for i in range(n_layers)]
    q = [w.q for w in layers]                      # static input buffers of the graph
    steps = [spd.DecodeStep.from_workload(ctx, w, device_pointer_tables=True) for w in layers]
    run = (lambda s, x: s.run_fused(x)) if fused else (lambda s, x: s.run(x))

    def eager():
        for s, x in zip(steps, q):
            run(s, x)
        torch.cuda.synchronize()
        return [s.y.clone() for s in steps]

    eager()                                        # schedules built and uploaded, scratch allocated
    builds0, _ = ctx.spd_get_schedule_stats()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for s, x in zip(steps, q):
            run(s, x)                              # stream=None: torch's current stream, here the capturing one
    assert ctx.spd_get_schedule_stats()[0] == builds0      # nothing was built while capturing
    g = torch.Generator(device=DEV).manual_seed(11)
    for rep in range(4):
        for x in q:
            x.copy_(torch.randn(x.shape, generator=g, device=DEV).to(x.dtype))
        want = eager()
        for s in steps:
            s.y.fill_(float("nan"))
            s.a_in.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for s, y in zip(steps, want):
            assert torch.equal(s.y, y), f"replay {rep}"
    for w, s in zip(layers, steps):
        assert _err(s, _oracle_y(w)) <= 2e-3
    ctx.close()


@pytest.mark.parametrize("storage", ["hnd", "hnd_exact", "nhd_hpw", "paged", "paged_tm_hpw"])
@pytest.mark.parametrize("fused", [True, False])
def test_decode_loop_reuses_the_public_schedule_while_the_cache_grows(storage, fused):
    """150 decode steps, one token appended per user and step: the public schedule is rebuilt only every 65th step
    (a schedule serves lengths up to 64 tokens beyond those it was built for), rows cross 32-token steps and pages on
    the way, and every step's result is right."""
    import paper_2409_19134_amd as spd
    hpw = storage.endswith("_hpw")
    storage = storage[:-4] if hpw else storage
    paged = {"paged": True, "paged_tm": "token_major"}.get(storage, False)
    ctx = spd.Context(0)
    ctx.spd_set_option(spd.SPD_OPT_HEAD_PER_WAVE, 1 if hpw else 0)
    U, Hq, Hkv, d, n_steps = 4, 16, 4, 128, 150
    lp, lo0 = [300, 33, 1500, 64], [1, 30, 700, 95]
    cap = [x + n_steps for x in lo0]
    wl = workloads.random_case(560, torch.bfloat16, U, Hq, Hkv, d, lp, cap, device=DEV,
                               layout="nhd" if paged else storage, paged=paged)
    sh = spd.make_shape(wl.dtype, Hq, Hkv, d, wl.scale)
    g = torch.Generator(device=DEV).manual_seed(9)
    builds0, hits0 = ctx.spd_get_schedule_stats()
    check_at = {0, 1, 2, 31, 63, 64, 65, 66, 100, 129, 130, 149}
    for s in range(n_steps):
        wl.public.lens = np.asarray([x + s for x in lo0], dtype=np.int32)        # step 0: the lengths as built
        if s > 0:        # the token of this step goes in with the call
            kn = torch.randn((U, Hkv, d), generator=g, device=DEV).to(torch.bfloat16)
            vn = torch.randn((U, Hkv, d), generator=g, device=DEV).to(torch.bfloat16)
        else:
            kn = vn = None
        wl.q = torch.randn((U, Hq, d), generator=g, device=DEV).to(torch.bfloat16)
        step = spd.DecodeStep.from_workload(ctx, wl)
        if fused:
            step.run_fused(wl.q, k_new=kn, v_new=vn)
        else:
            step.ctx.spd_partial_attn_private(sh, wl.q, step.private, step.a_in, step.lse_in)
            if kn is None:
                step.ctx.spd_partial_attn_public_batched(sh, wl.q, step.public, step.a_out, step.lse_out)
            else:
                step.ctx.spd_partial_attn_public_batched_append(sh, wl.q, kn, vn, step.public, step.a_out, step.lse_out)
            step.ctx.spd_lse_merge(step.a_in, step.lse_in, step.a_out, step.lse_out, step.y)
        if s in check_at:
            torch.cuda.synchronize()
            assert _err(step, _oracle_y(wl)) <= 2e-3, f"step {s}"
    torch.cuda.synchronize()
    builds, hits = ctx.spd_get_schedule_stats()
    assert builds - builds0 == 1 + 3           # private once; public at steps 0, 65 and 130
    assert hits - hits0 == 2 * n_steps - 4
    ctx.close()


def test_service_call_argument_errors_and_zero_users():
    import paper_2409_19134_amd as spd
    ctx = spd.Context(0)
    wl = workloads.random_case(580, torch.bfloat16, 2, 32, 8, 128, [100, 0], [5, 300], device=DEV)
    step = spd.DecodeStep.from_workload(ctx, wl)
    sh, pub = step.shape, step.public
    args = lambda **kw: [kw.get(k, getattr(step, k).data_ptr()) for k in ("a_in", "lse_in", "a_out", "lse_out", "y", "lse", "w_in")]
    call = lambda a, k_new=None, v_new=None: spd.lib.spd_public_attn_merge(ctx.handle, sh, wl.q.data_ptr(), pub.struct, k_new, v_new, *a, None)
    assert call(args(a_in=None)) == spd.SPD_ERR_NULL
    assert call(args(y=None)) == spd.SPD_ERR_NULL
    assert call(args(a_in=step.a_in.data_ptr() + 4)) == spd.SPD_ERR_ALIGN
    kn = torch.zeros((2, 8, 128), device=DEV, dtype=torch.bfloat16)
    assert call(args(), kn.data_ptr(), None) == spd.SPD_ERR_NULL          # the new token needs both rows
    empty = spd.KVView([], token_stride=128, head_stride=128, k=[], v=[])
    assert spd.lib.spd_public_attn_merge(ctx.handle, sh, None, empty.struct, None, None, *([None] * 7), None) == spd.SPD_OK
    step.run_two_parties(wl.q)
    torch.cuda.synchronize()
    assert _err(step, _oracle_y(wl)) <= 2e-3
    ctx.close()


def test_c_program_runs_the_path_without_python():
    """tests/host/abi_gpu_program.cpp knows only include/spd.h and the HIP runtime: the three calls and the fused step
    from a plain program, against a closed form (zero keys: the result is the mean of V)."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = os.path.join(root, "tests", "host", "abi_gpu_program")
    assert os.path.exists(exe), "build it first: python -c 'import __graft_entry__ as g; g.build()'"
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert run.returncode == 0 and run.stdout.strip().endswith("c abi gpu ok"), run.stdout[-2000:]


def test_two_host_threads_with_a_context_each():
    """A context is for one host thread at a time; two threads with a context and a stream each run side by side."""
    import threading
    import paper_2409_19134_amd as spd
    cases = [workloads.random_case(570 + i, torch.bfloat16, 3, 32, 8, 128, [900 + 100 * i, 40, 2100], [30, 0, 200],
                                   device=DEV, layout=("hnd", "nhd")[i]) for i in range(2)]
    want = [_oracle_y(w) for w in cases]
    errors = [None, None]

    def work(i):
        try:
            torch.cuda.set_device(0)
            ctx = spd.Context(0)
            stream = torch.cuda.Stream()
            step = spd.DecodeStep.from_workload(ctx, cases[i])
            worst = 0.0
            for rep in range(40):
                with torch.cuda.stream(stream):
                    if rep % 2:
                        step.run_fused(cases[i].q)
                    else:
                        step.run(cases[i].q)
                if rep % 10 == 9:
                    stream.synchronize()
                    worst = max(worst, _err(step, want[i]))
            stream.synchronize()
            ctx.close()
            errors[i] = worst
        except Exception as exc:        # surfaces in the main thread's assertion
            errors[i] = exc

    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert all(isinstance(e, float) and e <= 2e-3 for e in errors), errors


def test_contexts_give_their_memory_back():
    """Forty contexts created, used (both storage for small schedules and a schedule too large for it, scratch for
    split rows) and destroyed: the device's free memory ends where it began, so spd_destroy frees what a context
    allocated."""
    import paper_2409_19134_amd as spd
    wl_small = workloads.random_case(811, torch.bfloat16, 3, 8, 2, 128, [700, 40, 5000], [10, 0, 300], device=DEV, layout="hnd")
    wl_big = workloads.random_case(812, torch.bfloat16, 600, 8, 2, 64, [40] * 600, [7] * 600, device=DEV, layout="nhd")
    want = _oracle_y(wl_small)
    torch.cuda.synchronize()

    def one_context():
        ctx = spd.Context(0)
        for wl in (wl_small, wl_big):
            step = spd.DecodeStep.from_workload(ctx, wl)
            step.run_fused(wl.q)
            step.run(wl.q)
            if wl is wl_small:
                torch.cuda.synchronize()
                assert _err(step, want) <= 2e-3
        torch.cuda.synchronize()
        ctx.close()

    one_context()                     # whatever the first use of the library itself keeps is allocated now
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(40):
        one_context()
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free0 - free1 < 32 << 20, f"{(free0 - free1) >> 20} MiB not returned after 40 contexts"


def test_steps_in_flight_option_picks_the_kernel_form():
    """SPD_OPT_STEPS_IN_FLIGHT: the library picks the streaming kernel's form by the size of the launch (a small input
    runs with one step in flight, a launch of many more pieces than workgroup slots with two), the option forces either
    where the kernel has both, and the results agree with the oracle every time."""
    import paper_2409_19134_amd as spd
    ctx = spd.Context(0)
    small = workloads.random_case(821, torch.bfloat16, 3, 32, 8, 128, [700, 33, 1500], [40, 0, 129], device=DEV, layout="hnd")
    want = _oracle_y(small)

    def form(wl, expect_two):
        step = spd.DecodeStep.from_workload(ctx, wl)
        step.run_fused(wl.q)
        torch.cuda.synchronize()
        name = ctx.spd_last_kernel_name()
        assert name.split(", ")[3] == ("true" if expect_two else "false"), name
        return step

    assert ctx.spd_get_option(spd.SPD_OPT_STEPS_IN_FLIGHT) == -1
    assert _err(form(small, False), want) <= 2e-3
    ctx.spd_set_option(spd.SPD_OPT_STEPS_IN_FLIGHT, 2)
    assert ctx.spd_get_option(spd.SPD_OPT_STEPS_IN_FLIGHT) == 2
    assert _err(form(small, True), want) <= 2e-3
    ctx.spd_set_option(spd.SPD_OPT_STEPS_IN_FLIGHT, 1)
    assert _err(form(small, False), want) <= 2e-3
    for bad in (0, 3, -2):
        with pytest.raises(spd.binding.SpdError) as e:
            ctx.spd_set_option(spd.SPD_OPT_STEPS_IN_FLIGHT, bad)
        assert e.value.code == spd.binding.SPD_ERR_LEN
    assert ctx.spd_get_option(spd.SPD_OPT_STEPS_IN_FLIGHT) == 1

    # forms the option cannot change: fp32 has one step in flight, 128-byte rows always two
    f32 = workloads.random_case(822, torch.float32, 2, 8, 4, 128, [300, 77], [40, 5], device=DEV, layout="hnd")
    ctx.spd_set_option(spd.SPD_OPT_STEPS_IN_FLIGHT, 2)
    assert _err(form(f32, False), _oracle_y(f32)) <= 1e-5
    d64 = workloads.random_case(823, torch.bfloat16, 2, 16, 4, 64, [300, 77], [40, 5], device=DEV, layout="hnd")
    ctx.spd_set_option(spd.SPD_OPT_STEPS_IN_FLIGHT, 1)
    assert _err(form(d64, True), _oracle_y(d64)) <= 2e-3

    # by size: with pieces of at most 128 tokens, many users with short rows make several rounds of pieces, which take
    # the two-step form; forced to one step the same launch gives the same answer
    ctx.spd_set_option(spd.SPD_OPT_STEPS_IN_FLIGHT, -1)
    ctx.spd_set_option(spd.SPD_OPT_CHUNK_MAX, 128)
    rng = np.random.default_rng(5)
    U = 300
    big = workloads.random_case(824, torch.bfloat16, U, 16, 8, 128, rng.integers(1, 300, U).tolist(),
                                rng.integers(0, 40, U).tolist(), device=DEV, layout="hnd_exact")
    want_big = _oracle_y(big)
    assert _err(form(big, True), want_big) <= 2e-3
    ctx.spd_set_option(spd.SPD_OPT_STEPS_IN_FLIGHT, 1)
    assert _err(form(big, False), want_big) <= 2e-3
    ctx.close()
