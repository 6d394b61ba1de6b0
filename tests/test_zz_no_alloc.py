"""spd_decode_step_static (the decode step on the library's fixed scratch array, for callers that cannot allocate)
against spd_decode_step: same inputs, every output bit for bit, on two calls in a row, the second one smaller."""
import numpy as np
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
OUTPUTS = ("a_in", "lse_in", "a_out", "lse_out", "y", "lse", "w_in")


def _both(ctx, wl, k_new=None, v_new=None):
    """(outputs of spd_decode_step, outputs of spd_decode_step_static) for one workload."""
    import paper_2409_19134_amd as spd
    got = []
    for static in (False, True):
        step = spd.DecodeStep.from_workload(ctx, wl)
        for name in OUTPUTS:
            getattr(step, name).fill_(float("nan"))
        fn = ctx.spd_decode_step_static if static else ctx.spd_decode_step
        fn(step.shape, wl.q, step.private, step.public, step.a_in, step.lse_in, step.a_out, step.lse_out, step.y,
           step.lse, step.w_in, None, k_new, v_new)
        torch.cuda.synchronize()
        got.append({name: getattr(step, name).clone() for name in OUTPUTS})
    return got


def _same(a, b):
    for name in OUTPUTS:
        assert not torch.isnan(b[name]).any(), name
        assert torch.equal(a[name].view(torch.int32), b[name].view(torch.int32)), name


def test_static_step_equals_decode_step_twice_second_smaller():
    import paper_2409_19134_amd as spd
    ctx = spd.Context(0)
    big = workloads.make_workload(2, DEV)                       # the headline workload: 16 users, ~38 000 tokens
    small = workloads.random_case(77, torch.bfloat16, 3, 32, 8, 128, [700, 0, 33], [17, 64, 0], device=DEV)
    for wl in (big, small, big):
        ref, got = _both(ctx, wl)
        _same(ref, got)
    ctx.close()


def test_static_step_other_storage_modes_and_append():
    import paper_2409_19134_amd as spd
    ctx = spd.Context(0)
    paged = workloads.make_workload(5, DEV, len_div=64, n_users=6)
    f32 = workloads.make_workload(1, DEV)
    token_major = workloads.make_workload(4, DEV, len_div=8, n_users=40, layout="nhd")
    for wl in (paged, f32, token_major):
        ref, got = _both(ctx, wl)
        _same(ref, got)
    wl = workloads.random_case(78, torch.bfloat16, 4, 32, 8, 128, [3000, 100, 900, 64], [300, 900, 5, 1], device=DEV)
    gen = torch.Generator(device=DEV).manual_seed(79)
    k_new = torch.randn((4, 8, 128), generator=gen, device=DEV).to(torch.bfloat16)
    v_new = torch.randn((4, 8, 128), generator=gen, device=DEV).to(torch.bfloat16)
    ref, got = _both(ctx, wl, k_new, v_new)
    _same(ref, got)
    ctx.close()


def test_static_step_refuses_what_does_not_fit():
    """A schedule of more work items than the array has room for: an error before anything is launched."""
    import paper_2409_19134_amd as spd
    ctx = spd.Context(0)
    U = 2100                                     # 2100 users x 8 KV heads x 2 pieces x 48 bytes > 512 KiB
    lens = np.full(U, 40, dtype=np.int32)
    wl = workloads.random_case(80, torch.bfloat16, U, 32, 8, 128, lens, lens, device=DEV)
    step = spd.DecodeStep.from_workload(ctx, wl)
    step.y.fill_(7.0)
    with pytest.raises(spd.binding.SpdError) as e:
        ctx.spd_decode_step_static(step.shape, wl.q, step.private, step.public, step.a_in, step.lse_in, step.a_out,
                                   step.lse_out, step.y, step.lse, step.w_in)
    assert e.value.code == spd.binding.SPD_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert float(step.y.min()) == 7.0 == float(step.y.max())       # nothing ran
    step.run_fused(wl.q)                                           # the allocating entry point takes the same step
    torch.cuda.synchronize()
    assert not torch.isnan(step.y).any()
    ctx.close()


def test_static_step_in_a_hip_graph_without_warm_up():
    """Recorded into a graph as the very first call on its view (schedules travel in kernel arguments), replayed with
    fresh queries between other eager work."""
    import paper_2409_19134_amd as spd
    ctx = spd.Context(0)
    wl = workloads.random_case(81, torch.bfloat16, 5, 32, 8, 128, [2000, 100, 0, 900, 64], [300, 900, 5, 0, 1], device=DEV)
    other = workloads.random_case(82, torch.bfloat16, 2, 32, 8, 128, [500, 90], [30, 9], device=DEV)
    step = spd.DecodeStep.from_workload(ctx, wl)
    q = wl.q.clone()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        ctx.spd_decode_step_static(step.shape, q, step.private, step.public, step.a_in, step.lse_in, step.a_out,
                                   step.lse_out, step.y, step.lse, step.w_in, torch.cuda.current_stream())
    gen = torch.Generator(device=DEV).manual_seed(83)
    for rep in range(3):
        q.copy_(torch.randn(q.shape, generator=gen, device=DEV).to(q.dtype))
        torch.cuda.synchronize()
        ref_step = spd.DecodeStep.from_workload(ctx, wl)
        ref_step.run_fused(q)
        # eager work of another view on the same array between the replays
        o = spd.DecodeStep.from_workload(ctx, other)
        ctx.spd_decode_step_static(o.shape, other.q, o.private, o.public, o.a_in, o.lse_in, o.a_out, o.lse_out, o.y, o.lse,
                                   o.w_in)
        torch.cuda.synchronize()
        step.y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for name in OUTPUTS:
            assert torch.equal(getattr(step, name).view(torch.int32), getattr(ref_step, name).view(torch.int32)), (rep, name)
    ctx.close()
