"""KV append fused into the public partial (protocol step 3a + 3c): the new token must land in the cache bit for bit,
nothing else may change, and the partial / the whole step must equal the oracle on the cache that contains it."""
import copy

import numpy as np
import pytest
import torch

import workloads
from oracle import spd_oracle as orc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-3, torch.float16: 1e-4}    # as in test_gpu_parity.py


@pytest.fixture(scope="module")
def ctx():
    import paper_2409_19134_amd as spd
    c = spd.Context(0)
    yield c
    torch.cuda.synchronize()
    c.close()


def _set_last_token(side, u, k_row, v_row):
    """Plain copy of one token's rows ([Hkv, d]) into position lens[u]-1 of user u (torch indexing only)."""
    t = int(side.lens[u]) - 1
    if side.paged:
        page = int(side.block_table[u, t // side.page_tokens])
        if side.page_token_major:
            side.k_pool[page, t % side.page_tokens] = k_row
            side.v_pool[page, t % side.page_tokens] = v_row
        else:
            side.k_pool[page, :, t % side.page_tokens] = k_row
            side.v_pool[page, :, t % side.page_tokens] = v_row
    elif side.layout == "nhd":
        side.k[u][t] = k_row
        side.v[u][t] = v_row
    else:
        side.k[u][:, t] = k_row
        side.v[u][:, t] = v_row


def _clone_side(side):
    c = copy.copy(side)
    if side.paged:
        c.k_pool, c.v_pool = side.k_pool.clone(), side.v_pool.clone()
    else:
        c.k, c.v = [t.clone() for t in side.k], [t.clone() for t in side.v]
    return c


def _all_bytes(side):
    ts = [side.k_pool, side.v_pool] if side.paged else list(side.k) + list(side.v)
    return [t.view(torch.int32 if t.dtype == torch.float32 else torch.int16).cpu() for t in ts]


CASES = [
    (torch.bfloat16, 32, 8, 128, [40, 1, 700, 33], [1, 16, 17, 250], "nhd", False),
    (torch.bfloat16, 32, 8, 128, [40, 1, 700, 33], [1, 16, 17, 250], "nhd_hpw", False),
    (torch.bfloat16, 16, 4, 128, [2000, 10, 0], [1500, 3000, 1], "nhd_hpw", False),
    (torch.bfloat16, 32, 8, 128, [40, 1, 700, 33], [1, 16, 17, 250], "hnd", False),
    (torch.bfloat16, 64, 8, 128, [300, 0, 5000], [32, 1, 4097], "hnd_exact", False),
    (torch.bfloat16, 32, 8, 128, [40, 1, 700, 33], [1, 16, 17, 250], "nhd", True),
    (torch.bfloat16, 32, 8, 128, [2000, 10], [1500, 3000], "nhd", True),
    (torch.bfloat16, 32, 8, 128, [2000, 10, 0], [1500, 3000, 1], "nhd", "token_major"),
    (torch.bfloat16, 16, 4, 128, [40, 1, 700, 33], [1, 16, 17, 250], "nhd", "token_major"),
    (torch.bfloat16, 32, 8, 128, [2000, 10, 0], [1500, 3000, 1], "nhd_hpw", "token_major"),
    (torch.float32, 8, 8, 64, [128, 5], [16, 1], "nhd", False),
    (torch.float32, 8, 2, 128, [128, 5, 9], [33, 1, 900], "nhd", True),
    (torch.bfloat16, 32, 8, 64, [40, 1, 700, 33], [1, 16, 17, 250], "nhd", False),
    (torch.bfloat16, 12, 2, 64, [2000, 10, 0], [1500, 3000, 1], "hnd", False),
    (torch.bfloat16, 32, 8, 64, [128, 5, 9], [33, 1, 900], "nhd", "token_major"),
    (torch.bfloat16, 32, 8, 64, [2000, 10, 0], [1500, 3000, 1], "nhd_hpw", False),
    (torch.bfloat16, 16, 4, 64, [2000, 10, 0], [1500, 3000, 1], "nhd_hpw", "token_major"),
    (torch.bfloat16, 64, 8, 64, [300, 0, 5000], [32, 1, 4097], "nhd", True),
    (torch.float32, 8, 8, 64, [128, 5], [16, 1], "nhd", False),
    (torch.float32, 8, 2, 128, [128, 5, 9], [33, 1, 900], "nhd", True),
    (torch.float32, 16, 4, 128, [2000, 10, 0], [1500, 3000, 1], "hnd", False),
    (torch.float16, 32, 8, 128, [40, 1, 700, 33], [1, 16, 17, 250], "hnd", False),
    (torch.float16, 32, 8, 128, [2000, 10, 0], [1500, 3000, 1], "nhd_hpw", "token_major"),
    (torch.float16, 32, 8, 64, [2000, 10, 0], [1500, 3000, 1], "nhd", True),
    # many short rows: the pieces hold their result rows back (the result ring) while they append
    (torch.bfloat16, 16, 8, 128, [(37 * u) % 400 for u in range(220)], [1 + (53 * u) % 300 for u in range(220)], "hnd", False),
    (torch.bfloat16, 16, 8, 128, [(37 * u) % 400 for u in range(220)], [1 + (53 * u) % 300 for u in range(220)], "nhd_hpw4", "token_major"),
]


@pytest.mark.parametrize("page_tokens", [32, 128])
@pytest.mark.parametrize("paged", [True, "token_major"])
@pytest.mark.parametrize("fused", [False, True])
def test_append_with_larger_pages(ctx, page_tokens, paged, fused):
    """The new token lands in the right place of a 32- or 128-token page: first slot of a fresh page, last slot of a
    full one, somewhere in between."""
    import paper_2409_19134_amd as spd
    U, Hq, Hkv, d, dtype = 4, 16, 4, 128, torch.bfloat16
    lo = [page_tokens + 1, page_tokens, 5, 3 * page_tokens - 1]
    wl = workloads.random_case(212, dtype, U, Hq, Hkv, d, [40, 1, 700, 33], lo, device=DEV, paged=paged,
                               page_tokens=page_tokens)
    g = torch.Generator(device=DEV).manual_seed(978)
    k_new = torch.randn((U, Hkv, d), generator=g, device=DEV).to(dtype)
    v_new = torch.randn((U, Hkv, d), generator=g, device=DEV).to(dtype)
    want = copy.copy(wl)
    want.public = _clone_side(wl.public)
    for u in range(U):
        _set_last_token(want.public, u, k_new[u], v_new[u])
    step = spd.DecodeStep.from_workload(ctx, wl)
    if fused:
        step.run_fused(wl.q, k_new=k_new, v_new=v_new)
    else:
        step.run_two_parties(wl.q, k_new=k_new, v_new=v_new)
    torch.cuda.synchronize()
    Y, _ = orc.attention(orc.from_workload(want))
    assert np.abs(step.y.cpu().double().numpy().reshape(Y.shape) - Y).max() <= TOL[dtype]
    for a, b in zip(_all_bytes(wl.public), _all_bytes(want.public)):
        assert torch.equal(a, b)


@pytest.mark.parametrize("dtype,Hq,Hkv,d,lp,lo,layout,paged", CASES)
@pytest.mark.parametrize("fused", [False, True, "two_parties"])
@pytest.mark.parametrize("steps", [None, 2])
def test_append_then_attend(ctx, mapping_of, in_flight, dtype, Hq, Hkv, d, lp, lo, layout, paged, fused, steps):
    layout = mapping_of(layout)
    in_flight(steps)
    import paper_2409_19134_amd as spd
    U = len(lp)
    wl = workloads.random_case(211, dtype, U, Hq, Hkv, d, lp, lo, device=DEV, layout=layout, paged=paged)
    g = torch.Generator(device=DEV).manual_seed(977)
    k_new = torch.randn((U, Hkv, d), generator=g, device=DEV).to(dtype)
    v_new = torch.randn((U, Hkv, d), generator=g, device=DEV).to(dtype)
    # the slot the new token goes to holds something else beforehand
    for u in range(U):
        _set_last_token(wl.public, u, torch.full((Hkv, d), 3.0, device=DEV, dtype=dtype),
                        torch.full((Hkv, d), -5.0, device=DEV, dtype=dtype))
    # what the cache must look like afterwards: a plain copy of the new rows into that slot
    want = copy.copy(wl)
    want.public = _clone_side(wl.public)
    for u in range(U):
        _set_last_token(want.public, u, k_new[u], v_new[u])
    hw = orc.from_workload(want)
    A_out, m_out, g_out = orc.partial(hw, hw.public)
    tol = TOL[dtype]

    step = spd.DecodeStep.from_workload(ctx, wl)
    if fused == "two_parties":       # the users' call, then the service's call with the append
        step.run_two_parties(wl.q, k_new=k_new, v_new=v_new)
    elif fused:
        step.run_fused(wl.q, k_new=k_new, v_new=v_new)
    else:
        ctx.spd_partial_attn_public_batched_append(step.shape, wl.q, k_new, v_new, step.public, step.a_out, step.lse_out)
    torch.cuda.synchronize()

    got = step.a_out.cpu().double().numpy().reshape(A_out.shape)
    assert np.abs(got - A_out).max() <= tol
    lse_want = orc.lse_of(m_out, g_out)
    assert np.abs(step.lse_out.cpu().double().numpy().reshape(-1) - lse_want).max() <= tol
    if fused:
        Y, _ = orc.attention(hw)
        assert np.abs(step.y.cpu().double().numpy().reshape(Y.shape) - Y).max() <= tol
    # the cache: the new rows are in place bit for bit and no other byte moved
    for a, b in zip(_all_bytes(wl.public), _all_bytes(want.public)):
        assert torch.equal(a, b)
    # a plain call on the updated cache now gives the same partial
    a2, l2 = ctx.spd_partial_attn_public_batched(step.shape, wl.q, step.public)
    torch.cuda.synchronize()
    assert (a2 - step.a_out).abs().max().item() <= (1e-5 if fused is True else 0.0)


def test_append_argument_errors(ctx):
    import paper_2409_19134_amd as spd
    wl = workloads.random_case(223, torch.bfloat16, 2, 32, 8, 128, [10, 10], [5, 0], device=DEV)
    step = spd.DecodeStep.from_workload(ctx, wl)
    kn = torch.zeros((2, 8, 128), device=DEV, dtype=torch.bfloat16)
    with pytest.raises(spd.SpdError) as ei:      # a user whose length does not even count the new token
        ctx.spd_partial_attn_public_batched_append(step.shape, wl.q, kn, kn, step.public, step.a_out, step.lse_out)
    assert ei.value.code == spd.SPD_ERR_LEN
    with pytest.raises(spd.SpdError) as ei:      # only one of the two rows given
        ctx.spd_decode_step(step.shape, wl.q, step.private, step.public, step.a_in, step.lse_in, step.a_out,
                            step.lse_out, step.y, step.lse, step.w_in, None, kn, None)
    assert ei.value.code == spd.SPD_ERR_NULL
