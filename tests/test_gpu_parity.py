"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the same seeded inputs.

Tolerances are the ones the benchmark contract states: max abs error <= 1e-5 for fp32 inputs and <= 2e-3 for
bf16 inputs with fp32 accumulation (on A_in, A_out, Y and on the log-sum-exps).
"""
import numpy as np
import pytest
import torch

import workloads
from oracle import spd_oracle as orc

pytestmark = pytest.mark.gpu

# fp16: fp32 accumulation of exact products, probabilities carried with ~22 bits: the fp32 bar with room for the
# hardware exp2 / log2 over tens of thousands of tokens
TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-3, torch.float16: 1e-4}
DEV = "cuda:0"


@pytest.fixture(scope="module")
def ctx():
    import paper_2409_19134_amd as spd
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = spd.Context(0)
    yield c
    torch.cuda.synchronize()
    c.close()


def run_step(ctx, wl, fused=False):
    """One decode step: the three C-ABI calls in sequence, the fused spd_decode_step (fused=True), or the users' call
    followed by the service's spd_public_attn_merge (fused="two_parties")."""
    import paper_2409_19134_amd as spd
    step = spd.DecodeStep.from_workload(ctx, wl)
    for t in (step.a_in, step.a_out, step.y, step.lse_in, step.lse_out, step.lse, step.w_in):
        t.fill_(float("nan"))          # every output must be overwritten
    if fused == "two_parties":
        step.run_two_parties(wl.q)
    elif fused:
        step.run_fused(wl.q)
    else:
        step.run(wl.q)
    torch.cuda.synchronize()
    return step


def maxerr(got: torch.Tensor, want: np.ndarray) -> float:
    g = got.detach().cpu().double().numpy().reshape(want.shape)
    both_inf = np.isinf(g) & np.isinf(want) & (np.sign(g) == np.sign(want))
    with np.errstate(invalid="ignore"):          # inf - inf where both sides agree on the infinity
        diff = np.where(both_inf, 0.0, np.abs(g - want))
    assert not np.isnan(g).any(), "NaN in GPU result"
    return float(diff.max()) if diff.size else 0.0


def check_against_oracle(ctx, wl, rows=None, tol=None):
    """All three ways of running a step (three calls; fused call; users' call + service's call) against the oracle.
    Returns the three-call step."""
    hw = orc.from_workload(wl)
    want = _oracle_outputs(hw, rows)          # once: the three forms must all give this
    first = None
    for fused in (False, True, "two_parties"):
        step, errs = _check_one(ctx, wl, want, rows, tol, fused)
        first = first or (step, errs)
    return first


def _oracle_outputs(hw, rows):
    Y, lse = orc.attention(hw, rows=rows)
    A_in, m_in, g_in = orc.partial(hw, hw.private, rows=rows)
    A_out, m_out, g_out = orc.partial(hw, hw.public, rows=rows)
    _, _, _, w_in = orc.merge(A_in, m_in, g_in, A_out, m_out, g_out)
    return dict(Y=Y, lse=lse, A_in=A_in, A_out=A_out, w_in=w_in, lse_in=orc.lse_of(m_in, g_in),
                lse_out=orc.lse_of(m_out, g_out))


def _check_one(ctx, wl, want, rows, tol, fused):
    tol = TOL[wl.dtype] if tol is None else tol
    step = run_step(ctx, wl, fused)
    if rows is None:
        sel = slice(None)
    else:
        r = np.asarray(rows)
        sel = torch.as_tensor(r[:, 0] * wl.n_q_heads + r[:, 1], device=DEV)
    flat = lambda t: t.reshape(wl.n_users * wl.n_q_heads, -1)[sel]
    errs = {
        "A_in": maxerr(flat(step.a_in), want["A_in"]), "A_out": maxerr(flat(step.a_out), want["A_out"]),
        "Y": maxerr(flat(step.y), want["Y"]),
        "lse_in": maxerr(flat(step.lse_in), want["lse_in"][:, None]),
        "lse_out": maxerr(flat(step.lse_out), want["lse_out"][:, None]),
        "lse": maxerr(flat(step.lse), want["lse"][:, None]),
        "w_in": maxerr(flat(step.w_in), want["w_in"][:, None]),
    }
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"fused={fused}: beyond tolerance {tol}: {bad} (all: {errs})"
    return step, errs


# ---------------------------------------------------------------------------
# the five benchmark configurations at oracle-sized lengths (several tiles, ragged tails)


def test_config1_fp32_full_size(ctx):
    check_against_oracle(ctx, workloads.make_workload(1, DEV))


@pytest.mark.parametrize("cfg,len_div,n_users,layout", [(2, 4, None, None), (3, 64, 12, None), (4, 8, 48, None),
                                                        (4, 8, 48, "nhd"), (2, 8, None, "nhd"), (5, 128, 6, None),
                                                        (5, 128, 6, "nhd"), (3, 64, 12, "nhd"),
                                                        (4, 8, 48, "nhd_hpw"), (2, 8, None, "nhd_hpw"),
                                                        (3, 64, 12, "nhd_hpw"), (5, 128, 6, "nhd_hpw"),
                                                        (4, 8, 48, "nhd_hpw4"), (2, 8, None, "nhd_hpw4"),
                                                        (3, 64, 12, "nhd_hpw2"), (5, 128, 6, "nhd_hpw4")])
@pytest.mark.parametrize("steps", [1, 2])
def test_configs_reduced_lengths(ctx, mapping_of, in_flight, cfg, len_div, n_users, layout, steps):
    layout = mapping_of(layout)
    in_flight(steps)
    check_against_oracle(ctx, workloads.make_workload(cfg, DEV, len_div=len_div, n_users=n_users, layout=layout))


def test_config2_full_size_all_rows(ctx):
    """The headline workload at its real size; the oracle still finishes in seconds."""
    check_against_oracle(ctx, workloads.make_workload(2, DEV))


# ---------------------------------------------------------------------------
# full-size workloads, sampled output rows


def _one_row_per_stream(wl):
    """One query head of every (user, KV head) stream - every byte of K and V enters some checked row - with the head
    inside the group rotating, so that every position g = 0 .. G-1 of the MFMA tile is checked many times."""
    G = wl.n_q_heads // wl.n_kv_heads
    return [(u, kvh * G + (u + kvh) % G) for u in range(wl.n_users) for kvh in range(wl.n_kv_heads)]


@pytest.mark.parametrize("cfg,layout", [(3, None), (4, None), (5, None), (3, "nhd"),
                                        (4, "nhd"), (5, "nhd")])   # large and token-major: head per wave
def test_full_size_one_row_per_stream(ctx, cfg, layout):
    """The three big workloads at their real size, in the launch configurations the benchmark times (three calls, the
    fused step, the two parties), head-major and token-major."""
    wl = workloads.make_workload(cfg, DEV, layout=layout)
    rows = _one_row_per_stream(wl)
    assert len(rows) == wl.n_users * wl.n_kv_heads
    check_against_oracle(ctx, wl, rows=rows)


# ---------------------------------------------------------------------------
# edge cases


@pytest.mark.parametrize("lp,lo", [
    ([0], [0]), ([1], [0]), ([0], [1]), ([1], [1]),
    ([31], [33]), ([32], [32]), ([127, 128, 129], [0, 1, 2]),
    ([0, 0, 700], [5, 0, 0]), ([513, 1025, 2049], [95, 96, 97]),
])
@pytest.mark.parametrize("layout,paged", [("nhd", False), ("nhd_hpw", False), ("hnd", False), ("hnd_exact", False),
                                          ("nhd", True), ("nhd", "token_major"), ("nhd_hpw", "token_major"),
                                          ("nhd_hpw4", False), ("nhd_hpw2", "token_major")])
@pytest.mark.parametrize("steps", [None, 2])
def test_bf16_edge_lengths(ctx, mapping_of, in_flight, lp, lo, layout, paged, steps):
    layout = mapping_of(layout)
    in_flight(steps)
    wl = workloads.random_case(101, torch.bfloat16, len(lp), 32, 8, 128, lp, lo, device=DEV, layout=layout, paged=paged)
    step, _ = check_against_oracle(ctx, wl)
    for u in range(len(lp)):     # empty parts are exact: zeros and -inf
        if lp[u] == 0:
            assert (step.a_in[u] == 0).all() and torch.isneginf(step.lse_in[u]).all()
            assert (step.w_in[u] == 0).all()
        if lo[u] == 0:
            assert (step.a_out[u] == 0).all() and torch.isneginf(step.lse_out[u]).all()
        if lp[u] == 0 and lo[u] == 0:
            assert (step.y[u] == 0).all() and torch.isneginf(step.lse[u]).all()
        elif lo[u] == 0:
            assert torch.equal(step.y[u], step.a_in[u])       # merging with an empty part is the identity
        elif lp[u] == 0:
            assert torch.equal(step.y[u], step.a_out[u])


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (16, 8), (64, 8), (16, 1), (12, 4), (32, 2), (48, 16),
                                    (128, 8),    # G = 16 with 8 waves: head-per-wave results too big for the LDS tiles
                                    (24, 12), (27, 9), (32, 32)])   # head per wave in groups of 6, 3 and 8 heads
@pytest.mark.parametrize("layout", ["nhd", "nhd_hpw", "nhd_hpw4", "hnd"])   # nhd_hpw: one wave per KV head where Hkv is in 2..8; nhd_hpw4: groups of up to four heads
@pytest.mark.parametrize("steps", [None, 2])
def test_bf16_head_groupings(ctx, mapping_of, in_flight, Hq, Hkv, layout, steps):
    layout = mapping_of(layout)
    in_flight(steps)
    wl = workloads.random_case(103, torch.bfloat16, 3, Hq, Hkv, 128, [300, 77, 1500], [40, 0, 65], device=DEV,
                               layout=layout)
    check_against_oracle(ctx, wl)


def _random_case_spec(rng):
    """Shape, lengths, storage and mapping of one randomised case, drawn from the given numpy generator."""
    bf16 = rng.random() < 0.7
    Hkv = int(rng.choice([1, 2, 4, 8] if bf16 else [1, 2, 4]))
    G = int(rng.choice([1, 2, 3, 4, 8, 16] if bf16 else [1, 2, 4, 8]))
    d = 128 if bf16 else int(rng.choice([64, 128]))
    U = int(rng.integers(1, 7))
    kinds = [lambda: 0, lambda: int(rng.integers(1, 40)), lambda: int(rng.integers(40, 800)),
             lambda: int(rng.integers(800, 6000)), lambda: int(rng.choice([32, 64, 128, 512, 1024]))]
    weights = [0.1, 0.25, 0.3, 0.2, 0.15]
    lens = lambda: [kinds[int(rng.choice(len(kinds), p=weights))]() for _ in range(U)]
    storage = str(rng.choice(["nhd", "nhd_hpw", "nhd_hpw4", "hnd", "hnd_exact", "paged", "paged_tm", "paged_tm_hpw", "paged_tm_hpw2"]))
    return dict(dtype=torch.bfloat16 if bf16 else torch.float32, U=U, Hq=Hkv * G, Hkv=Hkv, d=d, lp=lens(), lo=lens(),
                storage=storage, scale=float(rng.choice([d ** -0.5, 0.02, 0.3])))


@pytest.mark.parametrize("steps", [1, 2])
@pytest.mark.parametrize("block", range(4))
def test_randomised_cases(ctx, mapping_of, in_flight, block, steps):
    """Seeded random shapes, lengths, storage modes and kernel mappings; every case through both step variants and
    both forms of the streaming kernel."""
    in_flight(steps)
    rng = np.random.default_rng(9000 + block)
    for i in range(10):
        c = _random_case_spec(rng)
        print(f"randomised case {block}.{i}: {c}", flush=True)       # names the case if the GPU run ends badly
        storage = mapping_of(c["storage"])
        paged = {"paged": True, "paged_tm": "token_major"}.get(storage, False)
        layout = "nhd" if paged else storage
        wl = workloads.random_case(9100 + 16 * block + i, c["dtype"], c["U"], c["Hq"], c["Hkv"], c["d"], c["lp"], c["lo"],
                                   device=DEV, layout=layout, paged=paged, scale=c["scale"])
        check_against_oracle(ctx, wl)


def _random_case_spec_wide(rng):
    """Like _random_case_spec, over all three element types, both head sizes, every head group size and KV-head
    counts that need head groups in the head-per-wave mapping."""
    kind = rng.random()
    dtype = torch.bfloat16 if kind < 0.45 else torch.float16 if kind < 0.8 else torch.float32
    f32 = dtype == torch.float32
    Hkv = int(rng.choice([1, 2, 3, 4, 8] if f32 else [1, 2, 3, 4, 8, 12, 16, 27]))
    G = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 16] if f32 else [1, 2, 3, 4, 8, 16]))
    G = min(G, max(1, 128 // Hkv))
    d = int(rng.choice([64, 128]))
    U = int(rng.integers(1, 7))
    kinds = [lambda: 0, lambda: int(rng.integers(1, 40)), lambda: int(rng.integers(40, 800)),
             lambda: int(rng.integers(800, 6000)), lambda: int(rng.choice([32, 64, 128, 512, 1024]))]
    weights = [0.1, 0.25, 0.3, 0.2, 0.15]
    lens = lambda: [kinds[int(rng.choice(len(kinds), p=weights))]() for _ in range(U)]
    storage = str(rng.choice(["nhd", "nhd_hpw", "nhd_hpw4", "nhd_hpw3", "hnd", "hnd_exact", "paged", "paged_tm", "paged_tm_hpw", "paged_tm_hpw4"]))
    return dict(dtype=dtype, U=U, Hq=Hkv * G, Hkv=Hkv, d=d, lp=lens(), lo=lens(), storage=storage,
                scale=float(rng.choice([d ** -0.5, 0.02, 0.3])), page_tokens=int(rng.choice([16, 32, 64, 128, 256])))


@pytest.mark.parametrize("steps", [1, 2])
@pytest.mark.parametrize("block", range(4))
def test_randomised_cases_all_dtypes_and_head_sizes(ctx, mapping_of, in_flight, block, steps):
    in_flight(steps)
    rng = np.random.default_rng(9500 + block)
    for i in range(10):
        c = _random_case_spec_wide(rng)
        print(f"randomised wide case {block}.{i}: {c}", flush=True)
        storage = mapping_of(c["storage"])
        paged = {"paged": True, "paged_tm": "token_major"}.get(storage, False)
        layout = "nhd" if paged else storage
        wl = workloads.random_case(9600 + 16 * block + i, c["dtype"], c["U"], c["Hq"], c["Hkv"], c["d"], c["lp"], c["lo"],
                                   device=DEV, layout=layout, paged=paged, scale=c["scale"], page_tokens=c["page_tokens"])
        check_against_oracle(ctx, wl)


def _pad_contiguous(side, Hkv, d, pad_tokens, pad_channels, token_major):
    """Re-house every user's K and V in buffers with unused channels after each row and unused rows after each head
    (head-major) or unused channels after each token's heads (token-major); fills the padding with a large value."""
    for name in ("k", "v"):
        out = []
        for t in getattr(side, name):
            if token_major:                                   # [L, Hkv, d] -> rows of Hkv*d + pad_channels elements
                L = t.shape[0]
                big = torch.full((max(L, 1), Hkv * d + pad_channels), 777.0, device=t.device, dtype=t.dtype)
                big[:L, :Hkv * d] = t.reshape(L, Hkv * d)
            else:                                             # [Hkv, cap, d] -> [Hkv, cap + pad_tokens, d + pad_channels]
                cap = t.shape[1]
                big = torch.full((Hkv, cap + pad_tokens, d + pad_channels), 777.0, device=t.device, dtype=t.dtype)
                big[:, :cap, :d] = t
            out.append(big)
        setattr(side, name, out)
    if token_major:
        side.token_stride = Hkv * d + pad_channels
    else:
        side.token_stride = d + pad_channels
        side.head_stride = (side.k[0].shape[1]) * (d + pad_channels)


@pytest.mark.parametrize("layout", ["hnd", "nhd", "nhd_hpw"])
@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64)])
def test_padded_strides(ctx, mapping_of, layout, dtype, d):
    """Token and head strides larger than the data they step over (rows and heads with unused space behind them)."""
    layout = mapping_of(layout)
    Hkv = 4
    wl = workloads.random_case(106, dtype, 3, 8, Hkv, d, [700, 33, 1500], [40, 0, 129], device=DEV, layout=layout)
    for side in (wl.private, wl.public):
        _pad_contiguous(side, Hkv, d, pad_tokens=3, pad_channels=32, token_major=layout == "nhd")
    check_against_oracle(ctx, wl)


def test_many_users_with_short_rows(ctx):
    """Thousands of workgroups that each take a whole short row (or only write an empty one)."""
    rng = np.random.default_rng(77)
    U = 1500
    lp = rng.integers(0, 300, U).tolist()
    lo = rng.integers(0, 40, U).tolist()
    wl = workloads.random_case(104, torch.bfloat16, U, 16, 8, 128, lp, lo, device=DEV, layout="hnd_exact")
    check_against_oracle(ctx, wl)


@pytest.mark.parametrize("chunk_max", [None, 128])
def test_one_very_long_row(chunk_max, monkeypatch):
    """A single KV head with a quarter of a million tokens: the row is cut into 512 chunks (one per resident workgroup);
    with the piece limit forced down to 128 tokens into ~2000, more than one staging pass of the combine holds.
    A context of its own (the piece limit is an option of the context), and the chunk count is checked, not assumed."""
    import paper_2409_19134_amd as spd
    own = spd.Context(0)
    lp, lo = 200_003, 70_001
    if chunk_max:
        own.spd_set_option(spd.SPD_OPT_CHUNK_MAX, chunk_max)
        assert own.spd_get_option(spd.SPD_OPT_CHUNK_MAX) == chunk_max
        monkeypatch.setenv("SPD_CHUNK_MAX", str(chunk_max))      # the host-only helper below reads the environment
    n_cus = torch.cuda.get_device_properties(0).multi_processor_count
    items, _ = spd.spd_build_schedule(spd.make_shape(torch.bfloat16, 4, 1, 128, 0.1), [lp], n_cus)
    assert all(it["n_chunks"] == len(items) for it in items)
    assert (len(items) >= 1500) == bool(chunk_max), len(items)          # beyond the combine's 512-chunk staging pass
    wl = workloads.random_case(105, torch.bfloat16, 1, 4, 1, 128, [lp], [lo], device=DEV, layout="hnd")
    builds0, _ = own.spd_get_schedule_stats()
    check_against_oracle(own, wl)
    builds1, _ = own.spd_get_schedule_stats()
    # both owners' schedules were built by this context, under its options: for the separate calls (an owner alone
    # gets a larger resident round) and for the fused step - except that the private row's pieces at the default
    # piece limit are short enough for the separate call to take the fused step's round, and so its schedule
    assert builds1 - builds0 == (4 if chunk_max else 3)
    own.close()


@pytest.mark.parametrize("rows_opt,layout,group", [(None, "hnd", 0), (0, "hnd", 0), (3, "hnd", 0), (None, "nhd", 4),
                                                  (2, "nhd", 4), (None, "nhd", 8), (None, "nhd", 2)])
def test_many_rows_per_piece_fused_step_and_result_ring(rows_opt, layout, group):
    """Many users with rows of a few hundred tokens on both sides: every piece crosses several rows, so the pieces hold
    their result rows back and store them together (the ring is filled and emptied several times per piece with
    rows_opt = 3, never used with 0), and the fused step - both owners would each fill the device - builds schedules of
    its own with half as many pieces per owner."""
    import paper_2409_19134_amd as spd
    own = spd.Context(0)
    if rows_opt is not None:
        own.spd_set_option(spd.SPD_OPT_RESULT_ROWS, rows_opt)
    own.spd_set_option(spd.SPD_OPT_HEAD_PER_WAVE, group)     # token-major: a ring per wave, `group` KV heads per workgroup
    rng = np.random.default_rng(77)
    U = 300
    lp = rng.integers(0, 700, size=U).tolist()
    lo = rng.integers(0, 500, size=U).tolist()
    lp[3] = lo[3] = 0
    lp[7], lo[8] = 5000, 3000                       # rows longer than the short-row rule allows
    wl = workloads.random_case(108, torch.bfloat16, U, 16, 8, 128, lp, lo, device=DEV, layout=layout)
    builds0, _ = own.spd_get_schedule_stats()
    check_against_oracle(own, wl)
    builds1, _ = own.spd_get_schedule_stats()
    assert builds1 - builds0 == 4          # the separate calls' schedules and the fused step's own
    own.close()


@pytest.mark.parametrize("dtype,Hq,Hkv,d,layout,paged,group", [
    (torch.float32, 8, 8, 64, "hnd", False, 0), (torch.float32, 12, 4, 128, "hnd", True, 0),
    (torch.float16, 24, 8, 64, "hnd_exact", False, 0), (torch.bfloat16, 40, 8, 128, "hnd", True, 0),
    (torch.bfloat16, 64, 8, 128, "hnd", False, 0),            # G = 8: fewer rows fit the ring
    (torch.bfloat16, 128, 8, 128, "hnd", False, 0),           # G = 16: no room for a ring beside the staging tiles
    (torch.float16, 12, 4, 64, "nhd", "token_major", 4), (torch.bfloat16, 48, 16, 128, "nhd", False, 8),
])
def test_result_ring_shapes(dtype, Hq, Hkv, d, layout, paged, group):
    """The result ring over element types, head sizes, group sizes, storage modes and both mappings, with the KV
    append in the fused step: many users with short rows, so that every piece holds rows back."""
    import paper_2409_19134_amd as spd
    own = spd.Context(0)
    own.spd_set_option(spd.SPD_OPT_HEAD_PER_WAVE, group)
    rng = np.random.default_rng(79)
    U = 200
    lp = rng.integers(0, 400, size=U).tolist()
    lo = rng.integers(1, 300, size=U).tolist()
    lp[5], lo[6] = 3000, 2000
    wl = workloads.random_case(109, dtype, U, Hq, Hkv, d, lp, lo, device=DEV, layout=layout, paged=paged)
    check_against_oracle(own, wl)
    own.close()


@pytest.mark.parametrize("d,Hq,Hkv", [(64, 8, 8), (64, 8, 2), (128, 8, 1), (128, 4, 4), (64, 16, 2)])
@pytest.mark.parametrize("paged", [False, True])
def test_fp32_shapes(ctx, d, Hq, Hkv, paged):
    wl = workloads.random_case(107, torch.float32, 4, Hq, Hkv, d, [128, 0, 1000, 3], [16, 5, 0, 77], device=DEV, paged=paged)
    check_against_oracle(ctx, wl)


@pytest.mark.parametrize("dtype,d,Hq,Hkv", [
    (torch.bfloat16, 64, 32, 8), (torch.bfloat16, 64, 8, 8), (torch.bfloat16, 64, 12, 2), (torch.bfloat16, 64, 14, 2),
    (torch.bfloat16, 64, 3, 1), (torch.bfloat16, 64, 40, 8), (torch.bfloat16, 64, 64, 4), (torch.bfloat16, 64, 16, 16),
    (torch.float32, 64, 9, 3), (torch.float32, 128, 5, 1), (torch.float32, 64, 12, 2), (torch.float32, 128, 14, 2)])
@pytest.mark.parametrize("storage", ["hnd", "nhd", "nhd_hpw", "paged", "paged_tm", "paged_tm_hpw"])
def test_small_head_dim_and_odd_groups(ctx, mapping_of, dtype, d, Hq, Hkv, storage):
    """bf16 with 64 channels per head (every storage mode and mapping), and fp32 head groups of 3, 5, 6 and 7."""
    storage = mapping_of(storage)
    paged = {"paged": True, "paged_tm": "token_major"}.get(storage, False)
    wl = workloads.random_case(108, dtype, 5, Hq, Hkv, d, [128, 0, 1000, 3, 2500], [16, 5, 0, 77, 300], device=DEV,
                               layout="nhd" if paged else storage, paged=paged)
    check_against_oracle(ctx, wl)


@pytest.mark.parametrize("lp,lo", [(0, 0), (1, 0), (31, 33), (32, 64), (127, 129), (4097, 1), (20000, 700)])
@pytest.mark.parametrize("storage", ["hnd", "nhd_hpw", "paged"])
def test_bf16_d64_edge_lengths(ctx, mapping_of, lp, lo, storage):
    storage = mapping_of(storage)
    paged = storage == "paged"
    wl = workloads.random_case(109, torch.bfloat16, 2, 32, 8, 64, [lp, 77], [lo, 5], device=DEV,
                               layout="nhd" if paged else storage, paged=paged)
    check_against_oracle(ctx, wl)


@pytest.mark.parametrize("d,Hq,Hkv", [(128, 32, 8), (128, 64, 4), (128, 6, 2), (64, 32, 8), (64, 16, 16), (64, 7, 1)])
@pytest.mark.parametrize("storage", ["hnd", "nhd", "nhd_hpw", "paged", "paged_tm", "paged_tm_hpw"])
def test_fp16_shapes(ctx, mapping_of, d, Hq, Hkv, storage):
    storage = mapping_of(storage)
    paged = {"paged": True, "paged_tm": "token_major"}.get(storage, False)
    wl = workloads.random_case(110, torch.float16, 5, Hq, Hkv, d, [128, 0, 1000, 3, 2500], [16, 5, 0, 77, 300], device=DEV,
                               layout="nhd" if paged else storage, paged=paged)
    check_against_oracle(ctx, wl)


@pytest.mark.parametrize("lp,lo", [(0, 0), (1, 0), (31, 33), (127, 129), (4097, 1), (40000, 700)])
@pytest.mark.parametrize("steps", [None, 2])
def test_fp16_edge_lengths(ctx, in_flight, lp, lo, steps):
    in_flight(steps)
    wl = workloads.random_case(111, torch.float16, 2, 32, 8, 128, [lp, 77], [lo, 5], device=DEV, layout="hnd")
    check_against_oracle(ctx, wl)


def test_fp16_small_probabilities_are_kept(ctx):
    """One dominant token and 30000 tokens whose probability (6e-8 of the largest) lies below fp16's smallest
    subnormal, with large values: together they hold 0.2 % of the mass and move the result by 1.8.  The kernel's
    probabilities therefore cannot be plain fp16 numbers."""
    L, d = 30001, 128
    wl = workloads.random_case(112, torch.float16, 1, 1, 1, d, [L], [0], device=DEV, layout="hnd")
    wl.q.zero_()
    wl.q[0, 0, 0] = 16.0
    k, v = wl.private.k[0], wl.private.v[0]          # [Hkv, capacity, d]
    k.zero_()
    k[0, 1234, 0] = 11.75                              # score 16 * 11.75 / sqrt(128) = 16.62 above all others
    v.fill_(1000.0)
    v[0, 1234] = 0.0
    step, errs = check_against_oracle(ctx, wl)
    assert 1.5 < float(step.y[0, 0, 0]) < 2.1


@pytest.mark.parametrize("d,Hq,Hkv", [(64, 8, 8), (64, 8, 2), (128, 8, 1), (128, 4, 4), (64, 16, 2), (128, 32, 8), (128, 14, 2),
                                      (64, 9, 3), (128, 32, 2), (64, 64, 4)])
@pytest.mark.parametrize("storage", ["hnd", "nhd", "hnd_exact", "paged", "paged_tm"])
def test_fp32_shapes_and_storage_modes(ctx, d, Hq, Hkv, storage):
    paged = {"paged": True, "paged_tm": "token_major"}.get(storage, False)
    wl = workloads.random_case(113, torch.float32, 5, Hq, Hkv, d, [128, 0, 1000, 3, 2500], [16, 5, 0, 77, 300], device=DEV,
                               layout="nhd" if paged else storage, paged=paged)
    check_against_oracle(ctx, wl)


@pytest.mark.parametrize("lp,lo", [(0, 0), (1, 0), (31, 33), (32, 64), (127, 129), (4097, 1), (40000, 700)])
@pytest.mark.parametrize("d", [64, 128])
def test_fp32_edge_lengths(ctx, lp, lo, d):
    wl = workloads.random_case(114, torch.float32, 2, 8, 2, d, [lp, 77], [lo, 5], device=DEV, layout="hnd")
    check_against_oracle(ctx, wl)


def test_fp32_large_launch(ctx):
    """64 users x 8 KV heads x 3000 tokens in fp32 (1.6 GB): several resident rounds of pieces; sampled rows."""
    wl = workloads.random_case(115, torch.float32, 64, 16, 8, 128, [3000] * 64, [100] * 64, device=DEV, layout="hnd")
    check_against_oracle(ctx, wl, rows=[(0, 0), (63, 15), (31, 7), (17, 9)])


def test_peaked_softmax_and_large_score_gap(ctx):
    """Scores spread far beyond the fp32 exp range between the two parts: weights saturate, nothing overflows."""
    wl = workloads.random_case(109, torch.bfloat16, 2, 32, 8, 128, [256, 256], [64, 64], device=DEV, scale=1.0)
    wl.private.k[0].mul_(6.0)        # user 0: private scores ~ N(0, 70): the max dominates
    wl.public.k[1].mul_(8.0)         # user 1: public side dominates
    check_against_oracle(ctx, wl)


def test_single_user_call_equals_batched_call(ctx):
    """A user's rows depend only on that user's buffers: the per-process call gives the same bits."""
    import paper_2409_19134_amd as spd
    wl = workloads.random_case(113, torch.bfloat16, 5, 32, 8, 128, [900, 31, 0, 2500, 128], [10, 300, 7, 0, 64], device=DEV)
    step = run_step(ctx, wl)
    sh = spd.make_shape(wl.dtype, 32, 8, 128, wl.scale)
    for u in range(5):
        v = spd.KVView(wl.private.lens[u:u + 1], wl.private.token_stride, wl.private.head_stride,
                       k=[wl.private.k[u]], v=[wl.private.v[u]],
                       head_strides=None if wl.private.head_strides is None else wl.private.head_strides[u:u + 1])
        a, l = ctx.spd_partial_attn_private(sh, wl.q[u:u + 1].contiguous(), v)
        torch.cuda.synchronize()
        # the split of a user's tokens depends on the batch's total work, so compare to tolerance, not bits
        assert (a[0] - step.a_in[u]).abs().max().item() <= 1e-5
        fin = torch.isfinite(l[0])
        assert torch.equal(fin, torch.isfinite(step.lse_in[u]))
        assert (l[0][fin] - step.lse_in[u][fin]).abs().max().item() <= 1e-5 if fin.any() else True


def test_run_to_run_determinism_and_user_permutation(ctx):
    wl = workloads.random_case(127, torch.bfloat16, 6, 32, 8, 128, [1500, 40, 700, 0, 3000, 64], [9, 100, 0, 50, 512, 1], device=DEV)
    s1 = run_step(ctx, wl)
    y1, l1 = s1.y.clone(), s1.lse.clone()
    s2 = run_step(ctx, wl)
    assert torch.equal(s2.y, y1) and torch.equal(s2.lse, l1)
    # permuting users permutes outputs; where a row is cut depends on the rows before it (a piece gives up steps for
    # reaching into a second row, and the halves of a resident round are unequal), so equal to rounding, not to the bit
    perm = [3, 0, 5, 1, 4, 2]
    import copy
    wp = copy.copy(wl)
    wp.q = wl.q[perm].contiguous()
    for name in ("private", "public"):
        side = copy.copy(getattr(wl, name))
        side.lens = side.lens[perm].copy()
        if side.head_strides is not None:
            side.head_strides = side.head_strides[perm].copy()
        side.k = [side.k[i] for i in perm]
        side.v = [side.v[i] for i in perm]
        setattr(wp, name, side)
    s3 = run_step(ctx, wp)
    assert (s3.y - y1[perm]).abs().max().item() <= 1e-5
    fin = torch.isfinite(l1[perm])
    assert torch.equal(torch.isfinite(s3.lse), fin)
    assert (s3.lse[fin] - l1[perm][fin]).abs().max().item() <= 1e-5
    # with the options that make the cuts depend on the neighbours switched off, it is the same chunking: bit for bit
    import paper_2409_19134_amd as spd
    own = spd.Context(0)
    own.spd_set_option(spd.SPD_OPT_SEG_COST, 0)
    own.spd_set_option(spd.SPD_OPT_HALF_SKEW, 0)
    p1, p3 = run_step(own, wl), run_step(own, wp)
    assert torch.equal(p3.y, p1.y[perm]) and torch.equal(p3.lse, p1.lse[perm])
    own.close()


def test_token_permutation_invariance(ctx):
    """A decode query attends to a set of tokens: shuffling a cache's tokens (K and V together) changes nothing
    beyond rounding."""
    wl = workloads.random_case(131, torch.bfloat16, 1, 32, 8, 128, [777], [100], device=DEV)
    s1 = run_step(ctx, wl)
    y1 = s1.y.clone()
    p = torch.randperm(777, generator=torch.Generator().manual_seed(1)).to(DEV)
    wl.private.k[0] = wl.private.k[0][p].contiguous()
    wl.private.v[0] = wl.private.v[0][p].contiguous()
    s2 = run_step(ctx, wl)
    assert (s2.y - y1).abs().max().item() <= 1e-5


def test_merge_standalone_against_oracle(ctx):
    rng = np.random.default_rng(7)
    n, d = 257, 128
    A0 = rng.standard_normal((n, d)); A1 = rng.standard_normal((n, d))
    l0 = rng.normal(0, 30, n); l1 = rng.normal(0, 30, n)
    l0[:5] = -np.inf; A0[:5] = 0
    l1[3:9] = -np.inf; A1[3:9] = 0
    l0[10], l1[10] = 500.0, -500.0
    l0[11], l1[11] = -3000.0, 2000.0
    l0[12] = l1[12] = 1.25
    t = lambda a: torch.tensor(a, dtype=torch.float32, device=DEV)
    a0, a1, t0, t1 = t(A0), t(A1), t(l0), t(l1)
    lse = torch.empty(n, device=DEV); w = torch.empty(n, device=DEV)
    y = ctx.spd_lse_merge(a0, t0, a1, t1, lse_out=lse, w0_out=w)
    torch.cuda.synchronize()
    # oracle in the paper's (m, gamma) form: m = lse, gamma = 1 (or 0 for an empty side), on the fp32-rounded inputs
    f64 = lambda x: x.cpu().double().numpy()
    g0 = np.where(np.isinf(f64(t0)), 0.0, 1.0); g1 = np.where(np.isinf(f64(t1)), 0.0, 1.0)
    Y, m, g, w0 = orc.merge(f64(a0), f64(t0), g0, f64(a1), f64(t1), g1)
    assert maxerr(y, Y) <= 1e-5
    assert maxerr(w, w0) <= 1e-6
    assert maxerr(lse, orc.lse_of(m, g)) <= 3e-4      # |lse| up to 3000 in fp32
    # in-place on either input and swapped operands
    y2 = ctx.spd_lse_merge(a1, t1, a0, t0)
    torch.cuda.synchronize()
    assert torch.equal(y2, y)
    a0c = a0.clone()
    ctx.spd_lse_merge(a0c, t0, a1, t1, y=a0c)
    torch.cuda.synchronize()
    assert torch.equal(a0c, y)


@pytest.mark.parametrize("n_parts,d", [(1, 128), (2, 128), (3, 64), (8, 128), (16, 256), (5, 4)])
def test_n_way_merge_against_oracle(ctx, n_parts, d):
    rng = np.random.default_rng(100 + n_parts)
    n = 259
    A = [rng.standard_normal((n, d)) for _ in range(n_parts)]
    L = [rng.normal(0, 30, n) for _ in range(n_parts)]
    for k in range(n_parts):                       # empty parts hold garbage that must not leak into the result
        rows = rng.choice(n, size=20, replace=False)
        L[k][rows] = -np.inf
        A[k][rows] = np.nan
    for k in range(n_parts):
        L[k][:3] = -np.inf                        # rows 0-2: every part empty
        A[k][:3] = 7.0
    L[0][3] = 3000.0                               # a gap far beyond the fp32 exponential range
    if n_parts > 1:
        L[1][3] = -3000.0
    t = lambda a: torch.tensor(a, dtype=torch.float32, device=DEV)
    a_t, l_t = [t(a) for a in A], [t(l) for l in L]
    y = torch.full((n, d), float("nan"), device=DEV)
    lse = torch.full((n,), float("nan"), device=DEV)
    w = torch.full((n_parts, n), float("nan"), device=DEV)
    ctx.spd_lse_merge_n(a_t, l_t, y, lse, w)
    torch.cuda.synchronize()
    # the oracle on the values the GPU saw (fp32-rounded inputs)
    Y, lse_o, W = orc.merge_n([(a.cpu().double().numpy(), l.cpu().double().numpy()) for a, l in zip(a_t, l_t)])
    assert maxerr(y, Y) <= 1e-5 * max(1.0, float(np.nanmax(np.abs(Y))))
    assert maxerr(w, W) <= 1e-6
    fin = np.isfinite(lse_o)
    assert maxerr(lse[torch.as_tensor(fin, device=DEV)], lse_o[fin]) <= 1e-3     # |lse| up to 3000 in fp32
    assert torch.isinf(lse[:3]).all() and (lse[:3] < 0).all() and (y[:3] == 0).all() and (w[:, :3] == 0).all()
    # in place over one of the parts, and without the optional outputs
    if n_parts > 1:
        want = y.clone()
        keep = a_t[1].clone()
        ctx.spd_lse_merge_n(a_t, l_t, a_t[1])
        torch.cuda.synchronize()
        assert torch.equal(a_t[1], want)
        a_t[1].copy_(keep)
    if n_parts == 2:                                # the two-owner call gives the same bits
        y2 = torch.empty_like(y)
        a0 = torch.nan_to_num(a_t[0]); a1 = torch.nan_to_num(a_t[1])
        ctx.spd_lse_merge(a0, l_t[0], a1, l_t[1], y2)
        torch.cuda.synchronize()
        assert (y2 - y).abs().max().item() <= 1e-5 * max(1.0, float(np.nanmax(np.abs(Y))))


def test_sequence_sharded_cache_merges_to_the_whole(ctx):
    """A user's cache cut into four consecutive token ranges, each attended to by its own call (what four devices
    holding a sequence-sharded cache would compute), then one n-way merge: equals attention over the whole cache."""
    import paper_2409_19134_amd as spd
    U, Hq, Hkv, d, n_shards = 3, 32, 8, 128, 4
    lens = [5000, 37, 1203]
    wl = workloads.random_case(140, torch.bfloat16, U, Hq, Hkv, d, lens, [0, 0, 0], device=DEV, layout="nhd")
    sh = spd.make_shape(wl.dtype, Hq, Hkv, d, wl.scale)
    outs, lses = [], []
    for s in range(n_shards):
        lo = [L * s // n_shards for L in lens]
        hi = [L * (s + 1) // n_shards for L in lens]
        ks = [k[a:b] for k, a, b in zip(wl.private.k, lo, hi)]          # views into the same buffers: [tokens, Hkv, d]
        vs = [v[a:b] for v, a, b in zip(wl.private.v, lo, hi)]
        view = spd.KVView([b - a for a, b in zip(lo, hi)], token_stride=Hkv * d, head_stride=d, k=ks, v=vs)
        o, l = ctx.spd_partial_attn_private(sh, wl.q, view)
        outs.append(o)
        lses.append(l)
    y = ctx.spd_lse_merge_n(outs, lses)
    torch.cuda.synchronize()
    Y, _ = orc.attention(orc.from_workload(wl))
    assert maxerr(y.reshape(U * Hq, d), Y) <= TOL[wl.dtype]


@pytest.mark.parametrize("dtype,scale", [
    (torch.bfloat16, 0.0), (torch.float16, 0.0), (torch.float32, 0.0),
    (torch.bfloat16, -0.25), (torch.float16, -0.25), (torch.float32, -0.25),
    (torch.bfloat16, 4.0), (torch.float16, 4.0),
    (torch.float32, 0.5)])   # fp32's 1e-5 bar is below half an fp32 ulp of scores (and log-sum-exps) of several hundred
def test_unusual_scales(ctx, dtype, scale):
    """scale = 0 (uniform weights: the mean of V), a negative scale (the least similar key wins) and a large one
    (scores of several hundred for the 16-bit types: nearly one-hot rows)."""
    wl = workloads.random_case(150, dtype, 3, 8, 2, 128, [700, 0, 65], [40, 3, 0], device=DEV, layout="hnd", scale=scale)
    check_against_oracle(ctx, wl)


@pytest.mark.parametrize("page_tokens", [32, 64, 128, 256])
@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float16, 64), (torch.float32, 128)])
@pytest.mark.parametrize("storage", ["paged", "paged_tm", "paged_tm_hpw"])
def test_page_sizes(ctx, mapping_of, page_tokens, dtype, d, storage):
    """Pages of 32 to 256 tokens (16 is what every other paged test uses), rows that end inside, at the end of and
    one token into a page."""
    storage = mapping_of(storage)
    paged = {"paged": True, "paged_tm": "token_major"}[storage]
    lp = [page_tokens * 3, 1, 2500, page_tokens + 1, 0]
    lo = [page_tokens - 1, 5, 0, 777, page_tokens]
    wl = workloads.random_case(160, dtype, 5, 16, 4, d, lp, lo, device=DEV, paged=paged, page_tokens=page_tokens)
    check_against_oracle(ctx, wl)


def test_owners_with_different_page_sizes(ctx):
    """The fused step with 64-token pages on the private side and 16-token pages on the public side."""
    import copy
    a = workloads.random_case(161, torch.bfloat16, 3, 32, 8, 128, [3000, 70, 0], [40, 0, 500], device=DEV, paged=True,
                              page_tokens=64)
    b = workloads.random_case(161, torch.bfloat16, 3, 32, 8, 128, [3000, 70, 0], [40, 0, 500], device=DEV, paged=True,
                              page_tokens=16)
    wl = copy.copy(a)
    wl.public = b.public
    check_against_oracle(ctx, wl)


def test_error_codes_from_device_calls(ctx):
    import paper_2409_19134_amd as spd
    wl = workloads.random_case(137, torch.bfloat16, 1, 32, 8, 128, [64], [8], device=DEV)
    sh = spd.make_shape(wl.dtype, 32, 8, 128, wl.scale)
    v = spd.KVView.from_side(wl.private)
    out = torch.full((1, 32, 128), 7.0, device=DEV)
    lse = torch.full((1, 32), 7.0, device=DEV)
    bad = spd.make_shape(wl.dtype, 30, 8, 128, wl.scale)
    with pytest.raises(spd.SpdError) as ei:
        ctx._partial(spd.lib.spd_partial_attn_private, "x", bad, wl.q[:, :30].contiguous(), v,
                     out[:, :30].contiguous(), lse[:, :30].contiguous(), None)
    assert ei.value.code == spd.SPD_ERR_SHAPE
    torch.cuda.synchronize()
    assert (out == 7.0).all()           # nothing was launched
    ctx.spd_partial_attn_private(sh, wl.q, v, out, lse)
    torch.cuda.synchronize()
    assert not (out == 7.0).any()
