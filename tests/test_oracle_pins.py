"""Pins for the CPU oracle: what the paper and the mathematics fix, computed by other means.

None of these re-type the oracle's own formula: they use a brute force without the
max shift, library softmax routines, closed forms, a hand-worked fixture and the
identity of Theorem 1 (section 4.2; proof in Appendix A) at every split point.
"""
import math
import os

import numpy as np
import pytest
import torch

import workloads
from oracle import spd_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _case(seed, dtype, U, Hq, Hkv, d, lp, lo, **kw):
    wl = workloads.random_case(seed, dtype, U, Hq, Hkv, d, lp, lo, **kw)
    return wl, orc.from_workload(wl)


def _rows_as_float64(wl, side, u, kv):
    """[L, d] float64 K and V rows of one (user, kv head), gathered with torch indexing only."""
    if side.paged:
        L = int(side.lens[u])
        n = -(-L // side.page_tokens)
        pages = side.block_table[u, :n].long()
        if side.page_token_major:
            k = side.k_pool[pages][:, :, kv].reshape(-1, wl.head_dim)[:L]
            v = side.v_pool[pages][:, :, kv].reshape(-1, wl.head_dim)[:L]
        else:
            k = side.k_pool[pages, kv].reshape(-1, wl.head_dim)[:L]
            v = side.v_pool[pages, kv].reshape(-1, wl.head_dim)[:L]
    else:
        L = int(side.lens[u])
        kt, vt = side.k[u], side.v[u]
        if side.layout in ("hnd", "hnd_exact"):
            k, v = kt[kv, :L], vt[kv, :L]
        else:                                      # nhd
            k, v = kt[:L, kv], vt[:L, kv]
    return k.double().numpy(), v.double().numpy()


def _concat_rows(wl, u, kv):
    kp, vp = _rows_as_float64(wl, wl.private, u, kv)
    ko, vo = _rows_as_float64(wl, wl.public, u, kv)
    return np.concatenate([kp, ko]), np.concatenate([vp, vo])


# ---------------------------------------------------------------------------
# 1. brute force: exp of the raw scores, no max shift, python floats / longdouble


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2), (8, 1)])
def test_brute_force_naive_exponentials(dtype, Hq, Hkv):
    d = 8
    wl, hw = _case(11, dtype, 3, Hq, Hkv, d, [5, 0, 17], [3, 4, 0], layout="nhd")
    Y, lse = orc.attention(hw)
    G = Hq // Hkv
    for u in range(3):
        for h in range(Hq):
            K, V = _concat_rows(wl, u, h // G)
            q = wl.q[u, h].double().numpy()
            num = [np.longdouble(0)] * d
            den = np.longdouble(0)
            for i in range(K.shape[0]):
                s = sum(float(q[c]) * float(K[i, c]) for c in range(d)) * wl.scale
                e = np.exp(np.longdouble(s))            # naive: no shift
                den += e
                for c in range(d):
                    num[c] += e * np.longdouble(V[i, c])
            got = Y[u * Hq + h]
            want = np.array([float(n / den) for n in num])
            np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
            assert lse[u * Hq + h] == pytest.approx(float(np.log(den)), rel=1e-12, abs=1e-12)


# ---------------------------------------------------------------------------
# 2. library routines: scipy softmax/logsumexp and torch fp64 scaled_dot_product_attention


@pytest.mark.parametrize("layout,paged", [("nhd", False), ("hnd", False), ("hnd_exact", False), ("nhd", True),
                                          ("nhd", "token_major")])
def test_against_library_softmax(layout, paged):
    from scipy.special import logsumexp, softmax
    U, Hq, Hkv, d = 4, 8, 2, 64
    wl, hw = _case(23, torch.bfloat16, U, Hq, Hkv, d, [33, 1, 100, 48], [16, 7, 0, 31], layout=layout, paged=paged)
    Y, lse = orc.attention(hw)
    G = Hq // Hkv
    for u in range(U):
        for h in range(Hq):
            K, V = _concat_rows(wl, u, h // G)
            q = wl.q[u, h].double().numpy()
            s = (K @ q) * wl.scale
            np.testing.assert_allclose(Y[u * Hq + h], softmax(s) @ V, rtol=1e-11, atol=1e-12)
            assert lse[u * Hq + h] == pytest.approx(logsumexp(s), rel=1e-12)
            # torch's attention routine, fp64, 1 query
            yt = torch.nn.functional.scaled_dot_product_attention(
                torch.from_numpy(q)[None, None], torch.from_numpy(K)[None], torch.from_numpy(V)[None],
                scale=wl.scale)
            np.testing.assert_allclose(Y[u * Hq + h], yt[0, 0].numpy(), rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------------------
# 3. closed forms


def _manual(q, kp, vp, ko, vo, scale=1.0, dtype=torch.float32, Hq=1, Hkv=1):
    """Workload from explicit arrays: q [Hq,d]; kp/vp [Lp,Hkv,d]; ko/vo [Lo,Hkv,d] (one user)."""
    q = torch.as_tensor(q, dtype=torch.float64).reshape(Hq, -1)
    d = q.shape[1]

    def t(a):
        return torch.as_tensor(a, dtype=torch.float64).reshape(-1, Hkv, d).to(dtype)
    kp, vp, ko, vo = t(kp), t(vp), t(ko), t(vo)
    mk = lambda k, v: orc.HostView([k.shape[0]], Hkv * d, d, k=[workloads.host_array(k)], v=[workloads.host_array(v)])
    hw = orc.HostWorkload(orc.F32 if dtype == torch.float32 else orc.BF16, Hq, Hkv, d, scale,
                          workloads.host_array(q.to(dtype))[None], mk(kp, vp), mk(ko, vo))
    return hw


def test_equal_keys_give_mean_of_values():
    d, L = 4, 9
    rng = np.random.default_rng(0)
    k_row = rng.standard_normal(d).astype(np.float32)
    V = rng.standard_normal((L, d)).astype(np.float32)
    q = rng.standard_normal(d).astype(np.float32)
    K = np.tile(k_row, (L, 1))
    hw = _manual(q, K[:4], V[:4], K[4:], V[4:], scale=0.5)
    Y, lse = orc.attention(hw)
    np.testing.assert_allclose(Y[0], V.astype(np.float64).mean(0), rtol=1e-13)
    s = 0.5 * float(np.dot(q.astype(np.float64), k_row.astype(np.float64)))
    assert lse[0] == pytest.approx(s + math.log(L), rel=1e-13)


def test_constant_values_single_token_and_dominant_score():
    d = 4
    rng = np.random.default_rng(1)
    q = rng.standard_normal(d).astype(np.float32)
    K = rng.standard_normal((6, d)).astype(np.float32)
    ones = np.ones((6, d), dtype=np.float32)
    Y, _ = orc.attention(_manual(q, K[:2], ones[:2], K[2:], ones[2:]))
    np.testing.assert_allclose(Y[0], 1.0, rtol=1e-14)
    # one token only (in the public part; private empty): Y = its value row, lse = its score
    V = rng.standard_normal((1, d)).astype(np.float32)
    Y, lse = orc.attention(_manual(q, np.zeros((0, d)), np.zeros((0, d)), K[:1], V, scale=0.25))
    np.testing.assert_array_equal(Y[0], V[0].astype(np.float64))
    assert lse[0] == pytest.approx(0.25 * float(q.astype(np.float64) @ K[0].astype(np.float64)), rel=1e-14)
    # a score far above the rest selects that token's value row
    Kd = K.copy()
    Kd[3] = 200.0 * q / float(q @ q)           # score 200 against O(1) others
    V = rng.standard_normal((6, d)).astype(np.float32)
    Y, _ = orc.attention(_manual(q, Kd[:2], V[:2], Kd[2:], V[2:]))
    np.testing.assert_allclose(Y[0], V[3].astype(np.float64), rtol=0, atol=1e-60)


def test_score_shift_leaves_output_and_moves_lse():
    """Appending a channel with q=1, k=c adds c to every score: Y unchanged, lse + c."""
    d = 4
    rng = np.random.default_rng(2)
    q = rng.standard_normal(d).astype(np.float32)
    K = rng.standard_normal((7, d)).astype(np.float32)
    V = rng.standard_normal((7, d)).astype(np.float32)
    Y0, lse0 = orc.attention(_manual(q, K[:3], V[:3], K[3:], V[3:]))
    c = 3.5
    q1 = np.concatenate([q, [1.0]]).astype(np.float32)
    K1 = np.concatenate([K, np.full((7, 1), c, dtype=np.float32)], axis=1)
    V1 = np.concatenate([V, np.zeros((7, 1), dtype=np.float32)], axis=1)
    Y1, lse1 = orc.attention(_manual(q1, K1[:3], V1[:3], K1[3:], V1[3:]))
    np.testing.assert_allclose(Y1[0, :d], Y0[0], rtol=1e-13)
    assert lse1[0] == pytest.approx(lse0[0] + c, rel=1e-13)


def test_empty_everything():
    d = 4
    hw = _manual(np.ones(d), np.zeros((0, d)), np.zeros((0, d)), np.zeros((0, d)), np.zeros((0, d)))
    Y, lse = orc.attention(hw)
    assert (Y == 0).all() and lse[0] == -np.inf
    A, m, g = orc.partial(hw, hw.private)
    assert (A == 0).all() and m[0] == -np.inf and g[0] == 0
    Ym, mm, gm, w = orc.merge(A, m, g, A, m, g)
    assert (Ym == 0).all() and gm[0] == 0 and not np.isnan(Ym).any()


# ---------------------------------------------------------------------------
# 4. hand-worked fixture


def _read_golden(name):
    vals = {}
    ln2 = None
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if not line:
                continue
            key, val = [x.strip() for x in line.split("=", 1)]
            if key == "ln2":
                ln2 = float(val)
                continue
            rows = []
            for row in val.split(";"):
                rows.append([{"LN2": ln2, "2LN2": 2 * ln2}.get(tok, None) if tok in ("LN2", "2LN2") else float(tok)
                             for tok in row.split()])
            vals[key] = np.array(rows, dtype=np.float64)
    return vals


def test_hand_worked_example():
    g = _read_golden("thm1_hand_example.txt")
    hw = _manual(g["q"][0], g["k_private"], g["v_private"], g["k_public"], g["v_public"], scale=1.0)
    Y, lse = orc.attention(hw)
    np.testing.assert_allclose(Y[0], g["Y"][0], rtol=2e-7)     # ln2 and 2 ln2 are rounded to fp32 on input (half-ulp 6e-8)
    assert lse[0] == pytest.approx(g["lse"][0, 0], rel=2e-7)
    A_in, m_in, g_in = orc.partial(hw, hw.private)
    A_out, m_out, g_out = orc.partial(hw, hw.public)
    np.testing.assert_allclose(A_in[0], g["A_in"][0], rtol=2e-7)
    np.testing.assert_allclose(A_out[0], g["A_out"][0], rtol=2e-7)
    assert m_in[0] == pytest.approx(g["m_in"][0, 0], rel=1e-7)
    assert g_in[0] == pytest.approx(g["gamma_in"][0, 0], rel=1e-7)
    assert m_out[0] == pytest.approx(g["m_out"][0, 0], rel=1e-7)
    assert g_out[0] == pytest.approx(g["gamma_out"][0, 0], rel=1e-7)
    assert orc.lse_of(m_in, g_in)[0] == pytest.approx(g["lse_in"][0, 0], rel=1e-7)
    Ym, m, gm, w = orc.merge(A_in, m_in, g_in, A_out, m_out, g_out)
    np.testing.assert_allclose(Ym[0], g["Y"][0], rtol=2e-7)
    assert w[0] == pytest.approx(g["w_in"][0, 0], rel=1e-7)
    assert 1.0 - w[0] == pytest.approx(g["w_out"][0, 0], rel=1e-7)


# ---------------------------------------------------------------------------
# 5. Theorem 1 at every split point; proof structure; merge algebra


def test_theorem1_every_split_point():
    U, Hq, Hkv, d = 2, 4, 2, 16
    L = 21
    wl, hw = _case(31, torch.bfloat16, U, Hq, Hkv, d, [L, L], [0, 0])
    only_private = [hw.private]
    Y, lse = orc.attention(hw, views=only_private)
    for s in range(L + 1):
        t = np.full(U, s, dtype=np.int32)
        A0, m0, g0 = orc.partial(hw, hw.private, t1=t)
        A1, m1, g1 = orc.partial(hw, hw.private, t0=t)
        Ym, m, g, w = orc.merge(A0, m0, g0, A1, m1, g1)
        np.testing.assert_allclose(Ym, Y, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(orc.lse_of(m, g), lse, rtol=1e-13)
        # lse = logaddexp of the parts; weights are gamma_x / gamma of the proof
        np.testing.assert_allclose(np.logaddexp(orc.lse_of(m0, g0), orc.lse_of(m1, g1)), lse, rtol=1e-13)
        np.testing.assert_allclose(w, np.exp(orc.lse_of(m0, g0) - lse), rtol=1e-12, atol=1e-300)
        # swapping the parts gives the same Y bit for bit and complementary weights
        Ys, ms, gs, ws = orc.merge(A1, m1, g1, A0, m0, g0)
        np.testing.assert_array_equal(Ys, Ym)
        np.testing.assert_allclose(w + ws, 1.0, rtol=1e-14)
        if s in (0, L):     # merging with an empty part is the identity
            full = A1 if s == 0 else A0
            np.testing.assert_array_equal(Ym, full)


def test_private_public_split_equals_concatenation():
    wl, hw = _case(37, torch.float32, 3, 6, 3, 32, [40, 0, 7], [9, 12, 0], layout="hnd")
    Y, lse = orc.attention(hw)
    A0, m0, g0 = orc.partial(hw, hw.private)
    A1, m1, g1 = orc.partial(hw, hw.public)
    Ym, m, g, w = orc.merge(A0, m0, g0, A1, m1, g1)
    np.testing.assert_allclose(Ym, Y, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(orc.lse_of(m, g), lse, rtol=1e-13)
    assert (w[6:12] == 0).all() and (w[12:] == 1).all()      # user 1 has no private part, user 2 no public part


def test_naive_gammas_of_the_proof_match_stabilised_coefficients():
    """gamma_x = sum exp(s) without any shift (Appendix A) gives the same weights where it is finite."""
    wl, hw = _case(41, torch.float32, 1, 2, 1, 8, [6], [5])
    A0, m0, g0 = orc.partial(hw, hw.private)
    A1, m1, g1 = orc.partial(hw, hw.public)
    _, _, _, w = orc.merge(A0, m0, g0, A1, m1, g1)
    for h in range(2):
        q = wl.q[0, h].double().numpy()
        Kp, _ = _rows_as_float64(wl, wl.private, 0, 0)
        Ko, _ = _rows_as_float64(wl, wl.public, 0, 0)
        gp = np.exp((Kp @ q) * wl.scale).sum()
        go = np.exp((Ko @ q) * wl.scale).sum()
        assert w[h] == pytest.approx(gp / (gp + go), rel=1e-13)
        # and the paper's alpha form written out independently
        alpha = math.exp(m1[h] - m0[h])
        assert w[h] == pytest.approx(g0[h] / (g0[h] + alpha * g1[h]), rel=1e-14)
        assert 1 - w[h] == pytest.approx(g1[h] / (g0[h] / alpha + g1[h]), rel=1e-13)


def test_attention_mass_is_the_softmax_mass_on_the_private_tokens():
    """w_in of the merge is the share of the unsplit softmax that falls on the private tokens (library softmax)."""
    from scipy.special import softmax
    wl, hw = _case(43, torch.float32, 2, 4, 2, 16, [9, 3], [4, 11], layout="hnd")
    A0, m0, g0 = orc.partial(hw, hw.private)
    A1, m1, g1 = orc.partial(hw, hw.public)
    _, _, _, w = orc.merge(A0, m0, g0, A1, m1, g1)
    for u in range(2):
        for h in range(4):
            K, _ = _concat_rows(wl, u, h // 2)
            p = softmax((K @ wl.q[u, h].double().numpy()) * wl.scale)
            assert w[u * 4 + h] == pytest.approx(p[:int(wl.private.lens[u])].sum(), rel=1e-13)


def test_attention_mass_track_closed_forms():
    # row 0: an arithmetic ramp 0.1 .. 1.0; row 1: constant; row 2: alternating 0 and 1
    steps = 10
    w = np.stack([np.linspace(0.1, 1.0, steps), np.full(steps, 0.25), np.arange(steps) % 2.0], axis=1)
    mn, sm, below = orc.attention_mass_track(w, 0.35)
    np.testing.assert_allclose(mn, [0.1, 0.25, 0.0], rtol=0, atol=0)
    np.testing.assert_allclose(sm, [steps * (0.1 + 1.0) / 2, 0.25 * steps, steps // 2], rtol=1e-14)
    assert below.tolist() == [3, steps, steps // 2]           # 0.1, 0.2, 0.3 | all | the zeros
    # strictly below: a mass equal to the threshold does not count; nothing to fold gives the neutral element
    assert orc.attention_mass_track(np.array([[0.5]]), 0.5)[2].tolist() == [0]
    mn0, sm0, b0 = orc.attention_mass_track(np.zeros((0, 2)), 0.5)
    assert mn0.tolist() == [1, 1] and sm0.tolist() == [0, 0] and b0.tolist() == [0, 0]
    # folding a sequence in two halves, carrying the state by hand, is folding it at once
    rng = np.random.default_rng(5)
    w = rng.random((7, 4))
    a = orc.attention_mass_track(w[:3], 0.4)
    b = orc.attention_mass_track(w[3:], 0.4)
    full = orc.attention_mass_track(w, 0.4)
    np.testing.assert_array_equal(np.minimum(a[0], b[0]), full[0])
    np.testing.assert_allclose(a[1] + b[1], full[1], rtol=1e-15)
    np.testing.assert_array_equal(a[2] + b[2], full[2])
    np.testing.assert_array_equal(full[0], w.min(axis=0))
    np.testing.assert_array_equal(full[2], (w < 0.4).sum(axis=0))


def test_merge_extreme_score_gap_stays_finite():
    """m_out - m_in far beyond the fp32 exp range (config 3 style outliers): weights saturate, no NaN."""
    d = 4
    A0 = np.full((1, d), 2.0); A1 = np.full((1, d), -3.0)
    Y, m, g, w = orc.merge(A0, [-900.0], [1.5], A1, [850.0], [2.0])
    assert w[0] == 0.0 and np.array_equal(Y, A1) and m[0] == 850.0 and g[0] == 2.0
    Y, m, g, w = orc.merge(A0, [900.0], [1.5], A1, [-850.0], [2.0])
    assert w[0] == 1.0 and np.array_equal(Y, A0)


def test_three_way_merge_any_bracketing():
    wl, hw = _case(43, torch.bfloat16, 2, 4, 1, 16, [30, 30], [0, 0])
    Y, lse = orc.attention(hw, views=[hw.private])
    cuts = [(0, 7), (7, 19), (19, 30)]
    parts = [orc.partial(hw, hw.private, t0=np.full(2, a, np.int32), t1=np.full(2, b, np.int32)) for a, b in cuts]
    def mg(x, y):
        Ym, m, g, _ = orc.merge(x[0], x[1], x[2], y[0], y[1], y[2])
        return (Ym, m, g)
    for order in [(0, 1, 2), (2, 0, 1), (1, 2, 0)]:
        a, b, c = [parts[i] for i in order]
        left = mg(mg(a, b), c)
        right = mg(a, mg(b, c))
        np.testing.assert_allclose(left[0], Y, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(right[0], Y, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(orc.lse_of(left[1], left[2]), lse, rtol=1e-13)


# ---------------------------------------------------------------------------
# 6. structure: GQA grouping, paging, batching, token order


def test_n_way_merge_of_any_partition_equals_unsplit_attention():
    """A row cut at random points into 1..7 ranges (some empty): the n-way merge of the ranges' partials equals the
    unsplit attention (Theorem 1 applied repeatedly), and equals folding the two-way merge from the left."""
    rng = np.random.default_rng(5)
    wl, hw = _case(71, torch.float32, 3, 4, 2, 16, [57, 0, 120], [0, 0, 0])
    Y, lse = orc.attention(hw)
    for n in (1, 2, 3, 5, 7):
        cuts = np.sort(rng.integers(0, np.maximum(hw.private.lens, 1)[None, :] + 1, size=(n - 1, hw.U)), axis=0)
        cuts = np.minimum(cuts, hw.private.lens[None, :])
        edges = np.concatenate([np.zeros((1, hw.U), dtype=np.int64), cuts, hw.private.lens[None, :].astype(np.int64)])
        raw = [orc.partial(hw, hw.private, edges[i], edges[i + 1]) for i in range(n)]
        parts = [(A, orc.lse_of(m, g)) for A, m, g in raw]
        Yn, lse_n, W = orc.merge_n(parts)
        np.testing.assert_allclose(Yn, Y, rtol=1e-12, atol=1e-13)
        both_empty = np.isinf(lse)
        np.testing.assert_allclose(lse_n[~both_empty], lse[~both_empty], rtol=1e-13)
        assert (lse_n[both_empty] == -np.inf).all() and (Yn[both_empty] == 0).all()
        np.testing.assert_allclose(W.sum(axis=0)[~both_empty], 1.0, rtol=1e-14)
        # fold of the two-way form
        A, m, g = raw[0]
        for A2, m2, g2 in raw[1:]:
            A, m, g, _ = orc.merge(A, m, g, A2, m2, g2)
        np.testing.assert_allclose(Yn, A, rtol=1e-12, atol=1e-13)
        # the order of the parts does not matter
        perm = rng.permutation(n)
        Yp, lse_p, Wp = orc.merge_n([parts[i] for i in perm])
        np.testing.assert_allclose(Yp, Yn, rtol=1e-13, atol=1e-14)
        np.testing.assert_allclose(Wp, W[perm], rtol=1e-13)


def test_n_way_merge_weights_are_shares_of_the_denominator():
    """Hand numbers: lse = ln 1, ln 2, ln 5, -inf: weights 1/8, 2/8, 5/8, 0 and lse = ln 8; a huge gap stays finite."""
    A = [np.full((1, 2), v) for v in (8.0, 16.0, -8.0, 123.0)]
    L = [np.array([np.log(1.0)]), np.array([np.log(2.0)]), np.array([np.log(5.0)]), np.array([-np.inf])]
    Y, lse, W = orc.merge_n(list(zip(A, L)))
    np.testing.assert_allclose(W[:, 0], [0.125, 0.25, 0.625, 0.0], rtol=1e-15)
    np.testing.assert_allclose(Y[0], [1.0 + 4.0 - 5.0] * 2, rtol=1e-15, atol=1e-15)
    assert lse[0] == pytest.approx(np.log(8.0), rel=1e-15)
    Y, lse, W = orc.merge_n([(A[0], np.array([900.0])), (A[1], np.array([-900.0]))])
    assert lse[0] == 900.0 and W[0, 0] == 1.0 and W[1, 0] == 0.0 and (Y[0] == 8.0).all()


def test_gqa_equals_mha_on_replicated_kv_heads():
    U, Hq, Hkv, d = 2, 8, 2, 16
    wl, hw = _case(51, torch.bfloat16, U, Hq, Hkv, d, [19, 5], [4, 0], layout="nhd")
    Y, lse = orc.attention(hw)
    G = Hq // Hkv
    def rep(side):
        ks = [workloads.host_array(t.repeat_interleave(G, dim=1)) for t in side.k]
        vs = [workloads.host_array(t.repeat_interleave(G, dim=1)) for t in side.v]
        return orc.HostView(side.lens, Hq * d, d, k=ks, v=vs)
    hw2 = orc.HostWorkload(orc.BF16, Hq, Hq, d, wl.scale, workloads.host_array(wl.q), rep(wl.private), rep(wl.public))
    Y2, lse2 = orc.attention(hw2)
    np.testing.assert_array_equal(Y, Y2)
    np.testing.assert_array_equal(lse, lse2)


def test_paged_equals_contiguous_and_layouts_agree():
    U, Hq, Hkv, d = 3, 4, 2, 32
    lp, lo = [50, 16, 1], [0, 33, 15]
    wl, hw = _case(53, torch.bfloat16, U, Hq, Hkv, d, lp, lo, paged=True)
    Y, lse = orc.attention(hw)
    # rebuild the same tokens as contiguous nhd and hnd buffers through torch indexing
    for layout in ("nhd", "hnd"):
        sides = []
        for side in (wl.private, wl.public):
            ks, vs = [], []
            cap = 64
            for u in range(U):
                L = int(side.lens[u])
                n = -(-L // side.page_tokens)
                pg = side.block_table[u, :n].long()
                k = side.k_pool[pg].permute(1, 0, 2, 3).reshape(Hkv, -1, d)[:, :L]   # [Hkv, L, d]
                v = side.v_pool[pg].permute(1, 0, 2, 3).reshape(Hkv, -1, d)[:, :L]
                if layout == "nhd":
                    ks.append(workloads.host_array(k.permute(1, 0, 2)))
                    vs.append(workloads.host_array(v.permute(1, 0, 2)))
                else:
                    kb = torch.zeros(Hkv, cap, d, dtype=k.dtype); kb[:, :L] = k
                    vb = torch.zeros(Hkv, cap, d, dtype=k.dtype); vb[:, :L] = v
                    ks.append(workloads.host_array(kb)); vs.append(workloads.host_array(vb))
            ts, hs = (Hkv * d, d) if layout == "nhd" else (d, cap * d)
            sides.append(orc.HostView(side.lens, ts, hs, k=ks, v=vs))
        hw2 = orc.HostWorkload(orc.BF16, Hq, Hkv, d, wl.scale, workloads.host_array(wl.q), *sides)
        Y2, lse2 = orc.attention(hw2)
        np.testing.assert_array_equal(Y, Y2)
        np.testing.assert_array_equal(lse, lse2)


@pytest.mark.parametrize("page_tokens", [32, 64, 256])
@pytest.mark.parametrize("token_major", [False, True])
def test_larger_pages_hold_the_same_attention(page_tokens, token_major):
    """The oracle on pages of 32, 64 and 256 tokens against the library softmax on rows gathered with torch indexing."""
    from scipy.special import softmax
    U, Hq, Hkv, d = 3, 4, 2, 16
    wl, hw = _case(73, torch.float32, U, Hq, Hkv, d, [300, 1, 64], [65, 0, 257],
                   paged="token_major" if token_major else True, page_tokens=page_tokens)
    assert hw.private.block_size == page_tokens
    Y, _ = orc.attention(hw)
    for u in range(U):
        for h in range(Hq):
            K, V = _concat_rows(wl, u, h // (Hq // Hkv))
            if K.shape[0] == 0:
                continue
            s = (K @ wl.q[u, h].double().numpy()) * wl.scale
            np.testing.assert_allclose(Y[u * Hq + h], softmax(s) @ V, rtol=1e-11, atol=1e-12)


def test_users_are_independent_and_rows_subset():
    U, Hq, Hkv, d = 4, 4, 2, 16
    wl, hw = _case(57, torch.float32, U, Hq, Hkv, d, [9, 30, 2, 14], [5, 0, 8, 1])
    Y, lse = orc.attention(hw)
    rows = [(3, 1), (0, 2), (2, 3)]
    Ys, ls = orc.attention(hw, rows=rows)
    for i, (u, h) in enumerate(rows):
        np.testing.assert_array_equal(Ys[i], Y[u * Hq + h])
        assert ls[i] == lse[u * Hq + h]
    for u in range(U):       # single-user call on that user's buffers
        one = lambda s: orc.HostView(s.lens[u:u + 1], s.token_stride, s.head_stride, k=[s.k[u]], v=[s.v[u]])
        hw1 = orc.HostWorkload(hw.dtype, Hq, Hkv, d, hw.scale, hw.q[u:u + 1], one(hw.private), one(hw.public))
        Y1, l1 = orc.attention(hw1)
        np.testing.assert_array_equal(Y1, Y[u * Hq:(u + 1) * Hq])


def test_token_permutation_invariance():
    U, Hq, Hkv, d = 1, 2, 1, 16
    wl, hw = _case(59, torch.float32, U, Hq, Hkv, d, [25], [6])
    Y, lse = orc.attention(hw)
    perm = np.random.default_rng(5).permutation(25)
    kp = hw.private.k[0][perm].copy(); vp = hw.private.v[0][perm].copy()
    pv = orc.HostView(hw.private.lens, Hkv * d, d, k=[kp], v=[vp])
    hw2 = orc.HostWorkload(hw.dtype, Hq, Hkv, d, hw.scale, hw.q, pv, hw.public)
    Y2, lse2 = orc.attention(hw2)
    np.testing.assert_allclose(Y2, Y, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(lse2, lse, rtol=1e-14)


def test_bf16_is_widened_exactly():
    """K = one-hot rows, q = bf16 values: the score must be exactly that bf16 value times scale."""
    d = 8
    vals = torch.tensor([1.0, -0.0078125, 3.140625, 1e-3, -65280.0, 2.0 ** -100, 0.33203125, 7.0]).to(torch.bfloat16)
    K = torch.eye(d).to(torch.bfloat16)
    V = torch.eye(d).to(torch.bfloat16)
    hw = _manual(vals.double().numpy(), K.double().numpy(), V.double().numpy(), np.zeros((0, d)), np.zeros((0, d)),
                 scale=2.0 ** -10, dtype=torch.bfloat16)
    A, m, g = orc.partial(hw, hw.private)
    s = vals.double().numpy() * 2.0 ** -10
    assert m[0] == s.max()
    w = np.exp(s - s.max())
    np.testing.assert_allclose(A[0], w / w.sum(), rtol=1e-14)
    assert g[0] == pytest.approx(w.sum(), rel=1e-15)


def test_fp16_decoding_of_every_bit_pattern():
    """The oracle's binary16 decoder against numpy's float16 on all 65536 patterns (zeros, subnormals, inf, NaN)."""
    import ctypes as C
    lib = orc._load()
    lib.orc_half_to_double.restype = C.c_double
    lib.orc_half_to_double.argtypes = [C.c_uint16]
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([lib.orc_half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert (np.isnan(got) == nan).all()
    assert (got[~nan] == want[~nan]).all()
    assert (np.signbit(got[~nan]) == np.signbit(want[~nan])).all()          # -0.0 keeps its sign


def test_fp16_inputs_against_library_softmax():
    """fp16 q, K, V (values torch rounded; widened by torch, not by the oracle) against scipy's softmax."""
    from scipy.special import logsumexp, softmax
    U, Hq, Hkv, d = 3, 4, 2, 16
    wl, hw = _case(67, torch.float16, U, Hq, Hkv, d, [33, 1, 100], [16, 0, 31], layout="nhd", paged=True)
    assert hw.dtype == orc.F16
    Y, lse = orc.attention(hw)
    for u in range(U):
        for h in range(Hq):
            K, V = _concat_rows(wl, u, h // (Hq // Hkv))
            s = (K @ wl.q[u, h].double().numpy()) * wl.scale
            np.testing.assert_allclose(Y[u * Hq + h], softmax(s) @ V, rtol=1e-11, atol=1e-12)
            assert lse[u * Hq + h] == pytest.approx(logsumexp(s), rel=1e-12)


def test_scale_is_applied_to_scores_not_outputs():
    wl, hw = _case(61, torch.float32, 1, 1, 1, 8, [5], [3], scale=0.0)
    Y, lse = orc.attention(hw)       # scale 0: uniform weights
    K, V = _concat_rows(wl, 0, 0)
    np.testing.assert_allclose(Y[0], V.mean(0), rtol=1e-14)
    assert lse[0] == pytest.approx(math.log(8), rel=1e-14)


def test_workload_configs_are_seeded_and_shaped():
    a = workloads.make_workload(2, len_div=64)
    b = workloads.make_workload(2, len_div=64)
    assert torch.equal(a.q, b.q) and all(torch.equal(x, y) for x, y in zip(a.private.k, b.private.k))
    assert a.n_q_heads == 32 and a.n_kv_heads == 8 and a.head_dim == 128 and a.dtype == torch.bfloat16
    lp, lo = workloads.draw_lengths(2, 16)
    assert lp.min() >= 512 and lp.max() <= 4096 and lo.min() >= 1 and lo.max() <= 512
    lp, lo = workloads.draw_lengths(3, 64)
    assert lp.min() >= 8192 and lp.max() <= 32768 and lo.min() >= 0 and lo.max() <= 1024
    lp, lo = workloads.draw_lengths(4, 256)
    assert lp.min() >= 16 and lp.max() <= 32768 and 700 < np.median(lp) < 1500 and lo.max() <= 2048
    lp, lo = workloads.draw_lengths(5, 32)
    assert lp.min() >= 32768 and lp.max() <= 131072 and lo.min() >= 1 and lo.max() <= 4096
    # the overrides the benchmark offers: another length law, a floor under the public lengths (buffers and block
    # tables are then made for the raised lengths, which is what lets a decode loop grow a cache up to them)
    lp, lo = workloads.draw_lengths(2, 200, len_ranges=(64, 512, 0, 256))
    assert lp.min() >= 64 and lp.max() <= 512 and lo.min() >= 0 and lo.max() <= 256 and lo.min() < 32
    lp2, lo2 = workloads.draw_lengths(2, 200, len_ranges=(64, 512, 0, 256), min_public_len=32)
    assert np.array_equal(lp, lp2) and np.array_equal(lo2, np.maximum(lo, 32))
    w4 = workloads.make_workload(4, n_users=12, len_div=4, min_public_len=32)
    assert w4.name.endswith("-variant") and int(w4.public.lens.min()) >= 32
    assert all(k.shape[1] == L for k, L in zip(w4.public.k, w4.public.lens))      # exactly sized per-user buffers
    w3 = workloads.make_workload(3, len_div=256, n_users=4)
    assert len(w3.outlier_channels) == 21
    kv, ch = divmod(int(w3.outlier_channels[0]), 128)
    k = w3.private.k[0].float()
    assert k[kv, :, ch].abs().mean() > 5 * k.abs().mean()
    w5 = workloads.make_workload(5, len_div=1024, n_users=3)
    assert w5.private.paged and w5.private.block_table.dtype == torch.int32
    used = torch.cat([w5.private.block_table[u, :-(-int(L) // 16)] for u, L in enumerate(w5.private.lens)])
    assert used.unique().numel() == used.numel()          # no page shared between users
