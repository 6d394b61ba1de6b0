"""Randomised pins of the oracle (hypothesis): library softmax on arbitrary small shapes, layouts and splits."""
import numpy as np
import torch
from hypothesis import given, settings, strategies as st
from scipy.special import logsumexp, softmax

import workloads
from oracle import spd_oracle as orc


@st.composite
def cases(draw):
    U = draw(st.integers(1, 3))
    Hkv = draw(st.sampled_from([1, 2, 3]))
    G = draw(st.sampled_from([1, 2, 4]))
    d = draw(st.sampled_from([4, 8, 16]))
    lp = [draw(st.integers(0, 40)) for _ in range(U)]
    lo = [draw(st.integers(0, 20)) for _ in range(U)]
    layout = draw(st.sampled_from(["nhd", "hnd", "hnd_exact", "paged", "paged_tm"]))
    dtype = draw(st.sampled_from([torch.float32, torch.bfloat16]))
    seed = draw(st.integers(0, 10_000))
    scale = draw(st.sampled_from([1.0, 0.25, 2.0]))
    return U, Hkv, G, d, lp, lo, layout, dtype, seed, scale


def _rows(wl, side, u, kv):
    L = int(side.lens[u])
    if side.paged:
        n = -(-L // side.page_tokens)
        pg = side.block_table[u, :n].long()
        if side.page_token_major:
            k = side.k_pool[pg][:, :, kv].reshape(-1, wl.head_dim)[:L]
            v = side.v_pool[pg][:, :, kv].reshape(-1, wl.head_dim)[:L]
        else:
            k = side.k_pool[pg, kv].reshape(-1, wl.head_dim)[:L]
            v = side.v_pool[pg, kv].reshape(-1, wl.head_dim)[:L]
    elif side.layout == "nhd":
        k, v = side.k[u][:L, kv], side.v[u][:L, kv]
    else:
        k, v = side.k[u][kv, :L], side.v[u][kv, :L]
    return k.double().numpy(), v.double().numpy()


@settings(max_examples=60, deadline=None)
@given(cases())
def test_oracle_matches_library_softmax_and_theorem1(case):
    U, Hkv, G, d, lp, lo, layout, dtype, seed, scale = case
    Hq = Hkv * G
    paged = {"paged": True, "paged_tm": "token_major"}.get(layout, False)
    wl = workloads.random_case(seed, dtype, U, Hq, Hkv, d, lp, lo, layout="nhd" if paged else layout,
                               paged=paged, scale=scale)
    hw = orc.from_workload(wl)
    Y, lse = orc.attention(hw)
    A0, m0, g0 = orc.partial(hw, hw.private)
    A1, m1, g1 = orc.partial(hw, hw.public)
    Ym, mm, gm, w = orc.merge(A0, m0, g0, A1, m1, g1)
    np.testing.assert_allclose(Ym, Y, rtol=1e-11, atol=1e-13)           # Theorem 1
    for u in range(U):
        for h in range(Hq):
            kp, vp = _rows(wl, wl.private, u, h // G)
            ko, vo = _rows(wl, wl.public, u, h // G)
            K, V = np.concatenate([kp, ko]), np.concatenate([vp, vo])
            r = u * Hq + h
            if K.shape[0] == 0:
                assert (Y[r] == 0).all() and lse[r] == -np.inf
                continue
            s = (K @ wl.q[u, h].double().numpy()) * scale
            np.testing.assert_allclose(Y[r], softmax(s) @ V, rtol=1e-10, atol=1e-12)
            assert abs(lse[r] - logsumexp(s)) <= 1e-11 * max(1.0, abs(lse[r]))
            if kp.shape[0]:
                sp = (kp @ wl.q[u, h].double().numpy()) * scale
                np.testing.assert_allclose(A0[r], softmax(sp) @ vp, rtol=1e-10, atol=1e-12)
                assert abs(orc.lse_of(m0, g0)[r] - logsumexp(sp)) <= 1e-11 * max(1.0, abs(logsumexp(sp)))
