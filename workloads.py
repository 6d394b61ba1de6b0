"""Seeded synthetic inputs for the SPD decode-attention path.

This module only *draws* inputs: query vectors, the two owners' KV caches
(private prompt cache, public output-token cache), their lengths, and, for
the paged workload, the block tables.  It holds none of the method's
arithmetic, so both the CPU oracle's tests and the HIP path's tests can use
it without sharing any computation.

The five workloads follow the benchmark configurations of this repository
(shapes of Llama-3-8B / Llama-3-70B attention, one layer, one decode step):

  1  fp32, 1 user, Hq=Hkv=8, d=64, private 128 tokens, public 16 tokens
  2  bf16, 16 users, Hq=32/Hkv=8, d=128, private U[512,4096], public U[1,512]
  3  bf16, 64 users, same heads, private U[8192,32768], public U[0,1024],
     21 of the 1024 (kv_head, channel) pairs of K scaled by 20
  4  bf16, 256 users, same heads, private lognormal(median 1024, sigma 1)
     clipped to [16,32768], public U[0,2048], separately allocated, exactly
     sized head-major buffers [Hkv][len][d] (a different head stride per user)
  5  bf16, 32 users, Hq=64/Hkv=8, d=128, private U[32768,131072],
     public U[1,4096], 16-token pages with a shuffled block table

All values are N(0,1) rounded to the workload dtype.  Seeds are
1000*config + k with k naming the tensor family (see SEED_FAMILIES).
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional

import numpy as np
import torch

SEED_FAMILIES = {
    "len_private": 0, "len_public": 1, "q": 2,
    "k_private": 3, "v_private": 4, "k_public": 5, "v_public": 6,
    "outlier_channels": 7, "table_private": 8, "table_public": 9,
}

PAGE_TOKENS = 16


def seed_of(cfg: int, family: str) -> int:
    return 1000 * cfg + SEED_FAMILIES[family]


@dataclasses.dataclass
class KVSide:
    """One owner's KV cache for all users.

    Contiguous mode: ``k[u]``/``v[u]`` are separately allocated tensors, one
    pair per user, shaped [Hkv, cap, d] ("hnd"), [Hkv, L, d] ("hnd_exact", per-user
    ``head_strides``) or [L, Hkv, d] ("nhd");
    ``token_stride``/``head_stride`` are in elements and the channel axis is
    unit stride.  Paged mode: ``k_pool``/``v_pool`` are
    [n_blocks, Hkv, PAGE_TOKENS, d] (or [n_blocks, PAGE_TOKENS, Hkv, d] with
    ``page_token_major``) and ``block_table`` is int32
    [U, max_blocks]; entries past a user's last page are 0 (a valid page that
    is never read).
    """
    lens: np.ndarray
    paged: bool
    token_stride: int
    head_stride: int
    k: Optional[List[torch.Tensor]] = None
    v: Optional[List[torch.Tensor]] = None
    k_pool: Optional[torch.Tensor] = None
    v_pool: Optional[torch.Tensor] = None
    block_table: Optional[torch.Tensor] = None
    block_stride: int = 0
    max_blocks: int = 0
    head_strides: Optional[np.ndarray] = None   # per-user head stride (layout "hnd_exact"), else None
    page_token_major: bool = False              # paged pools are [block, token, head, d] instead of [block, head, token, d]
    page_tokens: int = PAGE_TOKENS              # tokens per page (paged mode)
    layout: str = "nhd"      # contiguous mode: "nhd" or "hnd"; paged pools are [block, head, token, d]

    @property
    def n_tokens(self) -> int:
        return int(self.lens.sum())


@dataclasses.dataclass
class Workload:
    cfg: int
    name: str
    dtype: torch.dtype
    n_users: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    scale: float
    q: torch.Tensor            # [U, Hq, d]
    private: KVSide
    public: KVSide
    seeds: dict
    outlier_channels: Optional[np.ndarray] = None   # flat (kv_head*d + channel) indices

    @property
    def kv_bytes(self) -> int:
        """Bytes of K and V that one decode step must read (both owners)."""
        elt = 4 if self.dtype == torch.float32 else 2
        per_token = 2 * self.n_kv_heads * self.head_dim * elt
        return (self.private.n_tokens + self.public.n_tokens) * per_token


_SHAPES = {
    1: dict(name="fp32-tiny", dtype=torch.float32, U=1, Hq=8, Hkv=8, d=64),
    2: dict(name="llama3-8b-16users", dtype=torch.bfloat16, U=16, Hq=32, Hkv=8, d=128),
    3: dict(name="llama3-8b-64users-long-outliers", dtype=torch.bfloat16, U=64, Hq=32, Hkv=8, d=128),
    4: dict(name="llama3-8b-256users-skewed", dtype=torch.bfloat16, U=256, Hq=32, Hkv=8, d=128),
    5: dict(name="llama3-70b-32users-paged", dtype=torch.bfloat16, U=32, Hq=64, Hkv=8, d=128),
}


def draw_lengths(cfg: int, n_users: int, len_div: int = 1, len_ranges=None, min_public_len: int = 0):
    """Private and public token counts per user (int32), both ends inclusive.  len_ranges = (private low, private
    high, public low, public high) replaces the configuration's length law by uniform draws (same seeds);
    min_public_len raises every public length to at least that many tokens."""
    rp = np.random.default_rng(seed_of(cfg, "len_private"))
    ro = np.random.default_rng(seed_of(cfg, "len_public"))
    if len_ranges is not None:
        plo, phi, olo, ohi = (int(x) for x in len_ranges)
        assert 0 <= plo <= phi and 0 <= olo <= ohi
        lp = rp.integers(plo, phi, size=n_users, endpoint=True)
        lo = ro.integers(olo, ohi, size=n_users, endpoint=True)
    elif cfg == 1:
        lp = np.full(n_users, 128)
        lo = np.full(n_users, 16)
    elif cfg == 2:
        lp = rp.integers(512, 4096, size=n_users, endpoint=True)
        lo = ro.integers(1, 512, size=n_users, endpoint=True)
    elif cfg == 3:
        lp = rp.integers(8192, 32768, size=n_users, endpoint=True)
        lo = ro.integers(0, 1024, size=n_users, endpoint=True)
    elif cfg == 4:
        lp = np.exp(rp.normal(math.log(1024.0), 1.0, size=n_users))
        lp = np.clip(np.rint(lp), 16, 32768).astype(np.int64)
        lo = ro.integers(0, 2048, size=n_users, endpoint=True)
    elif cfg == 5:
        lp = rp.integers(32768, 131072, size=n_users, endpoint=True)
        lo = ro.integers(1, 4096, size=n_users, endpoint=True)
    else:
        raise ValueError(f"unknown config {cfg}")
    if len_div > 1:
        # shrink for CPU-sized tests; a length that was >= 1 stays >= 1, zeros stay zero
        lp = np.where(lp > 0, np.maximum(1, lp // len_div), 0)
        lo = np.where(lo > 0, np.maximum(1, lo // len_div), 0)
    lo = np.maximum(lo, min_public_len)
    return lp.astype(np.int32), lo.astype(np.int32)


def _randn(shape, gen, device, dtype):
    if int(np.prod(shape)) == 0:
        return torch.empty(shape, device=device, dtype=dtype)
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32).to(dtype)


def _make_contig(lens, Hkv, d, dtype, device, seed_k, seed_v, layout, ch_scale):
    """Per-user buffers.  'nhd': [L, Hkv, d] (token_stride = Hkv*d, head_stride = d).
    'hnd': [Hkv, cap, d] with a common capacity cap = max(lens) rounded up to 64
    tokens (token_stride = d, head_stride = cap*d), so one stride pair serves all users.
    'hnd_exact': [Hkv, L, d] exactly sized per user (token_stride = d, per-user head stride L*d)."""
    gk = torch.Generator(device=device).manual_seed(seed_k)
    gv = torch.Generator(device=device).manual_seed(seed_v)
    ks, vs = [], []
    if layout == "nhd":
        token_stride, head_stride = Hkv * d, d
    elif layout == "hnd":
        cap = max(64, int(-(-int(lens.max(initial=0)) // 64) * 64))
        token_stride, head_stride = d, cap * d
    elif layout == "hnd_exact":
        token_stride, head_stride = d, 0
    else:
        raise ValueError(layout)
    for L in lens.tolist():
        if layout == "nhd":
            k = _randn((L, Hkv, d), gk, device, dtype)
            v = _randn((L, Hkv, d), gv, device, dtype)
            if ch_scale is not None and L > 0:
                k = (k.float() * ch_scale.view(1, Hkv, d)).to(dtype)
        elif layout == "hnd_exact":
            k = _randn((Hkv, L, d), gk, device, dtype)
            v = _randn((Hkv, L, d), gv, device, dtype)
            if ch_scale is not None and L > 0:
                k = (k.float() * ch_scale.view(Hkv, 1, d)).to(dtype)
        else:
            k = torch.zeros((Hkv, cap, d), device=device, dtype=dtype)
            v = torch.zeros((Hkv, cap, d), device=device, dtype=dtype)
            if L > 0:
                kk = _randn((Hkv, L, d), gk, device, dtype)
                if ch_scale is not None:
                    kk = (kk.float() * ch_scale.view(Hkv, 1, d)).to(dtype)
                k[:, :L] = kk
                v[:, :L] = _randn((Hkv, L, d), gv, device, dtype)
        ks.append(k)
        vs.append(v)
    hs = (lens.astype(np.int64) * d) if layout == "hnd_exact" else None
    return KVSide(lens=lens, paged=False, token_stride=token_stride, head_stride=head_stride, k=ks, v=vs,
                  layout=layout, head_strides=hs)


def _make_paged(lens, Hkv, d, dtype, device, seed_k, seed_v, seed_t, ch_scale, spare_blocks=3, token_major=False,
                page_tokens=PAGE_TOKENS):
    """One pool per tensor; each user's pages are drawn from a seeded shuffle of the pool.  Pages are
    [Hkv, page_tokens, d] (head-major) or, with token_major, [page_tokens, Hkv, d]."""
    gk = torch.Generator(device=device).manual_seed(seed_k)
    gv = torch.Generator(device=device).manual_seed(seed_v)
    n_pages = [-(-int(L) // page_tokens) for L in lens.tolist()]
    n_blocks = sum(n_pages) + spare_blocks
    max_blocks = max(1, max(n_pages, default=0))
    perm = np.random.default_rng(seed_t).permutation(n_blocks).astype(np.int32)
    table = np.zeros((len(lens), max_blocks), dtype=np.int32)
    at = 0
    for u, n in enumerate(n_pages):
        table[u, :n] = perm[at:at + n]
        at += n
    shape = (n_blocks, page_tokens, Hkv, d) if token_major else (n_blocks, Hkv, page_tokens, d)
    k_pool = torch.empty(shape, device=device, dtype=dtype)
    v_pool = torch.empty(shape, device=device, dtype=dtype)
    step = 4096  # pages per draw, bounds the fp32 staging buffer
    for b0 in range(0, n_blocks, step):
        b1 = min(n_blocks, b0 + step)
        kk = _randn((b1 - b0,) + shape[1:], gk, device, dtype)
        if ch_scale is not None:
            cs = ch_scale.view(1, 1, Hkv, d) if token_major else ch_scale.view(1, Hkv, 1, d)
            kk = (kk.float() * cs).to(dtype)
        k_pool[b0:b1] = kk
        v_pool[b0:b1] = _randn((b1 - b0,) + shape[1:], gv, device, dtype)
    return KVSide(lens=lens, paged=True, token_stride=Hkv * d if token_major else d,
                  head_stride=d if token_major else page_tokens * d,
                  k_pool=k_pool, v_pool=v_pool,
                  block_table=torch.from_numpy(table).to(device),
                  block_stride=Hkv * page_tokens * d, max_blocks=max_blocks, page_token_major=token_major,
                  page_tokens=page_tokens)


def make_workload(cfg: int, device="cpu", len_div: int = 1, n_users: Optional[int] = None,
                  layout: Optional[str] = None, shape=None, dtype=None, page_tokens: int = PAGE_TOKENS,
                  len_ranges=None, min_public_len: int = 0) -> Workload:
    """Draw workload ``cfg`` on ``device``.

    ``len_div`` divides every drawn length (for CPU-sized parity cases);
    ``n_users`` overrides the user count; ``layout`` overrides the contiguous
    layout ("hnd" for configs 1-3, "hnd_exact" for config 4 by default; config 5 is paged).
    ``shape`` = (Hq, Hkv, d) and ``dtype`` replace the configuration's own (same users, lengths and seeds): for
    measurements on other model shapes, not part of the five configurations.  ``len_ranges`` likewise replaces the
    length law and ``min_public_len`` bounds the public lengths from below (see draw_lengths).
    """
    sh = _SHAPES[cfg]
    U = sh["U"] if n_users is None else n_users
    Hq, Hkv, d = shape if shape is not None else (sh["Hq"], sh["Hkv"], sh["d"])
    plain = shape is None and dtype is None and n_users is None and page_tokens == PAGE_TOKENS and len_ranges is None \
        and min_public_len == 0
    name = sh["name"] if plain else f'{sh["name"]}-variant'
    dtype = sh["dtype"] if dtype is None else dtype
    lp, lo = draw_lengths(cfg, U, len_div, len_ranges, min_public_len)
    seeds = {fam: seed_of(cfg, fam) for fam in SEED_FAMILIES}

    gq = torch.Generator(device=device).manual_seed(seeds["q"])
    q = _randn((U, Hq, d), gq, device, dtype)

    ch_scale, outliers = None, None
    if cfg == 3:
        n_out = math.ceil(0.02 * Hkv * d)   # 21 of 1024 (kv_head, channel) pairs
        outliers = np.sort(np.random.default_rng(seeds["outlier_channels"])
                           .permutation(Hkv * d)[:n_out])
        cs = np.ones(Hkv * d, dtype=np.float32)
        cs[outliers] = 20.0
        ch_scale = torch.from_numpy(cs).to(device).view(Hkv, d)

    if cfg == 5:
        tm = layout == "nhd"      # token-major pages [block, token, head, d]
        priv = _make_paged(lp, Hkv, d, dtype, device, seeds["k_private"], seeds["v_private"],
                           seeds["table_private"], ch_scale, token_major=tm, page_tokens=page_tokens)
        pub = _make_paged(lo, Hkv, d, dtype, device, seeds["k_public"], seeds["v_public"],
                          seeds["table_public"], ch_scale, token_major=tm, page_tokens=page_tokens)
    else:
        lay = layout or ("hnd_exact" if cfg == 4 else "hnd")
        priv = _make_contig(lp, Hkv, d, dtype, device, seeds["k_private"], seeds["v_private"], lay, ch_scale)
        pub = _make_contig(lo, Hkv, d, dtype, device, seeds["k_public"], seeds["v_public"], lay, ch_scale)

    return Workload(cfg=cfg, name=name, dtype=dtype, n_users=U, n_q_heads=Hq,
                    n_kv_heads=Hkv, head_dim=d, scale=1.0 / math.sqrt(d), q=q,
                    private=priv, public=pub, seeds=seeds, outlier_channels=outliers)


def random_case(seed: int, dtype, U: int, Hq: int, Hkv: int, d: int, lens_private, lens_public,
                device="cpu", layout: str = "nhd", paged=False, scale: Optional[float] = None,
                page_tokens: int = PAGE_TOKENS) -> Workload:
    """A free-form seeded case for edge-case tests (explicit shapes and lengths).  paged: False, True
    (head-major pages) or "token_major"; page_tokens: tokens per page."""
    lp = np.asarray(lens_private, dtype=np.int32)
    lo = np.asarray(lens_public, dtype=np.int32)
    assert lp.shape == (U,) and lo.shape == (U,)
    gq = torch.Generator(device=device).manual_seed(seed)
    q = _randn((U, Hq, d), gq, device, dtype)
    if paged:
        tm = paged == "token_major"
        priv = _make_paged(lp, Hkv, d, dtype, device, seed + 1, seed + 2, seed + 5, None, token_major=tm,
                           page_tokens=page_tokens)
        pub = _make_paged(lo, Hkv, d, dtype, device, seed + 3, seed + 4, seed + 6, None, token_major=tm,
                          page_tokens=page_tokens)
    else:
        priv = _make_contig(lp, Hkv, d, dtype, device, seed + 1, seed + 2, layout, None)
        pub = _make_contig(lo, Hkv, d, dtype, device, seed + 3, seed + 4, layout, None)
    return Workload(cfg=0, name=f"case-{seed}", dtype=dtype, n_users=U, n_q_heads=Hq, n_kv_heads=Hkv,
                    head_dim=d, scale=(1.0 / math.sqrt(d)) if scale is None else scale, q=q,
                    private=priv, public=pub, seeds={"base": seed})


# ---------------------------------------------------------------------------
# host copies (raw bits) for CPU consumers


def host_array(t: torch.Tensor) -> np.ndarray:
    """Host copy of a tensor with its exact bits: fp32 -> float32, bf16 and fp16 -> uint16."""
    t = t.detach().contiguous().cpu()
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    if t.dtype == torch.float32:
        return t.numpy().copy()
    raise TypeError(t.dtype)
