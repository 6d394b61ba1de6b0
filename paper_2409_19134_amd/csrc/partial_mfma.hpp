// Partial attention over one chunk of one (user, KV head): bf16, fp16 or fp32 K/V, head_dim D = 128 or 64, MFMA path.
//
// What it computes (paper section 4.2): for each of the G query heads that share this KV head,
//   A = softmax(s) V and lse = ln sum exp(s) over the chunk's tokens, s_i = scale * <q, k_i>,
// i.e. one owner's term of Theorem 1 restricted to a token range.  Chunks of one row are later
// combined with the n-way form of the same theorem (combine.hpp).
//
// Mapping onto a 64-lane wave (r = lane % 16, grp = lane / 16), 32 tokens per step:
//   S^T = K . Q^T   two v_mfma_f32_16x16x32_{bf16,f16} chains (D/32 MFMAs each):
//                   the A operand is K as loaded (lane reads 16 B = 8 channels of token row r),
//                   the B operand is Q (head r, rows >= G are zero).  The result lands with
//                   head = r and tokens tb + grp*8 + e (e = 0..7) in each lane.
//   softmax         online (running max m, running sum l) per lane; the max is made uniform across the
//                   four lane groups of a head with two cross-lane exchanges per step.
//   O^T += V^T P^T  D/16 MFMA pairs (one per channel phase cc): the A operand V^T needs 8 tokens of one
//                   channel per lane; the lane loaded D/16 channels of 8 tokens (16 B each at D = 128, 8 B
//                   at D = 64: 16 lanes read a full row either way), so the operand is formed in registers
//                   with v_perm_b32 (no LDS).
//                   P is split into hi + lo parts of the element type, so the product keeps ~16 (bf16) or ~22
//                   (fp16) mantissa bits.  fp16 has a narrow exponent range: there P carries a factor 2^14 (the
//                   running sum l carries it too, so it cancels in A; lse subtracts it), which keeps
//                   probabilities down to 4e-9 of the row's largest out of the subnormal range.
//                   The B operand P^T is exactly the lane's own 8 probabilities.
// fp32 inputs take the same route with v_mfma_f32_16x16x4_f32 (one k-value per lane instead of eight): the lane's
// loads, the token each of its values belongs to and the layout of the results are the same as above, only the
// number of MFMAs per step differs (D/4 for S^T, D/2 for O^T at fp32, against D/16 and D/8 at 16 bits); P needs no
// split.
// Every K/V byte is read once per KV head (all G heads share the tile).
// The four waves of a workgroup take interleaved 32-token steps and are combined through LDS; the result rows of a
// workgroup that crosses many rows wait in LDS too and are stored together (the result ring, below).
#pragma once
#include "common.hpp"

namespace spd {

// The element type's MFMA and conversions, by dtype code (SPD_BF16 / SPD_F16: an integer template argument keeps
// the kernel's name readable in profiler output).
template <int DT>
struct Elt;
template <>
struct Elt<SPD_BF16> {
    static constexpr int kBytes = 2;
    typedef __bf16 type;
    typedef __bf16 vec8 __attribute__((ext_vector_type(8)));
    static constexpr float kPShift = 0.f;  // log2 of the factor P carries into the second MFMA
    static __device__ __forceinline__ f32x4 mfma(vec8 a, vec8 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};
template <>
struct Elt<SPD_F16> {
    static constexpr int kBytes = 2;
    typedef _Float16 type;
    typedef _Float16 vec8 __attribute__((ext_vector_type(8)));
    static constexpr float kPShift = 14.f;  // P <= 2^14 < 65504
    static __device__ __forceinline__ f32x4 mfma(vec8 a, vec8 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
};

template <>
struct Elt<SPD_F32> {
    static constexpr int kBytes = 4;
    static constexpr float kPShift = 0.f;
    static __device__ __forceinline__ f32x4 mfma(float a, float b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
};

// One step's loads of a lane, for rows of RB bytes (D channels of 2 or 4 bytes): RB/64 16-byte pieces of each of its
// two K rows, and RB/16 bytes (D/16 channels) of each of its eight V rows.
// A lane's share of one V row (RB/16 bytes), kept in the registers its loads deliver it in.
template <int RB>
struct VRow;
template <>
struct VRow<128> {
    u32x2 w;
    __device__ __forceinline__ void load(const char *p) { w = stream_load<u32x2>(p); }
    __device__ __forceinline__ unsigned dword(int i) const { return w[i]; }
};
template <>
struct VRow<256> {
    u32x4 w;
    __device__ __forceinline__ void load(const char *p) { w = stream_load16(p); }
    __device__ __forceinline__ unsigned dword(int i) const { return w[i]; }
};
template <>
struct VRow<512> {
    u32x4 w0, w1;
    __device__ __forceinline__ void load(const char *p)
    {
        w0 = stream_load16(p);
        w1 = stream_load16(p + 16);
    }
    __device__ __forceinline__ unsigned dword(int i) const { return i < 4 ? w0[i] : w1[i - 4]; }  // i is a constant
};

template <int RB>
struct TileRegs {
    u32x4 k[2][RB / 64];  // [S tile a][piece kk]: token row r of tile a, bytes kk*64 + grp*16 .. +16
    VRow<RB> v[8];        // [e]: token tb + grp*8 + e, bytes r*(RB/16) .. +RB/16
};

struct LaneConst {
    int r, grp;
    const char *k_base;  // contiguous: user's K + head offset; paged: pool + head offset
    const char *v_base;
    const int32_t *bt_row;
    int page_shift, page_mask;  // paged: token t lies in the row's page t >> page_shift at place t & page_mask
    int64_t token_stride, block_stride;
    const char *k_new_row;  // KV append: this (user, KV head)'s new K / V row if the segment ends its row, else nullptr
    const char *v_new_row;
};

// The pages that hold the two 16-token halves of the 32-token step at tb (the same page twice if pages hold 32 tokens
// or more).  The ids are wave-uniform and come through the scalar cache.  Clamping keeps the lookups inside the
// user's pages; rows past the chunk re-read its last token, which lies in the page the clamped lookup names (an
// 8-token group never straddles a page).
struct PagePair {
    int p0, p1;
};

__device__ __forceinline__ PagePair load_pages(const LaneConst &L, int tb, int t_last)
{
    const int tbu = uniform(tb);
    PagePair P;
    P.p0 = scalar_load_i32(L.bt_row, min(tbu, t_last) >> L.page_shift);
    P.p1 = scalar_load_i32(L.bt_row, min(tbu + 16, t_last) >> L.page_shift);
    return P;
}

// Issues the 16 loads of the step at tb.  Paged: P holds that step's page ids on entry and the following step's
// (tb + step) on return: the lookup is issued behind the data loads, one whole step before it is needed, so that no
// wave ever waits for a block-table entry before it can ask for data.
template <int RB, bool PAGED, bool APPEND>
__device__ __forceinline__ void load_tile(TileRegs<RB> &T, const LaneConst &L, int tb, int t_last, PagePair &P, int step)
{
    const int gk = tb + (L.r >> 2) * 8;  // first token of the 8-token group this lane's K rows fall in
    const int gv = tb + L.grp * 8;       // first token of the group this lane's V rows fall in
    const char *kp = L.k_base, *vp = L.v_base;
    if (PAGED) {
        kp += (int64_t)((gk - tb) >= 16 ? P.p1 : P.p0) * L.block_stride;
        vp += (int64_t)((gv - tb) >= 16 ? P.p1 : P.p0) * L.block_stride;
    }
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const int t = min(gk + a * 4 + (L.r & 3), t_last);  // rows past the chunk re-read its last token (masked later)
        const char *p = kp + (int64_t)(PAGED ? (t & L.page_mask) : t) * L.token_stride + L.grp * 16;
        if (APPEND && L.k_new_row && t == t_last)  // the appended token is read from the caller's buffer, not the cache
            p = L.k_new_row + L.grp * 16;
#pragma unroll
        for (int kk = 0; kk < RB / 64; ++kk)
            T.k[a][kk] = stream_load16(p + kk * 64);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int t = min(gv + e, t_last);
        const char *p = vp + (int64_t)(PAGED ? (t & L.page_mask) : t) * L.token_stride + L.r * (RB / 16);
        if (APPEND && L.v_new_row && t == t_last)
            p = L.v_new_row + L.r * (RB / 16);
        T.v[e].load(p);
    }
    if (PAGED)
        P = load_pages(L, tb + step, t_last);
    // all loads of the step are issued before anything that follows: without this the compiler sinks the V loads
    // below the K wait to shorten live ranges, which serialises two memory round trips per step
    __builtin_amdgcn_sched_barrier(0);
}

// qB: Q as the B operand, loaded like a K row (head r instead of token r): bytes kk*64 + grp*16 .. +16 of the row.
template <int DT, int D>
__device__ __forceinline__ void compute_tile(const TileRegs<D * Elt<DT>::kBytes> &T,
                                             const u32x4 (&qB)[D * Elt<DT>::kBytes / 64], int tb, int grp, int t_end,
                                             float c, float &m, float &l, f32x4 (&acc)[D / 16])
{
    constexpr int RB = D * Elt<DT>::kBytes;
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
    if constexpr (DT == SPD_F32) {
#pragma unroll
        for (int kk = 0; kk < RB / 64; ++kk)
#pragma unroll
            for (int e = 0; e < 4; ++e) {  // four channels per piece, one MFMA (k = 4: the lane groups) each
                s0 = Elt<DT>::mfma(__uint_as_float(T.k[0][kk][e]), __uint_as_float(qB[kk][e]), s0);
                s1 = Elt<DT>::mfma(__uint_as_float(T.k[1][kk][e]), __uint_as_float(qB[kk][e]), s1);
            }
    } else {
        typedef typename Elt<DT>::vec8 vec8;
#pragma unroll
        for (int kk = 0; kk < RB / 64; ++kk) {
            s0 = Elt<DT>::mfma(__builtin_bit_cast(vec8, T.k[0][kk]), __builtin_bit_cast(vec8, qB[kk]), s0);
            s1 = Elt<DT>::mfma(__builtin_bit_cast(vec8, T.k[1][kk]), __builtin_bit_cast(vec8, qB[kk]), s1);
        }
    }
    // scores in log2 units; tokens past the chunk end get -inf
    const int t0 = tb + grp * 8;
    float x[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        x[e] = (t0 + e < t_end) ? s0[e] * c : -INFINITY;
        x[4 + e] = (t0 + 4 + e < t_end) ? s1[e] * c : -INFINITY;
    }
    float mt = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    mt = wave_xor_max<16>(mt);
    mt = wave_xor_max<32>(mt);
    const float m_new = fmaxf(m, mt);  // finite: every step holds at least one token of the chunk
    const float alpha = fast_exp2(m - m_new);
    const float m_p = m_new - Elt<DT>::kPShift;  // p (and with it l and acc) carries the factor 2^kPShift
    float p[8], ps = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        p[e] = fast_exp2(x[e] - m_p);
        ps += p[e];
    }
    l = l * alpha + ps;
    m = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {  // wave-uniform: rescale only when some max moved
#pragma unroll
        for (int cc = 0; cc < D / 16; ++cc)
            acc[cc] *= alpha;
    }
    if constexpr (DT == SPD_F32) {
        // channel phase cc: the lane's dword cc of each of its eight tokens; the MFMA's four k-values are the four
        // lane groups' tokens grp*8 + e, and the B operand is the lane's own probability of that token
#pragma unroll
        for (int cc = 0; cc < D / 16; ++cc)
#pragma unroll
            for (int e = 0; e < 8; ++e)
                acc[cc] = Elt<DT>::mfma(__uint_as_float(T.v[e].dword(cc)), p[e], acc[cc]);
    } else {
        typedef typename Elt<DT>::vec8 vec8;
        typedef typename Elt<DT>::type E;
        vec8 ph, pl;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            ph[e] = (E)p[e];
            pl[e] = (E)(p[e] - (float)ph[e]);
        }
#pragma unroll
        for (int cc = 0; cc < D / 16; ++cc) {
            const int w = cc >> 1;
            const unsigned sel = (cc & 1) ? 0x07060302u : 0x05040100u;  // odd channel: high halves, even: low halves
            u32x4 vt;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                vt[j] = __builtin_amdgcn_perm(T.v[2 * j + 1].dword(w), T.v[2 * j].dword(w), sel);  // (token 2j, token 2j+1) of channel cc
            const vec8 va = __builtin_bit_cast(vec8, vt);
            acc[cc] = Elt<DT>::mfma(va, ph, acc[cc]);
            acc[cc] = Elt<DT>::mfma(va, pl, acc[cc]);
        }
    }
}

// LDS row stride (floats) of one head's D channels: the four extra floats spread the heads over the banks
__host__ __device__ constexpr int o_stride(int D) { return D + 4; }

// LDS bytes of the result staging tiles of a workgroup of `waves` waves, and whether the head-per-wave mapping can have
// them (kernel and launch use the same rule; 64 KB is what a workgroup may ask for without special attributes).
__host__ __device__ constexpr size_t staging_bytes(int D, int waves, int G)
{
    return sizeof(float) * (size_t)waves * G * o_stride(D);
}
__host__ __device__ constexpr bool staging_fits(int D, int waves, int G) { return staging_bytes(D, waves, G) <= 64 * 1024; }

// The result ring.  A piece that crosses rows produces a result row ([G][D] values and G log-sum-exps, final or a chunk
// partial) at every segment end.  Written where they arise, those rows reach HBM as single lines scattered over the
// read stream, and each costs the memory system far more than its bytes: a plain streaming read of 2.8 GB at 768
// workgroups takes 414 us, 444 us with 8 MB of such rows written along the way, and 418 us with the same rows written
// when a workgroup is done (measured on this GPU; workload 4 writes 8 MB of them in 443 us).  So a head-major
// workgroup keeps its rows in LDS, up to `ring_rows` of them, and stores them together when the ring is full or the
// piece ends.  A row of the ring: G * D values, then G log-sum-exps, padded to a multiple of four floats.
constexpr int kRingMaxRows = 32;
__host__ __device__ constexpr int ring_row_floats(int D, int G) { return G * D + ((G + 3) & ~3); }
// LDS bytes a head-major workgroup may use for staging and ring together: a CU's 160 KB are shared by the three
// workgroups that the one-step kernel's registers allow, or by two (the two-step kernel, or a launch of no more than
// two workgroups per CU), and a workgroup may ask for 64 KB in all.
__host__ __device__ constexpr size_t ring_lds_budget(bool two_per_cu) { return (two_per_cu ? 60 : 40) * 1024; }
__host__ __device__ constexpr int ring_rows_that_fit(int D, int G, bool two_per_cu)
{
    const size_t staging = sizeof(float) * (size_t)kWaves * G * o_stride(D);
    const size_t row = sizeof(float) * (size_t)ring_row_floats(D, G);
    const size_t n = staging >= ring_lds_budget(two_per_cu) ? 0 : (ring_lds_budget(two_per_cu) - staging) / row;
    return n < 2 ? 0 : n > (size_t)kRingMaxRows ? kRingMaxRows : (int)n;  // a ring of one row holds nothing back
}

// The same for the head-per-wave mapping, where every wave owns a row per segment: a ring per wave, its rows in the
// layout of the wave's staging tile ([G][o_stride]), then G log-sum-exps (padded to four floats) and the two pointers
// the row goes to.
__host__ __device__ constexpr int hpw_ring_row_floats(int D, int G) { return G * o_stride(D) + ((G + 3) & ~3) + 4; }
__host__ __device__ constexpr int hpw_ring_rows_that_fit(int D, int G, int waves)
{
    const size_t staging = sizeof(float) * (size_t)waves * G * o_stride(D);
    const size_t row = sizeof(float) * (size_t)hpw_ring_row_floats(D, G) * waves;
    const size_t n = staging >= ring_lds_budget(true) ? 0 : (ring_lds_budget(true) - staging) / row;
    return n < 2 ? 0 : n > (size_t)kRingMaxRows ? kRingMaxRows : (int)n;
}

// Waves per SIMD the kernel is compiled for: a step's loads take RB/4 registers per lane (twice that with PREFETCH).
__host__ __device__ constexpr int mfma_waves_per_simd(int RB, bool prefetch, bool hpw)
{
    return RB == 512 ? 2 : RB == 256 ? (prefetch ? 2 : 3) : (hpw ? 2 : 3);
}

// One workgroup per piece (see DevItem); q: [U][Hq][D] of the element type DT (SPD_BF16, SPD_F16 or SPD_F32).  A
// segment that is its row's only one writes out/lse directly; otherwise it writes part_o[slot][G][D] /
// part_lse[slot][G], which combine_chunks_kernel then reduces.
//
// (Register counts below are those of 256-byte rows: 16-bit elements with D = 128.  Rows of 128 bytes need about half
// and always run with PREFETCH; fp32 rows of 512 bytes need ~245 with one step in flight and never run with it.)
// PREFETCH = true keeps two 32-token steps of loads in flight per wave (~245 VGPRs, two waves per SIMD): for launches
// that run several rounds of workgroups, and for small ones that fit two per CU anyway (half as many dependent round
// trips per wave).  PREFETCH = false holds one step (~160 VGPRs, three waves per SIMD): as fast when the private
// owner's pieces are one resident round, and it leaves room on every CU for the other owner's pieces.
//
// HPW ("head per wave") is the mapping for contiguous token-major storage, where the KV heads of a token are adjacent
// in memory ([token][head][d]).  A piece is then a token range of a *user* for a group of two to eight KV heads (the
// host picks the group size by the size of the launch), the workgroup has one wave per KV head of the group, and all waves walk the same tokens:
// together they read whole, consecutive DRAM pages, where one workgroup per head would touch every page eight times
// at different moments (a barrier per step keeps the waves together).  Each wave owns its head's result, so there is no cross-wave combine; the wave stores its
// result through an LDS tile of its own.  Without HPW (head-major storage: one contiguous stream per head) a piece is
// a token range of one (user, KV head) row and its four waves take interleaved steps.
//
// APPEND = true adds the KV append (the address substitution costs ~1 % when nothing is appended, hence a flag).
template <int DT, int D, bool PAGED, bool PREFETCH, bool HPW, bool APPEND>
__global__ __launch_bounds__(HPW ? 512 : kThreads, mfma_waves_per_simd(D *Elt<DT>::kBytes, PREFETCH, HPW)) void partial_mfma_kernel(
    PartialArgs A)
{
    const OwnerArgs &a0 = A.a0, &a1 = A.a1;
    const int n0 = A.n0, Hq = A.Hq, G = A.G;
    const char *__restrict__ q = A.q;
    const float scale_log2e = A.scale_log2e;
    const bool second = (int)blockIdx.x >= n0;  // workgroup-uniform: which owner this workgroup serves
    const DevItem *__restrict__ items = second ? a1.items : a0.items;
    const KvAddr kv = second ? a1.kv : a0.kv;
    const uintptr_t k_pool = reinterpret_cast<uintptr_t>(second ? a1.k_pool : a0.k_pool);  // 0 unless paged
    const uintptr_t v_pool = reinterpret_cast<uintptr_t>(second ? a1.v_pool : a0.v_pool);
    const char *const *k_ptrs = second ? a1.k_ptrs : a0.k_ptrs;  // null unless the view brought device pointer tables
    const char *const *v_ptrs = second ? a1.v_ptrs : a0.v_ptrs;
    float *__restrict__ part_o = second ? a1.part_o : a0.part_o;
    float *__restrict__ part_lse = second ? a1.part_lse : a0.part_lse;
    float *__restrict__ out = second ? a1.out : a0.out;
    float *__restrict__ lse = second ? a1.lse : a0.lse;
    const char *k_new = second ? a1.k_new : a0.k_new;
    const char *v_new = second ? a1.v_new : a0.v_new;
    const int grow = second ? a1.grow : a0.grow;
    __shared__ float sm_m[kWaves][16];
    __shared__ float sm_l[kWaves][16];
    __shared__ float *ring_dst_o[kRingMaxRows], *ring_dst_l[kRingMaxRows];  // where the ring's rows go
    extern __shared__ float sm_o[];  // [waves][G * kOStride], sized by the launch: only G heads are staged; then the ring
    constexpr int kOStride = o_stride(D);
    constexpr int CP = D / 16;  // channel phases of the O^T tile: a lane holds CP consecutive channels per accumulator row
    constexpr int kRowBytes = D * Elt<DT>::kBytes;
    constexpr int RB = kRowBytes;
    const int o_wave_stride = G * kOStride;
    // head-per-wave results go through a wave-private tile if the launch gave the room
    const bool staged = HPW && staging_fits(D, (int)(blockDim.x >> 6), G);

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    constexpr int kStep = HPW ? 32 : 32 * kWaves;

    // Everything a segment needs before its first MFMA: addresses, the KV append copy, Q, and the loads of the wave's
    // first 32-token step.  Issued for the *next* segment before the current one's epilogue, so that the barriers
    // and the result stores of the epilogue overlap the memory round trip instead of preceding it.
    auto begin_segment = [&](const DevItem &it, LaneConst &L, u32x4 (&qB)[RB / 64], int &tb, TileRegs<RB> &T0, PagePair &P) {
        L.r = lane & 15;
        L.grp = lane >> 4;
        L.token_stride = kv.token_stride;
        L.block_stride = kv.block_stride;
        L.page_shift = kv.page_shift;
        L.page_mask = (1 << kv.page_shift) - 1;
        const int kv_head = HPW ? it.kv_head + uniform(wave) : it.kv_head;  // head per wave: the group's first head + wave
        L.k_base = it.k_base + k_pool + (PAGED ? 0 : user_base(k_ptrs, it.user)) + (HPW ? (int64_t)kv_head * kv.head_stride : 0);
        L.v_base = it.v_base + v_pool + (PAGED ? 0 : user_base(v_ptrs, it.user)) + (HPW ? (int64_t)kv_head * kv.head_stride : 0);
        L.bt_row = PAGED ? kv.block_table + (int64_t)it.user * kv.max_blocks : nullptr;
        const int t_last = it.t_end - 1;
        L.k_new_row = L.v_new_row = nullptr;
        if (APPEND && k_new && (it.rot & kEndsRow)) {
            // KV append: this segment holds the row's last token, which is the new one.  Wave 0 copies its K and V
            // rows into the cache (16 bytes per lane, K in the first lanes, V in the next); every reader of that token
            // takes it from the caller's buffer instead, so nothing waits for the copy.
            constexpr int kRowLanes = kRowBytes / 16;
            const int64_t row = ((int64_t)it.user * (Hq / G) + kv_head) * kRowBytes;
            L.k_new_row = k_new + row;
            L.v_new_row = v_new + row;
            if ((HPW || wave == 0) && lane < 2 * kRowLanes) {
                int64_t off = (int64_t)(PAGED ? (t_last & L.page_mask) : t_last) * kv.token_stride + (lane % kRowLanes) * 16;
                if (PAGED)
                    off += (int64_t)scalar_load_i32(L.bt_row, t_last >> L.page_shift) * kv.block_stride;
                if (lane < kRowLanes)
                    copy16(const_cast<char *>(L.k_base) + off, L.k_new_row + lane * 16);
                else
                    copy16(const_cast<char *>(L.v_base) + off, L.v_new_row + (lane - kRowLanes) * 16);
            }
        }
        // Q as the B operand: head r (zero beyond G), read like a K row: bytes kk*64 + grp*16 .. +16
        const char *qrow = q + ((int64_t)it.user * Hq + (int64_t)kv_head * G + L.r) * kRowBytes + L.grp * 16;
#pragma unroll
        for (int kk = 0; kk < RB / 64; ++kk) {
            qB[kk] = u32x4{0u, 0u, 0u, 0u};
            if (L.r < G)
                qB[kk] = *reinterpret_cast<const u32x4 *>(qrow + kk * 64);
        }
        // head-major: the four waves take interleaved 32-token steps; token-major: every wave takes every step
        tb = HPW ? it.t_begin : it.t_begin + ((uniform(wave) - (it.rot & 3)) & (kWaves - 1)) * 32;
        if (PAGED)
            P = load_pages(L, tb, t_last);
        if (PREFETCH && tb < it.t_end)
            load_tile<RB, PAGED, APPEND>(T0, L, tb, t_last, P, kStep);
    };

    DevItem it = scalar_load_item(items, second ? (int)blockIdx.x - n0 : (int)blockIdx.x, grow);
    if (it.n_chunks == 0) {  // a row without tokens (head-per-wave: a user without tokens) is a piece of its own
        if (HPW) {
            const int64_t head0 = (int64_t)it.user * Hq + (int64_t)(it.kv_head + wave) * G;
            for (int idx = lane; idx < G * D; idx += 64)
                out[head0 * D + idx] = 0.f;
            if (lane < G)
                lse[head0 + lane] = -INFINITY;
        } else {
            write_empty_row<D>(it, G, Hq, out, lse);
        }
        return;
    }
    LaneConst L;
    u32x4 qB[RB / 64];
    int tb;
    TileRegs<RB> T0;
    PagePair P = {0, 0};
    int n_ring = 0;  // rows held in the result ring (head-major mapping only)
    begin_segment(it, L, qB, tb, T0, P);
    for (;;) {
        // the piece's next segment is fetched (scalar cache) long before it is looked at: with tens of MB of loads in
        // flight a dependent round trip costs microseconds, so none may sit between two segments
        DevItem nx = it;
        if (it.next >= 0)
            nx = scalar_load_item(items, it.next, grow);
        const int t_last = it.t_end - 1;

        float m = -INFINITY, l = 0.f;
        f32x4 acc[CP];
#pragma unroll
        for (int cc = 0; cc < CP; ++cc)
            acc[cc] = f32x4{0.f, 0.f, 0.f, 0.f};

        if (!PREFETCH) {
            for (; tb < it.t_end; tb += kStep) {
                TileRegs<RB> T;
                load_tile<RB, PAGED, APPEND>(T, L, tb, t_last, P, kStep);
                compute_tile<DT, D>(T, qB, tb, L.grp, it.t_end, scale_log2e, m, l, acc);
            }
        } else if (tb < it.t_end) {  // T0 already holds (the loads of) step tb
            {
                TileRegs<RB> T1;
                for (;;) {
                    const int tb1 = tb + kStep;
                    const bool more1 = tb1 < it.t_end;
                    // head per wave: the waves stay in step (they all run the same trip counts), so that together they
                    // ask for whole consecutive token rows at about the same time
                    if (HPW)
                        __builtin_amdgcn_s_barrier();
                    if (more1)
                        load_tile<RB, PAGED, APPEND>(T1, L, tb1, t_last, P, kStep);
                    compute_tile<DT, D>(T0, qB, tb, L.grp, it.t_end, scale_log2e, m, l, acc);
                    if (!more1)
                        break;
                    const int tb2 = tb1 + kStep;
                    const bool more2 = tb2 < it.t_end;
                    if (HPW)
                        __builtin_amdgcn_s_barrier();
                    if (more2)
                        load_tile<RB, PAGED, APPEND>(T0, L, tb2, t_last, P, kStep);
                    compute_tile<DT, D>(T1, qB, tb1, L.grp, it.t_end, scale_log2e, m, l, acc);
                    if (!more2)
                        break;
                    tb = tb2;
                }
            }
        }

        const int grp = L.grp, r = L.r;
        // the two-per-CU kernel has the registers to let the next segment's loads fly during the epilogue below
        if (PREFETCH && it.next >= 0)
            begin_segment(nx, L, qB, tb, T0, P);

        // ---- combine the lane groups (sum of l) ... ----
        l = wave_xor_sum<16>(l);
        l = wave_xor_sum<32>(l);
        const bool direct = it.n_chunks == 1;
        if (HPW) {
            // ... and that is all: the wave owns head `wave` of this token range.  Lane (r < G, grp) holds channels
            // (4*grp + v)*CP + cc of query head r: CP consecutive floats per v.
            const int kvh = it.kv_head + uniform(wave);
            const int64_t head0 = (int64_t)it.user * Hq + (int64_t)kvh * G;
            const int64_t slot = (int64_t)it.slot + (int64_t)uniform(wave) * it.n_chunks;  // it.slot: the group's first head
            const float inv = fast_rcp(l);  // l > 0: the segment holds at least one token
            float *res = direct ? out + head0 * D : part_o + slot * G * D;  // [G][D], contiguous
            float *res_l = direct ? lse + head0 : part_lse + slot * G;
            // the row waits in the wave's ring - unless the piece ends here with an empty ring, or there is no ring
            const bool last = it.next < 0;
            const bool to_ring = staged && A.ring_rows > 0 && !(last && n_ring == 0);
            const int hrow = hpw_ring_row_floats(D, G);
            float *const ring_w = sm_o + (int)(blockDim.x >> 6) * o_wave_stride + wave * A.ring_rows * hrow;
            if (staged) {
                // Through a wave-private LDS tile, so that the wave stores whole rows with consecutive lanes (storing
                // straight from the accumulator layout puts 16 bytes per lane into 16 different cache lines per
                // instruction; measured 2-3 % of the kernel on long token-major workloads).
                float *stage = to_ring ? ring_w + n_ring * hrow : sm_o + wave * o_wave_stride;
                if (r < G) {
                    float *dst = stage + r * kOStride + grp * 4 * CP;
#pragma unroll
                    for (int cc = 0; cc < CP; ++cc)
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            dst[v * CP + cc] = acc[cc][v] * inv;  // channel (4*grp + v)*CP + cc
                }
                if (to_ring) {
                    if (r < G && grp == 0)
                        stage[o_wave_stride + r] = (m + fast_log2(l) - Elt<DT>::kPShift) * kLn2;  // m is in log2 units
                    if (lane == 0) {
                        float **dst = reinterpret_cast<float **>(stage + o_wave_stride + ((G + 3) & ~3));
                        dst[0] = res;
                        dst[1] = res_l;
                    }
                    ++n_ring;
                }
                __builtin_amdgcn_wave_barrier();  // same wave: LDS executes its writes before its reads
                if (!to_ring) {
                    for (int i = lane * 4; i < G * D; i += 256) {
                        const f32x4 w = *reinterpret_cast<const f32x4 *>(stage + (i / D) * kOStride + (i % D));
                        *reinterpret_cast<f32x4 *>(res + i) = w;
                    }
                } else if (last || n_ring == A.ring_rows) {
                    typedef __attribute__((address_space(1))) float *global_f32;
                    for (int k = 0; k < n_ring; ++k) {
                        const float *row = ring_w + k * hrow;
                        float *const *dst = reinterpret_cast<float *const *>(row + o_wave_stride + ((G + 3) & ~3));
                        const global_f32 o = (global_f32)dst[0];
                        for (int i = lane * 4; i < G * D; i += 256) {
                            const f32x4 w = *reinterpret_cast<const f32x4 *>(row + (i / D) * kOStride + (i % D));
                            *reinterpret_cast<__attribute__((address_space(1))) f32x4 *>(o + i) = w;
                        }
                        if (lane < G)
                            ((global_f32)dst[1])[lane] = row[o_wave_stride + lane];
                    }
                    n_ring = 0;
                }
                __builtin_amdgcn_wave_barrier();
            }
            if (r < G) {
                if (!staged) {
                    float *dst = res + r * D + grp * 4 * CP;
#pragma unroll
                    for (int v = 0; v < 4; ++v)
#pragma unroll
                        for (int c4 = 0; c4 < CP; c4 += 4) {
                            const f32x4 w = {acc[c4][v] * inv, acc[c4 + 1][v] * inv, acc[c4 + 2][v] * inv, acc[c4 + 3][v] * inv};
                            *reinterpret_cast<f32x4 *>(dst + v * CP + c4) = w;
                        }
                }
                if (grp == 0 && !to_ring)
                    res_l[r] = (m + fast_log2(l) - Elt<DT>::kPShift) * kLn2;  // m is in log2 units
            }
            if (last)
                return;
            if (!PREFETCH)
                begin_segment(nx, L, qB, tb, T0, P);
            it = nx;
            continue;
        }

        // ---- ... and the four waves (LDS) ----
        if (grp == 0) {
            sm_m[wave][r] = m;
            sm_l[wave][r] = l;
        }
        __syncthreads();
        float M = sm_m[0][r];
#pragma unroll
        for (int w = 1; w < kWaves; ++w)
            M = fmaxf(M, sm_m[w][r]);
        const float f = fast_exp2(m - M);  // some wave holds tokens, so M is finite; an idle wave has m = -inf, f = 0
        if (r < G) {
            float *dst = &sm_o[wave * o_wave_stride + r * kOStride + grp * 4 * CP];
#pragma unroll
            for (int cc = 0; cc < CP; ++cc)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    dst[v * CP + cc] = acc[cc][v] * f;  // channel (4*grp + v)*CP + cc
        }
        __syncthreads();

        const int64_t head0 = (int64_t)it.user * Hq + (int64_t)it.kv_head * G;
        // the row goes to the ring - unless the piece ends here with an empty ring, or there is no ring
        const bool last = it.next < 0;
        const bool to_ring = A.ring_rows > 0 && !(last && n_ring == 0);
        const int GD = G * D, ring_stride = ring_row_floats(D, G);
        float *const ring = sm_o + kWaves * o_wave_stride;
        float *const dst_o = direct ? out + head0 * D : part_o + (int64_t)it.slot * GD;
        float *const dst_l = direct ? lse + head0 : part_lse + (int64_t)it.slot * G;
        // (two copies of the loop, so that each stores through pointers of one kind, LDS or global memory: a pointer
        // that may be either makes every store a flat one)
        typedef __attribute__((address_space(1))) float *global_f32;
        typedef __attribute__((address_space(3))) float *lds_f32;
        auto reduce_waves = [&](auto row_o, auto row_l) {
            for (int idx = threadIdx.x; idx < GD; idx += kThreads) {
                const int g = idx / D, ch = idx % D;
                float Mg = sm_m[0][g];
#pragma unroll
                for (int w = 1; w < kWaves; ++w)
                    Mg = fmaxf(Mg, sm_m[w][g]);
                float o = 0.f, lt = 0.f;
#pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    o += sm_o[w * o_wave_stride + g * kOStride + ch];
                    lt += sm_l[w][g] * fast_exp2(sm_m[w][g] - Mg);
                }
                row_o[idx] = o * fast_rcp(lt);
                if (ch == 0)
                    row_l[g] = (Mg + fast_log2(lt) - Elt<DT>::kPShift) * kLn2;  // Mg is in log2 units
            }
        };
        if (to_ring)
            reduce_waves((lds_f32)(ring + n_ring * ring_stride), (lds_f32)(ring + n_ring * ring_stride + GD));
        else
            reduce_waves((global_f32)dst_o, (global_f32)dst_l);
        if (to_ring) {
            if (threadIdx.x == 0) {
                ring_dst_o[n_ring] = dst_o;
                ring_dst_l[n_ring] = dst_l;
            }
            ++n_ring;
            if (last || n_ring == A.ring_rows) {
                __syncthreads();
                for (int i = 0; i < n_ring; ++i) {
                    const lds_f32 src = (lds_f32)(ring + i * ring_stride);
                    const global_f32 o = (global_f32)ring_dst_o[i];
                    for (int idx = threadIdx.x; idx < GD; idx += kThreads)
                        o[idx] = src[idx];
                    if ((int)threadIdx.x < G)
                        ((global_f32)ring_dst_l[i])[threadIdx.x] = src[GD + threadIdx.x];
                }
                n_ring = 0;
            }
        }
        if (last)
            return;
        if (!PREFETCH)
            begin_segment(nx, L, qB, tb, T0, P);
        it = nx;
        __syncthreads();  // the LDS staging arrays are reused by the next segment
    }
}

}  // namespace spd
