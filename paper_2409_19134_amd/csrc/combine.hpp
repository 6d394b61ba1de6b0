// Combination rules of Theorem 1 (paper section 4.2) written on log-sum-exps.
//
//   combine_chunks_kernel  n-way form, used inside one owner's call: the chunks c of a (user, KV head) row each hold
//                          (A_c, lse_c); lse = logsumexp_c lse_c and A = sum_c exp(lse_c - lse) A_c.
//                          A separate launch, not a last-workgroup-reduces scheme inside the partial kernel: on this
//                          multi-die GPU a device-scope release/acquire writes back and invalidates a whole L2, which
//                          cost more than the extra launch when every workgroup had to issue one.
//   finalize_step_kernel   last kernel of the fused step: combines whichever rows were split, for both owners, and
//                          merges the owners, in one launch
//   lse_merge_kernel       the two-owner merge itself: Y = w0 A_in + w1 A_out with w_x = exp(lse_x - lse).
//                          With lse_x = m_x + ln gamma_x these weights equal the paper's
//                          gamma_in / (gamma_in + alpha gamma_out) and gamma_out / (alpha^-1 gamma_in + gamma_out),
//                          alpha = exp(m_out - m_in), but never form alpha, which overflows fp32 for
//                          |m_out - m_in| > 88.
#pragma once
#include "common.hpp"

namespace spd {

constexpr int kCombineStage = 512;  // chunk weights staged in LDS per pass

// e^x through the hardware's 2^x (one instruction after the scaling; the library expf is a dozen, and these kernels
// are a few microseconds of pure latency in which every thread computes the same few weights).  fast_exp(0) is
// exactly 1 and fast_exp(-inf) exactly 0, which the merge relies on.
__device__ __forceinline__ float fast_exp(float x) { return fast_exp2(x * kLog2e); }
// ln x through the hardware's log2 (1 ulp), for the same reason
__device__ __forceinline__ float fast_log(float x) { return fast_log2(x) * kLn2; }

// n-way form for one (row, query head), executed by a workgroup of D threads (thread = channel): returns this
// thread's channel of A = sum_c exp(lse_c - lse) A_c and lse = logsumexp_c lse_c.  The chunk weights are staged in
// LDS by all threads in parallel, then every thread streams its channel of the chunks' partial vectors with
// independent loads, in chunk order (so the result does not depend on the order in which the partial workgroups
// ran).  sm_w: kCombineStage floats, sm_red: D floats.  n_chunks >= 1; chunks are never empty, so lse is finite.
template <int D>
__device__ __forceinline__ void combine_row(const float *__restrict__ pl, const float *__restrict__ po, int n_chunks,
                                            int G, float *sm_w, float *sm_red, float &a_out, float &lse_out)
{
    const int tid = threadIdx.x;
    float mloc = -INFINITY;
    for (int c = tid; c < n_chunks; c += D)
        mloc = fmaxf(mloc, pl[(int64_t)c * G]);
    __syncthreads();  // earlier readers of the LDS arrays are done
    sm_red[tid] = mloc;
    __syncthreads();
    for (int s = D / 2; s > 0; s >>= 1) {
        if (tid < s)
            sm_red[tid] = fmaxf(sm_red[tid], sm_red[tid + s]);
        __syncthreads();
    }
    const float M = sm_red[0];
    float o = 0.f, den = 0.f;
    for (int c0 = 0; c0 < n_chunks; c0 += kCombineStage) {
        const int nc = min(kCombineStage, n_chunks - c0);
        __syncthreads();
        for (int c = tid; c < nc; c += D)
            sm_w[c] = fast_exp(pl[(int64_t)(c0 + c) * G] - M);
        __syncthreads();
#pragma unroll 8
        for (int c = 0; c < nc; ++c) {
            den += sm_w[c];
            o = fmaf(sm_w[c], po[(int64_t)(c0 + c) * G * D], o);
        }
    }
    a_out = o * fast_rcp(den);
    lse_out = M + fast_log(den);
}

// The same for rows of at most MAXC chunks, without LDS or barriers: every load is issued at once (one memory round
// trip), same arithmetic and chunk order as combine_row.
template <int D, int MAXC>
__device__ __forceinline__ void combine_row_small(const float *__restrict__ pl, const float *__restrict__ po,
                                                  int n_chunks, int G, float &a_out, float &lse_out)
{
    float l[MAXC], x[MAXC];
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const bool on = c < n_chunks;
        l[c] = on ? pl[(int64_t)c * G] : -INFINITY;
        x[c] = on ? po[(int64_t)c * G * D] : 0.f;
    }
    float M = l[0];
#pragma unroll
    for (int c = 1; c < MAXC; ++c)
        M = fmaxf(M, l[c]);
    float o = 0.f, den = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        if (c < n_chunks) {
            const float w = fast_exp(l[c] - M);
            den += w;
            o = fmaf(w, x[c], o);
        }
    }
    a_out = o * fast_rcp(den);
    lse_out = M + fast_log(den);
}

// One owner's side of a row as combine_chunks_kernel reads it: up to MAXC (lse, value) pairs, all loaded at once.
// A row that was not split (or holds no token) is one pair read from the caller's own A / lse arrays.
template <int MAXC>
struct RowLoads {
    float l[MAXC], x[MAXC];
    int n;  // pairs held; 0 if the row has more chunks than MAXC (then combine_row takes it)
};

template <int D, int MAXC>
__device__ __forceinline__ RowLoads<MAXC> load_row(const RowInfo ri, int G, int g, int64_t row, const float *part_o,
                                                   const float *part_lse, const float *a, const float *lse)
{
    const bool split = ri.n_chunks > 1;
    const float *pl = split ? part_lse + (int64_t)ri.first_slot * G + g : lse + row;
    const float *po = split ? part_o + ((int64_t)ri.first_slot * G + g) * D + threadIdx.x : a + row * D + threadIdx.x;
    RowLoads<MAXC> r;
    r.n = split ? (ri.n_chunks <= MAXC ? ri.n_chunks : 0) : 1;
    const int GD = G * D;  // 32-bit offsets: at most MAXC * 16 * 128 floats from the row's first pair
    // groups of four pairs: a wave-uniform branch per group, unconditional loads inside it (a pair past the end re-reads
    // the row's first pair; reduce_row ignores it), so the loads leave back to back and few are redundant
    static_assert(MAXC % 4 == 0, "pairs are loaded in groups of four");
#pragma unroll
    for (int c0 = 0; c0 < MAXC; c0 += 4) {
        if (c0 < r.n) {
#pragma unroll
            for (int c = c0; c < c0 + 4; ++c) {
                const int ce = c < r.n ? c : 0;
                r.l[c] = pl[ce * G];  // masked where it is used: nothing here waits for a load
                r.x[c] = po[ce * GD];
            }
        } else {
#pragma unroll
            for (int c = c0; c < c0 + 4; ++c) {
                r.l[c] = -INFINITY;
                r.x[c] = 0.f;
            }
        }
    }
    return r;
}

// n-way form over the loaded pairs, same arithmetic and chunk order as combine_row; a single pair passes through
// unchanged (it may be an empty row: value 0, lse -inf).
template <int MAXC>
__device__ __forceinline__ void reduce_row(const RowLoads<MAXC> &r, float &a_out, float &lse_out)
{
    if (r.n == 1) {
        a_out = r.x[0];
        lse_out = r.l[0];
        return;
    }
    float M = r.l[0];
#pragma unroll
    for (int c = 1; c < MAXC; ++c)
        M = fmaxf(M, c < r.n ? r.l[c] : -INFINITY);
    float o = 0.f, den = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        if (c < r.n) {
            const float w = fast_exp(r.l[c] - M);
            den += w;
            o = fmaf(w, r.x[c], o);
        }
    }
    a_out = o * fast_rcp(den);
    lse_out = M + fast_log(den);
}

// One workgroup of D threads per (split row, query head); grid (split rows, G).
template <int D>
__global__ __launch_bounds__(D) void combine_chunks_kernel(const CombineRow *__restrict__ rows, int Hq, int G,
                                                           const float *__restrict__ part_o,
                                                           const float *__restrict__ part_lse,
                                                           float *__restrict__ out, float *__restrict__ lse)
{
    __shared__ float sm_w[kCombineStage];
    __shared__ float sm_red[D];
    const CombineRow r = rows[blockIdx.x];  // grid: (split rows, G) - no integer division on a latency-bound path
    const int g = blockIdx.y;
    const int64_t row = (int64_t)r.user * Hq + (int64_t)r.kv_head * G + g;
    float a, ls;
    constexpr int kSmall = 16;
    if (r.n_chunks <= kSmall)  // every load at once: one memory round trip
        reduce_row(load_row<D, kSmall>(RowInfo{r.first_slot, r.n_chunks}, G, g, row, part_o, part_lse, out, lse), a, ls);
    else
        combine_row<D>(part_lse + (int64_t)r.first_slot * G + g,
                       part_o + ((int64_t)r.first_slot * G + g) * D + threadIdx.x, r.n_chunks, G, sm_w, sm_red, a, ls);
    out[row * D + threadIdx.x] = a;
    if (threadIdx.x == 0)
        lse[row] = ls;
}

// Two-owner weights of Theorem 1 on log-sum-exps; a side with lse = -inf gets weight exactly 0.
__device__ __forceinline__ void merge_weights(float l0, float l1, float &w0, float &w1, float &ls)
{
    const float M = fmaxf(l0, l1);
    if (M == -INFINITY) {  // both owners hold no token for this row
        w0 = 0.f, w1 = 0.f, ls = -INFINITY;
        return;
    }
    const float e0 = fast_exp(l0 - M), e1 = fast_exp(l1 - M);  // the larger one is exactly 1
    const float den = e0 + e1;
    const float inv = fast_rcp(den);
    w0 = e0 * inv;
    w1 = e1 * inv;
    ls = M + fast_log(den);
}

// Last kernel of a fused decode step: one workgroup of D threads per (user, query head), grid (users, Hkv, G).  For each owner, a row
// that was split is combined here (and its A / lse written, so the caller still gets both partials); unsplit and
// empty rows were already written by the partial kernels and are read back.  Then the two owners are merged.
// The first owner's partials are read through a_in_r / lse_in_r and, for the rows combined here, written through
// a_in_w / lse_in_w (the same arrays for a fused step).  rows_in == nullptr says that the first owner's partials are
// finished results handed in by the caller: they are only read, and the write pointers may be null.
template <int D>
__global__ __launch_bounds__(D) void finalize_step_kernel(const RowInfo *__restrict__ rows_in,
                                                          const RowInfo *__restrict__ rows_out, int Hkv, int Hq, int G,
                                                          const float *__restrict__ part_o_in,
                                                          const float *__restrict__ part_lse_in,
                                                          const float *__restrict__ part_o_out,
                                                          const float *__restrict__ part_lse_out, const float *a_in_r,
                                                          const float *lse_in_r, float *a_in, float *lse_in,
                                                          float *a_out, float *lse_out, float *__restrict__ y,
                                                          float *__restrict__ lse, float *__restrict__ w_in)
{
    __shared__ float sm_w[kCombineStage];
    __shared__ float sm_red[D];
    // grid (users, Hkv, G): the indices come as they are (a 64-bit division here was ~150 dependent scalar instructions
    // in front of a kernel that lasts 4 us)
    const int user = blockIdx.x, kvh = blockIdx.y, g = blockIdx.z;
    const int64_t row = (int64_t)user * Hq + kvh * G + g;
    const int tid = threadIdx.x;
    const RowInfo ri = rows_in ? rows_in[user * Hkv + kvh] : RowInfo{0, 1}, ro = rows_out[user * Hkv + kvh];
    // Measured on this kernel (4 us, pure latency): the 8-wide straight-line form is the fastest for rows of up to 8
    // chunks; loading both owners' pairs in one go, or 16-wide for everything, made it 1.3-2.3 us slower.
    constexpr int kSmall = 8, kMedium = 16;
    float x0, l0, x1, l1;
    if (ri.n_chunks > 1 && ri.n_chunks <= kSmall) {
        combine_row_small<D, kSmall>(part_lse_in + (int64_t)ri.first_slot * G + g,
                                     part_o_in + ((int64_t)ri.first_slot * G + g) * D + tid, ri.n_chunks, G, x0, l0);
        a_in[row * D + tid] = x0;
        if (tid == 0)
            lse_in[row] = l0;
    } else if (ri.n_chunks > 1 && ri.n_chunks <= kMedium) {
        combine_row_small<D, kMedium>(part_lse_in + (int64_t)ri.first_slot * G + g,
                                      part_o_in + ((int64_t)ri.first_slot * G + g) * D + tid, ri.n_chunks, G, x0, l0);
        a_in[row * D + tid] = x0;
        if (tid == 0)
            lse_in[row] = l0;
    } else if (ri.n_chunks > 1) {
        combine_row<D>(part_lse_in + (int64_t)ri.first_slot * G + g,
                       part_o_in + ((int64_t)ri.first_slot * G + g) * D + tid, ri.n_chunks, G, sm_w, sm_red, x0, l0);
        a_in[row * D + tid] = x0;
        if (tid == 0)
            lse_in[row] = l0;
    } else {
        x0 = a_in_r[row * D + tid];
        l0 = lse_in_r[row];
    }
    if (ro.n_chunks > 1 && ro.n_chunks <= kSmall) {
        combine_row_small<D, kSmall>(part_lse_out + (int64_t)ro.first_slot * G + g,
                                     part_o_out + ((int64_t)ro.first_slot * G + g) * D + tid, ro.n_chunks, G, x1, l1);
        a_out[row * D + tid] = x1;
        if (tid == 0)
            lse_out[row] = l1;
    } else if (ro.n_chunks > 1) {
        combine_row<D>(part_lse_out + (int64_t)ro.first_slot * G + g,
                       part_o_out + ((int64_t)ro.first_slot * G + g) * D + tid, ro.n_chunks, G, sm_w, sm_red, x1, l1);
        a_out[row * D + tid] = x1;
        if (tid == 0)
            lse_out[row] = l1;
    } else {
        x1 = a_out[row * D + tid];
        l1 = lse_out[row];
    }
    float w0, w1, ls;
    merge_weights(l0, l1, w0, w1, ls);
    y[row * D + tid] = (w0 == 0.f ? 0.f : w0 * x0) + (w1 == 0.f ? 0.f : w1 * x1);
    if (tid == 0) {
        lse[row] = ls;
        w_in[row] = w0;
    }
}

// one thread per 4 channels of one row; block (vec_per_row, rows per block)
__global__ __launch_bounds__(256) void lse_merge_kernel(int n_rows, int vec_per_row, const float *a0,
                                                         const float *__restrict__ lse0, const float *a1,
                                                         const float *__restrict__ lse1, float *y,
                                                         float *__restrict__ lse_out, float *__restrict__ w0_out)
{
    const int64_t row = (int64_t)blockIdx.x * blockDim.y + threadIdx.y;
    if (row >= n_rows)
        return;
    const int64_t i = row * vec_per_row + threadIdx.x;
    float w0, w1, ls;
    merge_weights(lse0[row], lse1[row], w0, w1, ls);
    const f32x4 x0 = reinterpret_cast<const f32x4 *>(a0)[i];
    const f32x4 x1 = reinterpret_cast<const f32x4 *>(a1)[i];
    f32x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        r[e] = (w0 == 0.f ? 0.f : w0 * x0[e]) + (w1 == 0.f ? 0.f : w1 * x1[e]);  // a zero weight ignores its side entirely
    reinterpret_cast<f32x4 *>(y)[i] = r;
    if (threadIdx.x == 0) {
        if (lse_out)
            lse_out[row] = ls;
        if (w0_out)
            w0_out[row] = w0;
    }
}

// The merge for up to SPD_MAX_MERGE_PARTS owners; the part pointers travel in the kernel arguments.
struct MergeParts {
    const float *a[SPD_MAX_MERGE_PARTS];
    const float *lse[SPD_MAX_MERGE_PARTS];
};

// one thread per 4 channels of one row; block (vec_per_row, rows per block).  Every part's row is loaded before y is
// written, so y may alias a part.
__global__ __launch_bounds__(256) void lse_merge_n_kernel(int n_parts, int n_rows, int vec_per_row, MergeParts p,
                                                           float *y, float *__restrict__ lse_out,
                                                           float *__restrict__ w_out)
{
    const int64_t row = (int64_t)blockIdx.x * blockDim.y + threadIdx.y;
    if (row >= n_rows)
        return;
    const int64_t i = row * vec_per_row + threadIdx.x;
    float l[SPD_MAX_MERGE_PARTS];
    f32x4 x[SPD_MAX_MERGE_PARTS];
    float top = -INFINITY;
#pragma unroll
    for (int k = 0; k < SPD_MAX_MERGE_PARTS; ++k) {
        if (k < n_parts) {  // n_parts is uniform: the loads of all parts are in flight together
            l[k] = p.lse[k][row];
            x[k] = reinterpret_cast<const f32x4 *>(p.a[k])[i];
            top = fmaxf(top, l[k]);
        }
    }
    float den = 0.f;
    f32x4 r = {0.f, 0.f, 0.f, 0.f};
    float w[SPD_MAX_MERGE_PARTS];
#pragma unroll
    for (int k = 0; k < SPD_MAX_MERGE_PARTS; ++k) {
        if (k < n_parts) {
            w[k] = top == -INFINITY ? 0.f : fast_exp(l[k] - top);  // exactly 0 for an empty part, exactly 1 for the largest
            den += w[k];
        }
    }
    const float inv = den > 0.f ? 1.f / den : 0.f;
#pragma unroll
    for (int k = 0; k < SPD_MAX_MERGE_PARTS; ++k) {
        if (k < n_parts) {
            w[k] *= inv;
            if (w[k] != 0.f)  // a zero weight ignores its part entirely (it may hold anything)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    r[e] = fmaf(w[k], x[k][e], r[e]);
        }
    }
    reinterpret_cast<f32x4 *>(y)[i] = r;
    if (threadIdx.x == 0) {
        if (lse_out)
            lse_out[row] = den > 0.f ? top + fast_log(den) : -INFINITY;
        if (w_out)
#pragma unroll
            for (int k = 0; k < SPD_MAX_MERGE_PARTS; ++k)
                if (k < n_parts)
                    w_out[(int64_t)k * n_rows + row] = w[k];
    }
}

// Copies a freshly built schedule from its pinned host staging buffer to device memory (n16 16-byte words).
__global__ __launch_bounds__(256) void upload_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, unsigned n16)
{
    const unsigned i = blockIdx.x * 256u + threadIdx.x;
    if (i < n16)
        dst[i] = src[i];
}

// Folds one decode step's private attention masses into running per-row statistics (minimum, sum, count below a
// threshold); any of the three outputs may be null.
__global__ __launch_bounds__(256) void mass_track_kernel(int n_rows, const float *__restrict__ w_in, float threshold,
                                                          float *mass_min, float *mass_sum, int32_t *n_below)
{
    const int i = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    if (i >= n_rows)
        return;
    const float w = w_in[i];
    if (mass_min)
        mass_min[i] = fminf(mass_min[i], w);
    if (mass_sum)
        mass_sum[i] += w;
    if (n_below && w < threshold)
        n_below[i] += 1;
}

}  // namespace spd
