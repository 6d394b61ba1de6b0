// Combination rules of Theorem 1 (paper section 4.2) written on log-sum-exps.
//
//   combine_chunks_kernel  n-way form, used inside one owner's call: the chunks c of a (user, KV head) row each hold
//                          (A_c, lse_c); lse = logsumexp_c lse_c and A = sum_c exp(lse_c - lse) A_c.
//                          Rows with no token get A = 0, lse = -inf; rows with one chunk were already written by the
//                          partial kernel and are skipped.
//   lse_merge_kernel       the two-owner merge itself: Y = w0 A_in + w1 A_out with w_x = exp(lse_x - lse).
//                          With lse_x = m_x + ln gamma_x these weights equal the paper's
//                          gamma_in / (gamma_in + alpha gamma_out) and gamma_out / (alpha^-1 gamma_in + gamma_out),
//                          alpha = exp(m_out - m_in), but never form alpha, which overflows fp32 for
//                          |m_out - m_in| > 88.
#pragma once
#include "common.hpp"

namespace spd {

// grid: U * Hkv blocks of D threads (thread = channel), D in {64, 128}.  Chunks are read in index order, so the
// result does not depend on which workgroup finished first.
template <int D>
__global__ __launch_bounds__(D) void combine_chunks_kernel(const RowInfo *__restrict__ rows, int Hkv, int Hq, int G,
                                                           const float *__restrict__ part_o,
                                                           const float *__restrict__ part_lse,
                                                           float *__restrict__ out, float *__restrict__ lse)
{
    const RowInfo ri = rows[blockIdx.x];
    if (ri.n_chunks == 1)
        return;
    const int user = blockIdx.x / Hkv, kvh = blockIdx.x % Hkv;
    const int ch = threadIdx.x;
    for (int g = 0; g < G; ++g) {
        const int64_t row = (int64_t)user * Hq + (int64_t)kvh * G + g;
        float M = -INFINITY;
        for (int c = 0; c < ri.n_chunks; ++c)
            M = fmaxf(M, part_lse[(int64_t)(ri.first_slot + c) * G + g]);
        float o = 0.f, den = 0.f;
        for (int c = 0; c < ri.n_chunks; ++c) {
            const int64_t s = (int64_t)(ri.first_slot + c) * G + g;
            const float w = expf(part_lse[s] - M);   // chunks are never empty, so M is finite here
            den += w;
            o = fmaf(w, part_o[s * D + ch], o);
        }
        const bool empty = ri.n_chunks == 0;
        out[row * D + ch] = empty ? 0.f : o / den;
        if (ch == 0)
            lse[row] = empty ? -INFINITY : M + logf(den);
    }
}

// one thread per 4 channels of one row
__global__ __launch_bounds__(256) void lse_merge_kernel(int64_t n_vec, int vec_per_row, const float *__restrict__ a0,
                                                         const float *__restrict__ lse0, const float *__restrict__ a1,
                                                         const float *__restrict__ lse1, float *__restrict__ y,
                                                         float *__restrict__ lse_out, float *__restrict__ w0_out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_vec)
        return;
    const int64_t row = i / vec_per_row;
    const float l0 = lse0[row], l1 = lse1[row];
    const float M = fmaxf(l0, l1);
    float w0, w1, ls;
    if (M == -INFINITY) {  // both owners hold no token for this row
        w0 = 0.f, w1 = 0.f, ls = -INFINITY;
    } else {
        const float e0 = expf(l0 - M), e1 = expf(l1 - M);  // the larger one is exactly 1
        const float den = e0 + e1;
        w0 = e0 / den;
        w1 = e1 / den;
        ls = M + logf(den);
    }
    const f32x4 x0 = reinterpret_cast<const f32x4 *>(a0)[i];
    const f32x4 x1 = reinterpret_cast<const f32x4 *>(a1)[i];
    f32x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        r[e] = (w0 == 0.f ? 0.f : w0 * x0[e]) + (w1 == 0.f ? 0.f : w1 * x1[e]);  // a zero weight ignores its side entirely
    reinterpret_cast<f32x4 *>(y)[i] = r;
    if (i % vec_per_row == 0) {
        if (lse_out)
            lse_out[row] = ls;
        if (w0_out)
            w0_out[row] = w0;
    }
}

}  // namespace spd
