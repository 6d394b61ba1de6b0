// Partial attention over one chunk of one (user, KV head): vector-ALU path for fp32 inputs
// (head_dim 64 or 128) where products must be formed in fp32 and the tile is too thin for MFMA.
//
// Computes the same quantity as the MFMA kernel (paper section 4.2: A = softmax(s) V and
// lse = ln sum exp(s) over a token range).  A row of D channels is covered by LPR = D/4 lanes (16 bytes each),
// so one wave reads 64/LPR full rows per load; every lane group keeps its own online-softmax state
// (m, l, acc) for the G query heads of the KV head and the groups are merged at the end with the
// n-way form of Theorem 1 (first across lane groups by cross-lane exchanges, then across waves in LDS).
#pragma once
#include "common.hpp"

namespace spd {

template <int D, int G>
__global__ __launch_bounds__(kThreads) void partial_f32_kernel(
    OwnerArgs a0, OwnerArgs a1, int n0, const float *__restrict__ q, int Hq, float scale_log2e)
{
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
    constexpr int EPL = 4;          // fp32 elements per 16-byte lane load
    constexpr int LPR = D / EPL;    // lanes per row: 16 (D=64) or 32 (D=128)
    constexpr int RPW = 64 / LPR;   // rows per wave per step
    __shared__ float sm_m[kWaves][G];
    __shared__ float sm_l[kWaves][G];
    __shared__ float sm_o[kWaves][G][D];

    DevItem fetched = items[second ? (int)blockIdx.x - n0 : (int)blockIdx.x];
    for (;;) {
        const DevItem it = fetched;
        if (it.next >= 0)  // fetch the piece's next segment early; it is looked at only when this one is done
            fetched = items[it.next];
        if (it.n_chunks == 0) {  // a row without tokens is a piece of its own
            write_empty_row<D>(it, G, Hq, out, lse);
            return;
        }
        const int lane = threadIdx.x & 63;
        const int wave = threadIdx.x >> 6;
        const int cl = lane % LPR;      // which 4-channel slice of the row
        const int rs = lane / LPR;      // which row of the step

        const bool paged = kv.block_table != nullptr;
        const char *k_base = it.k_base + k_pool + user_base(k_ptrs, it.user);
        const char *v_base = it.v_base + v_pool + user_base(v_ptrs, it.user);
        const int32_t *bt_row = paged ? kv.block_table + (int64_t)it.user * kv.max_blocks : nullptr;

        float qr[G][EPL];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const f32x4 w = *reinterpret_cast<const f32x4 *>(
                q + ((int64_t)it.user * Hq + (int64_t)it.kv_head * G + g) * D + cl * EPL);
#pragma unroll
            for (int e = 0; e < EPL; ++e)
                qr[g][e] = w[e];
        }

        float m[G], l[G], acc[G][EPL];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            m[g] = -INFINITY;
            l[g] = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e)
                acc[g][e] = 0.f;
        }

        const int t_last = it.t_end - 1;
        // KV append: the row's last token is the new one; it is read from the caller's buffer and wave 0 copies it into
        // the cache (lanes [0, LPR): K, [LPR, 2*LPR): V; 2*LPR <= 64)
        const char *k_new_row = nullptr, *v_new_row = nullptr;
        if (k_new && (it.rot & kEndsRow)) {
            const int64_t row = ((int64_t)it.user * (Hq / G) + it.kv_head) * D * 4;
            k_new_row = k_new + row;
            v_new_row = v_new + row;
            if (wave == 0 && lane < 2 * LPR) {
                int64_t off = paged ? (int64_t)bt_row[t_last >> 4] * kv.block_stride + (int64_t)(t_last & 15) * kv.token_stride
                                    : (int64_t)t_last * kv.token_stride;
                off += (lane % LPR) * 16;
                if (lane < LPR)
                    copy16(const_cast<char *>(k_base) + off, k_new_row + (lane % LPR) * 16);
                else
                    copy16(const_cast<char *>(v_base) + off, v_new_row + (lane % LPR) * 16);
            }
        }
        // kUnroll steps of loads are issued before the first is used: the workloads that take this kernel are small and
        // latency-bound, so what counts is the number of dependent memory round trips per wave
        constexpr int kUnroll = 4;
        for (int tb = it.t_begin + wave * RPW; tb < it.t_end; tb += RPW * kWaves * kUnroll) {
            f32x4 kk[kUnroll], vv[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int tc = min(tb + u * RPW * kWaves + rs, t_last);  // rows past the chunk re-read its last token
                int64_t off;
                if (paged)
                    off = (int64_t)bt_row[tc >> 4] * kv.block_stride + (int64_t)(tc & 15) * kv.token_stride;
                else
                    off = (int64_t)tc * kv.token_stride;
                off += cl * 16;
                const bool is_new = k_new_row && tc == t_last;
                kk[u] = *reinterpret_cast<const f32x4 *>(is_new ? k_new_row + cl * 16 : k_base + off);
                vv[u] = *reinterpret_cast<const f32x4 *>(is_new ? v_new_row + cl * 16 : v_base + off);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int t = tb + u * RPW * kWaves + rs;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float s = qr[g][0] * kk[u][0];
                    s = fmaf(qr[g][1], kk[u][1], s);
                    s = fmaf(qr[g][2], kk[u][2], s);
                    s = fmaf(qr[g][3], kk[u][3], s);
#pragma unroll
                    for (int o = 1; o < LPR; o <<= 1)
                        s += __shfl_xor(s, o);          // all LPR lanes of the row end up with the full dot product
                    if (t < it.t_end) {
                        const float x = s * scale_log2e;
                        const float m_new = fmaxf(m[g], x);
                        const float alpha = fast_exp2(m[g] - m_new);
                        const float p = fast_exp2(x - m_new);
                        l[g] = l[g] * alpha + p;
#pragma unroll
                        for (int e = 0; e < EPL; ++e)
                            acc[g][e] = fmaf(p, vv[u][e], acc[g][e] * alpha);
                        m[g] = m_new;
                    }
                }
            }
        }

        // merge the RPW lane groups of the wave (they hold disjoint token subsets)
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float mw = m[g];
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1)
                mw = fmaxf(mw, __shfl_xor(mw, o));
            const float f = (mw == -INFINITY) ? 0.f : fast_exp2(m[g] - mw);
            float lw = l[g] * f;
            float a[EPL];
#pragma unroll
            for (int e = 0; e < EPL; ++e)
                a[e] = acc[g][e] * f;
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) {
                lw += __shfl_xor(lw, o);
#pragma unroll
                for (int e = 0; e < EPL; ++e)
                    a[e] += __shfl_xor(a[e], o);
            }
            if (rs == 0) {
                if (cl == 0) {
                    sm_m[wave][g] = mw;
                    sm_l[wave][g] = lw;
                }
#pragma unroll
                for (int e = 0; e < EPL; ++e)
                    sm_o[wave][g][cl * EPL + e] = a[e];
            }
        }
        __syncthreads();

        const bool direct = it.n_chunks == 1;
        const int64_t head0 = (int64_t)it.user * Hq + (int64_t)it.kv_head * G;
        const int64_t slot = it.slot;
        for (int idx = threadIdx.x; idx < G * D; idx += kThreads) {
            const int g = idx / D, ch = idx % D;
            float Mg = sm_m[0][g];
#pragma unroll
            for (int w = 1; w < kWaves; ++w)
                Mg = fmaxf(Mg, sm_m[w][g]);
            float o = 0.f, lt = 0.f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                const float f = (sm_m[w][g] == -INFINITY) ? 0.f : fast_exp2(sm_m[w][g] - Mg);
                o += sm_o[w][g][ch] * f;
                lt += sm_l[w][g] * f;
            }
            const float a = o * fast_rcp(lt);
            if (direct)
                out[(head0 + g) * D + ch] = a;
            else
                part_o[(slot * G + g) * D + ch] = a;
            if (ch == 0) {
                const float ls = (Mg + fast_log2(lt)) * kLn2;  // Mg is in log2 units
                if (direct)
                    lse[head0 + g] = ls;
                else
                    part_lse[slot * G + g] = ls;
            }
        }
        if (it.next < 0)
            return;
        __syncthreads();  // the LDS staging arrays are reused by the next segment
    }
}

}  // namespace spd
