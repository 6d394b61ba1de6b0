// Argument validation of the partial-attention calls (host only, no HIP calls): every condition the kernels rely
// on - shapes the kernels are instantiated for, 16-byte aligned rows, lengths inside the block table - is checked
// here before anything is enqueued.
#pragma once
#include <cmath>
#include <cstdint>

#include "../../include/spd.h"
#include "common.hpp"

namespace spd::host {

constexpr int32_t kMaxLen = 1 << 30;  // tokens per user: token indices and their 32-token steps stay inside int32

// log2 of a page size the kernels take (16, 32, 64, 128 or 256 tokens), else -1.
inline int page_shift(int block_size)
{
    for (int s = 4; s <= 8; ++s)
        if (block_size == (1 << s))
            return s;
    return -1;
}

inline int elt_size(int dtype) { return dtype == SPD_F32 ? 4 : 2; }

inline int validate_shape(const spd_shape *s)
{
    if (!s)
        return SPD_ERR_NULL;
    if (s->dtype != SPD_F32 && s->dtype != SPD_BF16 && s->dtype != SPD_F16)
        return SPD_ERR_SHAPE;
    if (s->n_q_heads <= 0 || s->n_kv_heads <= 0 || s->n_q_heads % s->n_kv_heads != 0)
        return SPD_ERR_SHAPE;
    if (s->n_kv_heads > 65535)  // a grid dimension of the closing kernel
        return SPD_ERR_SHAPE;
    const int G = s->n_q_heads / s->n_kv_heads;
    if (s->head_dim != 64 && s->head_dim != 128)
        return SPD_ERR_SHAPE;
    if (G > spd::kMaxGroup)  // an MFMA tile holds 16 heads
        return SPD_ERR_SHAPE;
    if (!std::isfinite(s->scale))
        return SPD_ERR_SHAPE;
    return SPD_OK;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int validate_view(const spd_shape *s, const spd_kv_view *v)
{
    if (!v)
        return SPD_ERR_NULL;
    if (v->n_users < 0)
        return SPD_ERR_LEN;
    if (v->n_users > 0 && !v->lens)
        return SPD_ERR_NULL;
    const int es = elt_size(s->dtype);
    if (v->block_size != 0 && page_shift(v->block_size) < 0)
        return SPD_ERR_SHAPE;
    bool any = false;
    for (int u = 0; u < v->n_users; ++u) {
        if (v->lens[u] < 0 || v->lens[u] > kMaxLen)
            return SPD_ERR_LEN;
        any = any || v->lens[u] > 0;
    }
    // rows are read with 16-byte loads: strides must keep every row 16-byte aligned and rows must not overlap
    if (v->token_stride < s->head_dim || (v->token_stride * es) % 16 != 0)
        return any ? SPD_ERR_ALIGN : SPD_OK;
    if (v->head_stride < 0 || (v->head_stride * es) % 16 != 0)
        return any ? SPD_ERR_ALIGN : SPD_OK;
    if (v->head_strides && v->block_size == 0)
        for (int u = 0; u < v->n_users; ++u)
            if (v->lens[u] > 0 && (v->head_strides[u] < 0 || (v->head_strides[u] * es) % 16 != 0))
                return SPD_ERR_ALIGN;
    if (v->block_size == 0) {
        if (any && (!v->k_ptrs || !v->v_ptrs))
            return SPD_ERR_NULL;
        if ((v->k_ptrs_dev != nullptr) != (v->v_ptrs_dev != nullptr))  // device pointer tables: both or neither
            return SPD_ERR_NULL;
        if ((reinterpret_cast<uintptr_t>(v->k_ptrs_dev) | reinterpret_cast<uintptr_t>(v->v_ptrs_dev)) & 7u)
            return SPD_ERR_ALIGN;
        for (int u = 0; u < v->n_users; ++u) {
            if (v->lens[u] == 0)
                continue;
            if (!v->k_ptrs[u] || !v->v_ptrs[u])
                return SPD_ERR_NULL;
            if (!aligned16(v->k_ptrs[u]) || !aligned16(v->v_ptrs[u]))
                return SPD_ERR_ALIGN;
        }
    } else {
        if (v->max_blocks < 0)
            return SPD_ERR_LEN;
        for (int u = 0; u < v->n_users; ++u)
            if (((int64_t)v->lens[u] + v->block_size - 1) / v->block_size > v->max_blocks)
                return SPD_ERR_LEN;
        if (any) {
            if (!v->k_pool || !v->v_pool || !v->block_table)
                return SPD_ERR_NULL;
            if (!aligned16(v->k_pool) || !aligned16(v->v_pool) || (reinterpret_cast<uintptr_t>(v->block_table) & 3u))
                return SPD_ERR_ALIGN;
            if (v->block_stride <= 0 || (v->block_stride * es) % 16 != 0)
                return SPD_ERR_ALIGN;
        }
    }
    return SPD_OK;
}

}  // namespace spd::host
