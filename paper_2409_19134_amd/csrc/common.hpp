// Shared device-side declarations of the SPD decode-attention kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/spd.h"

namespace spd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;            // waves per workgroup in the partial-attention kernels
constexpr int kThreads = kWaves * 64;
constexpr int kMaxGroup = 16;        // query heads per KV head the MFMA tile can hold
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Addressing of one owner's cache; all strides in BYTES.
struct KvAddr {
    const char *const *k_ptrs;   // contiguous mode: device array of per-user base pointers
    const char *const *v_ptrs;
    const char *k_pool;          // paged mode
    const char *v_pool;
    const int32_t *block_table;
    int32_t max_blocks;
    int64_t block_stride;
    int64_t token_stride;
    int64_t head_stride;
};

// first partial slot and chunk count of one (user, KV head) row
struct RowInfo {
    int32_t first_slot;
    int32_t n_chunks;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float wave_xor_max(float v, int mask) { return fmaxf(v, __shfl_xor(v, mask)); }

}  // namespace spd
