// Shared device-side declarations of the SPD decode-attention kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/spd.h"

namespace spd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 4;            // waves per workgroup in the partial-attention kernels
constexpr int kThreads = kWaves * 64;
constexpr int kMaxGroup = 16;        // query heads per KV head the MFMA tile can hold
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Addressing of one owner's cache; all strides in BYTES.  Base pointers travel in the work items.
struct KvAddr {
    const int32_t *block_table;  // paged mode only, else nullptr
    int32_t max_blocks;
    int32_t page_shift;  // paged mode: a page holds 1 << page_shift tokens (16 .. 256)
    int64_t block_stride;
    int64_t token_stride;
    int64_t head_stride;  // used by the head-per-wave kernel only (token-major storage: the same for every user)
};

// One segment of work as the kernels read it: tokens [t_begin, t_end) of one (user, KV head) row.  A workgroup
// processes a *piece*: a short list of segments linked by `next` (a piece that crosses a row boundary has one
// segment per row it touches).  k_base / v_base point at channel 0 of token 0 of the row (contiguous mode) or at the
// KV head's offset inside the pool (paged mode: a byte offset stored as a pointer, the pool base travels in OwnerArgs).  n_chunks == 0 marks a row without tokens: the workgroup only
// writes A = 0, lse = -inf.
struct DevItem {
    const char *k_base;
    const char *v_base;
    int32_t user, kv_head, t_begin, t_end;
    int32_t slot;      // where this segment's partial goes when the row has several segments (head-per-wave pieces:
                       // the slot of KV head 0; head h writes slot + h * n_chunks)
    int32_t n_chunks;  // segments of the row; 1: the segment writes the final result itself
    int32_t next;      // index of the piece's next segment, -1 if none
    int32_t rot;       // bits 0-1: 32-token steps the piece has already handed out (mod 4), keeps the four waves
                       // evenly loaded; bit 8 (kEndsRow): the segment ends at the last token of its row
};
constexpr int kEndsRow = 0x100;

// 16-byte load of K/V data that is read exactly once: the non-temporal hint keeps the stream from displacing
// other lines in L2 (measured: plain streaming reads reach ~6.3 TB/s on this GPU, non-temporal ones ~7.1 TB/s).
// The pointer is cast to the global address space: base pointers arrive through memory (the work items), where the
// compiler cannot see the address space and would otherwise emit slower FLAT loads that also tie up the LDS counter.
template <typename V>  // V: u32x4 (16 bytes) or u32x2 (8 bytes)
__device__ __forceinline__ V stream_load(const char *p)
{
    typedef const V __attribute__((address_space(1))) *global_ptr;
    return __builtin_nontemporal_load((global_ptr)(uintptr_t)p);
}
__device__ __forceinline__ u32x4 stream_load16(const char *p) { return stream_load<u32x4>(p); }

// Wave-uniform values (work item fields arrive through vector loads): tell the compiler, so that address arithmetic
// and the block-table lookups go to the scalar unit.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ const char *uniform(const char *p)
{
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const char *>(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ DevItem uniform(const DevItem &it)
{
    DevItem u;
    u.k_base = uniform(it.k_base);
    u.v_base = uniform(it.v_base);
    u.user = uniform(it.user);
    u.kv_head = uniform(it.kv_head);
    u.t_begin = uniform(it.t_begin);
    u.t_end = uniform(it.t_end);
    u.slot = uniform(it.slot);
    u.n_chunks = uniform(it.n_chunks);
    u.next = uniform(it.next);
    u.rot = uniform(it.rot);
    return u;
}

// A work item read through the scalar cache (items are constant during a launch, the index is wave-uniform): the
// fields land in scalar registers and cost no vector registers while they wait to be used.
typedef const uint32_t __attribute__((address_space(4))) *const_u32_ptr;
__device__ __forceinline__ DevItem scalar_load_item(const DevItem *items, int idx)
{
    static_assert(sizeof(DevItem) == 48, "DevItem is read as 12 dwords");
    const const_u32_ptr w = (const_u32_ptr)(uintptr_t)(items + idx);
    DevItem it;
    it.k_base = reinterpret_cast<const char *>(((uint64_t)w[1] << 32) | w[0]);
    it.v_base = reinterpret_cast<const char *>(((uint64_t)w[3] << 32) | w[2]);
    it.user = (int32_t)w[4];
    it.kv_head = (int32_t)w[5];
    it.t_begin = (int32_t)w[6];
    it.t_end = (int32_t)w[7];
    it.slot = (int32_t)w[8];
    it.n_chunks = (int32_t)w[9];
    it.next = (int32_t)w[10];
    it.rot = (int32_t)w[11];
    return it;
}

// Block-table entry read through the scalar cache (the table is constant during a launch and the index is
// wave-uniform): it neither waits behind the vector loads of the K/V stream nor delays them.
typedef const int32_t __attribute__((address_space(4))) *const_i32_ptr;
__device__ __forceinline__ int scalar_load_i32(const int32_t *p, int idx)
{
    return ((const_i32_ptr)(uintptr_t)p)[idx];
}

// A user's base pointer from a device pointer table, as an integer to add to the item's offset (0 without a table).
// Scalar cache: the table is constant during a launch and the index wave-uniform.
typedef const uint64_t __attribute__((address_space(4))) *const_u64_ptr;
__device__ __forceinline__ uintptr_t user_base(const char *const *table, int user)
{
    return table ? (uintptr_t)((const_u64_ptr)(uintptr_t)table)[user] : 0;
}

__device__ __forceinline__ void copy16(char *dst, const char *src)
{
    *reinterpret_cast<u32x4 *>(dst) = *reinterpret_cast<const u32x4 *>(src);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// hardware log2 and reciprocal (1 ulp): the epilogues are latency, every library call in them is a dozen instructions
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

// Exchanges between the four 16-lane groups of a wave (lane ^ 16, lane ^ 32) without a trip through the LDS crossbar:
// v_permlane16_swap trades the odd 16-lane rows of its first operand for the even rows of its second, v_permlane32_swap
// the upper half of the first for the lower half of the second.  Fed the same value twice, the two results hold, in
// every lane, the lane's own value and its partner's (in one order or the other), which is all a max or a sum needs.
template <int MASK>
__device__ __forceinline__ void wave_xor_pair(float v, float &a, float &b)
{
    static_assert(MASK == 16 || MASK == 32, "lane groups are 16 lanes wide");
    const unsigned u = __float_as_uint(v);
    if constexpr (MASK == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
        a = __uint_as_float(r[0]);
        b = __uint_as_float(r[1]);
    } else {
        const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
        a = __uint_as_float(r[0]);
        b = __uint_as_float(r[1]);
    }
}
template <int MASK>
__device__ __forceinline__ float wave_xor_max(float v)
{
    float a, b;
    wave_xor_pair<MASK>(v, a, b);
    return fmaxf(a, b);
}
template <int MASK>
__device__ __forceinline__ float wave_xor_sum(float v)
{
    float a, b;
    wave_xor_pair<MASK>(v, a, b);
    return a + b;
}

// Rows without tokens (Theorem 1 with an empty part): A = 0, lse = -inf for the G heads of the row.
template <int D>
__device__ __forceinline__ void write_empty_row(const DevItem &it, int G, int Hq, float *out, float *lse)
{
    const int64_t head0 = (int64_t)it.user * Hq + (int64_t)it.kv_head * G;
    for (int idx = threadIdx.x; idx < G * D; idx += blockDim.x)
        out[head0 * D + idx] = 0.f;
    if ((int)threadIdx.x < G)
        lse[head0 + threadIdx.x] = -INFINITY;
}

// Everything a partial kernel needs to know about one owner's call.  A launch serves one owner, or - for the fused
// decode step - both at once: workgroups [0, n0) take owner 0's pieces, the rest owner 1's.
struct OwnerArgs {
    const DevItem *items;
    const char *k_pool;  // paged mode: the items' k_base / v_base are byte offsets inside these; else nullptr
    const char *v_pool;
    // contiguous mode with device pointer tables: the items' k_base / v_base are byte offsets from k_ptrs[user] /
    // v_ptrs[user] (so that the schedule does not depend on the buffers' addresses); else nullptr
    const char *const *k_ptrs;
    const char *const *v_ptrs;
    KvAddr kv;
    float *part_o;    // [slots][G][D] chunk partials of split rows
    float *part_lse;  // [slots][G]
    float *out;       // [U][Hq][D]
    float *lse;       // [U][Hq]
    // KV append (protocol step 3a), or nullptr: [U][Hkv][D] rows of the new token's K and V.  The row's last token
    // (position lens[u] - 1) is then taken from here, and the segment that ends the row also writes it to the cache.
    const char *k_new;
    const char *v_new;
    // Tokens every row has gained since the schedule was built (a decode loop appends one token per user and step):
    // added to t_end of the segments that end their row, so that a schedule serves several consecutive steps.
    int32_t grow;
};

// A work item with the row's growth applied.
__device__ __forceinline__ DevItem scalar_load_item(const DevItem *items, int idx, int grow)
{
    DevItem it = scalar_load_item(items, idx);
    it.t_end += (it.rot & kEndsRow) ? grow : 0;
    return it;
}

// A row (user, KV head) whose tokens were split into several chunks.
struct CombineRow {
    int32_t first_slot, n_chunks, user, kv_head;
};

// Chunk bookkeeping of every (user, KV head) row, indexed user * Hkv + kv_head.
struct RowInfo {
    int32_t first_slot, n_chunks;
};

// The partial kernel's arguments.
struct PartialArgs {
    OwnerArgs a0, a1;
    int32_t n0;             // workgroups [0, n0) serve a0, the rest a1
    const char *q;          // [U][Hq][D]
    int32_t Hq, G;
    float scale_log2e;
    int32_t ring_rows;      // result rows a workgroup may hold back in LDS (see the result ring in partial_mfma.hpp); 0: none
};
}  // namespace spd
