// Host side of the SPD decode-attention library: C ABI, argument validation, split schedule, launches.
// The calls follow the paper's decode protocol (section 4, step 3b/3c) and Theorem 1 (section 4.2).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "combine.hpp"
#include "common.hpp"
#include "partial_bf16_mfma.hpp"
#include "partial_generic.hpp"

namespace {

using spd::KvAddr;
using spd::RowInfo;

constexpr int kCacheEntries = 8;     // remembered schedules per entry point
constexpr int kChunkAlign = 32;      // chunk boundaries are multiples of the MFMA kernel's 32-token step
constexpr int kChunkMin = 128;       // one step for each of the four waves
constexpr int kChunkMaxDefault = 1024;
constexpr int kTargetWgPerCuDefault = 3;

int env_int(const char *name, int dflt)
{
    const char *s = std::getenv(name);
    if (!s || !*s)
        return dflt;
    const long v = std::strtol(s, nullptr, 10);
    return v > 0 ? (int)v : dflt;
}

int elt_size(int dtype) { return dtype == SPD_F32 ? 4 : 2; }

int validate_shape(const spd_shape *s)
{
    if (!s)
        return SPD_ERR_NULL;
    if (s->dtype != SPD_F32 && s->dtype != SPD_BF16)
        return SPD_ERR_SHAPE;
    if (s->n_q_heads <= 0 || s->n_kv_heads <= 0 || s->n_q_heads % s->n_kv_heads != 0)
        return SPD_ERR_SHAPE;
    const int G = s->n_q_heads / s->n_kv_heads;
    if (s->dtype == SPD_BF16) {
        if (s->head_dim != 128 || G > spd::kMaxGroup)
            return SPD_ERR_SHAPE;
    } else {
        if (s->head_dim != 64 && s->head_dim != 128)
            return SPD_ERR_SHAPE;
        if (G != 1 && G != 2 && G != 4 && G != 8)
            return SPD_ERR_SHAPE;
    }
    if (!std::isfinite(s->scale))
        return SPD_ERR_SHAPE;
    return SPD_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int validate_view(const spd_shape *s, const spd_kv_view *v)
{
    if (!v)
        return SPD_ERR_NULL;
    if (v->n_users < 0)
        return SPD_ERR_LEN;
    if (v->n_users > 0 && !v->lens)
        return SPD_ERR_NULL;
    const int es = elt_size(s->dtype);
    if (v->block_size != 0 && v->block_size != 16)
        return SPD_ERR_SHAPE;
    bool any = false;
    for (int u = 0; u < v->n_users; ++u) {
        if (v->lens[u] < 0)
            return SPD_ERR_LEN;
        any = any || v->lens[u] > 0;
    }
    // rows are read with 16-byte loads: strides must keep every row 16-byte aligned and rows must not overlap
    if (v->token_stride < s->head_dim || (v->token_stride * es) % 16 != 0)
        return any ? SPD_ERR_ALIGN : SPD_OK;
    if (v->head_stride < 0 || (v->head_stride * es) % 16 != 0)
        return any ? SPD_ERR_ALIGN : SPD_OK;
    if (v->block_size == 0) {
        if (any && (!v->k_ptrs || !v->v_ptrs))
            return SPD_ERR_NULL;
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
            if (((int64_t)v->lens[u] + 15) / 16 > v->max_blocks)
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

// Target chunk length (tokens) for a total of `tokens` per KV head over all users.
int pick_chunk(int64_t tokens, int n_kv_heads, int n_cus)
{
    const int64_t target_items = (int64_t)std::max(1, n_cus) * env_int("SPD_TARGET_WG_PER_CU", kTargetWgPerCuDefault);
    const int chunk_max = std::max(kChunkMin, env_int("SPD_CHUNK_MAX", kChunkMaxDefault) / kChunkMin * kChunkMin);
    int64_t c = (tokens * n_kv_heads + target_items - 1) / target_items;
    c = (c + kChunkMin - 1) / kChunkMin * kChunkMin;
    return (int)std::min<int64_t>(std::max<int64_t>(c, kChunkMin), chunk_max);
}

struct Schedule {
    std::vector<spd_work_item> items;
    std::vector<RowInfo> rows;   // [U * Hkv]
    int64_t n_slots = 0;
    int chunk_tokens = 0;
    bool need_combine = false;   // some row has zero or several chunks
};

void build_schedule(int Hkv, int n_users, const int32_t *lens, int n_cus, Schedule &S)
{
    int64_t tokens = 0;
    for (int u = 0; u < n_users; ++u)
        tokens += lens[u];
    const int C = pick_chunk(tokens, Hkv, n_cus);
    S.chunk_tokens = C;
    S.items.clear();
    S.rows.assign((size_t)n_users * Hkv, RowInfo{0, 0});
    S.n_slots = 0;
    S.need_combine = false;
    for (int u = 0; u < n_users; ++u) {
        const int L = lens[u];
        int n_c = 0, per = 0;
        if (L > 0) {
            n_c = (L + C - 1) / C;
            per = ((L + n_c - 1) / n_c + kChunkAlign - 1) / kChunkAlign * kChunkAlign;  // balanced, 32-aligned
            n_c = (L + per - 1) / per;
        }
        if (n_c != 1)
            S.need_combine = true;
        for (int h = 0; h < Hkv; ++h) {
            S.rows[(size_t)u * Hkv + h] = RowInfo{(int32_t)S.n_slots, n_c};
            for (int c = 0; c < n_c; ++c) {
                spd_work_item it;
                it.user = u;
                it.kv_head = h;
                it.t_begin = c * per;
                it.t_end = std::min(L, (c + 1) * per);
                it.slot = (int32_t)(S.n_slots + c);
                it.n_chunks = n_c;
                it.chunk = c;
                it.reserved = 0;
                S.items.push_back(it);
            }
            S.n_slots += n_c;
        }
    }
    // longest first, so the last workgroups to start are the short ones
    std::stable_sort(S.items.begin(), S.items.end(), [](const spd_work_item &a, const spd_work_item &b) {
        return (a.t_end - a.t_begin) > (b.t_end - b.t_begin);
    });
}

uint64_t fnv1a(const uint8_t *p, size_t n)
{
    uint64_t h = 1469598103934665603ull;
    for (size_t i = 0; i < n; ++i) {
        h ^= p[i];
        h *= 1099511628211ull;
    }
    return h;
}

// A schedule resident on the device, remembered by the bytes that determine it.
struct CachedSchedule {
    bool valid = false;
    uint64_t hash = 0, last_use = 0;
    std::vector<uint8_t> key;
    int64_t n_items = 0, n_slots = 0;
    int n_rows = 0;
    bool need_combine = false;
    char *dev = nullptr;     // items | rows | k_ptrs | v_ptrs
    char *pinned = nullptr;  // host staging copy of the same blob
    size_t capacity = 0;
    size_t off_rows = 0, off_kptrs = 0, off_vptrs = 0;
};

struct Owner {
    CachedSchedule cache[kCacheEntries];
    float *part_o = nullptr;
    float *part_lse = nullptr;
    size_t part_o_cap = 0, part_lse_cap = 0;  // floats
    // optional timing of the partial kernel: a ring of event pairs recorded around its launch
    std::vector<hipEvent_t> ev_start, ev_stop;
    int ev_used = 0;
};

}  // namespace

struct spd_ctx {
    int device = 0;
    int n_cus = 0;
    int last_hip = 0;
    uint64_t tick = 0;
    bool timing = false;
    Owner owner[2];
};

namespace {

#define SPD_HIP(ctx, call)                                  \
    do {                                                    \
        hipError_t e_ = (call);                             \
        if (e_ != hipSuccess) {                             \
            (ctx)->last_hip = (int)e_;                      \
            return SPD_ERR_HIP;                             \
        }                                                   \
    } while (0)

void free_entry(CachedSchedule &e)
{
    if (e.dev)
        (void)hipFree(e.dev);
    if (e.pinned)
        (void)hipHostFree(e.pinned);
    e = CachedSchedule();
}

void make_key(const spd_shape *s, const spd_kv_view *v, std::vector<uint8_t> &key)
{
    key.clear();
    auto put = [&key](const void *p, size_t n) {
        const uint8_t *b = static_cast<const uint8_t *>(p);
        key.insert(key.end(), b, b + n);
    };
    const int32_t head[5] = {s->dtype, s->n_q_heads, s->n_kv_heads, v->n_users, v->block_size};
    put(head, sizeof head);
    put(v->lens, sizeof(int32_t) * (size_t)v->n_users);
    if (v->block_size == 0) {
        for (int u = 0; u < v->n_users; ++u) {  // pointers of empty users are never read: normalise them
            const void *kp = v->lens[u] ? v->k_ptrs[u] : nullptr;
            const void *vp = v->lens[u] ? v->v_ptrs[u] : nullptr;
            put(&kp, sizeof kp);
            put(&vp, sizeof vp);
        }
    }
}

// Find or build the device-resident schedule for this view.  Uploads are enqueued on `stream`.
int get_schedule(spd_ctx *ctx, Owner &own, const spd_shape *s, const spd_kv_view *v, hipStream_t stream,
                 CachedSchedule **out)
{
    std::vector<uint8_t> key;
    make_key(s, v, key);
    const uint64_t h = fnv1a(key.data(), key.size());
    ++ctx->tick;
    CachedSchedule *victim = &own.cache[0];
    for (auto &e : own.cache) {
        if (e.valid && e.hash == h && e.key == key) {
            e.last_use = ctx->tick;
            *out = &e;
            return SPD_OK;
        }
        if (!e.valid) {
            if (victim->valid)
                victim = &e;
        } else if (victim->valid && e.last_use < victim->last_use) {
            victim = &e;
        }
    }
    Schedule S;
    build_schedule(s->n_kv_heads, v->n_users, v->lens, ctx->n_cus, S);

    const size_t b_items = S.items.size() * sizeof(spd_work_item);
    const size_t b_rows = S.rows.size() * sizeof(RowInfo);
    const size_t b_ptrs = v->block_size == 0 ? sizeof(void *) * (size_t)v->n_users : 0;
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    const size_t off_rows = up(b_items), off_k = off_rows + up(b_rows), off_v = off_k + up(b_ptrs);
    const size_t total = off_v + up(b_ptrs) + 256;

    CachedSchedule &e = *victim;
    if (e.valid || e.capacity < total) {
        if (e.valid)
            SPD_HIP(ctx, hipDeviceSynchronize());  // a kernel or copy in flight may still read the evicted blob
        const size_t cap = std::max(total, e.capacity);
        if (e.capacity < total) {
            free_entry(e);
            SPD_HIP(ctx, hipMalloc(reinterpret_cast<void **>(&e.dev), cap));
            SPD_HIP(ctx, hipHostMalloc(reinterpret_cast<void **>(&e.pinned), cap, hipHostMallocDefault));
            e.capacity = cap;
        }
    }
    std::memset(e.pinned, 0, total);
    if (b_items)
        std::memcpy(e.pinned, S.items.data(), b_items);
    if (b_rows)
        std::memcpy(e.pinned + off_rows, S.rows.data(), b_rows);
    if (b_ptrs) {
        const void **kp = reinterpret_cast<const void **>(e.pinned + off_k);
        const void **vp = reinterpret_cast<const void **>(e.pinned + off_v);
        for (int u = 0; u < v->n_users; ++u) {
            kp[u] = v->lens[u] ? v->k_ptrs[u] : nullptr;
            vp[u] = v->lens[u] ? v->v_ptrs[u] : nullptr;
        }
    }
    SPD_HIP(ctx, hipMemcpyAsync(e.dev, e.pinned, total, hipMemcpyHostToDevice, stream));
    e.valid = true;
    e.hash = h;
    e.key.swap(key);
    e.last_use = ctx->tick;
    e.n_items = (int64_t)S.items.size();
    e.n_slots = S.n_slots;
    e.n_rows = (int)S.rows.size();
    e.need_combine = S.need_combine;
    e.off_rows = off_rows;
    e.off_kptrs = off_k;
    e.off_vptrs = off_v;
    *out = &e;
    return SPD_OK;
}

int ensure_scratch(spd_ctx *ctx, Owner &own, size_t o_floats, size_t lse_floats)
{
    if (own.part_o_cap < o_floats) {
        if (own.part_o)
            SPD_HIP(ctx, hipFree(own.part_o));  // hipFree waits for work that may still use the old buffer
        own.part_o = nullptr;
        own.part_o_cap = 0;
        const size_t cap = o_floats + o_floats / 4;
        if (hipMalloc(reinterpret_cast<void **>(&own.part_o), cap * sizeof(float)) != hipSuccess) {
            own.part_o = nullptr;
            return SPD_ERR_WORKSPACE;
        }
        own.part_o_cap = cap;
    }
    if (own.part_lse_cap < lse_floats) {
        if (own.part_lse)
            SPD_HIP(ctx, hipFree(own.part_lse));
        own.part_lse = nullptr;
        own.part_lse_cap = 0;
        const size_t cap = lse_floats + lse_floats / 4;
        if (hipMalloc(reinterpret_cast<void **>(&own.part_lse), cap * sizeof(float)) != hipSuccess) {
            own.part_lse = nullptr;
            return SPD_ERR_WORKSPACE;
        }
        own.part_lse_cap = cap;
    }
    return SPD_OK;
}

template <int D, int G>
void launch_f32(const CachedSchedule &e, const KvAddr &kv, const void *q, const spd_shape *s, float c, Owner &own,
                float *out, float *lse, hipStream_t stream)
{
    hipLaunchKernelGGL((spd::partial_f32_kernel<D, G>), dim3((unsigned)e.n_items), dim3(spd::kThreads), 0, stream,
                       reinterpret_cast<const spd_work_item *>(e.dev), kv, static_cast<const float *>(q),
                       s->n_q_heads, c, own.part_o, own.part_lse, out, lse);
}

template <int D>
void launch_f32_g(int G, const CachedSchedule &e, const KvAddr &kv, const void *q, const spd_shape *s, float c,
                  Owner &own, float *out, float *lse, hipStream_t stream)
{
    switch (G) {
    case 1: launch_f32<D, 1>(e, kv, q, s, c, own, out, lse, stream); break;
    case 2: launch_f32<D, 2>(e, kv, q, s, c, own, out, lse, stream); break;
    case 4: launch_f32<D, 4>(e, kv, q, s, c, own, out, lse, stream); break;
    default: launch_f32<D, 8>(e, kv, q, s, c, own, out, lse, stream); break;
    }
}

int partial_attention(spd_ctx *ctx, int which, const spd_shape *s, const void *q, const spd_kv_view *v, float *out,
                      float *lse, void *hip_stream)
{
    if (!ctx)
        return SPD_ERR_NULL;
    const int rc = spd_validate_partial(s, q, v, out, lse);
    if (rc != SPD_OK)
        return rc;
    if (v->n_users == 0)
        return SPD_OK;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    SPD_HIP(ctx, hipSetDevice(ctx->device));
    Owner &own = ctx->owner[which];
    CachedSchedule *e = nullptr;
    const int rs = get_schedule(ctx, own, s, v, stream, &e);
    if (rs != SPD_OK)
        return rs;
    const int G = s->n_q_heads / s->n_kv_heads;
    const int d = s->head_dim;
    const int rw = ensure_scratch(ctx, own, (size_t)e->n_slots * G * d + 4, (size_t)e->n_slots * G + 4);
    if (rw != SPD_OK)
        return rw;

    const int es = elt_size(s->dtype);
    KvAddr kv;
    kv.k_ptrs = reinterpret_cast<const char *const *>(e->dev + e->off_kptrs);
    kv.v_ptrs = reinterpret_cast<const char *const *>(e->dev + e->off_vptrs);
    kv.k_pool = static_cast<const char *>(v->k_pool);
    kv.v_pool = static_cast<const char *>(v->v_pool);
    kv.block_table = v->block_size ? v->block_table : nullptr;
    kv.max_blocks = v->max_blocks;
    kv.block_stride = v->block_stride * es;
    kv.token_stride = v->token_stride * es;
    kv.head_stride = v->head_stride * es;
    const float c = s->scale * spd::kLog2e;

    if (e->n_items > 0) {
        const bool timed = ctx->timing && own.ev_used < (int)own.ev_start.size();
        if (timed)
            SPD_HIP(ctx, hipEventRecord(own.ev_start[own.ev_used], stream));
        if (s->dtype == SPD_BF16) {
            if (v->block_size)
                hipLaunchKernelGGL((spd::partial_bf16_d128_kernel<true>), dim3((unsigned)e->n_items),
                                   dim3(spd::kThreads), 0, stream, reinterpret_cast<const spd_work_item *>(e->dev), kv,
                                   static_cast<const uint16_t *>(q), s->n_q_heads, G, c, own.part_o, own.part_lse, out,
                                   lse);
            else
                hipLaunchKernelGGL((spd::partial_bf16_d128_kernel<false>), dim3((unsigned)e->n_items),
                                   dim3(spd::kThreads), 0, stream, reinterpret_cast<const spd_work_item *>(e->dev), kv,
                                   static_cast<const uint16_t *>(q), s->n_q_heads, G, c, own.part_o, own.part_lse, out,
                                   lse);
        } else if (d == 64) {
            launch_f32_g<64>(G, *e, kv, q, s, c, own, out, lse, stream);
        } else {
            launch_f32_g<128>(G, *e, kv, q, s, c, own, out, lse, stream);
        }
        SPD_HIP(ctx, hipGetLastError());
        if (timed)
            SPD_HIP(ctx, hipEventRecord(own.ev_stop[own.ev_used++], stream));
    }
    if (e->need_combine) {
        const RowInfo *rows = reinterpret_cast<const RowInfo *>(e->dev + e->off_rows);
        if (d == 64)
            hipLaunchKernelGGL((spd::combine_chunks_kernel<64>), dim3((unsigned)e->n_rows), dim3(64), 0, stream, rows,
                               s->n_kv_heads, s->n_q_heads, G, own.part_o, own.part_lse, out, lse);
        else
            hipLaunchKernelGGL((spd::combine_chunks_kernel<128>), dim3((unsigned)e->n_rows), dim3(128), 0, stream,
                               rows, s->n_kv_heads, s->n_q_heads, G, own.part_o, own.part_lse, out, lse);
        SPD_HIP(ctx, hipGetLastError());
    }
    return SPD_OK;
}

}  // namespace

extern "C" {

const char *spd_strerror(int code)
{
    switch (code) {
    case SPD_OK: return "ok";
    case SPD_ERR_NULL: return "a required pointer is NULL";
    case SPD_ERR_SHAPE: return "unsupported dtype, head counts, head_dim or block size";
    case SPD_ERR_LEN: return "negative count or length, or a paged length beyond max_blocks";
    case SPD_ERR_ALIGN: return "pointer or stride breaks the 16-byte row alignment";
    case SPD_ERR_WORKSPACE: return "scratch memory could not be allocated or is too small";
    case SPD_ERR_HIP: return "a HIP runtime call failed";
    case SPD_ERR_NOMEM: return "host allocation failed";
    default: return "unknown error code";
    }
}

int spd_create(spd_ctx **out, int hip_device)
{
    if (!out)
        return SPD_ERR_NULL;
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || hip_device < 0 || hip_device >= n)
        return SPD_ERR_HIP;
    spd_ctx *ctx = new (std::nothrow) spd_ctx();
    if (!ctx)
        return SPD_ERR_NOMEM;
    ctx->device = hip_device;
    hipError_t e = hipSetDevice(hip_device);
    if (e == hipSuccess)
        e = hipDeviceGetAttribute(&ctx->n_cus, hipDeviceAttributeMultiprocessorCount, hip_device);
    if (e != hipSuccess) {
        delete ctx;
        return SPD_ERR_HIP;
    }
    *out = ctx;
    return SPD_OK;
}

int spd_destroy(spd_ctx *ctx)
{
    if (!ctx)
        return SPD_ERR_NULL;
    (void)hipSetDevice(ctx->device);
    (void)hipDeviceSynchronize();
    for (auto &own : ctx->owner) {
        for (auto &e : own.cache)
            free_entry(e);
        if (own.part_o)
            (void)hipFree(own.part_o);
        if (own.part_lse)
            (void)hipFree(own.part_lse);
        for (auto ev : own.ev_start)
            (void)hipEventDestroy(ev);
        for (auto ev : own.ev_stop)
            (void)hipEventDestroy(ev);
    }
    delete ctx;
    return SPD_OK;
}

int spd_last_hip_error(const spd_ctx *ctx) { return ctx ? ctx->last_hip : 0; }

int spd_validate_partial(const spd_shape *shape, const void *q, const spd_kv_view *view, const float *out,
                         const float *lse)
{
    const int rc = validate_shape(shape);
    if (rc != SPD_OK)
        return rc;
    const int rv = validate_view(shape, view);
    if (rv != SPD_OK)
        return rv;
    if (view->n_users > 0) {
        if (!q || !out || !lse)
            return SPD_ERR_NULL;
        if (!aligned16(q) || !aligned16(out) || (reinterpret_cast<uintptr_t>(lse) & 3u))
            return SPD_ERR_ALIGN;
    }
    return SPD_OK;
}

int spd_build_schedule(const spd_shape *shape, int32_t n_users, const int32_t *lens, int32_t n_compute_units,
                       spd_work_item *items, int64_t capacity, int64_t *n_items, int32_t *chunk_tokens)
{
    const int rc = validate_shape(shape);
    if (rc != SPD_OK)
        return rc;
    if (n_users < 0)
        return SPD_ERR_LEN;
    if ((n_users > 0 && !lens) || !n_items)
        return SPD_ERR_NULL;
    for (int u = 0; u < n_users; ++u)
        if (lens[u] < 0)
            return SPD_ERR_LEN;
    Schedule S;
    build_schedule(shape->n_kv_heads, n_users, lens, n_compute_units, S);
    *n_items = (int64_t)S.items.size();
    if (chunk_tokens)
        *chunk_tokens = S.chunk_tokens;
    if (items) {
        if (capacity < (int64_t)S.items.size())
            return SPD_ERR_WORKSPACE;
        std::memcpy(items, S.items.data(), S.items.size() * sizeof(spd_work_item));
    }
    return SPD_OK;
}

int spd_set_kernel_timing(spd_ctx *ctx, int32_t max_launches)
{
    if (!ctx)
        return SPD_ERR_NULL;
    if (max_launches < 0)
        return SPD_ERR_LEN;
    SPD_HIP(ctx, hipSetDevice(ctx->device));
    for (auto &own : ctx->owner) {
        while ((int)own.ev_start.size() < max_launches) {
            hipEvent_t a, b;
            SPD_HIP(ctx, hipEventCreate(&a));
            own.ev_start.push_back(a);
            SPD_HIP(ctx, hipEventCreate(&b));
            own.ev_stop.push_back(b);
        }
        own.ev_used = 0;
    }
    ctx->timing = max_launches > 0;
    return SPD_OK;
}

int spd_get_kernel_timing(spd_ctx *ctx, int32_t entry_point, int32_t *n_launches, double *mean_us, double *min_us)
{
    if (!ctx || !n_launches || !mean_us || !min_us)
        return SPD_ERR_NULL;
    if (entry_point != 0 && entry_point != 1)
        return SPD_ERR_SHAPE;
    Owner &own = ctx->owner[entry_point];
    double sum = 0.0, mn = 0.0;
    for (int i = 0; i < own.ev_used; ++i) {
        SPD_HIP(ctx, hipEventSynchronize(own.ev_stop[i]));
        float ms = 0.f;
        SPD_HIP(ctx, hipEventElapsedTime(&ms, own.ev_start[i], own.ev_stop[i]));
        sum += ms;
        mn = (i == 0 || ms < mn) ? ms : mn;
    }
    *n_launches = own.ev_used;
    *mean_us = own.ev_used ? 1e3 * sum / own.ev_used : 0.0;
    *min_us = 1e3 * mn;
    own.ev_used = 0;
    return SPD_OK;
}

int spd_partial_attn_private(spd_ctx *ctx, const spd_shape *shape, const void *q, const spd_kv_view *priv, float *out,
                             float *lse, void *hip_stream)
{
    return partial_attention(ctx, 0, shape, q, priv, out, lse, hip_stream);
}

int spd_partial_attn_public_batched(spd_ctx *ctx, const spd_shape *shape, const void *q, const spd_kv_view *pub,
                                    float *out, float *lse, void *hip_stream)
{
    return partial_attention(ctx, 1, shape, q, pub, out, lse, hip_stream);
}

int spd_lse_merge(spd_ctx *ctx, int32_t n_rows, int32_t head_dim, const float *a0, const float *lse0, const float *a1,
                  const float *lse1, float *y, float *lse_out, float *w0_out, void *hip_stream)
{
    if (!ctx)
        return SPD_ERR_NULL;
    if (n_rows < 0)
        return SPD_ERR_LEN;
    if (head_dim <= 0 || head_dim % 4 != 0 || head_dim > 1024)
        return SPD_ERR_SHAPE;
    if (n_rows == 0)
        return SPD_OK;
    if (!a0 || !lse0 || !a1 || !lse1 || !y)
        return SPD_ERR_NULL;
    if (!aligned16(a0) || !aligned16(a1) || !aligned16(y))
        return SPD_ERR_ALIGN;
    SPD_HIP(ctx, hipSetDevice(ctx->device));
    const int vpr = head_dim / 4;
    const int64_t n_vec = (int64_t)n_rows * vpr;
    const unsigned blocks = (unsigned)((n_vec + 255) / 256);
    hipLaunchKernelGGL(spd::lse_merge_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), n_vec,
                       vpr, a0, lse0, a1, lse1, y, lse_out, w0_out);
    SPD_HIP(ctx, hipGetLastError());
    return SPD_OK;
}

}  // extern "C"
