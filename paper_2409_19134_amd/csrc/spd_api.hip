// Host side of the SPD decode-attention library: C ABI, schedule cache, scratch memory, launches
// (argument validation: host_checks.hpp; the split schedule itself: schedule.hpp).
// The calls follow the paper's decode protocol (section 4, step 3b/3c) and Theorem 1 (section 4.2).
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <array>
#include <cmath>
#include <mutex>
#include <cstdlib>
#include <cstring>
#include <new>
#include <type_traits>
#include <utility>
#include <vector>

#include "combine.hpp"
#include "common.hpp"
#include "host_checks.hpp"
#include "partial_mfma.hpp"
#include "schedule.hpp"
#include "schedule_key.hpp"

namespace {

using spd::CombineRow;
using spd::DevItem;
using spd::KvAddr;
using spd::OwnerArgs;
using spd::RowInfo;
using namespace spd::host;

// Remembered schedules per entry point.  Views without device pointer tables need one per set of buffers, i.e. one per
// layer of a model: the default holds an 80-layer model with room to spare.  SPD_SCHEDULE_CACHE_ENTRIES (1..4096, read
// when a context is created) changes it.
constexpr int kCacheEntriesDefault = 128;

// A schedule resident on the device, remembered by the bytes that determine it.
struct CachedSchedule {
    bool valid = false;
    uint64_t hash = 0, last_use = 0;
    uint64_t hash_but_lens = 0;  // of the key without the lengths: finds the schedule of a view that has grown since
    bool growable = false;       // no user without tokens (a row that only writes A = 0 cannot gain tokens)
    int32_t grow = 0;            // set by every lookup: tokens each row has gained over the lengths in `key`
    std::vector<uint8_t> key;
    int64_t n_items = 0, n_slots = 0, n_segments = 0;
    int hpw = 0;             // 0, or the KV heads per workgroup of the head-per-wave kernel the pieces are for
    int n_split_rows = 0;    // rows with several chunks: CombineRow[n_split_rows] follows the items
    size_t off_rows = 0, off_info = 0;
    char *dev = nullptr;     // DevItem[n_items] | CombineRow[n_split_rows] | RowInfo[n_users * Hkv]
    char *pinned = nullptr;  // host staging copy of the same blob
    size_t capacity = 0;
    bool in_slab = false;    // dev / pinned are slots of the owner's slab, not allocations of their own
    hipStream_t last_stream = nullptr;  // stream of the latest call that used this entry
    hipEvent_t uploaded = nullptr;      // completes when the latest upload has left the staging copy
};

// Most schedules are a few tens of KB: the first kSlabEntries entries of an owner share one device and one pinned
// allocation of kSlabSlot bytes each (made when the first schedule is built), so that a run of new views - a serving
// loop whose batch keeps changing - does not pay two allocations per view.  Larger schedules get storage of their own.
constexpr size_t kSlabSlot = 64 * 1024;
constexpr size_t kSlabEntries = 128;

struct Owner {
    std::vector<CachedSchedule> cache;
    char *slab_dev = nullptr, *slab_pinned = nullptr;
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
    int64_t schedule_builds = 0, schedule_hits = 0;
    bool timing = false;
    int32_t last_instance[6] = {-1, -1, -1, -1, -1, -1};  // template arguments of the partial kernel launched last
    Tuning tuning;           // what shapes the split schedules (SPD_OPT_*)
    int result_rows = spd::kRingMaxRows;  // SPD_OPT_RESULT_ROWS: result rows a workgroup holds back in LDS at most (0: none)
    int steps_in_flight = -1;  // SPD_OPT_STEPS_IN_FLIGHT: 1 or 2 where the kernel has both forms, -1 by the size of the launch
    int head_per_wave = -1;  // SPD_OPT_HEAD_PER_WAVE: 0 never, 1 whenever the layout allows, 2..8 the same with that many heads per workgroup, -1 by the size rule
    std::vector<uint8_t> key_scratch;
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
    if (e.dev && !e.in_slab)
        (void)hipFree(e.dev);
    if (e.pinned && !e.in_slab)
        (void)hipHostFree(e.pinned);
    if (e.uploaded)
        (void)hipEventDestroy(e.uploaded);
    e = CachedSchedule();
}

// Token-major storage (the KV heads of a token adjacent in memory, plain or inside pages) can take the head-per-wave
// kernel: one wave per KV head, all waves on the same tokens.
bool head_per_wave_layout(const spd_shape *s, const spd_kv_view *v)
{
    return s->dtype != SPD_F32 && head_per_wave_waves(s->n_kv_heads) > 1 &&
           !(v->head_strides && v->block_size == 0) && v->head_stride == s->head_dim &&
           v->token_stride >= (int64_t)s->n_kv_heads * s->head_dim;
}

int64_t total_steps(const spd_kv_view *v)
{
    int64_t T = 0;
    for (int u = 0; u < v->n_users; ++u)
        T += (v->lens[u] + kChunkAlign - 1) / kChunkAlign;
    return T;
}

// KV heads (waves) per workgroup of the head-per-wave mapping for a launch of `steps` 32-token steps per KV head, or 0
// for the head-major mapping.  The mapping pays once the launch is bandwidth-bound, i.e. every workgroup gets several
// steps; below that the four interleaving waves of the head-major mapping finish a short piece sooner.  Workgroups of
// four heads (two or three per CU, 1 KB of every token) take over from ~280 MB of K/V; workgroups of eight (one per
// CU, a token's whole 2 KB with eight KV heads) are ahead from a few GB of long rows (workload 3: 1.2 %), and for more
// than eight KV heads.  Measured (256 CUs, 8 KV heads, token-major, us per fused step; head-major / four / eight):
// workload 2's lengths with 16 users 35.5 / 40.2 / 48.1, 24 users 46.8 / 50.0 / -, 32 users 63.2 / 59.5 / 66.5,
// 64 users 115.7 / 102.5 / 110.0; workload 4 - / 445.5 / 452.9; workload 3 - / 783 / 774.  The bounds are on
// steps * KV heads per CU, which is what fixed the earlier crossovers for 16 and 32 KV heads (~330 MB each).
// The option SPD_OPT_HEAD_PER_WAVE overrides the rule: 0 never, 1 whenever the layout allows (group size by the rule),
// 2..8 that many heads per workgroup (the largest divisor of the KV head count up to it): for tests and measurements.
int head_per_wave_choice(const spd_ctx *ctx, const spd_shape *s, int64_t steps)
{
    const int opt = ctx->head_per_wave;
    if (opt == 0)
        return 0;
    const int64_t head_steps = steps * std::max(8, s->n_kv_heads) / std::max(1, ctx->n_cus);
    if (opt < 0 && head_steps < kHeadPerWaveMinHeadSteps)
        return 0;
    int most = 8;
    if (opt >= 2)
        most = opt;
    else if (head_steps < kHeadPerWaveWideHeadSteps && s->n_kv_heads <= 8)
        most = 4;
    const int w = head_per_wave_waves(s->n_kv_heads, most);
    return w >= 2 ? w : 0;
}

// A schedule as the kernels read it, laid out for device memory:
// DevItem[items] | CombineRow[split rows] | RowInfo[n_users * Hkv], each part 256-byte aligned.
struct ScheduleBlob {
    std::vector<char> bytes;  // a multiple of 256
    size_t off_rows = 0, off_info = 0;
    int64_t n_items = 0;      // workgroups of the launch
    int64_t n_slots = 0;      // chunk partials
    int64_t n_segments = 0;   // segments with tokens
    int n_split_rows = 0;
};

void build_blob(const spd_shape *s, const spd_kv_view *v, int hpw, int n_cus, const Tuning &tune, ScheduleBlob &B)
{
    Schedule S;
    build_schedule(s->n_kv_heads, v->n_users, v->lens, n_cus, hpw, tune, S);
    DeviceTables T;
    build_device_tables(S, s->n_kv_heads, elt_size(s->dtype), v, hpw, T);
    const size_t b_items = T.items.size() * sizeof(DevItem);
    const size_t b_rows = T.split_rows.size() * sizeof(CombineRow);
    const size_t b_info = T.row_info.size() * sizeof(RowInfo);
    B.off_rows = (b_items + 255) / 256 * 256;
    B.off_info = B.off_rows + (b_rows + 255) / 256 * 256;
    B.bytes.assign(B.off_info + (b_info + 255) / 256 * 256 + 256, 0);
    if (b_items)
        std::memcpy(B.bytes.data(), T.items.data(), b_items);
    if (b_rows)
        std::memcpy(B.bytes.data() + B.off_rows, T.split_rows.data(), b_rows);
    if (b_info)
        std::memcpy(B.bytes.data() + B.off_info, T.row_info.data(), b_info);
    B.n_items = T.items_launched;
    B.n_slots = S.n_slots;
    B.n_segments = T.n_segments;
    B.n_split_rows = (int)T.split_rows.size();
}

// Find or build the device-resident schedule for this view (hpw: pieces for the head-per-wave kernel).  Uploads are
// enqueued on `stream`.
int get_schedule(spd_ctx *ctx, Owner &own, const spd_shape *s, const spd_kv_view *v, int hpw, const Tuning &tune,
                 hipStream_t stream, CachedSchedule **out)
{
    std::vector<uint8_t> &key = ctx->key_scratch;  // reused from call to call: no allocation on the hit path
    make_key(s, v, hpw, &tune.target_wg_per_cu, kTuningInts, key);
    const uint64_t h = hash_key(key.data(), key.size());
    ++ctx->tick;
    CachedSchedule *victim = &own.cache[0];
    for (auto &e : own.cache) {
        if (e.valid && e.hash == h && e.key == key) {
            e.last_use = ctx->tick;
            e.last_stream = stream;
            e.grow = 0;
            ++ctx->schedule_hits;
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
    // no schedule for exactly these lengths: one of the same view with uniformly shorter lengths will do
    const uint64_t h_but_lens = hash_key_but_lens(key, v->n_users);
    CachedSchedule *grown = nullptr;
    int32_t grown_by = 0;
    for (auto &e : own.cache) {
        if (e.valid && e.hash_but_lens == h_but_lens) {
            const int32_t g = e.growable ? uniform_growth(e.key, key, v->n_users) : 0;
            if (g > 0 && (!grown || g < grown_by)) {
                grown = &e;
                grown_by = g;
            }
        }
    }
    if (grown) {
        grown->last_use = ctx->tick;
        grown->last_stream = stream;
        grown->grow = grown_by;
        ++ctx->schedule_hits;
        *out = grown;
        return SPD_OK;
    }
    ScheduleBlob B;
    build_blob(s, v, hpw, ctx->n_cus, tune, B);
    const size_t total = B.bytes.size();

    CachedSchedule &e = *victim;
    ++ctx->schedule_builds;
    if (e.valid) {
        // Reusing an entry: work in flight may still read its device blob, and its last upload may still read the
        // staging copy.  On the same stream the new upload is ordered behind that work anyway.  If the entry was last
        // used on another stream, the whole device is waited for: that stream belongs to the caller and may be gone by
        // now, so it is never touched again (evictions are rare; recording an event per call to wait on instead would
        // put a marker between the kernels of every step).  The staging copy is only rewritten once its last upload
        // has completed.
        if (e.last_stream != stream)
            SPD_HIP(ctx, hipDeviceSynchronize());
        SPD_HIP(ctx, hipEventSynchronize(e.uploaded));
    }
    if (e.capacity < total) {
        // Rounded up to a power of two (at least 64 KB): a serving loop whose batch changes a little every step builds
        // schedules of slightly different sizes, and growing an entry costs a hipFree (which waits for the device)
        // and two allocations.
        size_t cap = kSlabSlot;
        while (cap < total)
            cap *= 2;
        const size_t idx = (size_t)(&e - own.cache.data());
        free_entry(e);  // hipFree (storage of its own only) waits for the device
        if (cap == kSlabSlot && idx < kSlabEntries) {
            if (!own.slab_dev) {
                const size_t bytes = kSlabSlot * std::min(kSlabEntries, own.cache.size());
                SPD_HIP(ctx, hipMalloc(reinterpret_cast<void **>(&own.slab_dev), bytes));
                SPD_HIP(ctx, hipHostMalloc(reinterpret_cast<void **>(&own.slab_pinned), bytes, hipHostMallocDefault));
            }
            e.dev = own.slab_dev + idx * kSlabSlot;
            e.pinned = own.slab_pinned + idx * kSlabSlot;
            e.in_slab = true;
        } else {
            SPD_HIP(ctx, hipMalloc(reinterpret_cast<void **>(&e.dev), cap));
            SPD_HIP(ctx, hipHostMalloc(reinterpret_cast<void **>(&e.pinned), cap, hipHostMallocDefault));
        }
        e.capacity = cap;
    }
    if (!e.uploaded)
        SPD_HIP(ctx, hipEventCreateWithFlags(&e.uploaded, hipEventDisableTiming));
    std::memcpy(e.pinned, B.bytes.data(), total);
    // The upload is a kernel that reads the pinned staging copy over the bus: a copy command would leave the compute
    // queue for a DMA engine and back, which costs the stream tens of microseconds per schedule.
    {
        const unsigned n16 = (unsigned)(total / 16);  // total is a multiple of 256
        hipLaunchKernelGGL(spd::upload_kernel, dim3((n16 + 255) / 256), dim3(256), 0, stream,
                           reinterpret_cast<const spd::u32x4 *>(e.pinned), reinterpret_cast<spd::u32x4 *>(e.dev), n16);
        SPD_HIP(ctx, hipGetLastError());
    }
    SPD_HIP(ctx, hipEventRecord(e.uploaded, stream));
    e.last_stream = stream;
    e.valid = true;
    e.hash = h;
    e.hash_but_lens = h_but_lens;
    e.growable = true;
    for (int u = 0; u < v->n_users; ++u)
        e.growable = e.growable && v->lens[u] > 0;
    e.grow = 0;
    e.key = key;
    e.last_use = ctx->tick;
    e.n_items = B.n_items;
    e.hpw = hpw;
    e.n_slots = B.n_slots;
    e.n_segments = B.n_segments;
    e.n_split_rows = B.n_split_rows;
    e.off_rows = B.off_rows;
    e.off_info = B.off_info;
    *out = &e;
    return SPD_OK;
}

int ensure_scratch(spd_ctx *ctx, Owner &own, size_t o_floats, size_t lse_floats)
{
    if (own.part_o_cap < o_floats) {
        float *old = own.part_o;  // forgotten before it is freed: a failing hipFree must not leave it behind in use
        own.part_o = nullptr;
        own.part_o_cap = 0;
        if (old)
            SPD_HIP(ctx, hipFree(old));  // hipFree waits for work that may still use the old buffer
        const size_t cap = o_floats + o_floats / 4;
        if (hipMalloc(reinterpret_cast<void **>(&own.part_o), cap * sizeof(float)) != hipSuccess) {
            own.part_o = nullptr;
            return SPD_ERR_WORKSPACE;
        }
        own.part_o_cap = cap;
    }
    if (own.part_lse_cap < lse_floats) {
        float *old = own.part_lse;
        own.part_lse = nullptr;
        own.part_lse_cap = 0;
        if (old)
            SPD_HIP(ctx, hipFree(old));
        const size_t cap = lse_floats + lse_floats / 4;
        if (hipMalloc(reinterpret_cast<void **>(&own.part_lse), cap * sizeof(float)) != hipSuccess) {
            own.part_lse = nullptr;
            return SPD_ERR_WORKSPACE;
        }
        own.part_lse_cap = cap;
    }
    return SPD_OK;
}

// A call for one owner has the device to itself: its resident round is half as many pieces again as an owner's share of
// a fused step (three per CU with the default two: the one-step-in-flight kernel then holds them all at once) - unless
// that round would be made of short pieces (up to kShortPieceSteps steps at two per CU): those run faster as two per
// CU.  Measured as two parties, us per step, 3 against 2 per CU (both on the one-step kernel): workload 2's length law
// with 8 / 16 / 24 / 32 users 25.4 / 38.7 / 49.6 / 62.2 against 25.2 / 38.1 / 49.2 / 61.8; with 64 users (72 steps per
// piece) 109.5 against 109.7, workloads 3 and 4 781.6 / 453.2 against 782.8 / 454.8.
Tuning standalone_tuning(const spd_ctx *ctx, const spd_shape *s, const spd_kv_view *v, int hpw)
{
    const Tuning base = ctx->tuning;
    Tuning t = base;
    t.target_wg_per_cu += t.target_wg_per_cu / 2;
    if (hpw || base.target_wg_per_cu < 2)
        return t;
    int64_t rows = 0, steps = 0;
    const int64_t wide = single_round_pieces(s->n_kv_heads, v->n_users, v->lens, ctx->n_cus, t, &rows);
    const int64_t narrow = single_round_pieces(s->n_kv_heads, v->n_users, v->lens, ctx->n_cus, base, &rows, &steps);
    if (wide > 0 && narrow > 0 && steps <= (int64_t)kShortPieceSteps * (narrow / s->n_kv_heads))
        return base;
    return t;
}

// Validation, schedule lookup and scratch growth of one partial-attention call.
int prepare_partial(spd_ctx *ctx, int which, const spd_shape *s, const void *q, const spd_kv_view *v, float *out,
                    float *lse, int mapping, const Tuning *tune, hipStream_t stream, CachedSchedule **e)
{
    const int rc = spd_validate_partial(s, q, v, out, lse);
    if (rc != SPD_OK)
        return rc;
    *e = nullptr;
    if (v->n_users == 0)
        return SPD_OK;
    Owner &own = ctx->owner[which];
    // mapping: KV heads per workgroup of the head-per-wave mapping, 0 = head-major, -1 = whatever suits this view on its own
    const int hpw = mapping >= 0 ? mapping : head_per_wave_layout(s, v) ? head_per_wave_choice(ctx, s, total_steps(v)) : 0;
    // tune: the fused step's; none for a call that serves one owner alone
    const int rs = get_schedule(ctx, own, s, v, hpw, tune ? *tune : standalone_tuning(ctx, s, v, hpw), stream, e);
    if (rs != SPD_OK)
        return rs;
    const int G = s->n_q_heads / s->n_kv_heads;
    return ensure_scratch(ctx, own, (size_t)(*e)->n_slots * G * s->head_dim + 4, (size_t)(*e)->n_slots * G + 4);
}

// Where one owner's chunk partials go: the context's own scratch memory, or a part of the library's fixed array.
struct ScratchPtrs {
    float *part_o = nullptr;      // [slots][G][D]
    float *part_lse = nullptr;    // [slots][G]
};
ScratchPtrs scratch_of(const Owner &own)
{
    ScratchPtrs sp;
    sp.part_o = own.part_o;
    sp.part_lse = own.part_lse;
    return sp;
}

OwnerArgs owner_args(const ScratchPtrs &own, const CachedSchedule *e, const spd_shape *s, const spd_kv_view *v, float *out,
                     float *lse, const void *k_new, const void *v_new)
{
    const int es = elt_size(s->dtype);
    OwnerArgs a;
    a.items = reinterpret_cast<const DevItem *>(e->dev);
    a.k_pool = v->block_size ? static_cast<const char *>(v->k_pool) : nullptr;
    a.v_pool = v->block_size ? static_cast<const char *>(v->v_pool) : nullptr;
    a.k_ptrs = v->block_size ? nullptr : reinterpret_cast<const char *const *>(v->k_ptrs_dev);
    a.v_ptrs = v->block_size ? nullptr : reinterpret_cast<const char *const *>(v->v_ptrs_dev);
    a.kv.block_table = v->block_size ? v->block_table : nullptr;
    a.kv.max_blocks = v->max_blocks;
    a.kv.page_shift = v->block_size ? page_shift(v->block_size) : 0;
    a.kv.block_stride = v->block_stride * es;
    a.kv.token_stride = v->token_stride * es;
    a.kv.head_stride = v->head_stride * es;
    a.part_o = own.part_o;
    a.part_lse = own.part_lse;
    a.out = out;
    a.lse = lse;
    a.k_new = static_cast<const char *>(k_new);
    a.v_new = static_cast<const char *>(v_new);
    a.grow = e->grow;
    return a;
}

// Run-time values to template arguments: f is called with a std::integral_constant of the matching candidate.
template <int V, int... Rest, class F>
bool with_value(int v, F &&f)
{
    if (v == V)
        return f(std::integral_constant<int, V>());
    if constexpr (sizeof...(Rest) > 0)
        return with_value<Rest...>(v, std::forward<F>(f));
    else
        return false;
}
template <class F>
bool with_bool(bool b, F &&f)
{
    return b ? f(std::true_type()) : f(std::false_type());
}

struct MfmaLaunch {
    dim3 grid, block;
    uint32_t lds;
    hipStream_t stream;
    hipEvent_t ev0, ev1;  // both null unless timing is armed: receive the kernel's own start and stop time stamps
    spd::PartialArgs args;
};

// The kernel instances that exist: the head-per-wave mapping always keeps two steps in flight, fp32 rows of 512 bytes
// always one (and have no head-per-wave mapping), rows of 128 bytes always two.
template <int DT, int D, bool PREFETCH, bool HPW>
constexpr bool mfma_instance_exists()
{
    constexpr int RB = D * (DT == SPD_F32 ? 4 : 2);
    return !(HPW && !PREFETCH) && !(DT == SPD_F32 && (HPW || PREFETCH)) && !(RB == 128 && !PREFETCH);
}

template <int DT, int D, bool PAGED, bool PREFETCH, bool HPW, bool APPEND>
bool launch_mfma(const MfmaLaunch &L)
{
    if constexpr (mfma_instance_exists<DT, D, PREFETCH, HPW>()) {
        hipExtLaunchKernelGGL((spd::partial_mfma_kernel<DT, D, PAGED, PREFETCH, HPW, APPEND>), L.grid, L.block, L.lds,
                              L.stream, L.ev0, L.ev1, 0, L.args);
        return true;
    } else {
        return false;
    }
}

// The partial kernel: every piece's workgroup writes final rows or chunk partials.  One owner per launch
// (e1 == nullptr), or both owners' pieces in one grid (the fused step; both views in the same storage mode).
struct NewToken {  // KV append for the public owner (protocol step 3a); both null if none
    const void *k = nullptr, *v = nullptr;
};

// sp0 / sp1: where the two owners' chunk partials go.
int launch_partial(spd_ctx *ctx, int which, const CachedSchedule *e0, const spd_kv_view *v0, float *out0, float *lse0,
                   const ScratchPtrs &sp0, const CachedSchedule *e1, const spd_kv_view *v1, float *out1, float *lse1,
                   const ScratchPtrs &sp1, const spd_shape *s, const void *q, NewToken nt, hipStream_t stream)
{
    const int64_t n0 = e0->n_items, n1 = e1 ? e1->n_items : 0;
    if (n0 + n1 == 0)
        return SPD_OK;
    // the public owner is entry point 1: the new token, if any, belongs to whichever of the two that is
    const OwnerArgs a0 = owner_args(sp0, e0, s, v0, out0, lse0, which == 1 ? nt.k : nullptr, which == 1 ? nt.v : nullptr);
    const OwnerArgs a1 = e1 ? owner_args(sp1, e1, s, v1, out1, lse1, which == 0 ? nt.k : nullptr,
                                         which == 0 ? nt.v : nullptr)
                            : a0;
    const int G = s->n_q_heads / s->n_kv_heads;
    const float c = s->scale * spd::kLog2e;
    Owner &town = ctx->owner[e1 ? 0 : which];  // a two-owner launch is booked under entry point 0
    const bool timed = ctx->timing && town.ev_used < (int)town.ev_start.size();
    const hipEvent_t ev0 = timed ? town.ev_start[town.ev_used] : nullptr;
    const hipEvent_t ev1 = timed ? town.ev_stop[town.ev_used] : nullptr;
    const bool f32 = s->dtype == SPD_F32;
    const bool hpw = e0->hpw != 0;  // a two-owner launch needs the same mapping on both sides (checked by the caller)
    const int waves = hpw ? e0->hpw : spd::kWaves;
    const int D = s->head_dim;
    MfmaLaunch L;
    L.grid = dim3((unsigned)(n0 + n1));
    L.block = dim3(64u * (unsigned)waves);
    // cross-wave staging; head-per-wave stages its per-wave results too if that fits (the kernel applies the same rule)
    L.lds = (hpw && !spd::staging_fits(D, waves, G)) ? 0 : (uint32_t)spd::staging_bytes(D, waves, G);

    L.stream = stream;
    L.ev0 = ev0;
    L.ev1 = ev1;
    L.args.a0 = a0;
    L.args.a1 = a1;
    L.args.n0 = (int)n0;
    L.args.q = static_cast<const char *>(q);
    L.args.Hq = s->n_q_heads;
    L.args.G = G;
    L.args.scale_log2e = c;
    // Two steps in flight (PREFETCH) or one.  Clearly more pieces than the one-step kernel holds at once, three per CU
    // (a few left over just start a little later), run on the two-step kernel, two per CU: fewer workgroup starts and
    // half as many dependent memory round trips per wave.  Everything that is resident at once runs on the one-step
    // kernel, also what fits two per CU (us per fused step, two steps / one: 1 and 2 users of workload 2's length law
    // 9.0 / 8.7 and 13.3 / 12.8; 16 users of 64-512 tokens 11.9 / 11.6; workload 4, 256 + 256 pieces, 433.3 / 430.8, with
    // 128 users 225.7 / 222.0, with 8 query heads per KV head 452.0 / 446.2; 128 users of 64-512 tokens 50.8 / 50.0; 256
    // such users 88.9 / 89.7; the standalone public call of workload 2 -0.3 us).  Head-per-wave workgroups fit one per
    // CU either way; with 128-byte rows a step is half the bytes, always two in flight; fp32 keeps one (at 128
    // channels a step is already 32 KB per wave and fills the registers).  SPD_OPT_STEPS_IN_FLIGHT overrides the size
    // rule (tests run both kernels on the same small inputs).
    const int64_t cus = std::max(1, ctx->n_cus);
    const int row_bytes = D * elt_size(s->dtype);
    const bool by_size = ctx->steps_in_flight < 0 ? n0 + n1 > cus * 4 : ctx->steps_in_flight == 2;
    const bool prefetch = !f32 && (hpw || row_bytes == 128 || by_size);
    // no more than two workgroups on a CU, whether the registers or the launch see to that: the larger LDS share
    const bool two_per_cu = prefetch || n0 + n1 <= cus * 2;
    // Result rows wait in LDS for the end of their piece (see the result ring in partial_mfma.hpp) - where a piece
    // has rows to wait for: with fewer than three segments per piece on average the ring only adds its copy (the
    // headline workload, 1.3 segments per piece: +0.4 us).  The head-per-wave mapping has fewer, wider segments and
    // takes it from 1.5 (workload 4 token-major, 2 segments per piece: 446 -> 442 us).
    const int64_t segments = e0->n_segments + (e1 ? e1->n_segments : 0);
    int ring_rows = 0;
    const int min_x2 = hpw ? 3 : 6;  // twice the segments per piece
    if (2 * segments >= min_x2 * (n0 + n1) && L.lds > 0)  // (head per wave without its staging tiles has no ring either)
        ring_rows = std::min(ctx->result_rows, hpw ? spd::hpw_ring_rows_that_fit(D, G, waves) : spd::ring_rows_that_fit(D, G, two_per_cu));
    L.lds += (uint32_t)(ring_rows * sizeof(float) * (hpw ? (size_t)spd::hpw_ring_row_floats(D, G) * waves : (size_t)spd::ring_row_floats(D, G)));
    L.args.ring_rows = ring_rows;
    const bool ok = with_value<SPD_F32, SPD_BF16, SPD_F16>(s->dtype, [&](auto dt) {
        return with_value<64, 128>(D, [&](auto d) {
            return with_bool(v0->block_size != 0, [&](auto paged) {
                return with_bool(prefetch, [&](auto pf) {
                    return with_bool(hpw, [&](auto hp) {
                        return with_bool(nt.k != nullptr, [&](auto app) {
                            return launch_mfma<decltype(dt)::value, decltype(d)::value, decltype(paged)::value,
                                               decltype(pf)::value, decltype(hp)::value, decltype(app)::value>(L);
                        });
                    });
                });
            });
        });
    });
    if (!ok)
        return SPD_ERR_SHAPE;  // no kernel instance for this combination: a bug in the rules above
    const int32_t inst[6] = {s->dtype, D, v0->block_size != 0, prefetch, hpw, nt.k != nullptr};
    std::memcpy(ctx->last_instance, inst, sizeof inst);
    SPD_HIP(ctx, hipGetLastError());
    if (timed)
        ++town.ev_used;
    return SPD_OK;
}

// The n-way combine of the rows that were split (a separate launch, see combine.hpp).
int launch_combine(spd_ctx *ctx, int which, const CachedSchedule *e, const spd_shape *s, float *out, float *lse,
                   hipStream_t stream)
{
    if (e->n_split_rows == 0)
        return SPD_OK;
    Owner &own = ctx->owner[which];
    const int G = s->n_q_heads / s->n_kv_heads;
    const CombineRow *rows = reinterpret_cast<const CombineRow *>(e->dev + e->off_rows);
    const dim3 grid((unsigned)e->n_split_rows, (unsigned)G);
    if (s->head_dim == 64)
        hipLaunchKernelGGL((spd::combine_chunks_kernel<64>), grid, dim3(64), 0, stream, rows, s->n_q_heads, G,
                           own.part_o, own.part_lse, out, lse);
    else
        hipLaunchKernelGGL((spd::combine_chunks_kernel<128>), grid, dim3(128), 0, stream, rows, s->n_q_heads, G,
                           own.part_o, own.part_lse, out, lse);
    SPD_HIP(ctx, hipGetLastError());
    return SPD_OK;
}

// An append needs both rows, 16-byte aligned, and at least the new token itself in every user's length.
int validate_new_token(const spd_kv_view *v, NewToken nt)
{
    if (!nt.k && !nt.v)
        return SPD_OK;
    if (!nt.k || !nt.v)
        return SPD_ERR_NULL;
    if (!aligned16(nt.k) || !aligned16(nt.v))
        return SPD_ERR_ALIGN;
    for (int u = 0; u < v->n_users; ++u)
        if (v->lens[u] < 1)
            return SPD_ERR_LEN;
    return SPD_OK;
}

int partial_attention(spd_ctx *ctx, int which, const spd_shape *s, const void *q, const spd_kv_view *v, float *out,
                      float *lse, NewToken nt, void *hip_stream)
{
    if (!ctx)
        return SPD_ERR_NULL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    SPD_HIP(ctx, hipSetDevice(ctx->device));
    CachedSchedule *e = nullptr;
    int rc = spd_validate_partial(s, q, v, out, lse);
    if (rc == SPD_OK)
        rc = validate_new_token(v, nt);
    if (rc != SPD_OK)
        return rc;
    rc = prepare_partial(ctx, which, s, q, v, out, lse, -1, nullptr, stream, &e);
    if (rc != SPD_OK || !e)
        return rc;
    rc = launch_partial(ctx, which, e, v, out, lse, scratch_of(ctx->owner[which]), nullptr, nullptr, nullptr, nullptr,
                        ScratchPtrs(), s, q, nt, stream);
    if (rc != SPD_OK)
        return rc;
    return launch_combine(ctx, which, e, s, out, lse, stream);
}

// The closing kernel of a step: combines whichever rows either owner had to split and merges the owners.
// ep == nullptr: the first owner's partials (a_in_r, lse_in_r) are finished results delivered by the caller; they are
// only read, and a_in_w / lse_in_w may be null.
int launch_finalize(spd_ctx *ctx, const spd_shape *shape, int n_users, const CachedSchedule *ep, const CachedSchedule *eo,
                    const ScratchPtrs &sp_in, const ScratchPtrs &sp_out, const float *a_in_r, const float *lse_in_r,
                    float *a_in_w, float *lse_in_w, float *a_out, float *lse_out, float *y, float *lse, float *w_in,
                    hipStream_t stream)
{
    const int G = shape->n_q_heads / shape->n_kv_heads;
    const RowInfo *ri = ep ? reinterpret_cast<const RowInfo *>(ep->dev + ep->off_info) : nullptr;
    const RowInfo *ro = reinterpret_cast<const RowInfo *>(eo->dev + eo->off_info);
    const dim3 grid((unsigned)n_users, (unsigned)shape->n_kv_heads, (unsigned)G);
    if (shape->head_dim == 64)
        hipLaunchKernelGGL((spd::finalize_step_kernel<64>), grid, dim3(64), 0, stream, ri, ro, shape->n_kv_heads,
                           shape->n_q_heads, G, (const float *)sp_in.part_o, (const float *)sp_in.part_lse,
                           (const float *)sp_out.part_o, (const float *)sp_out.part_lse, a_in_r, lse_in_r, a_in_w, lse_in_w,
                           a_out, lse_out, y, lse, w_in);
    else
        hipLaunchKernelGGL((spd::finalize_step_kernel<128>), grid, dim3(128), 0, stream, ri, ro, shape->n_kv_heads,
                           shape->n_q_heads, G, (const float *)sp_in.part_o, (const float *)sp_in.part_lse,
                           (const float *)sp_out.part_o, (const float *)sp_out.part_lse, a_in_r, lse_in_r, a_in_w, lse_in_w,
                           a_out, lse_out, y, lse, w_in);
    SPD_HIP(ctx, hipGetLastError());
    return SPD_OK;
}

// Everything spd_decode_step checks before anything is enqueued (also makes the context's device current).
int validate_decode_step(spd_ctx *ctx, const spd_shape *shape, const void *q, const spd_kv_view *priv,
                         const spd_kv_view *pub, NewToken nt, const float *a_in, const float *lse_in, const float *a_out,
                         const float *lse_out, const float *y, const float *lse, const float *w_in)
{
    if (!priv || !pub)
        return SPD_ERR_NULL;
    if (priv->n_users != pub->n_users)
        return SPD_ERR_LEN;
    SPD_HIP(ctx, hipSetDevice(ctx->device));
    int rc = spd_validate_partial(shape, q, priv, a_in, lse_in);
    if (rc == SPD_OK)
        rc = spd_validate_partial(shape, q, pub, a_out, lse_out);
    if (rc == SPD_OK)
        rc = validate_new_token(pub, nt);
    if (rc != SPD_OK)
        return rc;
    if (priv->n_users == 0)
        return SPD_OK;
    if (!y || !lse || !w_in)
        return SPD_ERR_NULL;
    if (!aligned16(y))
        return SPD_ERR_ALIGN;
    return SPD_OK;
}

// Both owners of a fused step share one launch, so they share the mapping: head per wave if both layouts allow it and
// the two together are bandwidth-bound (the value is the KV heads per workgroup, 0 for the head-major mapping).
int fused_step_mapping(const spd_ctx *ctx, const spd_shape *shape, const spd_kv_view *priv, const spd_kv_view *pub)
{
    if (!head_per_wave_layout(shape, priv) || !head_per_wave_layout(shape, pub))
        return 0;
    return head_per_wave_choice(ctx, shape, total_steps(priv) + total_steps(pub));
}

// Both owners of a fused step also share the device: if each would cut its rows into a full resident round of equal
// pieces, the two rounds together are more than fit at once, the second owner's pieces start when the first's end, and
// result rows are written all along (see the result ring in partial_mfma.hpp).  Where the pieces cross many rows -
// two rows per piece or more - each owner then gets half as many pieces, twice as long, all resident from the start
// and with more rows to hold back each (with the ring; us per fused step, 512 + 512 pieces against 256 + 256:
// workload 4 444.3 / 434.4, its length law with 128 users 230.7 / 227.0, 256 users of 64-512 tokens 92.7 / 91.3).
// With few, long rows the shorter pieces stay (workload 2's length law with 64 users: 103.9 / 107.2).
Tuning fused_step_tuning(const spd_ctx *ctx, const spd_shape *shape, const spd_kv_view *priv, const spd_kv_view *pub, int hpw)
{
    Tuning t = ctx->tuning;
    if (hpw || t.target_wg_per_cu < 2)
        return t;
    int64_t rows_p = 0, rows_o = 0;
    const int64_t np = single_round_pieces(shape->n_kv_heads, priv->n_users, priv->lens, ctx->n_cus, t, &rows_p);
    const int64_t no = single_round_pieces(shape->n_kv_heads, pub->n_users, pub->lens, ctx->n_cus, t, &rows_o);
    if (np > 0 && no > 0 && rows_p + rows_o >= 2 * (np + no))
        t.target_wg_per_cu /= 2;
    return t;
}

// The launches of a fused step, given both owners' schedules (device resident) and where their chunk partials go.
int launch_decode_step(spd_ctx *ctx, const spd_shape *shape, const void *q, const spd_kv_view *priv, const spd_kv_view *pub,
                       NewToken nt, const CachedSchedule *ep, const CachedSchedule *eo, const ScratchPtrs &sp_in,
                       const ScratchPtrs &sp_out, float *a_in, float *lse_in, float *a_out, float *lse_out, float *y,
                       float *lse, float *w_in, hipStream_t stream)
{
    int rc;
    // one grid for both owners, the private owner's long streams first (measured faster than public first): the
    // public owner's short, latency-bound pieces then run beside them on the workgroup slots that remain
    if ((priv->block_size != 0) == (pub->block_size != 0)) {
        rc = launch_partial(ctx, 0, ep, priv, a_in, lse_in, sp_in, eo, pub, a_out, lse_out, sp_out, shape, q, nt, stream);
        if (rc != SPD_OK)
            return rc;
    } else {  // different storage modes need different kernel instances
        rc = launch_partial(ctx, 1, eo, pub, a_out, lse_out, sp_out, nullptr, nullptr, nullptr, nullptr, ScratchPtrs(), shape, q,
                            nt, stream);
        if (rc != SPD_OK)
            return rc;
        rc = launch_partial(ctx, 0, ep, priv, a_in, lse_in, sp_in, nullptr, nullptr, nullptr, nullptr, ScratchPtrs(), shape, q,
                            NewToken(), stream);
        if (rc != SPD_OK)
            return rc;
    }
    // join: one kernel combines whichever rows were split and merges the owners
    return launch_finalize(ctx, shape, priv->n_users, ep, eo, sp_in, sp_out, a_in, lse_in, a_in, lse_in, a_out, lse_out, y, lse,
                           w_in, stream);
}

// ---- the fixed scratch array of spd_decode_step_static ------------------------------------------------------
// One array per GPU, resident from the moment the library's code object is loaded until the process ends.  `scratch`
// is only a host-side handle of the symbol: host code uses the device address that hipGetSymbolAddress returned for
// the GPU in question (static_scratch_of), never the name.
constexpr size_t kStaticSchedBytes = 512u << 10;   // per owner: its schedule as the kernels read it
constexpr size_t kStaticLseFloats = 64u << 10;     // per owner: chunk log-sum-exps (slots * G)
constexpr size_t kStaticOffLse = 2 * kStaticSchedBytes;
constexpr size_t kStaticOffPartO = kStaticOffLse + 2 * kStaticLseFloats * sizeof(float);
constexpr size_t kStaticPartOFloats = (SPD_STATIC_SCRATCH_BYTES - kStaticOffPartO) / 2 / sizeof(float) / 64 * 64;  // per owner
static_assert(kStaticOffPartO + 2 * kStaticPartOFloats * sizeof(float) <= SPD_STATIC_SCRATCH_BYTES, "layout exceeds the array");

static __device__ __align__(256) unsigned char scratch[SPD_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
struct StaticScratch {
    char *ptr = nullptr;          // this GPU's copy of `scratch`
    std::vector<uint8_t> key[2];  // the view whose schedule each owner's part holds (empty: unknown)
    bool replayed = false;        // a call has been recorded into a HIP graph: replays rewrite the array behind the
                                  // host's back, so its contents are no longer known here
};
std::mutex g_static_mutex;
std::array<StaticScratch, kMaxDevices> g_static;

// Looks up this GPU's address of the array (once per device, with that device current).
int static_scratch_init(spd_ctx *ctx)
{
    if (ctx->device >= kMaxDevices)
        return SPD_OK;  // spd_decode_step_static will refuse; everything else works
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticScratch &st = g_static[(size_t)ctx->device];
    if (st.ptr)
        return SPD_OK;
    void *p = nullptr;
    SPD_HIP(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    st.ptr = static_cast<char *>(p);
    return SPD_OK;
}

// A piece of a schedule handed to the GPU inside the kernel arguments (no staging memory, no copy command).
constexpr unsigned kUploadWords = 224;  // 16-byte words per launch (3.5 KB of the 4 KB a launch may carry)
struct UploadChunk {
    spd::u32x4 w[kUploadWords];
};
__global__ __launch_bounds__(256) void upload_args_kernel(UploadChunk c, spd::u32x4 *dst, unsigned n16)
{
    if (threadIdx.x < n16)
        dst[threadIdx.x] = c.w[threadIdx.x];
}

int upload_through_args(spd_ctx *ctx, const std::vector<char> &bytes, char *dst, hipStream_t stream)
{
    const size_t n16 = bytes.size() / 16;  // a multiple of 16 words
    for (size_t at = 0; at < n16; at += kUploadWords) {
        const unsigned n = (unsigned)std::min<size_t>(kUploadWords, n16 - at);
        UploadChunk c;
        std::memcpy(c.w, bytes.data() + at * 16, (size_t)n * 16);
        hipLaunchKernelGGL(upload_args_kernel, dim3(1), dim3(256), 0, stream, c, reinterpret_cast<spd::u32x4 *>(dst) + at, n);
        SPD_HIP(ctx, hipGetLastError());
    }
    return SPD_OK;
}

// No C++ exception leaves the library: a failed host allocation (the schedule builder and the cache use std::vector)
// becomes SPD_ERR_NOMEM.
template <class F>
int no_throw(F &&body)
{
    try {
        return body();
    } catch (...) {
        return SPD_ERR_NOMEM;
    }
}

}  // namespace

extern "C" {

int spd_abi_version(void) { return SPD_ABI_VERSION; }

const char *spd_strerror(int code)
{
    switch (code) {
    case SPD_OK: return "ok";
    case SPD_ERR_NULL: return "a required pointer is NULL";
    case SPD_ERR_SHAPE: return "unsupported dtype, head counts, head_dim or block size";
    case SPD_ERR_LEN: return "negative count or length, a length above 2^30, or a paged length beyond max_blocks";
    case SPD_ERR_ALIGN: return "pointer or stride breaks the 16-byte row alignment";
    case SPD_ERR_WORKSPACE: return "scratch memory could not be allocated, or the step exceeds the fixed scratch array of spd_decode_step_static";
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
    try {
        const int entries = std::min(4096, std::max(1, env_int("SPD_SCHEDULE_CACHE_ENTRIES", kCacheEntriesDefault)));
        for (auto &own : ctx->owner)
            own.cache.resize((size_t)entries);
    } catch (...) {
        delete ctx;
        return SPD_ERR_NOMEM;
    }
    ctx->device = hip_device;
    ctx->tuning = tuning_from_env();
    ctx->result_rows = std::min(spd::kRingMaxRows, env_int("SPD_RESULT_ROWS", spd::kRingMaxRows, 0));
    ctx->steps_in_flight = env_int("SPD_STEPS_IN_FLIGHT", -1, 1);
    if (ctx->steps_in_flight > 2)
        ctx->steps_in_flight = -1;
    ctx->head_per_wave = env_int("SPD_HEAD_PER_WAVE", -1, 0);
    if (ctx->head_per_wave > 8)
        ctx->head_per_wave = -1;
    hipError_t e = hipSetDevice(hip_device);
    if (e == hipSuccess)
        e = hipDeviceGetAttribute(&ctx->n_cus, hipDeviceAttributeMultiprocessorCount, hip_device);
    if (e != hipSuccess) {
        delete ctx;
        return SPD_ERR_HIP;
    }
    if (static_scratch_init(ctx) != SPD_OK) {
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
        if (own.slab_dev)
            (void)hipFree(own.slab_dev);
        if (own.slab_pinned)
            (void)hipHostFree(own.slab_pinned);
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

namespace {
int32_t *option_slot(spd_ctx *ctx, int32_t option)
{
    switch (option) {
    case SPD_OPT_HEAD_PER_WAVE: return &ctx->head_per_wave;
    case SPD_OPT_RESULT_ROWS: return &ctx->result_rows;
    case SPD_OPT_STEPS_IN_FLIGHT: return &ctx->steps_in_flight;
    case SPD_OPT_TARGET_WG_PER_CU: return &ctx->tuning.target_wg_per_cu;
    case SPD_OPT_NO_SPLIT_MAX: return &ctx->tuning.no_split_max;
    case SPD_OPT_CHUNK_MAX: return &ctx->tuning.chunk_max;
    case SPD_OPT_SEG_COST: return &ctx->tuning.seg_cost;
    case SPD_OPT_HALF_SKEW: return &ctx->tuning.half_skew;
    default: return nullptr;
    }
}
}  // namespace

int spd_set_option(spd_ctx *ctx, int32_t option, int32_t value)
{
    if (!ctx)
        return SPD_ERR_NULL;
    int32_t *slot = option_slot(ctx, option);
    if (!slot)
        return SPD_ERR_SHAPE;
    bool ok;
    switch (option) {
    case SPD_OPT_HEAD_PER_WAVE: ok = value >= -1 && value <= 8; break;
    case SPD_OPT_RESULT_ROWS: ok = value >= 0 && value <= spd::kRingMaxRows; break;
    case SPD_OPT_STEPS_IN_FLIGHT: ok = value == -1 || value == 1 || value == 2; break;
    case SPD_OPT_SEG_COST: ok = value >= 0 && value <= (1 << 20); break;
    case SPD_OPT_HALF_SKEW: ok = value >= 0 && value <= 90; break;
    default: ok = value >= 1 && value <= (1 << 30); break;
    }
    if (!ok)
        return SPD_ERR_LEN;
    *slot = value;
    return SPD_OK;
}

int spd_get_option(spd_ctx *ctx, int32_t option, int32_t *value)
{
    if (!ctx || !value)
        return SPD_ERR_NULL;
    const int32_t *slot = option_slot(ctx, option);
    if (!slot)
        return SPD_ERR_SHAPE;
    *value = *slot;
    return SPD_OK;
}

int spd_get_last_kernel_instance(const spd_ctx *ctx, int32_t instance[6])
{
    if (!ctx || !instance)
        return SPD_ERR_NULL;
    std::memcpy(instance, ctx->last_instance, sizeof ctx->last_instance);
    return SPD_OK;
}

int spd_get_schedule_stats(const spd_ctx *ctx, int64_t *builds, int64_t *hits)
{
    if (!ctx || !builds || !hits)
        return SPD_ERR_NULL;
    *builds = ctx->schedule_builds;
    *hits = ctx->schedule_hits;
    return SPD_OK;
}

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
                       int32_t head_per_wave, spd_work_item *items, int64_t capacity, int64_t *n_items,
                       int32_t *chunk_tokens)
try {
    const int rc = validate_shape(shape);
    if (rc != SPD_OK)
        return rc;
    if (n_users < 0)
        return SPD_ERR_LEN;
    if ((n_users > 0 && !lens) || !n_items)
        return SPD_ERR_NULL;
    for (int u = 0; u < n_users; ++u)
        if (lens[u] < 0 || lens[u] > kMaxLen)
            return SPD_ERR_LEN;
    if (head_per_wave < 0 || head_per_wave > 8)
        return SPD_ERR_SHAPE;
    // 1: the widest group; 2..8: the largest divisor of the KV head count up to that
    const int hpw = head_per_wave == 0 ? 0 : head_per_wave_waves(shape->n_kv_heads, head_per_wave == 1 ? 8 : head_per_wave);
    Schedule S;
    build_schedule(shape->n_kv_heads, n_users, lens, n_compute_units, hpw, tuning_from_env(), S);
    *n_items = (int64_t)S.items.size();
    if (chunk_tokens)
        *chunk_tokens = S.chunk_tokens;
    if (items) {
        if (capacity < (int64_t)S.items.size())
            return SPD_ERR_WORKSPACE;
        if (!S.items.empty())
            std::memcpy(items, S.items.data(), S.items.size() * sizeof(spd_work_item));
    }
    return SPD_OK;
} catch (...) {  // a failed host allocation (std::vector): no C++ exception leaves the library
    return SPD_ERR_NOMEM;
}

int spd_set_kernel_timing(spd_ctx *ctx, int32_t max_launches)
try {
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
} catch (...) {  // a failed host allocation (std::vector): no C++ exception leaves the library
    return SPD_ERR_NOMEM;
}

int spd_get_kernel_timing_samples(spd_ctx *ctx, int32_t entry_point, int32_t capacity, float *us, int32_t *n_launches)
{
    if (!ctx || !n_launches || (capacity > 0 && !us))
        return SPD_ERR_NULL;
    if (entry_point != 0 && entry_point != 1)
        return SPD_ERR_SHAPE;
    if (capacity < 0)
        return SPD_ERR_LEN;
    Owner &own = ctx->owner[entry_point];
    for (int i = 0; i < own.ev_used; ++i) {
        SPD_HIP(ctx, hipEventSynchronize(own.ev_stop[i]));
        float ms = 0.f;
        SPD_HIP(ctx, hipEventElapsedTime(&ms, own.ev_start[i], own.ev_stop[i]));
        if (i < capacity)
            us[i] = 1e3f * ms;
    }
    *n_launches = own.ev_used;
    own.ev_used = 0;
    return SPD_OK;
}

int spd_get_kernel_timing(spd_ctx *ctx, int32_t entry_point, int32_t *n_launches, double *mean_us, double *min_us)
try {
    if (!ctx || !n_launches || !mean_us || !min_us)
        return SPD_ERR_NULL;
    if (entry_point != 0 && entry_point != 1)
        return SPD_ERR_SHAPE;
    std::vector<float> us((size_t)ctx->owner[entry_point].ev_used);
    const int rc = spd_get_kernel_timing_samples(ctx, entry_point, (int32_t)us.size(), us.data(), n_launches);
    if (rc != SPD_OK)
        return rc;
    double sum = 0.0, mn = 0.0;
    for (size_t i = 0; i < us.size(); ++i) {
        sum += us[i];
        mn = (i == 0 || us[i] < mn) ? us[i] : mn;
    }
    *mean_us = us.empty() ? 0.0 : sum / (double)us.size();
    *min_us = mn;
    return SPD_OK;
} catch (...) {  // a failed host allocation (std::vector): no C++ exception leaves the library
    return SPD_ERR_NOMEM;
}

int spd_partial_attn_private(spd_ctx *ctx, const spd_shape *shape, const void *q, const spd_kv_view *priv, float *out,
                             float *lse, void *hip_stream)
{
    return no_throw([&] { return partial_attention(ctx, 0, shape, q, priv, out, lse, NewToken(), hip_stream); });
}

int spd_partial_attn_public_batched(spd_ctx *ctx, const spd_shape *shape, const void *q, const spd_kv_view *pub,
                                    float *out, float *lse, void *hip_stream)
{
    return no_throw([&] { return partial_attention(ctx, 1, shape, q, pub, out, lse, NewToken(), hip_stream); });
}

int spd_partial_attn_public_batched_append(spd_ctx *ctx, const spd_shape *shape, const void *q, const void *k_new,
                                           const void *v_new, const spd_kv_view *pub, float *out, float *lse,
                                           void *hip_stream)
{
    if (!k_new || !v_new)
        return SPD_ERR_NULL;
    NewToken nt;
    nt.k = k_new;
    nt.v = v_new;
    return no_throw([&] { return partial_attention(ctx, 1, shape, q, pub, out, lse, nt, hip_stream); });
}

int spd_decode_step(spd_ctx *ctx, const spd_shape *shape, const void *q, const spd_kv_view *priv,
                    const spd_kv_view *pub, const void *k_new, const void *v_new, float *a_in, float *lse_in,
                    float *a_out, float *lse_out, float *y, float *lse, float *w_in, void *hip_stream)
try {
    NewToken nt;
    nt.k = k_new;
    nt.v = v_new;
    if (!ctx)
        return SPD_ERR_NULL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int rc = validate_decode_step(ctx, shape, q, priv, pub, nt, a_in, lse_in, a_out, lse_out, y, lse, w_in);
    if (rc != SPD_OK || priv->n_users == 0)
        return rc;
    CachedSchedule *ep = nullptr, *eo = nullptr;
    const int hpw = fused_step_mapping(ctx, shape, priv, pub);
    const Tuning tune = fused_step_tuning(ctx, shape, priv, pub, hpw);
    rc = prepare_partial(ctx, 0, shape, q, priv, a_in, lse_in, hpw, &tune, stream, &ep);
    if (rc != SPD_OK)
        return rc;
    rc = prepare_partial(ctx, 1, shape, q, pub, a_out, lse_out, hpw, &tune, stream, &eo);  // an upload, if any, stays on `stream`
    if (rc != SPD_OK)
        return rc;
    return launch_decode_step(ctx, shape, q, priv, pub, nt, ep, eo, scratch_of(ctx->owner[0]), scratch_of(ctx->owner[1]), a_in,
                              lse_in, a_out, lse_out, y, lse, w_in, stream);
} catch (...) {  // a failed host allocation (std::vector): no C++ exception leaves the library
    return SPD_ERR_NOMEM;
}

int spd_decode_step_static(spd_ctx *ctx, const spd_shape *shape, const void *q, const spd_kv_view *priv,
                           const spd_kv_view *pub, const void *k_new, const void *v_new, float *a_in, float *lse_in,
                           float *a_out, float *lse_out, float *y, float *lse, float *w_in, void *hip_stream)
try {
    NewToken nt;
    nt.k = k_new;
    nt.v = v_new;
    if (!ctx)
        return SPD_ERR_NULL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int rc = validate_decode_step(ctx, shape, q, priv, pub, nt, a_in, lse_in, a_out, lse_out, y, lse, w_in);
    if (rc != SPD_OK || priv->n_users == 0)
        return rc;
    if (ctx->device >= kMaxDevices)
        return SPD_ERR_WORKSPACE;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticScratch &st = g_static[(size_t)ctx->device];
    if (!st.ptr)
        return SPD_ERR_WORKSPACE;
    const int hpw = fused_step_mapping(ctx, shape, priv, pub);
    const Tuning tune = fused_step_tuning(ctx, shape, priv, pub, hpw);
    const int G = shape->n_q_heads / shape->n_kv_heads;
    // both schedules are built and checked against the array's limits before anything is enqueued
    ScheduleBlob B[2];
    const spd_kv_view *views[2] = {priv, pub};
    std::vector<uint8_t> key[2];
    for (int w = 0; w < 2; ++w) {
        build_blob(shape, views[w], hpw, ctx->n_cus, tune, B[w]);
        make_key(shape, views[w], hpw, &tune.target_wg_per_cu, kTuningInts, key[w]);
        if (B[w].bytes.size() > kStaticSchedBytes || (size_t)B[w].n_slots * G + 4 > kStaticLseFloats ||
            (size_t)B[w].n_slots * G * shape->head_dim + 4 > kStaticPartOFloats)
            return SPD_ERR_WORKSPACE;
    }
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    SPD_HIP(ctx, hipStreamIsCapturing(stream, &capture));
    if (capture != hipStreamCaptureStatusNone)
        st.replayed = true;
    CachedSchedule e[2];
    ScratchPtrs sp[2];
    for (int w = 0; w < 2; ++w) {
        char *dst = st.ptr + (size_t)w * kStaticSchedBytes;
        // a schedule that the array already holds is not sent again - unless graph replays may have replaced it since
        if (st.replayed || st.key[w] != key[w]) {
            st.key[w].clear();
            rc = upload_through_args(ctx, B[w].bytes, dst, stream);
            if (rc != SPD_OK)
                return rc;
            if (!st.replayed)
                st.key[w] = key[w];
        }
        e[w].valid = true;
        e[w].dev = dst;
        e[w].n_items = B[w].n_items;
        e[w].n_slots = B[w].n_slots;
        e[w].n_segments = B[w].n_segments;
        e[w].hpw = hpw;
        e[w].n_split_rows = B[w].n_split_rows;
        e[w].off_rows = B[w].off_rows;
        e[w].off_info = B[w].off_info;
        sp[w].part_lse = reinterpret_cast<float *>(st.ptr + kStaticOffLse) + (size_t)w * kStaticLseFloats;
        sp[w].part_o = reinterpret_cast<float *>(st.ptr + kStaticOffPartO) + (size_t)w * kStaticPartOFloats;
    }
    return launch_decode_step(ctx, shape, q, priv, pub, nt, &e[0], &e[1], sp[0], sp[1], a_in, lse_in, a_out, lse_out, y, lse,
                              w_in, stream);
} catch (...) {  // a failed host allocation (std::vector): no C++ exception leaves the library
    return SPD_ERR_NOMEM;
}

int spd_public_attn_merge(spd_ctx *ctx, const spd_shape *shape, const void *q, const spd_kv_view *pub, const void *k_new,
                          const void *v_new, const float *a_in, const float *lse_in, float *a_out, float *lse_out,
                          float *y, float *lse, float *w_in, void *hip_stream)
try {
    NewToken nt;
    nt.k = k_new;
    nt.v = v_new;
    if (!ctx || !pub)
        return SPD_ERR_NULL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    SPD_HIP(ctx, hipSetDevice(ctx->device));
    int rc = spd_validate_partial(shape, q, pub, a_out, lse_out);
    if (rc == SPD_OK)
        rc = validate_new_token(pub, nt);
    if (rc != SPD_OK)
        return rc;
    if (pub->n_users == 0)
        return SPD_OK;
    if (!a_in || !lse_in || !y || !lse || !w_in)
        return SPD_ERR_NULL;
    if (!aligned16(a_in) || !aligned16(y))
        return SPD_ERR_ALIGN;
    CachedSchedule *eo = nullptr;
    rc = prepare_partial(ctx, 1, shape, q, pub, a_out, lse_out, -1, nullptr, stream, &eo);
    if (rc != SPD_OK)
        return rc;
    rc = launch_partial(ctx, 1, eo, pub, a_out, lse_out, scratch_of(ctx->owner[1]), nullptr, nullptr, nullptr, nullptr,
                        ScratchPtrs(), shape, q, nt, stream);
    if (rc != SPD_OK)
        return rc;
    // the closing kernel: combines the public rows that were split and merges; the private side arrives finished
    return launch_finalize(ctx, shape, pub->n_users, nullptr, eo, ScratchPtrs(), scratch_of(ctx->owner[1]), a_in, lse_in, nullptr,
                           nullptr, a_out, lse_out, y, lse, w_in, stream);
} catch (...) {  // a failed host allocation (std::vector): no C++ exception leaves the library
    return SPD_ERR_NOMEM;
}

int spd_attention_mass_track(spd_ctx *ctx, int32_t n_rows, const float *w_in, float threshold, float *mass_min,
                             float *mass_sum, int32_t *n_below, void *hip_stream)
{
    if (!ctx)
        return SPD_ERR_NULL;
    if (n_rows < 0)
        return SPD_ERR_LEN;
    if (n_rows == 0)
        return SPD_OK;
    if (!w_in)
        return SPD_ERR_NULL;
    SPD_HIP(ctx, hipSetDevice(ctx->device));
    hipLaunchKernelGGL(spd::mass_track_kernel, dim3((unsigned)((n_rows + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), n_rows, w_in, threshold, mass_min, mass_sum, n_below);
    SPD_HIP(ctx, hipGetLastError());
    return SPD_OK;
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
    const int vpr = head_dim / 4;              // at most 256
    const int rows_per_block = std::max(1, 256 / vpr);
    const unsigned blocks = (unsigned)(((int64_t)n_rows + rows_per_block - 1) / rows_per_block);
    hipLaunchKernelGGL(spd::lse_merge_kernel, dim3(blocks), dim3((unsigned)vpr, (unsigned)rows_per_block), 0,
                       static_cast<hipStream_t>(hip_stream), n_rows, vpr, a0, lse0, a1, lse1, y, lse_out, w0_out);
    SPD_HIP(ctx, hipGetLastError());
    return SPD_OK;
}

int spd_lse_merge_n(spd_ctx *ctx, int32_t n_parts, int32_t n_rows, int32_t head_dim, const float *const *a_parts,
                    const float *const *lse_parts, float *y, float *lse_out, float *w_out, void *hip_stream)
{
    if (!ctx)
        return SPD_ERR_NULL;
    if (n_rows < 0 || n_parts < 1 || n_parts > SPD_MAX_MERGE_PARTS)
        return SPD_ERR_LEN;
    if (head_dim <= 0 || head_dim % 4 != 0 || head_dim > 1024)
        return SPD_ERR_SHAPE;
    if (n_rows == 0)
        return SPD_OK;
    if (!a_parts || !lse_parts || !y)
        return SPD_ERR_NULL;
    spd::MergeParts parts = {};
    for (int k = 0; k < n_parts; ++k) {
        if (!a_parts[k] || !lse_parts[k])
            return SPD_ERR_NULL;
        if (!aligned16(a_parts[k]))
            return SPD_ERR_ALIGN;
        parts.a[k] = a_parts[k];
        parts.lse[k] = lse_parts[k];
    }
    if (!aligned16(y))
        return SPD_ERR_ALIGN;
    SPD_HIP(ctx, hipSetDevice(ctx->device));
    const int vpr = head_dim / 4;              // at most 256
    const int rows_per_block = std::max(1, 256 / vpr);
    const unsigned blocks = (unsigned)(((int64_t)n_rows + rows_per_block - 1) / rows_per_block);
    hipLaunchKernelGGL(spd::lse_merge_n_kernel, dim3(blocks), dim3((unsigned)vpr, (unsigned)rows_per_block), 0,
                       static_cast<hipStream_t>(hip_stream), (int)n_parts, (int)n_rows, vpr, parts, y, lse_out, w_out);
    SPD_HIP(ctx, hipGetLastError());
    return SPD_OK;
}

}  // extern "C"
