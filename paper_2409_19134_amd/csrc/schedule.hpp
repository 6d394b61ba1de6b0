// The split schedule of a partial-attention launch (host only, no HIP calls).
#pragma once
#include <algorithm>
#include <cstdint>
#include <cstdlib>
#include <vector>

#include "../../include/spd.h"
#include "common.hpp"

namespace spd::host {

constexpr int kChunkAlign = 32;      // chunk boundaries are multiples of the MFMA kernel's 32-token step
constexpr int kChunkMin = 128;       // one 32-token step for each of the four waves
constexpr int kShortPieceSteps = 64;  // 32-token steps per piece up to which Tuning::seg_cost and half_skew apply
// (32-token steps * KV heads) per CU from which the head-per-wave mapping is used, and from which its workgroups take
// eight heads instead of four (see head_per_wave_choice in spd_api.hip)
constexpr int kHeadPerWaveMinHeadSteps = 65;
constexpr int kHeadPerWaveWideHeadSteps = 900;

// What shapes a schedule besides the lengths.  A context starts from the defaults below, replaced by SPD_* variables
// of the environment that spd_create finds set (tuning_from_env), and spd_set_option changes them per context; all
// of them are part of the key a cached schedule is remembered by.
struct Tuning {
    // workgroups of the MFMA kernel resident per CU (2 waves per SIMD)                        SPD_TARGET_WG_PER_CU
    int32_t target_wg_per_cu = 2;
    // if no row is longer than this the work is latency-bound: every row is cut into chunks of one step per wave
    //                                                                                          SPD_NO_SPLIT_MAX
    int32_t no_split_max = 768;
    // tokens per piece when the work exceeds one resident round: a new workgroup costs a few microseconds of an idle
    // slot, more than the longer tail of bigger pieces (4096: 3 % slower on the longest workload)  SPD_CHUNK_MAX
    int32_t chunk_max = 16384;
    // 32-token steps a piece gives up for every further row it reaches into (a second segment costs an epilogue and a
    // memory round trip before the new row's first tile; measured on the headline workload: 0 -> 2 steps takes
    // 0.45 us off a 32.5 us step, 4 and more give it back)                                      SPD_SEG_COST
    int32_t seg_cost = 2;
    // When the pieces are exactly one resident round, the half dispatched first gets (100 + s) % of the mean piece and
    // the other half (100 - s) %: every workgroup asks for its first tile in the same microsecond, the memory system
    // serves those ~35 MB in launch order, and the half served last stays ~4 us behind to the end (measured with
    // in-kernel time stamps); unequal shares let both halves finish together (0 -> 12 %: -0.35 us)  SPD_HALF_SKEW
    int32_t half_skew = 12;
};
constexpr int kTuningInts = 5;
static_assert(sizeof(Tuning) == kTuningInts * sizeof(int32_t), "the key takes the struct as kTuningInts integers");

inline int env_int(const char *name, int dflt, int least = 1)
{
    const char *s = std::getenv(name);
    if (!s || !*s)
        return dflt;
    const long v = std::strtol(s, nullptr, 10);
    return v >= least && v <= (1 << 30) ? (int)v : dflt;
}

inline Tuning tuning_from_env()
{
    Tuning t;
    t.target_wg_per_cu = env_int("SPD_TARGET_WG_PER_CU", t.target_wg_per_cu);
    t.no_split_max = env_int("SPD_NO_SPLIT_MAX", t.no_split_max);
    t.chunk_max = env_int("SPD_CHUNK_MAX", t.chunk_max);
    t.seg_cost = env_int("SPD_SEG_COST", t.seg_cost, 0);
    t.half_skew = std::min(90, env_int("SPD_HALF_SKEW", t.half_skew, 0));
    return t;
}

// The split schedule ("stream-K" over tokens).  All KV heads of a user hold the same tokens, so the schedule is laid
// out on token steps (32 tokens) per user and replicated over the KV heads: the steps of all users, laid end to end,
// are divided into groups of equal length (+-1 step), and every group becomes one piece (one workgroup) per KV head.
// The pieces of a group are adjacent in launch order, so with token-major storage the heads that share DRAM pages
// stream them at the same time.  A group that crosses a user boundary gives pieces with several segments.
// Equal pieces matter because the path is HBM-bound: a launch lasts as long as its longest workgroup.
//   - if no user is longer than a few hundred tokens the work is latency-bound: every row is cut into chunks of 128
//     tokens (one step per wave: one memory round trip).  That also holds for a standalone call, although it then
//     needs the combine launch: whole rows of up to 512 tokens per workgroup measured 2.4 us slower;
//   - work that fits one resident wave of workgroups (2 per CU) gets exactly that many pieces;
//   - larger work gets pieces of at most `piece_max` tokens, their number rounded up to a multiple of the resident
//     wave, and relies on the hardware's dynamic workgroup dispatch.
struct Schedule {
    std::vector<spd_work_item> items;  // segments in piece order (rows with tokens only)
    std::vector<int32_t> piece_first;  // [n_pieces + 1] first segment of each piece
    int64_t n_slots = 0;
    int chunk_tokens = 0;              // tokens per piece (rounded up)
};

// hpw: pieces for the head-per-wave kernel (token-major storage).  A piece then covers all KV heads of its token
// range (a group of up to eight of them, see head_per_wave_waves): one item per cut and group (kv_head and slot are
// those of the group's first head) and one resident workgroup per CU.  The same
// token limit per piece serves both mappings (smaller pieces measured slower here too), although every wave now
// walks the whole range instead of a quarter of it.
// Waves (KV heads) per workgroup of the head-per-wave mapping: the largest divisor of Hkv that is at most `most`
// (8: two waves per SIMD is what the kernel's registers allow); Hkv / that many head groups share a token range.
inline int head_per_wave_waves(int Hkv, int most = 8)
{
    for (int w = std::min(Hkv, std::min(most, 8)); w >= 1; --w)
        if (Hkv % w == 0)
            return w;
    return 1;
}

// The number of pieces build_schedule makes for the head-major mapping if they are exactly one resident round of
// equal pieces (target_wg_per_cu per CU), else 0 (short rows cut into one-step chunks, less work than a round, or
// several rounds).  Costs a pass over the lengths: the fused step asks before it looks its schedules up.
// *rows: the (user, KV head) rows that hold tokens; *steps (if asked for): the 32-token steps of one KV head.
inline int64_t single_round_pieces(int Hkv, int n_users, const int32_t *lens, int n_cus, const Tuning &tune, int64_t *rows,
                                   int64_t *steps_out = nullptr)
{
    int64_t T = 0, short_chunks = 0;
    int max_len = 0;
    *rows = 0;
    for (int u = 0; u < n_users; ++u) {
        const int64_t steps = (lens[u] + kChunkAlign - 1) / kChunkAlign;
        T += steps;
        short_chunks += (steps + spd::kWaves - 1) / spd::kWaves;
        max_len = std::max(max_len, lens[u]);
        *rows += lens[u] > 0 ? Hkv : 0;
    }
    if (steps_out)
        *steps_out = T;
    const int64_t resident = (int64_t)std::max(1, n_cus) * tune.target_wg_per_cu;
    if (T == 0 || (max_len <= tune.no_split_max && short_chunks * Hkv <= resident))
        return 0;
    const int64_t wg = std::max<int64_t>(1, resident / Hkv);
    const int64_t piece_max = std::max(kChunkMin, (int)tune.chunk_max) / kChunkAlign;
    if (T > wg * piece_max || (T + spd::kWaves - 1) / spd::kWaves < wg)
        return 0;
    return wg * Hkv;
}

// hpw: 0 for the head-major mapping, else the KV heads (waves) per workgroup of the head-per-wave mapping, a divisor
// of Hkv that is at most 8.
inline void build_schedule(int Hkv, int n_users, const int32_t *lens, int n_cus, int hpw, const Tuning &tune, Schedule &S)
{
    const int hpw_waves = hpw ? hpw : 1;
    const int hpw_groups = hpw ? Hkv / hpw_waves : 1;
    S.items.clear();
    S.piece_first.assign(1, 0);
    S.n_slots = 0;
    S.chunk_tokens = 0;
    int64_t T = 0;  // total 32-token steps per KV head
    int max_len = 0;
    for (int u = 0; u < n_users; ++u) {
        T += (lens[u] + kChunkAlign - 1) / kChunkAlign;
        max_len = std::max(max_len, lens[u]);
    }
    if (T == 0)
        return;

    // a group: user-local step ranges; cut[g] lists (user, first step, end step)
    struct Cut {
        int user;
        int64_t s0, s1;
    };
    std::vector<std::vector<Cut>> groups;
    // Short rows are cut into chunks of one step per wave - unless that makes more workgroups than fit the machine
    // at once: many users with short rows are bandwidth-bound like any large launch and get equal pieces instead
    // (measured, 64 users x <= 512 + 256 tokens, 117 MB: 31.7 us against 35.6 us per fused step).
    int64_t short_chunks = 0;
    for (int u = 0; u < n_users; ++u)
        short_chunks += ((lens[u] + kChunkAlign - 1) / kChunkAlign + spd::kWaves - 1) / spd::kWaves;
    const int64_t resident = (int64_t)std::max(1, n_cus) * tune.target_wg_per_cu;
    if (max_len <= tune.no_split_max && short_chunks * (hpw ? hpw_groups : Hkv) <= resident) {
        const int64_t per = spd::kWaves;  // steps per chunk
        for (int u = 0; u < n_users; ++u) {
            const int64_t steps = (lens[u] + kChunkAlign - 1) / kChunkAlign;
            for (int64_t s0 = 0; s0 < steps; s0 += per)
                groups.push_back({Cut{u, s0, std::min(steps, s0 + per)}});
        }
        S.chunk_tokens = (int)std::min<int64_t>(per, (max_len + kChunkAlign - 1) / kChunkAlign) * kChunkAlign;
    } else {
        const int64_t slots = resident;
        // groups per resident wave of workgroups
        // head per wave: a CU holds eight such waves, i.e. 8 / waves workgroups
        const int64_t wg = hpw ? std::max<int64_t>(1, (int64_t)std::max(1, n_cus) * (8 / hpw_waves) / hpw_groups)
                               : std::max<int64_t>(1, slots / Hkv);
        const int64_t piece_max = std::max(kChunkMin, (int)tune.chunk_max) / kChunkAlign;
        // group boundaries (cumulative step counts)
        std::vector<int64_t> ends;
        std::vector<int64_t> cut_num;  // group i ends at the fraction cut_num[i] / cut_den of the line
        int64_t cut_den = 1;
        if (T <= wg * piece_max) {
            // at least one step per wave
            // (measured on the headline workload: fewer, round-aligned pieces or more pieces than fit at once are
            // both slower - 55 groups of 20 steps +2 us, 80 groups +1.5 us against 64 groups of 17-18 steps)
            const int64_t W = std::min<int64_t>(wg, hpw ? T : (T + spd::kWaves - 1) / spd::kWaves);
            // exactly one resident round of head-major pieces of 8 to kShortPieceSteps steps: unequal halves (see Tuning;
            // the ~4 us by which the second half trails do not matter to longer pieces: workload 4, 214 steps, +0.2 %)
            const int64_t skew = (!hpw && W == wg && W >= 2 && T >= 8 * W && T <= kShortPieceSteps * W) ? tune.half_skew : 0;
            for (int64_t i = 0; i < W; ++i) {
                const int64_t h = W / 2;
                // cumulative weight up to group i (inclusive), in percent-groups
                const int64_t cum = (i + 1 <= h) ? (i + 1) * (100 + skew) : h * (100 + skew) + (i + 1 - h) * (100 - skew);
                const int64_t tot = h * (100 + skew) + (W - h) * (100 - skew);
                ends.push_back(T * cum / tot);
                cut_num.push_back(cum);
                cut_den = tot;
            }
        } else {
            // several resident waves of equal pieces; the hardware hands them out in launch order.  (Cutting the last
            // wave's share finer to shorten the tail was measured and lost 1-3 %: short pieces cost more than the tail.)
            const int64_t W = wg * ((T + wg * piece_max - 1) / (wg * piece_max));
            for (int64_t i = 0; i < W; ++i) {
                ends.push_back(T * (i + 1) / W);
                cut_num.push_back(i + 1);
            }
            cut_den = W;
        }
        // A piece that crosses into another user's row pays for a second segment (an epilogue, and a memory round
        // trip before the new row's first tile): such pieces get `seg_cost` steps fewer.  The cuts are made on a line
        // that holds seg_cost extra steps in front of every user but the first; a cut that lands in such a gap moves
        // to the user's boundary.
        // Only for pieces of up to kShortPieceSteps steps: measured, 2 steps take 1.4 % off the headline workload's step
        // (pieces of 17 steps) and 3 % off 256 users with 64-512-token rows (36 steps), but add 0.9 % to workload 4
        // (pieces of 214 steps over four rows each), where the unequal lengths cost more than the segments.
        const int64_t seg_cost = T <= kShortPieceSteps * (int64_t)ends.size() ? tune.seg_cost : 0;
        if (seg_cost > 0) {
            int64_t n_rows_with_tokens = 0;
            for (int u = 0; u < n_users; ++u)
                n_rows_with_tokens += lens[u] > 0;
            const int64_t Tv = T + seg_cost * std::max<int64_t>(0, n_rows_with_tokens - 1);
            size_t i = 0;
            int64_t real0 = 0, virt0 = 0;  // the current user's first step on the real and on the stretched line
            bool first = true;
            for (int u = 0; u < n_users && i < ends.size(); ++u) {
                const int64_t steps = (lens[u] + kChunkAlign - 1) / kChunkAlign;
                if (steps == 0)
                    continue;
                if (!first)
                    virt0 += seg_cost;
                first = false;
                // cuts (on the stretched line) up to the end of this user's steps
                while (i < ends.size()) {
                    const int64_t cut = Tv * cut_num[i] / cut_den;
                    if (cut > virt0 + steps)
                        break;
                    ends[i++] = real0 + std::max<int64_t>(0, cut - virt0);
                }
                real0 += steps;
                virt0 += steps;
            }
            for (; i < ends.size(); ++i)
                ends[i] = T;
            ends.back() = T;
        }
        const int64_t W = (int64_t)ends.size();
        int64_t longest = ends[0];
        for (size_t i = 1; i < ends.size(); ++i)
            longest = std::max(longest, ends[i] - ends[i - 1]);
        S.chunk_tokens = (int)longest * kChunkAlign;
        groups.resize((size_t)W);
        int64_t g0 = 0;  // global step index of the current user's first step
        int64_t g = 0;
        for (int u = 0; u < n_users; ++u) {
            const int64_t steps = (lens[u] + kChunkAlign - 1) / kChunkAlign;
            int64_t s = 0;
            while (s < steps) {
                while (ends[(size_t)g] <= g0 + s)
                    ++g;
                const int64_t e = std::min(steps, ends[(size_t)g] - g0);
                groups[(size_t)g].push_back(Cut{u, s, e});
                s = e;
            }
            g0 += steps;
        }
    }

    // chunks per user (same for all its KV heads) and the first partial slot of every row
    std::vector<int32_t> n_chunks((size_t)n_users, 0), seen((size_t)n_users, 0);
    for (const auto &grp : groups)
        for (const Cut &c : grp)
            ++n_chunks[(size_t)c.user];
    std::vector<int64_t> user_slot0((size_t)n_users, 0);
    for (int u = 0; u < n_users; ++u) {
        user_slot0[(size_t)u] = S.n_slots;
        S.n_slots += (int64_t)n_chunks[(size_t)u] * Hkv;
    }
    int32_t piece = 0;
    for (const auto &grp : groups) {
        if (grp.empty())
            continue;
        for (int hh = 0; hh < (hpw ? hpw_groups : Hkv); ++hh) {
            const int h = hpw ? hh * hpw_waves : hh;  // head per wave: the first head of the group
            for (const Cut &c : grp) {
                spd_work_item it;
                it.user = c.user;
                it.kv_head = h;
                it.t_begin = (int32_t)(c.s0 * kChunkAlign);
                it.t_end = (int32_t)std::min<int64_t>(lens[c.user], c.s1 * kChunkAlign);
                it.n_chunks = n_chunks[(size_t)c.user];
                it.chunk = seen[(size_t)c.user];
                it.slot = (int32_t)(user_slot0[(size_t)c.user] + (int64_t)h * it.n_chunks + it.chunk);
                it.piece = piece;
                S.items.push_back(it);
            }
            ++piece;
            S.piece_first.push_back((int32_t)S.items.size());
        }
        for (const Cut &c : grp)
            ++seen[(size_t)c.user];
    }
}

// What the kernels read of a schedule, as it is laid out in device memory.
struct DeviceTables {
    std::vector<spd::DevItem> items;          // [items_launched] first segments and empty rows, then the continuation segments
    std::vector<spd::CombineRow> split_rows;  // rows held in more than one partial slot
    std::vector<spd::RowInfo> row_info;       // [n_users * Hkv] first slot and slot count of every row
    int64_t items_launched = 0;               // workgroups of the launch
    int64_t n_segments = 0;                   // segments with tokens, all pieces together
};

// es: bytes per K/V element.  Row addresses come from the view's host pointer arrays (contiguous mode without device
// pointer tables); in the other modes the items hold offsets and the kernel adds the pool or the user's pointer.
inline void build_device_tables(const Schedule &S, int Hkv, int es, const spd_kv_view *v, int hpw, DeviceTables &T)
{
    using spd::CombineRow;
    using spd::DevItem;
    using spd::RowInfo;
    // device items: the first segment of every piece (index = workgroup id), then one per row without tokens (it only
    // writes A = 0, lse = -inf), then the continuation segments, linked through `next`
    const int hpw_waves = hpw ? hpw : 1;  // heads an item stands for
    const int64_t n_pieces = (int64_t)S.piece_first.size() - 1;
    int64_t n_empty_rows = 0;  // workgroups that only write A = 0, lse = -inf (head-per-wave: one per empty user)
    for (int u = 0; u < v->n_users; ++u)
        n_empty_rows += v->lens[u] == 0 ? (hpw ? Hkv / hpw_waves : Hkv) : 0;
    const int64_t n_groups = n_pieces + n_empty_rows;  // launched workgroups
    std::vector<DevItem> &dev_items = T.items;
    dev_items.assign((size_t)n_groups, DevItem{});
    dev_items.reserve((size_t)n_groups + S.items.size());
    // the row's address - or, where the kernel adds the pool or the user's pointer itself, its offset from that
    auto row_base = [&](int u, int h, bool is_v) -> const char * {
        const uintptr_t base = (v->block_size || v->k_ptrs_dev) ? 0 : reinterpret_cast<uintptr_t>(is_v ? v->v_ptrs[u] : v->k_ptrs[u]);
        const int64_t hs = (v->head_strides && v->block_size == 0) ? v->head_strides[u] : v->head_stride;
        // head per wave: every wave adds its own head's offset (from head 0)
        return reinterpret_cast<const char *>(base + (uintptr_t)(hpw ? 0 : (int64_t)h * hs * es));
    };
    auto to_dev = [&](const spd_work_item &w, int rot) {
        DevItem d;
        d.k_base = row_base(w.user, w.kv_head, false);
        d.v_base = row_base(w.user, w.kv_head, true);
        d.user = w.user;
        d.kv_head = w.kv_head;
        d.t_begin = w.t_begin;
        d.t_end = w.t_end;
        d.slot = w.slot;
        d.n_chunks = w.n_chunks;
        d.next = -1;
        d.rot = (rot & (spd::kWaves - 1)) | (w.t_end == v->lens[w.user] ? spd::kEndsRow : 0);
        return d;
    };
    for (int64_t pc = 0; pc < n_pieces; ++pc) {
        int rot = 0;
        size_t prev = 0;
        for (int32_t i = S.piece_first[(size_t)pc]; i < S.piece_first[(size_t)pc + 1]; ++i) {
            const spd_work_item &w = S.items[(size_t)i];
            const DevItem d = to_dev(w, rot);
            size_t at;
            if (i == S.piece_first[(size_t)pc]) {
                at = (size_t)pc;
                dev_items[at] = d;
            } else {
                at = dev_items.size();
                dev_items.push_back(d);
                dev_items[prev].next = (int32_t)at;
            }
            prev = at;
            rot += (w.t_end - w.t_begin + kChunkAlign - 1) / kChunkAlign;
        }
    }
    {
        size_t at = (size_t)n_pieces;
        for (int u = 0; u < v->n_users; ++u) {
            if (v->lens[u] != 0)
                continue;
            for (int hh = 0; hh < (hpw ? Hkv / hpw_waves : Hkv); ++hh) {
                DevItem d;
                d.k_base = d.v_base = nullptr;
                d.user = u;
                d.kv_head = hpw ? hh * hpw_waves : hh;
                d.t_begin = d.t_end = 0;
                d.slot = d.n_chunks = d.rot = 0;
                d.next = -1;
                dev_items[at++] = d;
            }
        }
    }
    std::vector<CombineRow> &split_rows = T.split_rows;
    split_rows.clear();
    for (size_t i = 0; i < S.items.size(); ++i) {
        const spd_work_item &w = S.items[i];
        if (w.chunk == 0 && w.n_chunks > 1)
            for (int h = 0; h < hpw_waves; ++h)  // a head-per-wave item stands for the KV heads of its group
                split_rows.push_back(CombineRow{w.slot + h * w.n_chunks, w.n_chunks, w.user, w.kv_head + h});
    }
    std::vector<RowInfo> &row_info = T.row_info;
    row_info.assign((size_t)v->n_users * Hkv, RowInfo{0, 0});
    for (const spd_work_item &w : S.items)
        if (w.chunk == 0)
            for (int h = 0; h < hpw_waves; ++h)
                row_info[(size_t)w.user * Hkv + w.kv_head + h] = RowInfo{w.slot + h * w.n_chunks, w.n_chunks};
    T.items_launched = n_groups;
    T.n_segments = (int64_t)S.items.size();
}

}  // namespace spd::host
