// Host-only fuzz driver for the tables the kernels read of a schedule (work items linked into pieces, split rows,
// per-row slot bookkeeping).  Built by tests/test_host_sanitizers.py with AddressSanitizer and UBSan, run without a
// GPU: it includes the library's host headers and makes no HIP call.
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "../../paper_2409_19134_amd/csrc/schedule.hpp"

using namespace spd::host;

static uint64_t state = 0x243f6a8885a308d3ull;
static uint64_t rnd()
{
    state ^= state << 7;
    state ^= state >> 9;
    return state * 0x2545f4914f6cdd1dull;
}

#define FAIL(...)                 \
    do {                          \
        std::printf(__VA_ARGS__); \
        std::printf("\n");        \
        return 1;                 \
    } while (0)

int main()
{
    int checked = 0;
    for (int iter = 0; iter < 600; ++iter) {
        const int n_users = (int)(rnd() % 24);
        static const int kv_choices[] = {1, 2, 4, 8, 3, 12, 16, 7};
        const int Hkv = kv_choices[rnd() % 8];
        // 0: head-major mapping; else the KV heads per workgroup of the head-per-wave mapping (any divisor up to 8)
        const int hpw = rnd() % 2 ? head_per_wave_waves(Hkv, 1 + (int)(rnd() % 8)) : 0;
        const int waves = hpw ? hpw : 1;
        const int es = rnd() % 2 ? 2 : 4;
        const int d = rnd() % 2 ? 64 : 128;
        const bool offsets = rnd() % 3 == 0;  // paged mode: the items hold offsets from head 0, no addresses
        std::vector<int32_t> lens((size_t)n_users);
        for (auto &l : lens) {
            const unsigned kind = rnd() % 5;
            l = kind == 0 ? 0 : kind == 1 ? (int32_t)(rnd() % 700) : kind == 2 ? (int32_t)(rnd() % 3000)
                                                                             : (int32_t)(rnd() % 90000);
        }
        const int n_cus = 1 + (int)(rnd() % 300);
        // addresses are only computed, never read
        std::vector<const void *> kp((size_t)n_users), vp((size_t)n_users);
        for (int u = 0; u < n_users; ++u) {
            kp[(size_t)u] = reinterpret_cast<const void *>((uintptr_t)0x100000000ull * (uintptr_t)(2 * u + 1));
            vp[(size_t)u] = reinterpret_cast<const void *>((uintptr_t)0x100000000ull * (uintptr_t)(2 * u + 2));
        }
        spd_kv_view v = {};
        v.n_users = n_users;
        v.lens = lens.data();
        v.k_ptrs = kp.data();
        v.v_ptrs = vp.data();
        v.block_size = offsets ? 16 : 0;
        v.token_stride = hpw ? (int64_t)d * Hkv : d;
        v.head_stride = hpw ? d : (int64_t)d * 100000;

        Tuning tune;  // the defaults, or anything a context's options allow
        if (rnd() % 2) {
            tune.target_wg_per_cu = 1 + (int)(rnd() % 4);
            tune.no_split_max = 1 + (int)(rnd() % 2000);
            tune.chunk_max = 1 + (int)(rnd() % 40000);
            tune.seg_cost = (int)(rnd() % 9);
            tune.half_skew = (int)(rnd() % 91);
        }
        Schedule S;
        build_schedule(Hkv, n_users, lens.data(), n_cus, hpw, tune, S);
        DeviceTables T;
        build_device_tables(S, Hkv, es, &v, hpw, T);

        const int64_t n_launched = T.items_launched;
        const int64_t n_pieces = (int64_t)S.piece_first.size() - 1;
        if (n_launched < n_pieces || n_launched > (int64_t)T.items.size())
            FAIL("launched %lld of %zu items, %lld pieces", (long long)n_launched, T.items.size(), (long long)n_pieces);
        if (T.n_segments != (int64_t)S.items.size())
            FAIL("segment count %lld of %zu", (long long)T.n_segments, S.items.size());
        if (!hpw) {
            // what the fused step asks before it looks a schedule up: one resident round of equal pieces, or not
            int64_t rows = -1, steps = -1;
            const int64_t round = single_round_pieces(Hkv, n_users, lens.data(), n_cus, tune, &rows, &steps);
            int64_t rows_with_tokens = 0, steps_per_head = 0;
            for (int u = 0; u < n_users; ++u) {
                rows_with_tokens += lens[(size_t)u] > 0 ? Hkv : 0;
                steps_per_head += (lens[(size_t)u] + 31) / 32;
            }
            if (rows != rows_with_tokens || steps != steps_per_head)
                FAIL("rows %lld, expected %lld; steps %lld, expected %lld", (long long)rows, (long long)rows_with_tokens,
                     (long long)steps, (long long)steps_per_head);
            const int64_t resident = (int64_t)n_cus * tune.target_wg_per_cu;
            if (round < 0 || round > std::max<int64_t>(resident, Hkv) || round % Hkv)
                FAIL("round of %lld pieces with %lld resident", (long long)round, (long long)resident);
            // (a cut moved to a row boundary can leave a piece without steps, so the schedule may hold fewer)
            if (round > 0 && (n_pieces > round || (tune.seg_cost == 0 && n_pieces != round)))
                FAIL("%lld pieces where a round of %lld was announced", (long long)n_pieces, (long long)round);
        }

        // every item is reached exactly once: launched ones by their index, the others through one `next` link
        std::vector<int> reached(T.items.size(), 0);
        std::vector<int64_t> covered((size_t)n_users * Hkv, 0), slots_used;
        std::vector<int> empty_seen((size_t)n_users * Hkv, 0);
        for (int64_t first = 0; first < n_launched; ++first) {
            int steps = 0;  // 32-token steps the piece has handed out before the segment
            for (int64_t at = first; at >= 0; at = T.items[(size_t)at].next) {
                if (at >= (int64_t)T.items.size() || (at != first && at < n_launched))
                    FAIL("link to %lld leaves the continuation range", (long long)at);
                if (reached[(size_t)at]++)
                    FAIL("item %lld reached twice", (long long)at);
                const spd::DevItem &it = T.items[(size_t)at];
                if (it.user < 0 || it.user >= n_users || it.kv_head < 0 || it.kv_head % waves || it.kv_head + waves > Hkv)
                    FAIL("item %lld names no row", (long long)at);
                const int32_t len = lens[(size_t)it.user];
                if (it.t_begin == it.t_end) {
                    // a row without tokens: a launched item of its own that only writes the empty partial
                    if (len != 0 || it.t_begin != 0 || at != first || it.next != -1 || first < n_pieces)
                        FAIL("empty item %lld", (long long)at);
                    for (int j = 0; j < waves; ++j)
                        ++empty_seen[(size_t)it.user * Hkv + it.kv_head + j];
                    continue;
                }
                if (it.t_begin < 0 || it.t_begin % 32 || it.t_begin > it.t_end || it.t_end > len)
                    FAIL("item %lld token range", (long long)at);
                if (((it.rot & spd::kEndsRow) != 0) != (it.t_end == len))
                    FAIL("item %lld end-of-row flag", (long long)at);
                if ((it.rot & ~spd::kEndsRow) != (steps & (spd::kWaves - 1)))
                    FAIL("item %lld rotation %d after %d steps", (long long)at, it.rot, steps);
                steps += (it.t_end - it.t_begin + 31) / 32;
                const spd::RowInfo &row = T.row_info[(size_t)it.user * Hkv + it.kv_head];
                if (it.n_chunks != row.n_chunks || it.slot < row.first_slot || it.slot >= row.first_slot + row.n_chunks)
                    FAIL("item %lld slot outside its row's", (long long)at);
                // the row address: the user's pointer plus the head's offset, or the offset alone; head per wave:
                // head 0's, every wave adds its own
                const int64_t off = hpw ? 0 : (int64_t)it.kv_head * v.head_stride * es;
                const uintptr_t want_k = (offsets ? 0 : (uintptr_t)kp[(size_t)it.user]) + (uintptr_t)off;
                const uintptr_t want_v = (offsets ? 0 : (uintptr_t)vp[(size_t)it.user]) + (uintptr_t)off;
                if ((uintptr_t)it.k_base != want_k || (uintptr_t)it.v_base != want_v)
                    FAIL("item %lld row address", (long long)at);
                for (int j = 0; j < waves; ++j) {
                    covered[(size_t)it.user * Hkv + it.kv_head + j] += it.t_end - it.t_begin;
                    slots_used.push_back((int64_t)it.slot + (int64_t)j * it.n_chunks);
                }
            }
        }
        for (size_t i = 0; i < reached.size(); ++i)
            if (reached[i] != 1)
                FAIL("item %zu reached %d times", i, reached[i]);
        std::sort(slots_used.begin(), slots_used.end());
        if ((int64_t)slots_used.size() != S.n_slots)
            FAIL("%zu slots used, %lld counted", slots_used.size(), (long long)S.n_slots);
        for (size_t i = 0; i < slots_used.size(); ++i)
            if (slots_used[i] != (int64_t)i)
                FAIL("slot %lld used twice or skipped", (long long)slots_used[i]);

        // rows: tokens covered once, bookkeeping of every row, split rows listed exactly once
        std::vector<int> listed((size_t)n_users * Hkv, 0);
        for (const spd::CombineRow &r : T.split_rows) {
            if (r.user < 0 || r.user >= n_users || r.kv_head < 0 || r.kv_head >= Hkv)
                FAIL("split row names no row");
            const spd::RowInfo &row = T.row_info[(size_t)r.user * Hkv + r.kv_head];
            if (r.n_chunks < 2 || r.n_chunks != row.n_chunks || r.first_slot != row.first_slot)
                FAIL("split row %d/%d disagrees with its bookkeeping", r.user, r.kv_head);
            ++listed[(size_t)r.user * Hkv + r.kv_head];
        }
        for (int u = 0; u < n_users; ++u)
            for (int h = 0; h < Hkv; ++h) {
                const size_t r = (size_t)u * Hkv + h;
                if (covered[r] != lens[(size_t)u])
                    FAIL("coverage of user %d head %d", u, h);
                if (empty_seen[r] != (lens[(size_t)u] == 0 ? 1 : 0))
                    FAIL("empty row %d/%d written %d times", u, h, empty_seen[r]);
                if (lens[(size_t)u] == 0 ? T.row_info[r].n_chunks != 0 : T.row_info[r].n_chunks < 1)
                    FAIL("chunk count of row %d/%d", u, h);
                if (listed[r] != (T.row_info[r].n_chunks > 1 ? 1 : 0))
                    FAIL("row %d/%d listed %d times among the split rows", u, h, listed[r]);
            }
        ++checked;
    }
    std::printf("ok %d\n", checked);
    return 0;
}
