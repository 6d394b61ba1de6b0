// Host-only fuzz driver for the split schedule and the argument checks of the SPD library.
// Built by tests/test_host_sanitizers.py with AddressSanitizer and UBSan on the host pass, run without a GPU:
// it calls only spd_build_schedule and spd_validate_partial, which never touch the device.
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/spd.h"

static uint64_t state = 0x9e3779b97f4a7c15ull;
static uint64_t rnd()
{
    state ^= state << 7;
    state ^= state >> 9;
    return state * 0x2545f4914f6cdd1dull;
}

int main()
{
    int checked = 0;
    for (int iter = 0; iter < 400; ++iter) {
        const int n_users = (int)(rnd() % 40);
        static const int kv_choices[] = {1, 2, 4, 8, 3, 12, 16, 7, 32, 27};
        const int hkv = kv_choices[rnd() % 10];
        const int G = 1 << (rnd() % 4);
        // head-per-wave schedules: an item stands for `waves` consecutive KV heads
        // 0 head-major, 1 the widest group (up to 8 heads), 2..8 the widest group up to that many
        const int hpw = rnd() % 2 ? 1 + (int)(rnd() % 8) : 0;
        int waves = 1;
        if (hpw)
            for (int w = std::min(hkv, hpw == 1 ? 8 : hpw); w >= 1; --w)
                if (hkv % w == 0) {
                    waves = w;
                    break;
                }
        spd_shape sh = {SPD_BF16, hkv * G, hkv, 128, 0.088f};
        std::vector<int32_t> lens((size_t)n_users);
        for (auto &l : lens) {
            const unsigned kind = rnd() % 5;
            l = kind == 0 ? 0 : kind == 1 ? (int32_t)(rnd() % 64) : kind == 2 ? (int32_t)(rnd() % 3000)
                                                                             : (int32_t)(rnd() % 140000);
        }
        const int n_cus = 1 + (int)(rnd() % 300);
        int64_t n = -1;
        int32_t chunk = -1;
        int rc = spd_build_schedule(&sh, n_users, lens.data(), n_cus, hpw, nullptr, 0, &n, &chunk);
        if (rc != SPD_OK || n < 0) {
            std::printf("query failed rc=%d\n", rc);
            return 1;
        }
        std::vector<spd_work_item> items((size_t)n + 1);
        if (n > 0 && spd_build_schedule(&sh, n_users, lens.data(), n_cus, hpw, items.data(), n - 1, &n, &chunk) != SPD_ERR_WORKSPACE) {
            std::printf("short buffer accepted\n");
            return 1;
        }
        rc = spd_build_schedule(&sh, n_users, lens.data(), n_cus, hpw, items.data(), n, &n, &chunk);
        if (rc != SPD_OK) {
            std::printf("build failed rc=%d\n", rc);
            return 1;
        }
        // every token of every row exactly once, every partial slot used by exactly one (segment, head)
        std::vector<int64_t> covered((size_t)n_users * hkv, 0);
        std::vector<int64_t> slot_rows;
        for (int64_t i = 0; i < n; ++i) {
            const spd_work_item &w = items[(size_t)i];
            if (w.user < 0 || w.user >= n_users || w.kv_head < 0 || w.kv_head + waves > hkv || w.kv_head % waves != 0 ||
                w.t_begin < 0 || w.t_begin >= w.t_end || w.t_end > lens[(size_t)w.user] || w.t_begin % 32 != 0 ||
                w.n_chunks < 1 || w.chunk < 0 || w.chunk >= w.n_chunks || w.slot < 0) {
                std::printf("bad item %lld\n", (long long)i);
                return 1;
            }
            for (int j = 0; j < waves; ++j) {
                covered[(size_t)w.user * hkv + w.kv_head + j] += w.t_end - w.t_begin;
                slot_rows.push_back((int64_t)w.slot + (int64_t)j * w.n_chunks);
            }
        }
        std::sort(slot_rows.begin(), slot_rows.end());
        for (size_t i = 0; i < slot_rows.size(); ++i)
            if (slot_rows[i] != (int64_t)i) {   // dense and unique: the partial buffers are sized by their count
                std::printf("slot %lld used twice or skipped\n", (long long)slot_rows[i]);
                return 1;
            }
        for (int u = 0; u < n_users; ++u)
            for (int h = 0; h < hkv; ++h)
                if (covered[(size_t)u * hkv + h] != lens[(size_t)u]) {
                    std::printf("coverage mismatch user %d head %d\n", u, h);
                    return 1;
                }
        // validation with consistent fake addresses never reads through them
        std::vector<const void *> kp((size_t)n_users, (const void *)0x10000), vp((size_t)n_users, (const void *)0x20000);
        spd_kv_view v = {};
        v.n_users = n_users;
        v.lens = lens.data();
        v.k_ptrs = kp.data();
        v.v_ptrs = vp.data();
        v.token_stride = 128 * (int64_t)hkv;
        v.head_stride = 128;
        rc = spd_validate_partial(&sh, (const void *)0x1000, &v, (const float *)0x2000, (const float *)0x3000);
        if (rc != SPD_OK) {
            std::printf("validate rc=%d\n", rc);
            return 1;
        }
        ++checked;
    }
    std::printf("ok %d\n", checked);
    return 0;
}
