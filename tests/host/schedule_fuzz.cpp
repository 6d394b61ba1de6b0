// Host-only fuzz driver for the split schedule and the argument checks of the SPD library.
// Built by tests/test_host_sanitizers.py with AddressSanitizer and UBSan on the host pass, run without a GPU:
// it calls only spd_build_schedule and spd_validate_partial, which never touch the device.
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
        const int hkv = 1 << (rnd() % 4);
        const int G = 1 << (rnd() % 4);
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
        int rc = spd_build_schedule(&sh, n_users, lens.data(), n_cus, nullptr, 0, &n, &chunk);
        if (rc != SPD_OK || n < 0) {
            std::printf("query failed rc=%d\n", rc);
            return 1;
        }
        std::vector<spd_work_item> items((size_t)n + 1);
        if (n > 0 && spd_build_schedule(&sh, n_users, lens.data(), n_cus, items.data(), n - 1, &n, &chunk) != SPD_ERR_WORKSPACE) {
            std::printf("short buffer accepted\n");
            return 1;
        }
        rc = spd_build_schedule(&sh, n_users, lens.data(), n_cus, items.data(), n, &n, &chunk);
        if (rc != SPD_OK) {
            std::printf("build failed rc=%d\n", rc);
            return 1;
        }
        // every token of every row exactly once
        std::vector<int64_t> covered((size_t)n_users * hkv, 0);
        for (int64_t i = 0; i < n; ++i) {
            const spd_work_item &w = items[(size_t)i];
            if (w.user < 0 || w.user >= n_users || w.kv_head < 0 || w.kv_head >= hkv || w.t_begin < 0 ||
                w.t_begin >= w.t_end || w.t_end > lens[(size_t)w.user] || w.t_begin % 32 != 0) {
                std::printf("bad item %lld\n", (long long)i);
                return 1;
            }
            covered[(size_t)w.user * hkv + w.kv_head] += w.t_end - w.t_begin;
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
        v.token_stride = 128 * hkv;
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
