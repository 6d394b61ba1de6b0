// Host-only checks of the key a schedule is remembered by, and of the rule by which a schedule serves a view whose
// lengths have all grown by the same few tokens.  Built by tests/test_host_sanitizers.py with AddressSanitizer and
// UBSan (plain C++: the header makes no HIP call).
#include <cstdint>
#include <cstdio>
#include <vector>

#include "../../paper_2409_19134_amd/csrc/schedule_key.hpp"

using namespace spd::host;

static uint64_t state = 0x13198a2e03707344ull;
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

struct View {
    std::vector<int32_t> lens;
    std::vector<const void *> kp, vp;
    std::vector<int64_t> hs;
    spd_kv_view v = {};
    void bind()
    {
        v.n_users = (int32_t)lens.size();
        v.lens = lens.data();
        v.k_ptrs = kp.data();
        v.v_ptrs = vp.data();
    }
};

static int32_t g_tuning[5] = {2, 768, 16384, 2, 12};  // the schedule-shaping options of a context

static std::vector<uint8_t> key_of(const spd_shape &s, View &w, int mapping)
{
    w.bind();
    std::vector<uint8_t> k;
    make_key(&s, &w.v, mapping != 0, g_tuning, 5, k);
    return k;
}

int main()
{
    int checked = 0;
    for (int iter = 0; iter < 2000; ++iter) {
        const int n = 1 + (int)(rnd() % 12);
        spd_shape s = {SPD_BF16, 32, 8, 128, 0.088f};
        View a;
        for (int u = 0; u < n; ++u) {
            a.lens.push_back(rnd() % 6 == 0 ? 0 : (int32_t)(1 + rnd() % 5000));
            a.kp.push_back(reinterpret_cast<const void *>((uintptr_t)0x100000 * (uintptr_t)(2 * u + 1)));
            a.vp.push_back(reinterpret_cast<const void *>((uintptr_t)0x100000 * (uintptr_t)(2 * u + 2)));
        }
        const bool paged = rnd() % 3 == 0;
        a.v.token_stride = 128;
        a.v.head_stride = 128 * 8192;
        if (paged) {
            a.v.block_size = 16;
            a.v.k_pool = reinterpret_cast<const void *>((uintptr_t)0x7000000);
            a.v.v_pool = reinterpret_cast<const void *>((uintptr_t)0x9000000);
        }
        const std::vector<uint8_t> ka = key_of(s, a, 0);

        // the same view gives the same key; the mapping, a stride or a length changes it
        View b = a;
        if (key_of(s, b, 0) != ka)
            FAIL("same view, different key");
        if (key_of(s, b, 1) == ka)
            FAIL("the mapping is not part of the key");
        b.v.head_stride += 16;
        if (key_of(s, b, 0) == ka)
            FAIL("the head stride is not part of the key");
        // every schedule-shaping option of the context is part of the key
        for (int opt = 0; opt < 5; ++opt) {
            b = a;
            g_tuning[opt] += 1;
            const bool same = key_of(s, b, 0) == ka;
            g_tuning[opt] -= 1;
            if (same)
                FAIL("option %d is not part of the key", opt);
        }
        b = a;
        const int pick = (int)(rnd() % n);
        b.lens[(size_t)pick] += 1;
        const std::vector<uint8_t> kb = key_of(s, b, 0);
        if (kb == ka)
            FAIL("a length is not part of the key");
        // (a user that held no token has its pointers left out of the key: its first token changes more than a length)
        if ((paged || a.lens[(size_t)pick] > 0) && hash_key_but_lens(kb, n) != hash_key_but_lens(ka, n))
            FAIL("the hash without lengths depends on a length");
        if (n > 1 && uniform_growth(ka, kb, n) != 0)
            FAIL("growth of one user out of %d taken for uniform growth", n);

        // buffers: part of the key in contiguous mode (the items hold addresses) unless the user holds no token;
        // pools are never part of it
        b = a;
        b.kp[(size_t)pick] = reinterpret_cast<const void *>((uintptr_t)0x5550000);
        const bool matters = !paged && a.lens[(size_t)pick] > 0;
        if ((key_of(s, b, 0) != ka) != matters)
            FAIL("buffer address: key %s although it %s", matters ? "unchanged" : "changed", matters ? "matters" : "does not matter");
        if (paged) {
            b = a;
            b.v.k_pool = reinterpret_cast<const void *>((uintptr_t)0xabc0000);
            if (key_of(s, b, 0) != ka)
                FAIL("the pool is part of the key");
        }

        // uniform growth by g: recognised for 1..kMaxGrow, and only then
        for (int g : {0, 1, 2, 63, 64, 65, 1000, -1}) {
            b = a;
            bool shrunk_below_zero = false;
            for (auto &l : b.lens) {
                l += g;
                shrunk_below_zero = shrunk_below_zero || l < 0;
            }
            if (shrunk_below_zero)
                continue;
            const int32_t got = uniform_growth(ka, key_of(s, b, 0), n);
            // (an empty user's pointers are left out of the key, so growth from zero changes more than the lengths: the
            // library never reuses such a schedule anyway - a row without tokens has no segment to extend)
            bool any_empty = false;
            for (int32_t l : a.lens)
                any_empty = any_empty || l == 0;
            const int32_t want = (g >= 1 && g <= kMaxGrow && (paged || !any_empty)) ? g : 0;
            if (got != want)
                FAIL("growth by %d: got %d, want %d (paged %d, empty user %d)", g, got, want, (int)paged, (int)any_empty);
        }
        // another number of users is never growth
        b = a;
        b.lens.push_back(5);
        b.kp.push_back(a.kp[0]);
        b.vp.push_back(a.vp[0]);
        if (uniform_growth(ka, key_of(s, b, 0), n) != 0 || uniform_growth(ka, key_of(s, b, 0), n + 1) != 0)
            FAIL("a view with one more user taken for growth");
        ++checked;
    }
    std::printf("ok %d\n", checked);
    return 0;
}
