// The key a schedule is remembered by: the bytes of a view that determine its split schedule (host only, no HIP calls).
#pragma once
#include <cstdint>
#include <cstring>
#include <vector>

#include "../../include/spd.h"

namespace spd::host {

// Hash of a schedule key, eight bytes at a time (keys grow with the number of users and are hashed on every call).
// Only a filter: a hit is confirmed by comparing the keys themselves.
inline uint64_t hash_key(const uint8_t *p, size_t n)
{
    uint64_t h = 1469598103934665603ull ^ n;
    size_t i = 0;
    for (; i + 8 <= n; i += 8) {
        uint64_t w;
        std::memcpy(&w, p + i, 8);
        h = (h ^ w) * 0x9E3779B97F4A7C15ull;
        h ^= h >> 29;
    }
    for (; i < n; ++i)
        h = (h ^ p[i]) * 1099511628211ull;
    return h;
}

// A decode loop appends one token per user and step: a schedule built for the lengths L serves L + g for
// 1 <= g <= kMaxGrow as well (the kernels add g to the end of every row's last segment), which spares the loop a
// rebuild and an upload per step.  Beyond that the pieces would drift out of balance and a new schedule is built.
constexpr int32_t kMaxGrow = 64;
constexpr size_t kKeyLensOffset = 6 * sizeof(int32_t);  // the lengths follow the key's six-integer head

inline uint64_t hash_key_but_lens(const std::vector<uint8_t> &key, int n_users)
{
    const size_t tail = kKeyLensOffset + sizeof(int32_t) * (size_t)n_users;
    return hash_key(key.data(), kKeyLensOffset) ^ (hash_key(key.data() + tail, key.size() - tail) * 0x9E3779B97F4A7C15ull);
}

// g if `key` is `old_key` with every length g larger (1 <= g <= kMaxGrow), else 0.
inline int32_t uniform_growth(const std::vector<uint8_t> &old_key, const std::vector<uint8_t> &key, int n_users)
{
    if (n_users == 0 || old_key.size() != key.size())
        return 0;
    const size_t tail = kKeyLensOffset + sizeof(int32_t) * (size_t)n_users;
    if (std::memcmp(old_key.data(), key.data(), kKeyLensOffset) != 0 ||
        std::memcmp(old_key.data() + tail, key.data() + tail, key.size() - tail) != 0)
        return 0;
    int32_t g = 0;
    for (int u = 0; u < n_users; ++u) {
        int32_t was, now;
        std::memcpy(&was, old_key.data() + kKeyLensOffset + sizeof(int32_t) * (size_t)u, sizeof was);
        std::memcpy(&now, key.data() + kKeyLensOffset + sizeof(int32_t) * (size_t)u, sizeof now);
        if (u == 0)
            g = now - was;
        if (now - was != g || g < 1 || g > kMaxGrow)
            return 0;
    }
    return g;
}

// tuning: the kTuningInts integers of the context's Tuning (they shape the schedule like the lengths do).
inline void make_key(const spd_shape *s, const spd_kv_view *v, int hpw, const int32_t *tuning, int n_tuning,
                     std::vector<uint8_t> &key)
{
    key.clear();
    auto put = [&key](const void *p, size_t n) {
        const uint8_t *b = static_cast<const uint8_t *>(p);
        key.insert(key.end(), b, b + n);
    };
    const int32_t head[6] = {s->dtype, s->n_q_heads, s->n_kv_heads, v->n_users, v->block_size,
                             hpw};
    static_assert(sizeof head == kKeyLensOffset, "the lengths follow the head");
    put(head, sizeof head);
    put(v->lens, sizeof(int32_t) * (size_t)v->n_users);
    // the items carry row base addresses (contiguous mode) or row offsets inside the pools (paged mode): the key holds
    // everything those depend on.  The pools themselves are not part of it, so the layers of a model, which share
    // lengths and block table but have a pool each, share one schedule.
    const int32_t tables = (v->block_size == 0 && v->k_ptrs_dev) ? 1 : 0;  // the items then hold offsets, not addresses
    put(&tables, sizeof tables);
    put(tuning, sizeof(int32_t) * (size_t)n_tuning);
    put(&v->head_stride, sizeof v->head_stride);
    if (v->head_strides && v->block_size == 0)
        put(v->head_strides, sizeof(int64_t) * (size_t)v->n_users);
    if (v->block_size == 0 && !tables) {
        for (int u = 0; u < v->n_users; ++u) {  // pointers of empty users are never read: normalise them
            const void *kp = v->lens[u] ? v->k_ptrs[u] : nullptr;
            const void *vp = v->lens[u] ? v->v_ptrs[u] : nullptr;
            put(&kp, sizeof kp);
            put(&vp, sizeof vp);
        }
    }
}

}  // namespace spd::host
