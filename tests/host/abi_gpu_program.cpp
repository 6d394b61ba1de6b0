// The whole path from a program that knows only include/spd.h and the HIP runtime (no Python, no PyTorch): the three
// calls of the protocol (paper section 4, step 3), the fused step and the two-party form, checked against a closed form.
// All keys are zero, so every score is 0, the softmax is uniform and the result is the mean of the user's V rows
// over both caches, with lse = ln(number of tokens).  Built by paper_2409_19134_amd/build.py, run by a GPU test.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "spd.h"

#define HIP_OK(x)                                                                   \
    do {                                                                            \
        hipError_t e_ = (x);                                                        \
        if (e_ != hipSuccess) {                                                     \
            std::printf("HIP error %d at line %d\n", (int)e_, __LINE__);            \
            return 2;                                                               \
        }                                                                           \
    } while (0)
#define SPD_CALL(x)                                                                 \
    do {                                                                            \
        int rc_ = (x);                                                              \
        if (rc_ != SPD_OK) {                                                        \
            std::printf("%s at line %d\n", spd_strerror(rc_), __LINE__);            \
            return 3;                                                               \
        }                                                                           \
    } while (0)

static uint16_t bf16_of(float f)  // exact for the small integers used here
{
    uint32_t b;
    std::memcpy(&b, &f, sizeof b);
    return (uint16_t)(b >> 16);
}

int main()
{
    const int U = 2, Hq = 8, Hkv = 2, d = 128, G = Hq / Hkv;
    const int32_t lp[U] = {300, 40}, lo[U] = {5, 0};
    const int cap_p = 320, cap_o = 64;  // tokens each per-user buffer has room for; layout [Hkv][cap][d]
    auto value = [](int u, int owner, int h, int t, int c) { return (float)((t + 3 * h + u + 5 * owner) % 7 - 3 + c % 3); };

    std::vector<uint16_t> hq((size_t)U * Hq * d);
    for (size_t i = 0; i < hq.size(); ++i)
        hq[i] = bf16_of((float)((int)(i % 5) - 2));
    void *q = nullptr;
    HIP_OK(hipMalloc(&q, hq.size() * 2));
    HIP_OK(hipMemcpy(q, hq.data(), hq.size() * 2, hipMemcpyHostToDevice));

    const void *kp[2][U], *vp[2][U];  // [owner][user]
    std::vector<double> want((size_t)U * Hq * d, 0.0);
    for (int owner = 0; owner < 2; ++owner) {
        const int cap = owner ? cap_o : cap_p;
        for (int u = 0; u < U; ++u) {
            const int L = owner ? lo[u] : lp[u];
            std::vector<uint16_t> hv((size_t)Hkv * cap * d, bf16_of(77.f));  // beyond L: never read
            for (int h = 0; h < Hkv; ++h)
                for (int t = 0; t < L; ++t)
                    for (int c = 0; c < d; ++c) {
                        const float x = value(u, owner, h, t, c);
                        hv[((size_t)h * cap + t) * d + c] = bf16_of(x);
                        for (int g = 0; g < G; ++g)
                            want[((size_t)u * Hq + h * G + g) * d + c] += x;
                    }
            void *k = nullptr, *v = nullptr;
            HIP_OK(hipMalloc(&k, hv.size() * 2));
            HIP_OK(hipMalloc(&v, hv.size() * 2));
            HIP_OK(hipMemset(k, 0, hv.size() * 2));  // all keys zero
            HIP_OK(hipMemcpy(v, hv.data(), hv.size() * 2, hipMemcpyHostToDevice));
            kp[owner][u] = k;
            vp[owner][u] = v;
        }
    }
    for (int u = 0; u < U; ++u)
        for (int i = 0; i < Hq * d; ++i)
            want[(size_t)u * Hq * d + i] /= (double)(lp[u] + lo[u]);

    spd_shape shape = {SPD_BF16, Hq, Hkv, d, 0.0883883f};
    spd_kv_view priv, pub;
    std::memset(&priv, 0, sizeof priv);
    std::memset(&pub, 0, sizeof pub);
    priv.n_users = pub.n_users = U;
    priv.lens = lp;
    pub.lens = lo;
    priv.k_ptrs = kp[0];
    priv.v_ptrs = vp[0];
    pub.k_ptrs = kp[1];
    pub.v_ptrs = vp[1];
    priv.token_stride = pub.token_stride = d;
    priv.head_stride = (int64_t)cap_p * d;
    pub.head_stride = (int64_t)cap_o * d;

    const size_t n_rows = (size_t)U * Hq;
    float *a_in, *a_out, *y, *lse_in, *lse_out, *lse, *w_in;
    HIP_OK(hipMalloc((void **)&a_in, n_rows * d * 4));
    HIP_OK(hipMalloc((void **)&a_out, n_rows * d * 4));
    HIP_OK(hipMalloc((void **)&y, n_rows * d * 4));
    HIP_OK(hipMalloc((void **)&lse_in, n_rows * 4));
    HIP_OK(hipMalloc((void **)&lse_out, n_rows * 4));
    HIP_OK(hipMalloc((void **)&lse, n_rows * 4));
    HIP_OK(hipMalloc((void **)&w_in, n_rows * 4));
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));

    if (spd_abi_version() != SPD_ABI_VERSION) {
        std::printf("library built from another version of spd.h\n");
        return 4;
    }
    spd_ctx *ctx = nullptr;
    SPD_CALL(spd_create(&ctx, 0));
    std::vector<float> hy(n_rows * d), hl(n_rows), hw(n_rows);
    for (int variant = 0; variant < 3; ++variant) {
        HIP_OK(hipMemsetAsync(y, 0xff, n_rows * d * 4, stream));  // NaN bits: every output must be overwritten
        HIP_OK(hipMemsetAsync(lse, 0xff, n_rows * 4, stream));
        if (variant == 0) {  // the three calls of the protocol
            SPD_CALL(spd_partial_attn_private(ctx, &shape, q, &priv, a_in, lse_in, stream));
            SPD_CALL(spd_partial_attn_public_batched(ctx, &shape, q, &pub, a_out, lse_out, stream));
            SPD_CALL(spd_lse_merge(ctx, (int32_t)n_rows, d, a_in, lse_in, a_out, lse_out, y, lse, w_in, stream));
        } else if (variant == 1) {  // one call
            SPD_CALL(spd_decode_step(ctx, &shape, q, &priv, &pub, nullptr, nullptr, a_in, lse_in, a_out, lse_out, y, lse,
                                     w_in, stream));
        } else {  // the users' call, then the service's call
            SPD_CALL(spd_partial_attn_private(ctx, &shape, q, &priv, a_in, lse_in, stream));
            SPD_CALL(spd_public_attn_merge(ctx, &shape, q, &pub, nullptr, nullptr, a_in, lse_in, a_out, lse_out, y, lse,
                                           w_in, stream));
        }
        HIP_OK(hipStreamSynchronize(stream));
        HIP_OK(hipMemcpy(hy.data(), y, hy.size() * 4, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(hl.data(), lse, hl.size() * 4, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(hw.data(), w_in, hw.size() * 4, hipMemcpyDeviceToHost));
        double worst = 0.0;
        for (size_t i = 0; i < hy.size(); ++i)
            worst = std::fmax(worst, std::fabs((double)hy[i] - want[i]));
        for (int u = 0; u < U; ++u)
            for (int h = 0; h < Hq; ++h) {
                worst = std::fmax(worst, std::fabs((double)hl[(size_t)u * Hq + h] - std::log((double)(lp[u] + lo[u]))));
                worst = std::fmax(worst, std::fabs((double)hw[(size_t)u * Hq + h] - (double)lp[u] / (lp[u] + lo[u])));
            }
        std::printf("variant %d: max abs error against the closed form %.3g\n", variant, worst);
        if (!(worst <= 1e-5))
            return 1;
    }
    SPD_CALL(spd_destroy(ctx));
    std::printf("c abi gpu ok\n");
    return 0;
}
