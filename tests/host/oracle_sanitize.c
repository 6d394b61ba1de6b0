/* Runs the CPU oracle on small random inputs (contiguous and paged, both dtypes) under ASan/UBSan and checks the
 * Theorem 1 identity merge(partial(private), partial(public)) == attention(concat) on the way.
 * Built and run by tests/test_host_sanitizers.py; includes the oracle's source directly. */
#include <stdio.h>
#include "../../oracle/spd_oracle.c"

static unsigned long long st = 88172645463325252ull;
static double rnd(void)
{
    st ^= st << 13; st ^= st >> 7; st ^= st << 17;
    return (double)(st % 2000001ull) / 1000000.0 - 1.0;
}
static uint16_t to_bf16(float f)
{
    uint32_t b; memcpy(&b, &f, 4);
    return (uint16_t)((b + 0x7fffu + ((b >> 16) & 1u)) >> 16);
}

int main(void)
{
    int checked = 0;
    for (int iter = 0; iter < 60; ++iter) {
        const int dtype = iter & 1, paged = (iter >> 1) & 1;
        const int U = 1 + iter % 3, Hkv = 1 + iter % 2, G = 1 + iter % 4, Hq = Hkv * G, d = 8 * (1 + iter % 3);
        const int es = dtype == ORC_F32 ? 4 : 2;
        int32_t lens[2][3];
        orc_view views[2];
        void *bufs[2][2][3] = {{{0}}};
        void *pools[2][2] = {{0}};
        int32_t *tables[2] = {0, 0};
        for (int p = 0; p < 2; ++p) {
            memset(&views[p], 0, sizeof views[p]);
            views[p].n_users = U;
            views[p].lens = lens[p];
            int total_pages = 0, max_blocks = 1;
            for (int u = 0; u < U; ++u) {
                lens[p][u] = (int32_t)((iter * 7 + u * 5 + p * 3) % 37);
                if ((iter + u + p) % 9 == 0) lens[p][u] = 0;
                const int pages = (lens[p][u] + 15) / 16;
                total_pages += pages;
                if (pages > max_blocks) max_blocks = pages;
            }
            if (!paged) {
                views[p].token_stride = (int64_t)Hkv * d;
                views[p].head_stride = d;
                static const void *kp[2][3], *vp[2][3];
                for (int u = 0; u < U; ++u)
                    for (int t = 0; t < 2; ++t) {
                        const size_t n = (size_t)lens[p][u] * Hkv * d;
                        char *b = (char *)malloc(n * es + 1);
                        for (size_t i = 0; i < n; ++i) {
                            float f = (float)rnd();
                            if (dtype == ORC_F32) ((float *)b)[i] = f; else ((uint16_t *)b)[i] = to_bf16(f);
                        }
                        bufs[p][t][u] = b;
                        if (t == 0) kp[p][u] = b; else vp[p][u] = b;
                    }
                views[p].k_ptrs = kp[p];
                views[p].v_ptrs = vp[p];
            } else {
                views[p].block_size = 16;
                views[p].token_stride = d;
                views[p].head_stride = 16 * d;
                views[p].block_stride = (int64_t)Hkv * 16 * d;
                views[p].max_blocks = max_blocks;
                tables[p] = (int32_t *)calloc((size_t)U * max_blocks, sizeof(int32_t));
                int next = total_pages - 1;      /* pages handed out in reverse order */
                for (int u = 0; u < U; ++u)
                    for (int b = 0; b < (lens[p][u] + 15) / 16; ++b)
                        tables[p][u * max_blocks + b] = next--;
                views[p].block_table = tables[p];
                for (int t = 0; t < 2; ++t) {
                    const size_t n = (size_t)(total_pages > 0 ? total_pages : 1) * Hkv * 16 * d;
                    char *b = (char *)malloc(n * es);
                    for (size_t i = 0; i < n; ++i) {
                        float f = (float)rnd();
                        if (dtype == ORC_F32) ((float *)b)[i] = f; else ((uint16_t *)b)[i] = to_bf16(f);
                    }
                    pools[p][t] = b;
                }
                views[p].k_pool = pools[p][0];
                views[p].v_pool = pools[p][1];
            }
        }
        const size_t nq = (size_t)U * Hq * d;
        char *q = (char *)malloc(nq * es);
        for (size_t i = 0; i < nq; ++i) {
            float f = (float)rnd();
            if (dtype == ORC_F32) ((float *)q)[i] = f; else ((uint16_t *)q)[i] = to_bf16(f);
        }
        const int R = U * Hq;
        double *Y = malloc(sizeof(double) * R * d), *lse = malloc(sizeof(double) * R);
        double *A0 = malloc(sizeof(double) * R * d), *A1 = malloc(sizeof(double) * R * d), *Ym = malloc(sizeof(double) * R * d);
        double *m0 = malloc(sizeof(double) * R), *g0 = malloc(sizeof(double) * R), *m1 = malloc(sizeof(double) * R);
        double *g1 = malloc(sizeof(double) * R), *mm = malloc(sizeof(double) * R), *gm = malloc(sizeof(double) * R);
        const orc_view *vv[2] = {&views[0], &views[1]};
        if (orc_attention(U, Hq, Hkv, d, 0.3, dtype, q, 2, vv, 0, NULL, Y, lse)) return 2;
        if (orc_partial(U, Hq, Hkv, d, 0.3, dtype, q, &views[0], NULL, NULL, 0, NULL, A0, m0, g0)) return 2;
        if (orc_partial(U, Hq, Hkv, d, 0.3, dtype, q, &views[1], NULL, NULL, 0, NULL, A1, m1, g1)) return 2;
        orc_merge(R, d, A0, m0, g0, A1, m1, g1, Ym, mm, gm, NULL);
        for (int i = 0; i < R * d; ++i)
            if (fabs(Ym[i] - Y[i]) > 1e-12 * (1.0 + fabs(Y[i]))) {
                printf("identity violated iter %d idx %d: %g vs %g\n", iter, i, Ym[i], Y[i]);
                return 1;
            }
        free(Y); free(lse); free(A0); free(A1); free(Ym); free(m0); free(g0); free(m1); free(g1); free(mm); free(gm); free(q);
        for (int p = 0; p < 2; ++p) {
            for (int t = 0; t < 2; ++t) {
                for (int u = 0; u < 3; ++u) free(bufs[p][t][u]);
                free(pools[p][t]);
            }
            free(tables[p]);
        }
        ++checked;
    }
    printf("ok %d\n", checked);
    return 0;
}
