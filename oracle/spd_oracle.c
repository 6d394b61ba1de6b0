/*
 * CPU oracle for Secure Partitioned Decoding (SPD) decode-step attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of
 * what the GPU path must compute.  It shares no code, header, table or helper
 * with the HIP library and must never be called from the product path; only
 * the tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * What it states (paper section 4.2, Theorem 1 and its proof in Appendix A):
 *
 *   orc_attention   Y = softmax(Q K^T) V with K = concat(K_in, K_out),
 *                   V = concat(V_in, V_out): the plain definition over the
 *                   concatenated cache, two passes (max, then exp-sum).
 *   orc_partial     one owner's message: A_x = softmax(Q K_x^T) V_x together
 *                   with m_x = max(Q K_x^T) and gamma_x = sum exp(Q K_x^T - m_x)
 *                   (the stabilised denominators of section 4.2, last paragraph).
 *   orc_merge       Theorem 1 with the stabilised coefficients
 *                   gamma_in/(gamma_in + alpha gamma_out) and
 *                   gamma_out/(alpha^-1 gamma_in + gamma_out),
 *                   alpha = exp(m_out - m_in).
 *
 * Readings the paper leaves open (each also listed in the design notes):
 *   - scores are scale * <q, k>; the caller passes scale (1/sqrt(d) in every
 *     workload).  The theorem holds for any scores.
 *   - the theorem is applied independently per (user, query head); query head h
 *     reads KV head h / (Hq / Hkv) (consecutive grouping).
 *   - a decode query attends to every cached token of both parts; no mask.
 *   - an empty part has A = 0, m = -inf, gamma = 0 and weight 0; if both parts
 *     are empty Y = 0 and lse = -inf.
 *   - inputs are the already-rounded bf16 / fp16 / fp32 values, widened exactly to
 *     fp64; every sum, max and exponential is fp64.
 *
 * Parity pins live in tests/test_oracle_pins.py (brute force without the max
 * shift, library softmax, closed forms, Theorem 1 at every split point).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F16 = 2 };

/* One owner's cache for all users, in host memory. */
typedef struct {
    int32_t n_users;
    const int32_t *lens;          /* [n_users] tokens held for each user              */
    /* contiguous mode (block_size == 0): one base pointer per user                   */
    const void *const *k_ptrs;    /* [n_users]                                        */
    const void *const *v_ptrs;
    int64_t token_stride;         /* elements between consecutive tokens              */
    int64_t head_stride;          /* elements between consecutive KV heads            */
    const int64_t *head_strides;  /* [n_users] per-user head stride, or NULL (contiguous mode only) */
    /* paged mode (block_size > 0): one pool per tensor and a block table             */
    const void *k_pool;
    const void *v_pool;
    int32_t block_size;           /* tokens per page                                   */
    const int32_t *block_table;   /* [n_users][max_blocks] page ids                    */
    int32_t max_blocks;
    int64_t block_stride;         /* elements between consecutive pages                */
} orc_view;

/* IEEE binary16 (1 sign, 5 exponent, 10 fraction bits) to fp64, exactly. */
double orc_half_to_double(uint16_t h)
{
    const int sign = h >> 15, e = (h >> 10) & 31, f = h & 1023;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);                 /* zero and subnormals: f * 2^-10 * 2^-14 */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return sign ? -v : v;
}

static double widen(const void *base, int dtype, int64_t idx)
{
    if (dtype == ORC_F32)
        return (double)((const float *)base)[idx];
    if (dtype == ORC_F16)
        return orc_half_to_double(((const uint16_t *)base)[idx]);
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;  /* bf16 = top half of fp32 */
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* Element offset of channel 0 of token i, KV head kv, user u; *base gets the tensor. */
static int64_t row_offset(const orc_view *w, int is_v, int u, int64_t i, int kv, const void **base)
{
    if (w->block_size == 0) {
        *base = is_v ? w->v_ptrs[u] : w->k_ptrs[u];
        return i * w->token_stride + (int64_t)kv * (w->head_strides ? w->head_strides[u] : w->head_stride);
    }
    int64_t page = w->block_table[(int64_t)u * w->max_blocks + i / w->block_size];
    *base = is_v ? w->v_pool : w->k_pool;
    return page * w->block_stride + (int64_t)kv * w->head_stride + (i % w->block_size) * w->token_stride;
}

/* s = scale * <q, k_i> in fp64 */
static double score(const void *q, int dtype, int64_t q_off, const orc_view *w, int u, int64_t i, int kv,
                    int d, double scale)
{
    const void *kb;
    int64_t off = row_offset(w, 0, u, i, kv, &kb);
    double acc = 0.0;
    for (int c = 0; c < d; ++c)
        acc += widen(q, dtype, q_off + c) * widen(kb, dtype, off + c);
    return scale * acc;
}

/*
 * Unsplit attention over the concatenation of n_views caches (Theorem 1's left-hand side).
 * rows: n_rows pairs (user, query head), or NULL for all U*Hq rows in (u, h) order.
 * Y: [n_rows][d], lse: [n_rows] (natural log of the softmax denominator; -inf if no token).
 * Returns 0, or -1 on allocation failure.
 */
int orc_attention(int U, int Hq, int Hkv, int d, double scale, int dtype, const void *q,
                  int n_views, const orc_view *const *views,
                  int n_rows, const int32_t *rows, double *Y, double *lse)
{
    const int G = Hq / Hkv;
    if (rows == NULL)
        n_rows = U * Hq;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        const int u = rows ? rows[2 * r] : r / Hq;
        const int h = rows ? rows[2 * r + 1] : r % Hq;
        const int kv = h / G;
        const int64_t q_off = ((int64_t)u * Hq + h) * d;
        int64_t len = 0;
        for (int p = 0; p < n_views; ++p)
            len += views[p]->lens[u];
        double *y = Y + (int64_t)r * d;
        for (int c = 0; c < d; ++c)
            y[c] = 0.0;
        if (len == 0) {
            lse[r] = -INFINITY;
            continue;
        }
        double *s = (double *)malloc((size_t)len * sizeof(double));
        if (!s) {
            failed = 1;
            continue;
        }
        /* scores of the concatenated cache, in cache order */
        int64_t at = 0;
        double m = -INFINITY;
        for (int p = 0; p < n_views; ++p)
            for (int64_t i = 0; i < views[p]->lens[u]; ++i, ++at) {
                s[at] = score(q, dtype, q_off, views[p], u, i, kv, d, scale);
                if (s[at] > m)
                    m = s[at];
            }
        /* softmax denominator and the weighted sum of value rows */
        double gamma = 0.0;
        at = 0;
        for (int p = 0; p < n_views; ++p)
            for (int64_t i = 0; i < views[p]->lens[u]; ++i, ++at) {
                const double e = exp(s[at] - m);
                gamma += e;
                const void *vb;
                int64_t off = row_offset(views[p], 1, u, i, kv, &vb);
                for (int c = 0; c < d; ++c)
                    y[c] += e * widen(vb, dtype, off + c);
            }
        for (int c = 0; c < d; ++c)
            y[c] /= gamma;
        lse[r] = m + log(gamma);
        free(s);
    }
    return failed ? -1 : 0;
}

/*
 * One owner's partial over tokens [t0[u], t1[u]) of its cache (t0/t1 NULL: the whole cache):
 * A = softmax(s) V, m = max s, gamma = sum exp(s - m).  Empty range: A = 0, m = -inf, gamma = 0.
 */
int orc_partial(int U, int Hq, int Hkv, int d, double scale, int dtype, const void *q,
                const orc_view *view, const int32_t *t0, const int32_t *t1,
                int n_rows, const int32_t *rows, double *A, double *m_out, double *gamma_out)
{
    const int G = Hq / Hkv;
    if (rows == NULL)
        n_rows = U * Hq;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        const int u = rows ? rows[2 * r] : r / Hq;
        const int h = rows ? rows[2 * r + 1] : r % Hq;
        const int kv = h / G;
        const int64_t q_off = ((int64_t)u * Hq + h) * d;
        const int64_t lo = t0 ? t0[u] : 0;
        const int64_t hi = t1 ? t1[u] : view->lens[u];
        const int64_t len = hi > lo ? hi - lo : 0;
        double *a = A + (int64_t)r * d;
        for (int c = 0; c < d; ++c)
            a[c] = 0.0;
        if (len == 0) {
            m_out[r] = -INFINITY;
            gamma_out[r] = 0.0;
            continue;
        }
        double *s = (double *)malloc((size_t)len * sizeof(double));
        if (!s) {
            failed = 1;
            continue;
        }
        double m = -INFINITY;
        for (int64_t i = 0; i < len; ++i) {
            s[i] = score(q, dtype, q_off, view, u, lo + i, kv, d, scale);
            if (s[i] > m)
                m = s[i];
        }
        double gamma = 0.0;
        for (int64_t i = 0; i < len; ++i) {
            const double e = exp(s[i] - m);
            gamma += e;
            const void *vb;
            int64_t off = row_offset(view, 1, u, lo + i, kv, &vb);
            for (int c = 0; c < d; ++c)
                a[c] += e * widen(vb, dtype, off + c);
        }
        for (int c = 0; c < d; ++c)
            a[c] /= gamma;
        m_out[r] = m;
        gamma_out[r] = gamma;
        free(s);
    }
    return failed ? -1 : 0;
}

/*
 * Theorem 1 with the stabilised coefficients.  Per row:
 *   alpha = exp(m_out - m_in)
 *   Y = gamma_in / (gamma_in + alpha gamma_out) * A_in + gamma_out / (alpha^-1 gamma_in + gamma_out) * A_out
 * and the merged statistics m = max(m_in, m_out), gamma = gamma_in e^{m_in - m} + gamma_out e^{m_out - m},
 * which make the rule usable again on the result (n-way splits).  w_in (may be NULL) receives the first
 * coefficient.  A part with gamma = 0 is empty and gets weight 0; both empty gives Y = 0.
 */
void orc_merge(int n_rows, int d,
               const double *A_in, const double *m_in, const double *g_in,
               const double *A_out, const double *m_out, const double *g_out,
               double *Y, double *m, double *gamma, double *w_in)
{
    for (int r = 0; r < n_rows; ++r) {
        double c_in, c_out;
        if (g_in[r] == 0.0 && g_out[r] == 0.0) {
            c_in = c_out = 0.0;
        } else if (g_out[r] == 0.0) {
            c_in = 1.0, c_out = 0.0;
        } else if (g_in[r] == 0.0) {
            c_in = 0.0, c_out = 1.0;
        } else {
            const double alpha = exp(m_out[r] - m_in[r]);
            const double alpha_inv = exp(m_in[r] - m_out[r]);
            c_in = g_in[r] / (g_in[r] + alpha * g_out[r]);
            c_out = g_out[r] / (alpha_inv * g_in[r] + g_out[r]);
        }
        for (int c = 0; c < d; ++c)
            Y[(int64_t)r * d + c] = c_in * A_in[(int64_t)r * d + c] + c_out * A_out[(int64_t)r * d + c];
        const double mm = m_in[r] > m_out[r] ? m_in[r] : m_out[r];
        m[r] = mm;
        double g = 0.0;
        if (g_in[r] != 0.0)
            g += g_in[r] * exp(m_in[r] - mm);
        if (g_out[r] != 0.0)
            g += g_out[r] * exp(m_out[r] - mm);
        gamma[r] = g;
        if (w_in)
            w_in[r] = c_in;
    }
}

/* Number of threads an "omp parallel for" here uses (reported beside timings). */
int orc_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
