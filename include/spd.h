/*
 * spd.h - C ABI of the Secure Partitioned Decoding (SPD) decode-attention library for AMD MI355X (gfx950).
 *
 * SPD splits the attention of one decode step between two owners of the KV cache
 * (paper section 4, protocol step 3; section 4.2, Theorem 1):
 *
 *   - each user's process holds that user's *private* KV cache (the prompt) and answers a query with a
 *     partial attention over it                                   -> spd_partial_attn_private
 *   - the service process holds the *public* KV cache (generated tokens) of all users and computes the
 *     same kind of partial for every user in one batch            -> spd_partial_attn_public_batched
 *   - the service merges the two partials so that the result equals softmax attention over the
 *     concatenated cache (Theorem 1, stabilised as in the last paragraph of section 4.2)
 *                                                                  -> spd_lse_merge
 *
 * A partial is the pair (A, lse): A = softmax(s) V over the owner's tokens and lse = ln sum_i exp(s_i),
 * with scores s_i = scale * <q, k_i>.  In the paper's notation lse = m + ln(gamma); carrying lse instead of
 * (m, gamma) keeps the merge free of the overflow that alpha = exp(m_out - m_in) has in fp32.
 *
 * Conventions common to all calls
 *   - Every pointer marked DEVICE is memory of the HIP device the context was created on; HOST pointers are
 *     ordinary host memory read during the call only.  The library keeps no caller pointer after a call returns
 *     (it may keep *copies* of the small host arrays to recognise a repeated view, see below).
 *   - The caller owns all tensors and the stream.  Calls validate on the host, enqueue work on `hip_stream`
 *     (a hipStream_t passed as void*; NULL is the default stream) and return without synchronising.
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads).  The head_dim axis is unit stride everywhere.
 *   - Outputs are fp32 and fully overwritten.  An owner that holds no token for a user returns A = 0 and
 *     lse = -inf for that user's rows; this is legal, not an error.
 *   - Return value: SPD_OK or a negative error code; on any validation error nothing is launched.
 *   - Calls on one context that use the same entry point must not overlap in time (they share scratch memory);
 *     the private and the public call may run concurrently on two streams.  A context is not thread-safe: its
 *     calls must come from one host thread at a time (use a context per thread).
 *   - A call whose view the context has seen before (same lengths, strides and - without device pointer arrays -
 *     buffers) and whose scratch memory is large enough only launches kernels: it allocates nothing, copies nothing
 *     and may be recorded into a HIP graph (stream capture).  A call that has to build a schedule or grow scratch
 *     memory under capture fails with SPD_ERR_HIP and invalidates the capture, so run the step once eagerly first.
 *     The context remembers 128 views per entry point (SPD_SCHEDULE_CACHE_ENTRIES in the environment, read by
 *     spd_create, changes that), least recently used first out.
 */
#ifndef SPD_H
#define SPD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPD_OK 0
#define SPD_ERR_NULL (-1)      /* a required pointer is NULL                                         */
#define SPD_ERR_SHAPE (-2)     /* unsupported dtype / head counts / head_dim / block size            */
#define SPD_ERR_LEN (-3)       /* negative count or length, a length above 2^30, or a paged length
                                  beyond max_blocks                                                   */
#define SPD_ERR_ALIGN (-4)     /* a base pointer or stride breaks the 16-byte row alignment          */
#define SPD_ERR_WORKSPACE (-5) /* scratch memory could not be (re)allocated, or the step exceeds the
                                  fixed scratch array of spd_decode_step_static                       */
#define SPD_ERR_HIP (-6)       /* a HIP runtime call failed; see spd_last_hip_error                  */
#define SPD_ERR_NOMEM (-7)     /* host allocation failed                                             */

enum { SPD_F32 = 0, SPD_BF16 = 1, SPD_F16 = 2 };

/* Opaque library context: device id, scratch memory for split partials, cached schedules. */
typedef struct spd_ctx spd_ctx;

/* Attention shape shared by q, K and V of one call. */
typedef struct spd_shape {
    int32_t dtype;      /* SPD_F32, SPD_BF16 or SPD_F16: element type of q, K and V                   */
    int32_t n_q_heads;  /* Hq                                                                         */
    int32_t n_kv_heads; /* Hkv, must divide Hq; Hq / Hkv in 1..16                                      */
    int32_t head_dim;   /* d: 64 or 128                                                               */
    float scale;        /* multiplies <q,k> before the softmax; 1/sqrt(d) in the usual case           */
} spd_shape;

/*
 * One owner's KV cache for n_users users.
 *
 * Contiguous mode (block_size == 0): user u's K and V start at k_ptrs[u] / v_ptrs[u]; element (token i, KV head j,
 * channel c) is at offset i*token_stride + j*head_stride + c (in elements; head_strides[u] instead of head_stride if
 * that array is given).  Buffers of different users may be separate allocations.  A user with lens[u] == 0 may
 * have NULL pointers.
 *
 * Paged mode (block_size B = 16, 32, 64, 128 or 256 tokens per page): element (token i, head j, channel c) of user u is
 * at pool + block_table[u*max_blocks + i/B]*block_stride + j*head_stride + (i%B)*token_stride + c.
 * The table lives on the device and only entries [0, ceil(lens[u]/B)) of each row are read; they must name
 * pages inside the pool (the library cannot check device-resident entries).
 */
typedef struct spd_kv_view {
    int32_t n_users;
    const int32_t *lens;        /* HOST [n_users] tokens held per user, 0 .. 2^30                         */
    const void *const *k_ptrs;  /* HOST array [n_users] of DEVICE pointers (contiguous mode)              */
    const void *const *v_ptrs;  /* HOST array [n_users] of DEVICE pointers (contiguous mode)              */
    int64_t token_stride;       /* elements, multiple of 16 bytes                                         */
    int64_t head_stride;        /* elements, multiple of 16 bytes                                         */
    const int64_t *head_strides; /* HOST [n_users] or NULL: per-user head stride (contiguous mode), replacing
                                    head_stride; lets exactly sized head-major buffers [Hkv][len][d] of different
                                    lengths share one view                                                   */
    const void *k_pool;         /* DEVICE (paged mode)                                                    */
    const void *v_pool;         /* DEVICE (paged mode)                                                    */
    int32_t block_size;         /* 0 = contiguous; paged: tokens per page, 16 / 32 / 64 / 128 / 256       */
    const int32_t *block_table; /* DEVICE [n_users][max_blocks] (paged mode)                              */
    int32_t max_blocks;
    int64_t block_stride;       /* elements between pages, multiple of 16 bytes                           */
    const void *const *k_ptrs_dev; /* optional, DEVICE copies [n_users] of k_ptrs / v_ptrs (contiguous mode; both */
    const void *const *v_ptrs_dev; /* or neither): with them the split schedule does not depend on the buffers'
                                      addresses - views that differ only in their buffers, such as the layers of
                                      a model, share one cached schedule - and the kernels read each user's base
                                      pointer from these arrays.  k_ptrs / v_ptrs are still required (validation) */
} spd_kv_view;

/* Bumped whenever a struct layout or a signature of this header changes; spd_abi_version() returns the value the
 * library was built with, so a program can check that header and library belong together. */
#define SPD_ABI_VERSION 4
int spd_abi_version(void);

/* Create a context on HIP device `hip_device` (host call; allocates a small amount of device memory). */
int spd_create(spd_ctx **out, int hip_device);

/* Synchronise the device and free everything the context owns. */
int spd_destroy(spd_ctx *ctx);

/* Static description of an error code. */
const char *spd_strerror(int code);

/* hipError_t of the last failed HIP call made through this context (0 if none). */
int spd_last_hip_error(const spd_ctx *ctx);

/*
 * Options of a context: what shapes its split schedules, and the choice of kernel mapping.  spd_create takes each
 * option's default or, if set, the value of the environment variable of the same name with the prefix SPD_ (e.g.
 * SPD_CHUNK_MAX=4096), read once at that moment; spd_set_option changes it for later calls of this context.  The
 * schedule-shaping options are part of the key a cached schedule is found by, so a change never reuses a schedule
 * built under other options.  Out-of-range values are refused with SPD_ERR_LEN, unknown options with SPD_ERR_SHAPE.
 */
enum {
    SPD_OPT_HEAD_PER_WAVE = 0,    /* -1 (default): head-per-wave mapping for large token-major views; 0 never; 1 whenever
                                     the layout allows it; 2..8 the same, with at most that many KV heads per workgroup */
    SPD_OPT_TARGET_WG_PER_CU = 1, /* pieces per compute unit that count as one resident round for an owner of a fused
                                     step (default 2); a call for one owner alone takes half as many again, unless
                                     its round would then be made of pieces of 64 steps (2048 tokens) or less       */
    SPD_OPT_NO_SPLIT_MAX = 2,     /* rows up to this many tokens are cut into one-step-per-wave chunks if all of them
                                     fit the device at once (default 768)                                          */
    SPD_OPT_CHUNK_MAX = 3,        /* tokens per piece when the work exceeds one resident round (default 16384)       */
    SPD_OPT_SEG_COST = 4,         /* 32-token steps a piece gives up for every further row it reaches into (default 2) */
    SPD_OPT_HALF_SKEW = 5,        /* one resident round of pieces: per cent by which the half dispatched first is made
                                     longer and the other half shorter (default 12, 0..90)                          */
    SPD_OPT_RESULT_ROWS = 6,      /* result rows a workgroup (head-per-wave mapping: each of its waves) may hold back
                                     in on-chip memory and store together at the end of its piece (default 32, 0..32;
                                     fewer if they do not fit); not part of the schedule: changing it rebuilds nothing */
    SPD_OPT_STEPS_IN_FLIGHT = 7   /* 32-token steps a wave of the streaming kernel has in flight: -1 (default) by the
                                     size of the launch (two where the pieces outnumber the workgroup slots), 1 or 2
                                     always - where the kernel has both forms: fp32 always takes one, 128-byte rows
                                     and the head-per-wave mapping always two; not part of the schedule either       */
};
int spd_set_option(spd_ctx *ctx, int32_t option, int32_t value);
int spd_get_option(spd_ctx *ctx, int32_t option, int32_t *value);

/*
 * How often a call had to build and upload a split schedule (`builds`) and how often it found the one it needed among
 * those it remembers (`hits`).  A schedule is determined by the lengths, the storage mode and strides and, in
 * contiguous mode without device pointer arrays, the per-user base pointers - not by q, the outputs, the block table
 * or the pools; so the layers of a model that share lengths (and a block table, or pass k_ptrs_dev / v_ptrs_dev) share
 * one schedule.  A view whose lengths have all grown by the same 1..64 tokens since its schedule was built (a decode
 * loop that appends a token per user and step) is served by that schedule too and counts as a hit.
 */
int spd_get_schedule_stats(const spd_ctx *ctx, int64_t *builds, int64_t *hits);

/*
 * Private partial attention (protocol step 3b; A_in of Theorem 1): for every user u of `priv` and query head h,
 *   out[u][h][:] = softmax(scale * q[u][h] . K_in[u]^T) V_in[u],   lse[u][h] = ln sum_i exp(scale * <q[u][h], k_i>).
 * A user's rows depend only on that user's q row and buffers, so n_users == 1 is the paper's per-process call and
 * n_users > 1 computes many users' private partials in one launch.
 *   q    DEVICE [n_users][Hq][d], shape->dtype, 16-byte aligned
 *   out  DEVICE [n_users][Hq][d] fp32        lse  DEVICE [n_users][Hq] fp32
 * Long caches are split into chunks internally; chunk partials are combined with the n-way form of Theorem 1.
 */
int spd_partial_attn_private(spd_ctx *ctx, const spd_shape *shape, const void *q, const spd_kv_view *priv,
                             float *out, float *lse, void *hip_stream);

/*
 * Public batched partial attention (protocol step 3c; A_out of Theorem 1): the same quantity over the service's
 * output-token cache, for all users in one batch.  Arguments as for spd_partial_attn_private.
 */
int spd_partial_attn_public_batched(spd_ctx *ctx, const spd_shape *shape, const void *q, const spd_kv_view *pub,
                                    float *out, float *lse, void *hip_stream);

/*
 * KV append fused into the public partial (protocol step 3a followed by 3c; Figure 3 steps 2 and 3): the new token's
 * K and V rows, k_new / v_new DEVICE [n_users][Hkv][d] in shape->dtype, become token lens[u] - 1 of every user's
 * public cache - `pub->lens` already counts the new token, so every length must be >= 1 - and the partial is
 * computed over the cache including it.  The same launch writes the rows into the cache (contiguous: the buffer must
 * have room for lens[u] tokens; paged: the block table must already name the page of position lens[u] - 1) and reads
 * them from k_new / v_new, so no separate copy kernel and no ordering between the two is needed.  The cache memory
 * behind `pub` is written by this call although the view type is const.  Other arguments as for
 * spd_partial_attn_public_batched.
 */
int spd_partial_attn_public_batched_append(spd_ctx *ctx, const spd_shape *shape, const void *q, const void *k_new,
                                           const void *v_new, const spd_kv_view *pub, float *out, float *lse,
                                           void *hip_stream);

/*
 * Merge two partials row by row (Theorem 1 with the coefficients of section 4.2 rewritten on log-sum-exps):
 *   lse = logaddexp(lse0, lse1); w0 = exp(lse0 - lse); w1 = exp(lse1 - lse); y = w0*a0 + w1*a1.
 * A row whose lse is -inf on one side takes the other side unchanged; -inf on both sides gives y = 0, lse = -inf,
 * w0 = 0.  n_rows = n_users * Hq.  All arrays DEVICE fp32: a0, a1, y [n_rows][head_dim]; lse0, lse1 [n_rows];
 * lse_out and w0_out ([n_rows], the merged log-sum-exp and the weight of side 0) may be NULL.  y may alias a0 or a1.
 * head_dim must be a multiple of 4 and at most 1024.
 */
int spd_lse_merge(spd_ctx *ctx, int32_t n_rows, int32_t head_dim, const float *a0, const float *lse0,
                  const float *a1, const float *lse1, float *y, float *lse_out, float *w0_out, void *hip_stream);

/*
 * The same for n owners of disjoint token sets (Theorem 1 applied n - 1 times, in one launch): e.g. the partials of
 * a cache that is sharded by sequence over several devices, gathered on one.
 *   lse = logsumexp_i(lse_i);  w_i = exp(lse_i - lse);  y = sum_i w_i * a_i   (parts in the order given).
 * a_parts, lse_parts: HOST arrays of n_parts DEVICE pointers ([n_rows][head_dim] and [n_rows] fp32 each), read during
 * the call only; 1 <= n_parts <= SPD_MAX_MERGE_PARTS.  Parts with lse = -inf have weight 0 and their a_i is ignored;
 * if all are, y = 0 and lse = -inf.  lse_out [n_rows] and w_out [n_parts][n_rows] (the weights) may be NULL.
 * y may alias one of the a_i.  head_dim as for spd_lse_merge.
 */
#define SPD_MAX_MERGE_PARTS 16
int spd_lse_merge_n(spd_ctx *ctx, int32_t n_parts, int32_t n_rows, int32_t head_dim, const float *const *a_parts,
                    const float *const *lse_parts, float *y, float *lse_out, float *w_out, void *hip_stream);

/*
 * One whole decode step of one layer for a caller that holds both owners' caches in one process (section 4, step 3).
 * The paper's prototype overlaps the users' private computation with the service's public one; here both owners'
 * work is placed in one launch (the public owner's short pieces run beside the private owner's long streams on the
 * same compute units) and a single closing kernel combines whatever rows either owner had to split and merges the
 * two owners.  Results are those of the three calls above made in sequence, all of them still delivered:
 *   a_in, lse_in   = spd_partial_attn_private(q, priv)            [n_users][Hq][d], [n_users][Hq]
 *   a_out, lse_out = spd_partial_attn_public_batched(q, pub)
 *   y, lse, w_in   = spd_lse_merge(a_in, lse_in, a_out, lse_out)   (all three required here)
 * With k_new and v_new non-NULL (both or neither) the public part is spd_partial_attn_public_batched_append.
 * priv and pub must describe the same users.  Uses the scratch memory of both partial entry points: it must not
 * overlap in time with any other call on the same context.
 */
int spd_decode_step(spd_ctx *ctx, const spd_shape *shape, const void *q, const spd_kv_view *priv,
                    const spd_kv_view *pub, const void *k_new, const void *v_new, float *a_in, float *lse_in,
                    float *a_out, float *lse_out, float *y, float *lse, float *w_in, void *hip_stream);

/*
 * spd_decode_step for callers that cannot allocate device memory: code that is being recorded into a HIP graph,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results; but the split schedules and the
 * chunk partials live in one fixed array of SPD_STATIC_SCRATCH_BYTES of device memory that
 * belongs to the library (one copy per GPU, held until the process ends), the schedules reach it through kernel
 * arguments, and the call makes no hipMalloc, hipFree, hipHostMalloc or copy command - it only launches kernels.
 * A step that does not fit the array fails with SPD_ERR_WORKSPACE before anything is enqueued.  It fits if, for each
 * owner, the schedule takes at most 512 KiB (about 10 000 work items) and the chunk partials number at most
 * 65 536 / G and take at most ~7.2 MiB (slots * G * head_dim fp32): all five benchmark workloads do.
 * Every call on a GPU, from any context, uses that GPU's one array and keeps the previous call's contents in it:
 * calls that overlap in time on one GPU race (run them on one stream, or order them with events).  The call may be
 * recorded into a HIP graph without a warm-up call; once any call has been recorded, later calls send their schedules
 * every time (the library cannot know what replays have left in the array).  Devices 0..63.
 */
#define SPD_STATIC_SCRATCH_BYTES (16u << 20)
int spd_decode_step_static(spd_ctx *ctx, const spd_shape *shape, const void *q, const spd_kv_view *priv,
                           const spd_kv_view *pub, const void *k_new, const void *v_new, float *a_in, float *lse_in,
                           float *a_out, float *lse_out, float *y, float *lse, float *w_in, void *hip_stream);

/*
 * The service's half of a decode step in one call (section 4, step 3c): the public batched partial attention (with the
 * KV append if k_new / v_new are given, else pass NULL for both) and the merge with the private partials
 * (a_in, lse_in) that the users' processes have delivered.  Equivalent to spd_partial_attn_public_batched[_append]
 * followed by spd_lse_merge, with one launch less: the kernel that closes the public call also merges.
 * a_in, lse_in are inputs here (DEVICE, complete on `hip_stream` before the call's work runs); a_out, lse_out, y, lse
 * and w_in are outputs as in spd_decode_step.
 */
int spd_public_attn_merge(spd_ctx *ctx, const spd_shape *shape, const void *q, const spd_kv_view *pub,
                          const void *k_new, const void *v_new, const float *a_in, const float *lse_in, float *a_out,
                          float *lse_out, float *y, float *lse, float *w_in, void *hip_stream);

/*
 * Running statistics of the private part's attention mass (sections 2.4 and 7.1: a user's process can notice a
 * prompt-leakage injection by watching how much attention its prompt still receives; Theorem 1's weight of A_in,
 * w_in = gamma_in / (gamma_in + gamma_out), is that share, and spd_lse_merge / spd_decode_step emit it).
 * One call folds one decode step's masses into the statistics, row by row:
 *   mass_min[i] = min(mass_min[i], w_in[i]);  mass_sum[i] += w_in[i];  n_below[i] += (w_in[i] < threshold).
 * All arrays DEVICE, [n_rows] (w_in, mass_min, mass_sum fp32; n_below int32).  The caller owns and initialises the
 * statistics (mass_min = 1, the others 0) and divides mass_sum by its own step count for the mean; any of the
 * three may be NULL.  The comparison with `threshold` is made on the fp32 values as stored.
 */
int spd_attention_mass_track(spd_ctx *ctx, int32_t n_rows, const float *w_in, float threshold, float *mass_min,
                             float *mass_sum, int32_t *n_below, void *hip_stream);

/*
 * Built-in timing of the partial-attention kernel (the HBM-streaming kernel of both partial calls), measured with HIP
 * events on the stream each call launches on.  spd_set_kernel_timing(ctx, n) arms timing for the next n launches of
 * each entry point (n = 0 disarms); while armed, every partial call launches its partial kernel with a start and a
 * stop event attached to the dispatch itself (hipExtLaunchKernel), so the pair measures the kernel alone.
 * spd_get_kernel_timing waits for the recorded launches of one entry point (0 = private, 1 = public batched), returns
 * their count and mean / minimum duration in microseconds, and clears them.  spd_decode_step's single two-owner
 * launch is booked under entry point 0.
 */
int spd_set_kernel_timing(spd_ctx *ctx, int32_t max_launches);
/* Which instance of the partial kernel the context launched last, as its template arguments
 * {dtype, head_dim, paged, two steps in flight, head per wave, append} (all -1 before the first launch): lets a
 * measurement say which kernel it timed, e.g. partial_mfma_kernel<1, 128, false, false, false, false>. */
int spd_get_last_kernel_instance(const spd_ctx *ctx, int32_t instance[6]);
int spd_get_kernel_timing(spd_ctx *ctx, int32_t entry_point, int32_t *n_launches, double *mean_us, double *min_us);
/* The same, handing out every recorded duration (microseconds, in launch order) instead of their mean and minimum:
 * the first min(*n_launches, capacity) of them are written to us (HOST [capacity]); also clears the record. */
int spd_get_kernel_timing_samples(spd_ctx *ctx, int32_t entry_point, int32_t capacity, float *us, int32_t *n_launches);

/* ------------------------------------------------------------------------------------------------------------
 * Host-only helpers (no GPU needed): the argument checks and the split schedule the calls above use.
 */

/* The validation every partial-attention call performs first.  Returns SPD_OK or the error the call would return. */
int spd_validate_partial(const spd_shape *shape, const void *q, const spd_kv_view *view, const float *out,
                         const float *lse);

/*
 * One segment of split work: tokens [t_begin, t_end) of one (user, KV head) row.  A workgroup processes a *piece*:
 * consecutive segments with the same `piece` index (a piece that crosses a row boundary has one segment per row).
 */
typedef struct spd_work_item {
    int32_t user, kv_head, t_begin, t_end;
    int32_t slot;      /* index of the partial this segment writes when its row has several segments            */
    int32_t n_chunks;  /* segments of this (user, KV head) row; 1 means the segment writes the final result      */
    int32_t chunk;     /* index of this segment within its row                                                  */
    int32_t piece;     /* workgroup that processes this segment                                                  */
} spd_work_item;

/*
 * Build the split schedule for `lens` (HOST, [n_users]) on a device with `n_compute_units` CUs, under the default
 * options (see spd_set_option) or what the SPD_* environment variables say at the time of the call, as an owner of a
 * fused step gets it (a call for one owner alone takes half as many pieces per compute unit again).  The 32-token steps
 * of all rows, laid end to end, are cut into pieces of equal length (+-1 step, apart from what SPD_OPT_SEG_COST and
 * SPD_OPT_HALF_SKEW take from or add to a piece).  Every token of every (user, KV head)
 * is covered by exactly one segment; segment boundaries inside a row are multiples of 32 tokens.
 * items may be NULL to query the count.  On return *n_items is the number of segments (written only if it fits
 * `capacity`, else SPD_ERR_WORKSPACE) and *chunk_tokens the tokens per piece (rounded up to 32).
 * head_per_wave != 0 asks for the schedule of the token-major kernel mapping: a segment then stands for a group of
 * w consecutive KV heads starting at `kv_head` (one wave each), and head kv_head + j writes partial
 * `slot + j * n_chunks`; w = the largest divisor of n_kv_heads that is <= 8 (head_per_wave = 1) or <= head_per_wave
 * (2..8; other values are refused with SPD_ERR_SHAPE).
 */
int spd_build_schedule(const spd_shape *shape, int32_t n_users, const int32_t *lens, int32_t n_compute_units,
                       int32_t head_per_wave, spd_work_item *items, int64_t capacity, int64_t *n_items,
                       int32_t *chunk_tokens);

#ifdef __cplusplus
}
#endif
#endif /* SPD_H */
