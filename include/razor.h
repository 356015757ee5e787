/*
 * razor.h -- C ABI of the RazorAttention hot path for AMD MI355X (gfx950).
 *
 * Two device operations, one host-only planner (and razor_column_sums, a stand-in for the
 * prefill epilogue that lets razor_compress skip the dropped rows):
 *
 *   razor_plan         Algorithm 1, steps 2-3 as integer arithmetic: which rows
 *                      every (sequence, KV head) keeps, and where they live.
 *   razor_compress     Algorithm 1, steps 1-4: builds the per-head heterogeneous
 *                      cache from a full post-RoPE K/V cache -- retrieval heads
 *                      keep every row; the others keep n_sink leading rows, the
 *                      last `window` rows and one compensation token, the mean
 *                      of the dropped keys / values (Eq.(4)).
 *   razor_decode_attn  Algorithm 1, step 5: one query per sequence attends the
 *                      compressed cache; the compensation token enters the
 *                      softmax with multiplicity N_d exactly as in Eq.(5).
 *
 * Conventions
 *   - Pointers are DEVICE pointers unless their name ends in _host.
 *   - The library owns no memory and keeps no state between calls.  The caller
 *     allocates every buffer with the sizes razor_plan reports.  Device calls
 *     only enqueue work on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream); they never allocate, never synchronise.  Two exceptions, both
 *     opt-in: razor_decode_attn_static works in a fixed device array owned by the
 *     library, and the measurement hooks of razor_bench.h keep per-thread state.
 *   - All functions return RAZOR_OK (0) or a negative razor_status.  Arguments
 *     are validated on the host before anything is enqueued; a failing call
 *     enqueues nothing.
 *   - One call handles one transformer layer.  The retrieval mask is a model
 *     property: one byte per KV head, shared by every sequence of the batch.
 *     Under GQA a KV head is retrieval if any query head of its group is
 *     (Sec. 4.1 of the paper); that OR is taken by the caller.
 *   - K, V, Q are expected after the rotary transform (Algorithm 1 input); the
 *     library never applies positions.
 *
 * Cache layout (opaque to callers except through razor_head_desc)
 *   arena   per (b, kv head): a K plane of `cap` rows followed by a V plane of
 *           `cap` rows, head_dim elements per row, starting at element offset
 *           row_off * 2 * head_dim.  `cap` is a multiple of 16.  V rows are
 *           stored row-major.  K rows are stored in blocks of 16 rows; inside a
 *           block the 16-byte piece c of row r sits at byte (c * 16 + r) * 16,
 *           so that one wavefront-wide 128-bit load yields a matrix-core
 *           operand without a transpose.
 *   comp    float32 [batch, n_kv_heads, 2, head_dim]: khat then vhat of Eq.(4)
 *           (zeros for heads that dropped nothing).  With params.sliding = 1 a second array
 *           of the same shape follows: the low-order parts of the running means, which
 *           keep their update exact over generations of any length (comp_bytes of
 *           razor_sizes covers both).
 *   desc    razor_head_desc[batch * n_kv_heads], index b * n_kv_heads + h; the device copy
 *           must be 16-byte aligned like every other device buffer handed to the library.
 */
#ifndef RAZOR_H
#define RAZOR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RAZOR_API __attribute__((visibility("default")))

typedef enum razor_dtype { RAZOR_F32 = 0, RAZOR_BF16 = 1 } razor_dtype;

typedef enum razor_status {
    RAZOR_OK = 0,
    RAZOR_EINVAL = -1,     /* null pointer, unsupported dtype / head_dim / group size, bad length or stride */
    RAZOR_ECAPACITY = -2,  /* a workspace is smaller than asked for (razor_strerror names it) */
    RAZOR_EHIP = -3        /* a HIP runtime call failed (razor_strerror gives its text) */
} razor_status;

/* flags of razor_head_desc */
#define RAZOR_HEAD_RETRIEVAL 1u /* mask bit was set: full cache kept                          */
#define RAZOR_HEAD_COMP 2u      /* rows were dropped: comp[] holds a compensation token        */
#define RAZOR_HEAD_OVERFLOW 4u  /* a decode append found the head full and was not stored      */

#define RAZOR_BLOCK_ROWS 16    /* K rows per arena block                                       */
#define RAZOR_MAX_GROUP 16     /* largest n_q_heads / n_kv_heads                               */
#define RAZOR_MAX_WORKERS 8192 /* upper bound on wavefronts a decode launch splits the cache over */
#define RAZOR_MAX_HEADS 65535  /* largest batch * n_kv_heads of one call                          */

typedef struct razor_params {
    int32_t batch;       /* B >= 1; batch * n_kv_heads <= RAZOR_MAX_HEADS */
    int32_t n_q_heads;   /* H_q, multiple of n_kv_heads, group size <= RAZOR_MAX_GROUP */
    int32_t n_kv_heads;  /* H_kv */
    int32_t head_dim;    /* 64 or 128 */
    int32_t n_sink;      /* N_0 of Algorithm 1 (Table 2 uses 4), >= 0 */
    int32_t window;      /* buffer length L_h = max(S_0, N / C) already evaluated by the caller, >= 0 */
    int32_t max_new;     /* rows reserved per head for decode-time appends, >= 0 */
    int32_t use_comp;    /* 1: Eq.(5).  0: drop the compensation term (sinks + window only) */
    int32_t dtype;       /* razor_dtype of Q, K, V, k_new, v_new and of the arena */
    int32_t out_dtype;   /* razor_dtype of O */
    float scale;         /* multiplies every logit, the compensation logit included; 1.0f is
                            Eq.(5) as printed, 1/sqrt(head_dim) what the evaluated models use */
    int32_t n_workers;   /* wavefronts to split a pass over; 0 = pick from the device: one per SIMD
                            (four per compute unit), two for decode over 128-byte rows */
    int32_t sliding;     /* 0: compress once, decode appends and never evicts.
                            1: Algorithm 1 re-applied after every generated token: once a
                            non-retrieval head holds n_sink + window rows, an append overwrites its
                            oldest window row, and that row first moves into the compensation token
                            (khat += (k - khat) / (N_d + 1), likewise vhat, N_d += 1: Eq.(4) over the
                            enlarged dropped set).  Needs window >= 1 and every seq_len >= n_sink. */
    int32_t reserved0;   /* must be 0 */
    const int32_t *head_window_host; /* HOST, [n_kv_heads] or NULL: buffer length per KV head, used
                            instead of `window` (ALiBi models: the vision scope L_h of Eq.(2),
                            evaluated by the caller; a value >= the sequence keeps everything) */
    const float *alibi_slopes;       /* DEVICE, [n_q_heads] or NULL.  Non-NULL selects Eq.(1): every
                            logit becomes scale * q.k_n - slope[head] * (m - n), m the position of
                            the query (the newest token), n of the key.  The compensation token has
                            no position, so use_comp must be 0.  Only razor_decode_attn reads it. */
} razor_params;

/* One entry per (sequence b, KV head h).  Written by razor_plan (host copy) and
 * razor_compress (device copy); `rows`, `n_dropped`, `evicted` and flags of the device
 * copy are updated by razor_decode_attn when it appends. */
typedef struct razor_head_desc {
    int64_t row_off;   /* first row of this head's region, in rows of 2*head_dim elements */
    int64_t kept_off;  /* first entry of this head in kept_idx                             */
    int32_t rows;      /* cached rows (compensation token not counted)                     */
    int32_t cap;       /* rows reserved; multiple of 16, >= rows at plan time + max_new
                          (sliding, non-retrieval: >= min(that, n_sink + window))          */
    int32_t n_dropped; /* N_d of Eq.(4)/(5); 0 when nothing was dropped                    */
    uint32_t flags;    /* RAZOR_HEAD_*                                                     */
    int32_t evicted;   /* sliding mode: rows overwritten so far; the next one is row
                          n_sink + evicted % window                                        */
    int32_t window;    /* buffer length of this head (p->window or head_window_host[h])    */
    int32_t reserved[2]; /* zero; pads an entry to 48 bytes so that {rows, cap, n_dropped,
                          flags} of every entry of a 16-byte aligned table can be fetched
                          with one aligned 128-bit load                                    */
} razor_head_desc;

typedef struct razor_sizes {
    uint64_t arena_bytes;
    uint64_t comp_bytes;
    uint64_t desc_bytes;
    uint64_t kept_idx_bytes;
    uint64_t workspace_bytes; /* enough for razor_compress and for razor_decode_attn */
    int64_t total_rows;       /* sum of rows over all heads */
    int64_t total_cap;        /* sum of cap over all heads  */
} razor_sizes;

/*
 * Host-only; touches no GPU.  Algorithm 1 steps 2-3 for every (b, h):
 *   retrieval head, or seq_len <= n_sink + window:  keep rows [0, seq_len), N_d = 0;
 *   otherwise keep [0, n_sink) and [seq_len - window, seq_len), N_d = seq_len - n_sink - window
 *   (window = p->window, or p->head_window_host[h] when that table is given).
 * seq_lens_host[batch] (each >= 1), retrieval_mask_host[n_kv_heads] (non-zero = retrieval).
 * desc_host[batch * n_kv_heads] and kept_idx_host[total_rows] may each be NULL (sizes only;
 * kept positions ascending per head, heads in desc order).  sizes must not be NULL.
 */
RAZOR_API int razor_plan(const razor_params *p, const int32_t *seq_lens_host,
               const uint8_t *retrieval_mask_host, razor_head_desc *desc_host,
               int32_t *kept_idx_host, razor_sizes *sizes);

/*
 * Builds arena, comp and desc_dev from the full cache (Eq.(4) + Algorithm 1 step 3).
 * K, V: element [b, h, n, c] at b*stride_b + h*stride_h + n*stride_n + c (strides in
 * elements, last dimension contiguous, 16-byte aligned rows); rows n >= seq_lens[b] are
 * never read.  kept_idx_dev (int32[total_rows], nullable) receives the kept positions.
 * After the call the arena is self-contained: the caller may release K and V.
 * Means are accumulated in fp32 in a fixed order (bit-reproducible run to run).
 * col_sums (float32 [batch, n_kv_heads, 2, head_dim], nullable): sums of K and of V over rows
 * [0, seq_len) of every head, e.g. accumulated by the kernel that wrote K and V during prefill
 * (or by razor_column_sums).  When given, the dropped rows are not read at all: Eq.(4) is
 * evaluated as (col_sums - sum of the kept rows) / N_d, the kept rows being added up while
 * they are copied, which roughly halves the traffic of this call.  The subtraction loses accuracy when N_d is tiny against the sequence length.
 */
RAZOR_API int razor_compress(const razor_params *p, const void *K, const void *V,
                   int64_t stride_b, int64_t stride_h, int64_t stride_n,
                   const int32_t *seq_lens_host, const uint8_t *retrieval_mask_host,
                   void *arena, float *comp, razor_head_desc *desc_dev,
                   int32_t *kept_idx_dev, const float *col_sums, void *workspace,
                   size_t workspace_bytes, void *stream);

/*
 * Column sums of K and V over rows [0, seq_len) of every (sequence, KV head): what a prefill
 * kernel's epilogue can accumulate while it writes the cache.  col_sums: float32
 * [batch, n_kv_heads, 2, head_dim] (K sums, then V sums), fixed summation order.  Of p only
 * batch, n_kv_heads, head_dim, dtype and n_workers matter (the rest must still be valid).
 * The workspace is the one razor_plan sizes.
 */
RAZOR_API int razor_column_sums(const razor_params *p, const void *K, const void *V,
                      int64_t stride_b, int64_t stride_h, int64_t stride_n,
                      const int32_t *seq_lens_host, float *col_sums, void *workspace,
                      size_t workspace_bytes, void *stream);

/*
 * One decode step.  If k_new and v_new ([batch, n_kv_heads, head_dim]) are non-NULL the
 * new token is first appended to every head (rows += 1; a full head sets
 * RAZOR_HEAD_OVERFLOW and skips the append; in sliding mode a non-retrieval head that holds
 * n_sink + window rows instead moves its oldest window row into comp and overwrites it),
 * then Q [batch, n_q_heads, head_dim] attends:
 * retrieval heads by plain softmax attention, the others by Eq.(5), logits scaled by
 * p->scale, accumulation in fp32.  O [batch, n_q_heads, head_dim] in p->out_dtype.
 * p must describe the same batch / heads / head_dim / dtype the cache was built with.
 * Results are bit-reproducible run to run (no floating-point atomics).
 */
RAZOR_API int razor_decode_attn(const razor_params *p, const void *Q, const void *k_new,
                      const void *v_new, void *arena, float *comp,
                      razor_head_desc *desc_dev, void *O, void *workspace,
                      size_t workspace_bytes, void *stream);

/*
 * razor_decode_attn for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and same results as razor_decode_attn, but the split-K scratch of the
 * step (block-prefix table, per-step N_d, partial softmax states) lives in a device array of
 * RAZOR_STATIC_SCRATCH_BYTES that belongs to the library: every GPU the library runs on holds
 * its own copy from the first call on that GPU until the process ends.  The call allocates
 * nothing and frees nothing; its first call on a device only looks up the array's address.
 * The scratch a step needs grows with the wavefronts it is split over (n_workers, or four per
 * compute unit), the (sequence, KV head) pairs and the query group:
 *   (workers + batch * n_kv_heads) * (n_q_heads / n_kv_heads) * (head_dim + 2) * 4 bytes + tables;
 * a step that needs more than the array returns RAZOR_ECAPACITY and enqueues nothing (every
 * benchmark configuration fits: at most 4.8 MB).  All calls on one GPU share that GPU's array,
 * which keeps the last call's contents (nothing in it has to start at zero): calls that overlap
 * in time on one GPU -- different streams, or different threads -- race; calls on one stream
 * are safe.
 */
#define RAZOR_STATIC_SCRATCH_BYTES (8u << 20)
RAZOR_API int razor_decode_attn_static(const razor_params *p, const void *Q, const void *k_new,
                             const void *v_new, void *arena, float *comp,
                             razor_head_desc *desc_dev, void *O, void *stream);

/*
 * Sec. 3.3, identification of retrieval heads: echo and induction score of every query head
 * on a prompt made of `period` random tokens repeated up to n_tokens (the paper: 2500 tokens,
 * four times).  For a query position m >= period the echo token is the previous copy of the
 * current token, position m - period; the induction token follows it, position m - period + 1.
 *   echo[h]      = mean over m in [period, n_tokens) of A_h[m, m - period]
 *   induction[h] = mean over m in [period, n_tokens) of A_h[m, m - period + 1]
 * with A_h the causal softmax(scale * Q_h K_h^T) attention map (query head h reads KV head
 * h / (n_q_heads / n_kv_heads)).  all_copies != 0 sums the weight over every previous copy,
 * m - j * period (+ 1), j = 1, 2, ..., instead of the nearest one.  The map is never stored.
 *
 * Q  device, [n_q_heads, n_tokens, head_dim] with element strides q_stride_h, q_stride_n, last
 *    dimension contiguous, values as after the rotary transformation; K likewise
 *    [n_kv_heads, n_tokens, head_dim].  Layers may be stacked along the head dimension.
 *    dtype must be RAZOR_BF16 (matrix-core kernel), head_dim 64 or 128, strides multiples of 8
 *    elements, base pointers 16-byte aligned, scale > 0, 1 <= period < n_tokens,
 *    n_q_heads <= 65535.
 * echo, induction  device, float32 [n_q_heads], written.
 * workspace        device, at least razor_head_scores_workspace(n_q_heads, n_tokens) bytes
 *                  (returns 0 for non-positive arguments); RAZOR_ECAPACITY if smaller.
 * Everything is enqueued on `stream`; sums are taken in a fixed order (bit-reproducible).
 */
RAZOR_API size_t razor_head_scores_workspace(int n_q_heads, int n_tokens);
RAZOR_API int razor_head_scores(const void *Q, const void *K, int dtype, int n_q_heads,
                      int n_kv_heads, int head_dim, int n_tokens, int64_t q_stride_h,
                      int64_t q_stride_n, int64_t k_stride_h, int64_t k_stride_n, float scale,
                      int period, int all_copies, float *echo, float *induction,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * Sec. 3.3 / Table 2 / Sec. 4.1, host only: turn scores into the retrieval mask razor_plan
 * takes.  Of the n_heads query heads (all layers of the model, layer-major) the
 * round(frac_induction * n_heads) with the highest induction score and the
 * round(frac_echo * n_heads) with the highest echo score are retrieval heads (halves round up;
 * equal scores: lower index first; the paper uses 0.14 and 0.01).  mask_host
 * (uint8 [n_heads / group]) gets 1 for a KV head when any of its `group` query heads was
 * chosen.  RAZOR_EINVAL for NaN scores, fractions outside [0, 1] or n_heads % group != 0.
 */
RAZOR_API int razor_select_heads(const float *echo_host, const float *induction_host,
                       int n_heads, int group, double frac_induction, double frac_echo,
                       uint8_t *mask_host);

/* Text for a razor_status; for RAZOR_EHIP the text of the last HIP error seen by the
 * calling thread, for RAZOR_ECAPACITY the buffer its last such failure found too small.
 * The pointer stays valid until the thread's next failing call. */
RAZOR_API const char *razor_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* RAZOR_H */
