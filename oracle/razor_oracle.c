/*
 * RazorAttention reference oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 CPU statement of what the compressed-KV hot path
 * computes, written from the paper (arXiv 2407.15891).  It shares no code,
 * header, table or helper with the HIP library; only tests, the smoke check
 * and the cpu_baseline leg of the benchmark may call it.
 *
 *   oracle_select       Algorithm 1, steps 2-3: which cache rows a head keeps
 *   oracle_comp_token   Eq.(4): the compensation token (mean of dropped rows)
 *   oracle_comp_token2  Eq.(4) over a dropped set that reaches into the appended rows
 *   oracle_attn_head    Eq.(5): attention over kept rows + compensation token
 *   oracle_decode_batch Algorithm 1, step 5: per-head dispatch over a batch
 *   oracle_head_scores  Sec. 3.3: echo and induction score of every head on a repeated prompt
 *
 * No tiling, no online softmax, no fusion: two passes over the logits and
 * straight sums, so every line can be held against the paper by eye.
 * Inputs are read from their stored bits (bf16 or fp32) and widened to
 * double without rounding.
 *
 * Parity status: the numeric value of Eq.(5) on general data is not printed
 * anywhere in the paper ("parity unpinned" by a worked example); it is
 * pinned through the special cases, closed forms and brute force listed in
 * tests/test_oracle_pins.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

/* One stored element -> double (exact for both formats). */
static double widen(const void *base, int dtype, int64_t idx)
{
    if (dtype == ORACLE_F32) {
        return (double)((const float *)base)[idx];
    } else {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
}

/*
 * Algorithm 1, steps 2-3 (selection).  A retrieval head keeps every token.
 * A non-retrieval head keeps the first n_sink tokens and the most recent
 * `window` tokens; everything in between is the dropped set D = [d_lo, d_hi).
 * When sinks and window already cover the sequence nothing is dropped
 * (Eq.(4) would be 0/0), so the head is treated like a retrieval head.
 * kept[] receives the kept positions in ascending order; returns their count.
 */
int64_t oracle_select(int64_t N, int retrieval, int64_t n_sink, int64_t window,
                      int64_t *kept, int64_t *d_lo, int64_t *d_hi)
{
    int64_t n = 0;
    if (retrieval || N <= n_sink + window) {
        for (int64_t t = 0; t < N; ++t) kept[n++] = t;
        *d_lo = 0;
        *d_hi = 0;
        return n;
    }
    for (int64_t t = 0; t < n_sink; ++t) kept[n++] = t;
    for (int64_t t = N - window; t < N; ++t) kept[n++] = t;
    *d_lo = n_sink;
    *d_hi = N - window;
    return n;
}

/*
 * Eq.(4): khat = (1/N_d) sum_{m in D} k_m, vhat likewise, D = [d_lo, d_hi).
 * K_head / V_head point at row 0 of one head; row stride in elements.
 */
void oracle_comp_token(const void *K_head, const void *V_head, int dtype,
                       int64_t stride_n, int d, int64_t d_lo, int64_t d_hi,
                       double *khat, double *vhat)
{
    int64_t N_d = d_hi - d_lo;
    for (int c = 0; c < d; ++c) khat[c] = vhat[c] = 0.0;
    for (int64_t m = d_lo; m < d_hi; ++m) {
        for (int c = 0; c < d; ++c) {
            khat[c] += widen(K_head, dtype, m * stride_n + c);
            vhat[c] += widen(V_head, dtype, m * stride_n + c);
        }
    }
    for (int c = 0; c < d; ++c) {
        khat[c] /= (double)N_d;
        vhat[c] /= (double)N_d;
    }
}

/*
 * Eq.(4) when the dropped set spans two stores: positions [d_lo, d_hi) of the prefill
 * cache and rows [n_lo, n_hi) of the rows appended during decoding (sliding mode, where
 * Algorithm 1 is re-applied to the whole sequence after every generated token).
 */
void oracle_comp_token2(const void *K_head, const void *V_head, int dtype, int64_t stride_n,
                        int d, int64_t d_lo, int64_t d_hi,
                        const void *K_new, const void *V_new, int64_t stride_new,
                        int64_t n_lo, int64_t n_hi, double *khat, double *vhat)
{
    int64_t N_d = (d_hi - d_lo) + (n_hi - n_lo);
    for (int c = 0; c < d; ++c) khat[c] = vhat[c] = 0.0;
    for (int64_t m = d_lo; m < d_hi; ++m)
        for (int c = 0; c < d; ++c) {
            khat[c] += widen(K_head, dtype, m * stride_n + c);
            vhat[c] += widen(V_head, dtype, m * stride_n + c);
        }
    for (int64_t m = n_lo; m < n_hi; ++m)
        for (int c = 0; c < d; ++c) {
            khat[c] += widen(K_new, dtype, m * stride_new + c);
            vhat[c] += widen(V_new, dtype, m * stride_new + c);
        }
    for (int c = 0; c < d; ++c) {
        khat[c] /= (double)N_d;
        vhat[c] /= (double)N_d;
    }
}

/*
 * Eq.(5) for one query vector q (length d):
 *
 *        N_d e^{q.khat} vhat + sum_{n kept} e^{q.k_n} v_n
 *   o = ---------------------------------------------------
 *        N_d e^{q.khat}      + sum_{n kept} e^{q.k_n}
 *
 * with every logit multiplied by `scale` (scale = 1 is the printed form).
 * Kept rows come from two places: positions kept[0..n_kept) of the prefill
 * cache (K_head/V_head, row stride stride_n) and n_new rows appended during
 * decoding (K_new/V_new, row stride stride_new).  N_d == 0 means no
 * compensation term (retrieval head, nothing dropped, or ablation).
 * The exponentials are shifted by the largest logit, which cancels in the
 * quotient.  scratch must hold n_kept + n_new doubles.
 *
 * ALiBi models (Eq.(1)): the logit of the key at position n for the query at position
 * q_pos is scale * q.k_n - slope * (q_pos - n).  Prefill rows sit at their kept position,
 * appended row a at new_pos0 + a.  slope = 0 gives the RoPE form (Eq.(3)).  The
 * compensation token has no position; ALiBi callers pass N_d = 0.
 */
void oracle_attn_head(const double *q, int d, double scale,
                      const void *K_head, const void *V_head, int dtype,
                      int64_t stride_n, const int64_t *kept, int64_t n_kept,
                      const void *K_new, const void *V_new, int64_t stride_new,
                      int64_t n_new,
                      const double *khat, const double *vhat, int64_t N_d,
                      double slope, int64_t q_pos, int64_t new_pos0,
                      double *scratch, double *out)
{
    int64_t n_rows = n_kept + n_new;
    double s_c = 0.0, M = -INFINITY;

    /* pass 1: logits */
    for (int64_t r = 0; r < n_rows; ++r) {
        const void *kb = r < n_kept ? K_head : K_new;
        int64_t off = r < n_kept ? kept[r] * stride_n : (r - n_kept) * stride_new;
        double s = 0.0;
        for (int c = 0; c < d; ++c) s += q[c] * widen(kb, dtype, off + c);
        s *= scale;
        if (slope != 0.0) {
            int64_t pos = r < n_kept ? kept[r] : new_pos0 + (r - n_kept);
            s -= slope * (double)(q_pos - pos);
        }
        scratch[r] = s;
        if (s > M) M = s;
    }
    if (N_d > 0) {
        for (int c = 0; c < d; ++c) s_c += q[c] * khat[c];
        s_c *= scale;
        /* the term N_d e^{s_c} equals e^{s_c + ln N_d}; only used to pick the shift */
        if (s_c + log((double)N_d) > M) M = s_c + log((double)N_d);
    }

    /* pass 2: numerator and denominator */
    double den = 0.0;
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    for (int64_t r = 0; r < n_rows; ++r) {
        const void *vb = r < n_kept ? V_head : V_new;
        int64_t off = r < n_kept ? kept[r] * stride_n : (r - n_kept) * stride_new;
        double e = exp(scratch[r] - M);
        den += e;
        for (int c = 0; c < d; ++c) out[c] += e * widen(vb, dtype, off + c);
    }
    if (N_d > 0) {
        double e = (double)N_d * exp(s_c - M);
        den += e;
        for (int c = 0; c < d; ++c) out[c] += e * vhat[c];
    }
    for (int c = 0; c < d; ++c) out[c] /= den;
}

/*
 * Algorithm 1, step 5 over a batch: query head j of sequence b uses KV head
 * h = j / g (g = n_q_heads / n_kv_heads; a KV group shares one decision).
 *
 *   Q        [B, n_q_heads, d] stored dtype
 *   K, V     prefill cache, element strides (stride_b, stride_h, stride_n)
 *   kept     concatenated kept positions, head (b,h) owns
 *            kept[kept_off[b*Hkv+h] .. kept_off[b*Hkv+h+1])
 *   K_new,V_new [B, n_kv_heads, cap_new, d] appended rows, n_new of them valid; head (b,h)
 *            keeps rows [new_lo[b*Hkv+h], n_new) of them (new_lo == NULL: all)
 *   khat,vhat   [B, n_kv_heads, d] doubles;  N_d [B, n_kv_heads]
 *   slopes   ALiBi slope per query head (NULL: none); seq_lens[b] = prefill length, which
 *            places appended row a at position seq_lens[b] + a and the query at the last one
 *   out      [B, n_q_heads, d] doubles
 * Returns the number of threads used.
 */
int oracle_decode_batch(const void *Q, const void *K, const void *V, int dtype,
                        int B, int n_q_heads, int n_kv_heads, int d,
                        int64_t stride_b, int64_t stride_h, int64_t stride_n,
                        const int64_t *kept, const int64_t *kept_off,
                        const void *K_new, const void *V_new, int64_t cap_new,
                        int64_t n_new, const int64_t *new_lo,
                        const double *khat, const double *vhat,
                        const int64_t *N_d, const double *slopes, const int64_t *seq_lens,
                        double scale, double *out)
{
    int g = n_q_heads / n_kv_heads;
    int n_threads = 1;
    int64_t esz = dtype == ORACLE_F32 ? 4 : 2;
#ifdef _OPENMP
    n_threads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int bj = 0; bj < B * n_q_heads; ++bj) {
        int b = bj / n_q_heads, j = bj % n_q_heads, h = j / g;
        int64_t bh = (int64_t)b * n_kv_heads + h;
        int64_t n_kept = kept_off[bh + 1] - kept_off[bh];
        double *qd = (double *)malloc(sizeof(double) * (size_t)d);
        double *scratch = (double *)malloc(sizeof(double) * (size_t)(n_kept + n_new + 1));
        for (int c = 0; c < d; ++c) qd[c] = widen(Q, dtype, (int64_t)bj * d + c);
        const char *Kh = (const char *)K + (b * stride_b + h * stride_h) * esz;
        const char *Vh = (const char *)V + (b * stride_b + h * stride_h) * esz;
        int64_t lo_new = new_lo ? new_lo[bh] : 0;
        const char *Kn = K_new ? (const char *)K_new + (bh * cap_new + lo_new) * d * esz : NULL;
        const char *Vn = V_new ? (const char *)V_new + (bh * cap_new + lo_new) * d * esz : NULL;
        oracle_attn_head(qd, d, scale, Kh, Vh, dtype, stride_n,
                         kept + kept_off[bh], n_kept, Kn, Vn, d, n_new - lo_new,
                         khat + bh * d, vhat + bh * d, N_d[bh],
                         slopes ? slopes[j] : 0.0, seq_lens[b] + n_new - 1, seq_lens[b] + lo_new,
                         scratch, out + (int64_t)bj * d);
        free(qd);
        free(scratch);
    }
    return n_threads;
}

/*
 * Algorithm 1, steps 1-4 over a batch: selection and compensation tokens
 * for every (sequence, KV head).  mask[h] != 0 marks a retrieval KV head
 * (a model property, shared by all sequences).  kept must have room for
 * sum_b n_kv_heads * seq_lens[b] entries; kept_off gets B*Hkv+1 entries.
 */
int oracle_compress_batch(const void *K, const void *V, int dtype,
                          int B, int n_kv_heads, int d,
                          int64_t stride_b, int64_t stride_h, int64_t stride_n,
                          const int64_t *seq_lens, const uint8_t *mask,
                          int64_t n_sink, int64_t window, const int64_t *head_window,
                          int64_t *kept, int64_t *kept_off,
                          double *khat, double *vhat, int64_t *N_d)
{
    int n_threads = 1;
    int64_t esz = dtype == ORACLE_F32 ? 4 : 2;
    int64_t *d_lo = (int64_t *)malloc(sizeof(int64_t) * (size_t)(B * n_kv_heads));
    int64_t *d_hi = (int64_t *)malloc(sizeof(int64_t) * (size_t)(B * n_kv_heads));
    kept_off[0] = 0;
    for (int bh = 0; bh < B * n_kv_heads; ++bh) {
        int b = bh / n_kv_heads, h = bh % n_kv_heads;
        /* head_window: a buffer length per KV head (the vision scope L_h of Eq.(2)) */
        int64_t n = oracle_select(seq_lens[b], mask[h] != 0, n_sink,
                                  head_window ? head_window[h] : window,
                                  kept + kept_off[bh], &d_lo[bh], &d_hi[bh]);
        kept_off[bh + 1] = kept_off[bh] + n;
        N_d[bh] = d_hi[bh] - d_lo[bh];
    }
#ifdef _OPENMP
    n_threads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int bh = 0; bh < B * n_kv_heads; ++bh) {
        int b = bh / n_kv_heads, h = bh % n_kv_heads;
        for (int c = 0; c < d; ++c) khat[(int64_t)bh * d + c] = vhat[(int64_t)bh * d + c] = 0.0;
        if (N_d[bh] > 0) {
            const char *Kh = (const char *)K + (b * stride_b + h * stride_h) * esz;
            const char *Vh = (const char *)V + (b * stride_b + h * stride_h) * esz;
            oracle_comp_token(Kh, Vh, dtype, stride_n, d, d_lo[bh], d_hi[bh],
                              khat + (int64_t)bh * d, vhat + (int64_t)bh * d);
        }
    }
    free(d_lo);
    free(d_hi);
    return n_threads;
}

/*
 * Sec. 3.3 (identification of retrieval heads): the prompt is `period` random tokens
 * repeated several times, n_tokens in all.  For a query position m >= period the echo
 * token is the previous copy of the current token, position m - period, and the
 * induction token is the one right after it, position m - period + 1.  A head's echo
 * (induction) score is its causal softmax attention weight on that position, averaged
 * over the positions m in [period, n_tokens) (earlier positions have no previous copy).
 * With all_copies != 0 the weight is summed over every previous copy, m - j * period
 * (+1), j = 1, 2, ... while that position is not negative.
 *
 * Q [n_q_heads, n_tokens, d], K [n_kv_heads, n_tokens, d] contiguous, after the rotary
 * transformation; query head h reads KV head h / (n_q_heads / n_kv_heads).
 * Every row of the attention map is formed in full: logits, maximum, sum, division.
 */
int oracle_head_scores(const void *Q, const void *K, int dtype, int n_q_heads, int n_kv_heads,
                       int64_t n_tokens, int d, double scale, int64_t period, int all_copies,
                       double *echo, double *induction)
{
    if (n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads || period < 1 || period >= n_tokens)
        return -1;
    const int g = n_q_heads / n_kv_heads;
#pragma omp parallel for schedule(dynamic)
    for (int h = 0; h < n_q_heads; ++h) {
        double *w = (double *)malloc(sizeof(double) * (size_t)n_tokens);
        double *q = (double *)malloc(sizeof(double) * (size_t)d);
        double sum_echo = 0.0, sum_ind = 0.0;
        for (int64_t m = period; m < n_tokens; ++m) {
            for (int c = 0; c < d; ++c) q[c] = widen(Q, dtype, ((int64_t)h * n_tokens + m) * d + c);
            double top = -INFINITY;
            for (int64_t n = 0; n <= m; ++n) {                 /* causal: keys 0..m */
                double dot = 0.0;
                for (int c = 0; c < d; ++c)
                    dot += q[c] * widen(K, dtype, ((int64_t)(h / g) * n_tokens + n) * d + c);
                w[n] = scale * dot;
                if (w[n] > top) top = w[n];
            }
            double denom = 0.0;
            for (int64_t n = 0; n <= m; ++n) {
                w[n] = exp(w[n] - top);
                denom += w[n];
            }
            for (int64_t prev = m - period; prev >= 0; prev -= period) {
                sum_echo += w[prev] / denom;
                sum_ind += w[prev + 1] / denom;                /* prev + 1 <= m since period >= 1 */
                if (!all_copies) break;
            }
        }
        echo[h] = sum_echo / (double)(n_tokens - period);
        induction[h] = sum_ind / (double)(n_tokens - period);
        free(w);
        free(q);
    }
    return 0;
}
