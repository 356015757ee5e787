/*
 * Driver for the fp64 oracle built with -fsanitize=address,undefined (tests/test_sanitizers.py
 * compiles this file together with oracle/razor_oracle.c and runs it; test infrastructure).
 * It walks every exported oracle routine over exactly-sized heap buffers -- the hand-worked
 * four-token case of Eq.(5) whose value is known (33/10, 45/12 for the full cache), then seeded
 * random shapes in both storage formats, ragged lengths, strided rows, appended rows, the
 * sliding dropped set and the head scores -- so that an out-of-bounds index, a misaligned access
 * or an integer overflow anywhere in the oracle stops the run.  Prints "oracle sanitize ok".
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int64_t oracle_select(int64_t N, int retrieval, int64_t n_sink, int64_t window, int64_t *kept,
                      int64_t *d_lo, int64_t *d_hi);
void oracle_comp_token2(const void *K_head, const void *V_head, int dtype, int64_t stride_n, int d,
                        int64_t d_lo, int64_t d_hi, const void *K_new, const void *V_new,
                        int64_t stride_new, int64_t n_lo, int64_t n_hi, double *khat, double *vhat);
int oracle_decode_batch(const void *Q, const void *K, const void *V, int dtype, int B, int n_q_heads,
                        int n_kv_heads, int d, int64_t stride_b, int64_t stride_h, int64_t stride_n,
                        const int64_t *kept, const int64_t *kept_off, const void *K_new,
                        const void *V_new, int64_t cap_new, int64_t n_new, const int64_t *new_lo,
                        const double *khat, const double *vhat, const int64_t *N_d,
                        const double *slopes, const int64_t *seq_lens, double scale, double *out);
int oracle_compress_batch(const void *K, const void *V, int dtype, int B, int n_kv_heads, int d,
                          int64_t stride_b, int64_t stride_h, int64_t stride_n,
                          const int64_t *seq_lens, const uint8_t *mask, int64_t n_sink,
                          int64_t window, const int64_t *head_window, int64_t *kept,
                          int64_t *kept_off, double *khat, double *vhat, int64_t *N_d);
int oracle_head_scores(const void *Q, const void *K, int dtype, int n_q_heads, int n_kv_heads,
                       int64_t n_tokens, int d, double scale, int64_t period, int all_copies,
                       double *echo, double *induction);

static uint64_t rng_state = 88172645463325252ull;
static double uniform(void)   /* xorshift64, (-1, 1) */
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}

/* n random values stored as fp32 (dtype 0) or as bf16 bit patterns (dtype 1), exactly n elements */
static void *random_store(size_t n, int dtype)
{
    void *p = malloc(n * (dtype ? 2 : 4) + (n == 0));
    for (size_t i = 0; i < n; ++i) {
        float f = (float)(2.0 * uniform());
        if (dtype) {
            uint32_t bits;
            memcpy(&bits, &f, 4);
            ((uint16_t *)p)[i] = (uint16_t)(bits >> 16);
        } else {
            ((float *)p)[i] = f;
        }
    }
    return p;
}

static int fails = 0;
#define CHECK(cond, ...)                                                  \
    do {                                                                  \
        if (!(cond)) { ++fails; printf("FAILED: " __VA_ARGS__); printf("\n"); } \
    } while (0)

static void hand_worked(void)
{
    float K[4] = {0.f, logf(2.f), logf(8.f), 0.f}, V[4] = {1, 2, 4, 8}, Q[1] = {1};
    for (int retrieval = 0; retrieval < 2; ++retrieval) {
        int64_t lens[1] = {4}, kept[4], off[2], Nd[1];
        uint8_t mask[1] = {(uint8_t)retrieval};
        double khat[1], vhat[1], out[1];
        oracle_compress_batch(K, V, 0, 1, 1, 1, 4, 4, 1, lens, mask, 1, 1, NULL, kept, off, khat, vhat, Nd);
        oracle_decode_batch(Q, K, V, 0, 1, 1, 1, 1, 4, 4, 1, kept, off, K, V, 1, 0, NULL, khat, vhat, Nd, NULL,
                            lens, 1.0, out);
        const double want = retrieval ? 45.0 / 12.0 : 33.0 / 10.0;
        CHECK(fabs(out[0] - want) < 1e-6, "hand-worked Eq.(5): %.9f, expected %.9f", out[0], want);
        CHECK(Nd[0] == (retrieval ? 0 : 2), "hand-worked N_d %lld", (long long)Nd[0]);
    }
}

static void random_case(int dtype, int B, int H, int g, int d, int N, int pad, int n_sink, int window,
                        int n_new, int per_head_windows, int with_slopes)
{
    const int64_t stride_n = d + pad, stride_h = (int64_t)N * stride_n, stride_b = (int64_t)H * stride_h;
    /* the last row of the last head ends exactly at the end of the allocation */
    const size_t n_store = (size_t)(B * stride_b) - (size_t)pad;
    void *K = random_store(n_store, dtype), *V = random_store(n_store, dtype);
    void *Kn = random_store((size_t)B * H * n_new * d, dtype), *Vn = random_store((size_t)B * H * n_new * d, dtype);
    void *Q = random_store((size_t)B * H * g * d, dtype);
    int64_t *lens = malloc(sizeof(int64_t) * B), total = 0;
    for (int b = 0; b < B; ++b) {
        lens[b] = 1 + (int64_t)((uniform() * 0.5 + 0.5) * (N - 1));
        if (b == 0) lens[b] = N;
        total += lens[b];
    }
    uint8_t *mask = malloc(H);
    int64_t *hw = per_head_windows ? malloc(sizeof(int64_t) * H) : NULL;
    for (int h = 0; h < H; ++h) {
        mask[h] = (uint8_t)(uniform() > 0.4);
        if (hw) hw[h] = h % 2 ? 1000000 : 1 + h;
    }
    int64_t *kept = malloc(sizeof(int64_t) * (size_t)(total * H) + 8), *off = malloc(sizeof(int64_t) * (B * H + 1));
    int64_t *Nd = malloc(sizeof(int64_t) * B * H);
    double *khat = malloc(sizeof(double) * B * H * d), *vhat = malloc(sizeof(double) * B * H * d);
    double *out = malloc(sizeof(double) * B * H * g * d), *slopes = NULL;
    if (with_slopes) {
        slopes = malloc(sizeof(double) * H * g);
        for (int j = 0; j < H * g; ++j) slopes[j] = 0.05 * (j + 1);
        memset(Nd, 0, sizeof(int64_t) * B * H);
    }
    oracle_compress_batch(K, V, dtype, B, H, d, stride_b, stride_h, stride_n, lens, mask, n_sink, window, hw, kept,
                          off, khat, vhat, Nd);
    CHECK(off[B * H] <= total * H, "kept rows exceed the sequence rows");
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            const int64_t win = hw ? hw[h] : window;
            const int64_t rows = off[b * H + h + 1] - off[b * H + h];
            const int drops = !mask[h] && lens[b] > n_sink + win;
            CHECK(rows == (drops ? n_sink + win : lens[b]), "rows of (%d, %d)", b, h);
            CHECK(Nd[b * H + h] == (drops ? lens[b] - n_sink - win : 0), "N_d of (%d, %d)", b, h);
        }
    if (with_slopes) memset(Nd, 0, sizeof(int64_t) * B * H);   /* no compensation token with positions */
    oracle_decode_batch(Q, K, V, dtype, B, H * g, H, d, stride_b, stride_h, stride_n, kept, off, Kn, Vn, n_new,
                        n_new, NULL, khat, vhat, Nd, slopes, lens, 1.0 / sqrt((double)d), out);
    /* Eq.(5) is a convex combination of the kept values and vhat: bounded by the largest stored value */
    for (int i = 0; i < B * H * g * d; ++i)
        CHECK(isfinite(out[i]) && fabs(out[i]) <= 2.0 + 1e-9, "output %d = %g", i, out[i]);
    free(K); free(V); free(Kn); free(Vn); free(Q); free(lens); free(mask); free(hw); free(kept); free(off);
    free(Nd); free(khat); free(vhat); free(out); free(slopes);
}

static void sliding_dropped_set(int dtype)
{
    enum { N = 23, T = 9, D = 8 };
    void *K = random_store(N * D, dtype), *V = random_store(N * D, dtype);
    void *Kn = random_store(T * D, dtype), *Vn = random_store(T * D, dtype);
    double kh[D], vh[D], kh2[D], vh2[D];
    /* dropped set = prefill [3, 23) and appended [0, 4); equals the 24-term mean taken in two parts */
    oracle_comp_token2(K, V, dtype, D, D, 3, N, Kn, Vn, D, 0, 4, kh, vh);
    oracle_comp_token2(K, V, dtype, D, D, 3, N, Kn, Vn, D, 0, 0, kh2, vh2);
    for (int c = 0; c < D; ++c) CHECK(isfinite(kh[c]) && isfinite(vh[c]) && isfinite(kh2[c]), "sliding mean");
    int64_t kept[64], lo, hi;
    for (int64_t n = 1; n <= 40; ++n)
        for (int64_t w = 0; w <= 41; w += 5) {
            const int64_t cnt = oracle_select(n, 0, 4, w, kept, &lo, &hi);
            CHECK(cnt + (hi - lo) == n, "select(%lld, window %lld) does not partition the sequence", (long long)n, (long long)w);
        }
    free(K); free(V); free(Kn); free(Vn);
}

static void head_scores(int dtype)
{
    enum { HQ = 4, HKV = 2, N = 61, D = 16, PERIOD = 17 };
    void *Q = random_store((size_t)HQ * N * D, dtype), *K = random_store((size_t)HKV * N * D, dtype);
    double echo[HQ], ind[HQ];
    for (int all = 0; all < 2; ++all) {
        const int rc = oracle_head_scores(Q, K, dtype, HQ, HKV, N, D, 0.25, PERIOD, all, echo, ind);
        CHECK(rc == 0, "oracle_head_scores rc %d", rc);
        for (int h = 0; h < HQ; ++h)
            CHECK(echo[h] > 0 && echo[h] < 1 && ind[h] > 0 && ind[h] < 1, "score of head %d outside (0, 1)", h);
    }
    CHECK(oracle_head_scores(Q, K, dtype, HQ, 3, N, D, 0.25, PERIOD, 0, echo, ind) != 0, "bad group accepted");
    free(Q); free(K);
}

int main(void)
{
    hand_worked();
    for (int dtype = 0; dtype < 2; ++dtype) {
        random_case(dtype, 1, 1, 1, 8, 40, 0, 4, 6, 1, 0, 0);
        random_case(dtype, 3, 4, 2, 16, 97, 0, 4, 20, 3, 0, 0);
        random_case(dtype, 2, 3, 4, 8, 64, 8, 0, 7, 5, 0, 0);      /* strided rows, no sinks */
        random_case(dtype, 2, 2, 1, 8, 33, 0, 4, 0, 2, 0, 0);      /* no window */
        random_case(dtype, 2, 4, 2, 8, 50, 0, 0, 0, 2, 1, 1);      /* per-head windows + ALiBi slopes */
        random_case(dtype, 2, 2, 3, 64, 300, 0, 4, 1000, 4, 0, 0); /* window covers everything */
        sliding_dropped_set(dtype);
        head_scores(dtype);
    }
    if (fails) return 1;
    printf("oracle sanitize ok\n");
    return 0;
}
