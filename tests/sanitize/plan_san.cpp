// Driver for the host-only part of the razor library (csrc/razor_plan.cpp) built with
// -fsanitize=address,undefined (tests/test_sanitizers.py compiles and runs it; no GPU is touched:
// razor_plan, razor_select_heads and razor_strerror are plain host arithmetic).  Every output
// buffer is allocated at exactly the size razor_plan reports, so a write past a table ends the
// run; the tables themselves are checked against Algorithm 1's counts.  Prints "plan sanitize ok".
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "razor.h"

static int fails = 0;
#define CHECK(cond, ...)                                                          \
    do {                                                                          \
        if (!(cond)) { ++fails; std::printf("FAILED: " __VA_ARGS__); std::printf("\n"); } \
    } while (0)

int main()
{
    std::mt19937 rng(20240715);
    auto pick = [&](int lo, int hi) { return lo + (int)(rng() % (unsigned)(hi - lo + 1)); };
    for (int trial = 0; trial < 400; ++trial) {
        razor_params p{};
        p.batch = pick(1, 6);
        p.n_kv_heads = pick(1, 9);
        p.n_q_heads = p.n_kv_heads * pick(1, 4);
        p.head_dim = pick(0, 1) ? 64 : 128;
        p.n_sink = pick(0, 5);
        p.window = pick(trial % 7 == 0 ? 0 : 1, 70);
        p.max_new = pick(0, 40);
        p.use_comp = 1;
        p.dtype = pick(0, 1);
        p.out_dtype = RAZOR_F32;
        p.scale = 0.125f;
        p.sliding = p.window >= 1 ? pick(0, 1) : 0;
        std::vector<int32_t> lens(p.batch), hw(p.n_kv_heads);
        for (auto &n : lens) n = pick(p.sliding ? (p.n_sink > 0 ? p.n_sink : 1) : 1, 200);
        std::vector<uint8_t> mask(p.n_kv_heads);
        for (auto &m : mask) m = (uint8_t)(pick(0, 3) == 0);
        if (trial % 5 == 0) {
            for (auto &w : hw) w = pick(1, 300);
            p.head_window_host = hw.data();
        }
        razor_sizes sz{};
        int rc = razor_plan(&p, lens.data(), mask.data(), nullptr, nullptr, &sz);
        CHECK(rc == RAZOR_OK, "trial %d: razor_plan (sizes only) returned %d", trial, rc);
        if (rc != RAZOR_OK) continue;
        const size_t n_heads = (size_t)p.batch * p.n_kv_heads;
        CHECK(sz.desc_bytes == n_heads * sizeof(razor_head_desc), "trial %d: desc_bytes", trial);
        // exactly-sized heap buffers: one entry too many written by the planner is a heap overflow
        razor_head_desc *desc = (razor_head_desc *)std::malloc(sz.desc_bytes);
        int32_t *idx = (int32_t *)std::malloc(sz.kept_idx_bytes ? sz.kept_idx_bytes : 1);
        rc = razor_plan(&p, lens.data(), mask.data(), desc, idx, &sz);
        CHECK(rc == RAZOR_OK, "trial %d: razor_plan returned %d", trial, rc);
        int64_t rows = 0, cap = 0;
        for (size_t i = 0; i < n_heads && rc == RAZOR_OK; ++i) {
            const razor_head_desc &e = desc[i];
            const int64_t N = lens[i / p.n_kv_heads], win = p.head_window_host ? hw[i % p.n_kv_heads] : p.window;
            const bool drops = !mask[i % p.n_kv_heads] && N > p.n_sink + win;
            CHECK(e.rows == (drops ? p.n_sink + win : N) && e.n_dropped == (drops ? N - p.n_sink - win : 0),
                  "trial %d head %zu: rows %d, N_d %d", trial, i, e.rows, e.n_dropped);
            CHECK(e.row_off == cap && e.kept_off == rows && e.cap % RAZOR_BLOCK_ROWS == 0 && e.cap >= e.rows,
                  "trial %d head %zu: layout", trial, i);
            for (int32_t t = 0; t < e.rows; ++t) {
                const int32_t pos = idx[e.kept_off + t];
                const bool sink = drops && t < p.n_sink;
                CHECK(pos == (drops && !sink ? t + e.n_dropped : t), "trial %d head %zu: kept position %d", trial, i, t);
            }
            rows += e.rows;
            cap += e.cap;
        }
        CHECK(rows == sz.total_rows && cap == sz.total_cap, "trial %d: totals", trial);
        CHECK(sz.kept_idx_bytes == (uint64_t)rows * 4, "trial %d: kept_idx_bytes", trial);
        std::free(desc);
        std::free(idx);
    }
    // head selection: exactly-sized score and mask buffers
    for (int trial = 0; trial < 100; ++trial) {
        const int group = pick(1, 8), n_kv = pick(1, 40), n = group * n_kv;
        float *echo = (float *)std::malloc(sizeof(float) * n), *ind = (float *)std::malloc(sizeof(float) * n);
        uint8_t *mask = (uint8_t *)std::malloc(n_kv);
        for (int i = 0; i < n; ++i) { echo[i] = (float)(rng() % 1000) / 1000.f; ind[i] = (float)(rng() % 1000) / 1000.f; }
        const int rc = razor_select_heads(echo, ind, n, group, 0.14, 0.01, mask);
        CHECK(rc == RAZOR_OK, "select trial %d rc %d", trial, rc);
        int chosen = 0;
        for (int i = 0; i < n_kv; ++i) chosen += mask[i];
        const int most = (int)(0.14 * n + 0.5) + (int)(0.01 * n + 0.5);
        CHECK(chosen <= most, "select trial %d: %d KV heads for at most %d protected query heads", trial, chosen, most);
        std::free(echo); std::free(ind); std::free(mask);
    }
    razor_params bad{};
    CHECK(razor_plan(&bad, nullptr, nullptr, nullptr, nullptr, nullptr) == RAZOR_EINVAL, "zeroed params accepted");
    CHECK(razor_strerror(RAZOR_EINVAL) != nullptr && razor_strerror(12345) != nullptr, "strerror");
    if (fails) return 1;
    std::printf("plan sanitize ok\n");
    return 0;
}
