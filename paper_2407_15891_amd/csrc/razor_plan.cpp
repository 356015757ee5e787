// Host-only part of the razor library: argument checks, the selection table of
// Algorithm 1 (steps 2-3), buffer sizes and error text.  No GPU work happens here.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>

#include "razor_internal.h"

namespace razor {

static thread_local char g_hip_error_text[256] = "no HIP error recorded";

int hip_failure(const char *what, int hip_error)
{
    std::snprintf(g_hip_error_text, sizeof g_hip_error_text, "%s: %s", what,
                  hipGetErrorString(static_cast<hipError_t>(hip_error)));
    return RAZOR_EHIP;
}

static thread_local const char *g_capacity_text = "workspace too small";

int capacity_failure(const char *what)
{
    g_capacity_text = what;   // string literals only
    return RAZOR_ECAPACITY;
}

int check_params(const razor_params *p)
{
    if (!p) return RAZOR_EINVAL;
    if (p->batch < 1 || p->n_kv_heads < 1 || p->n_q_heads < 1) return RAZOR_EINVAL;
    if (p->n_q_heads % p->n_kv_heads != 0) return RAZOR_EINVAL;
    if (p->n_q_heads / p->n_kv_heads > RAZOR_MAX_GROUP) return RAZOR_EINVAL;
    if (p->head_dim != 64 && p->head_dim != 128) return RAZOR_EINVAL;
    if (p->n_sink < 0 || p->window < 0 || p->max_new < 0) return RAZOR_EINVAL;
    if (p->dtype != RAZOR_F32 && p->dtype != RAZOR_BF16) return RAZOR_EINVAL;
    if (p->out_dtype != RAZOR_F32 && p->out_dtype != RAZOR_BF16) return RAZOR_EINVAL;
    if (p->use_comp != 0 && p->use_comp != 1) return RAZOR_EINVAL;
    if (!(p->scale == p->scale) || p->scale <= 0.0f) return RAZOR_EINVAL;
    if (p->n_workers < 0 || p->n_workers > RAZOR_MAX_WORKERS) return RAZOR_EINVAL;
    // (sequence, KV head) pairs index gridDim.y of the compaction launches (limit 65535)
    if ((int64_t)p->batch * p->n_kv_heads > RAZOR_MAX_HEADS) return RAZOR_EINVAL;
    if (p->sliding != 0 && p->sliding != 1) return RAZOR_EINVAL;
    if (p->reserved0 != 0) return RAZOR_EINVAL;
    for (int h = 0; h < p->n_kv_heads; ++h) {
        const int win = p->head_window_host ? p->head_window_host[h] : p->window;
        if (win < 0 || (p->sliding && win < 1)) return RAZOR_EINVAL;
    }
    if (p->alibi_slopes && p->use_comp) return RAZOR_EINVAL;   // a mean of keys has no position
    return RAZOR_OK;
}

DecodeWorkspace decode_workspace(const razor_params &p, int workers)
{
    const size_t n_heads = (size_t)p.batch * p.n_kv_heads;
    const size_t g = (size_t)(p.n_q_heads / p.n_kv_heads);
    DecodeWorkspace w;
    // a (worker, head) segment owns slot worker + head, so slots <= workers + heads
    w.slots = (int)(workers + n_heads);
    w.prefix_off = 0;
    w.nd_off = round_up((n_heads + 2) * sizeof(int32_t), 256);
    w.ml_off = w.nd_off + round_up(n_heads * sizeof(int32_t), 256);
    w.acc_off = w.ml_off + round_up((size_t)w.slots * g * 2 * sizeof(float), 256);
    w.bytes = w.acc_off + (size_t)w.slots * g * p.head_dim * sizeof(float);
    return w;
}

CompressWorkspace compress_workspace(const razor_params &p)
{
    const size_t n_heads = (size_t)p.batch * p.n_kv_heads;
    CompressWorkspace w;
    w.prefix_off = 0;
    w.partial_off = round_up((n_heads + 2) * sizeof(int32_t), 256);
    w.desc_off = w.partial_off + (RAZOR_MAX_WORKERS + n_heads) * 2 * p.head_dim * sizeof(float);
    w.bytes = w.desc_off + round_up(n_heads * sizeof(razor_head_desc), 256);
    return w;
}

int auto_workers(int *out)
{
    static thread_local int cached_dev = -1, cached = 0;
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return hip_failure("hipGetDevice", (int)err);
    if (dev != cached_dev) {
        int cus = 0;
        err = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (err != hipSuccess) return hip_failure("hipDeviceGetAttribute", (int)err);
        cached = cus * 4 < RAZOR_MAX_WORKERS ? cus * 4 : RAZOR_MAX_WORKERS;   // one wave per SIMD: measured best for streaming
        cached_dev = dev;
    }
    *out = cached;
    return RAZOR_OK;
}

int build_plan(const razor_params &p, const int32_t *seq_lens, const uint8_t *mask,
               std::vector<razor_head_desc> &desc, razor_sizes &sizes, int &max_dropped,
               size_t *partial_sum_bytes)
{
    const int n_heads = p.batch * p.n_kv_heads;
    desc.assign((size_t)n_heads, razor_head_desc{});
    int64_t row_off = 0, kept_off = 0, groups = 0, chunks = 0;
    max_dropped = 0;
    for (int b = 0; b < p.batch; ++b) {
        const int64_t N = seq_lens[b];
        if (N < 1) return RAZOR_EINVAL;
        if (p.sliding && N < p.n_sink) return RAZOR_EINVAL;   // the sinks must lie inside the prefill
        for (int h = 0; h < p.n_kv_heads; ++h) {
            razor_head_desc &e = desc[(size_t)b * p.n_kv_heads + h];
            const bool retrieval = mask[h] != 0;
            const int64_t window = p.head_window_host ? p.head_window_host[h] : p.window;
            // Nothing is dropped when sinks and window already cover the sequence: the
            // mean over an empty set in Eq.(4) is undefined, so the head keeps every row.
            const bool drops = !retrieval && N > (int64_t)p.n_sink + window;
            const int64_t rows = drops ? (int64_t)p.n_sink + window : N;
            int64_t want = rows + p.max_new;
            // a sliding head stops growing at n_sink + window rows
            if (p.sliding && !retrieval && want > (int64_t)p.n_sink + window) want = (int64_t)p.n_sink + window;
            const int64_t cap = (int64_t)round_up((size_t)want, kBlockRows);
            if (cap > INT32_MAX) return RAZOR_EINVAL;
            e.row_off = row_off;
            e.kept_off = kept_off;
            e.rows = (int32_t)rows;
            e.cap = (int32_t)cap;
            e.n_dropped = drops ? (int32_t)(N - rows) : 0;
            e.window = (int32_t)window;
            e.flags = (retrieval ? RAZOR_HEAD_RETRIEVAL : 0u) | (drops ? RAZOR_HEAD_COMP : 0u);
            if (e.n_dropped > max_dropped) max_dropped = e.n_dropped;
            if (drops) {   // partial column sums razor_compress may leave: per copy group, or per chunk of dropped rows
                groups += ((rows + kBlockRows - 1) / kBlockRows + kGroupBlocks - 1) / kGroupBlocks;
                chunks += ((N - rows + kBlockRows - 1) / kBlockRows + kSumBlocks - 1) / kSumBlocks;
            }
            row_off += cap;
            kept_off += rows;
        }
    }
    const size_t row_bytes = (size_t)2 * p.head_dim * elem_size(p.dtype);
    sizes.arena_bytes = (uint64_t)row_off * row_bytes;
    // sliding mode carries every running mean as an fp32 pair: a second array of low-order parts
    sizes.comp_bytes = (uint64_t)n_heads * 2 * p.head_dim * sizeof(float) * (p.sliding ? 2 : 1);
    sizes.desc_bytes = (uint64_t)n_heads * sizeof(razor_head_desc);
    sizes.kept_idx_bytes = (uint64_t)kept_off * sizeof(int32_t);
    const size_t group_bytes = (size_t)std::max(groups, chunks + n_heads) * 2 * p.head_dim * sizeof(float);
    if (partial_sum_bytes) *partial_sum_bytes = group_bytes;
    const size_t wd = decode_workspace(p).bytes, wc = compress_workspace(p).bytes + group_bytes;
    sizes.workspace_bytes = round_up(wd > wc ? wd : wc, 256);
    sizes.total_rows = kept_off;
    sizes.total_cap = row_off;
    return RAZOR_OK;
}

}  // namespace razor

extern "C" int razor_plan(const razor_params *p, const int32_t *seq_lens_host,
                          const uint8_t *retrieval_mask_host, razor_head_desc *desc_host,
                          int32_t *kept_idx_host, razor_sizes *sizes)
{
    if (razor::check_params(p) != RAZOR_OK) return RAZOR_EINVAL;
    if (!seq_lens_host || !retrieval_mask_host || !sizes) return RAZOR_EINVAL;
    std::vector<razor_head_desc> desc;
    int max_dropped = 0;
    int rc = razor::build_plan(*p, seq_lens_host, retrieval_mask_host, desc, *sizes, max_dropped);
    if (rc != RAZOR_OK) return rc;
    if (desc_host) std::memcpy(desc_host, desc.data(), desc.size() * sizeof(razor_head_desc));
    if (kept_idx_host) {
        for (size_t i = 0; i < desc.size(); ++i) {
            const razor_head_desc &e = desc[i];
            int32_t *out = kept_idx_host + e.kept_off;
            // kept position of cache row t: the sinks come first, the window follows the gap
            const int32_t head = e.n_dropped > 0 ? p->n_sink : e.rows;
            for (int32_t t = 0; t < e.rows; ++t) out[t] = t < head ? t : t + e.n_dropped;
        }
    }
    return RAZOR_OK;
}

extern "C" int razor_select_heads(const float *echo_host, const float *induction_host, int n_heads,
                                  int group, double frac_induction, double frac_echo,
                                  uint8_t *mask_host)
{
    if (!echo_host || !induction_host || !mask_host || n_heads <= 0 || group <= 0 || n_heads % group)
        return RAZOR_EINVAL;
    if (!(frac_induction >= 0.0 && frac_induction <= 1.0) || !(frac_echo >= 0.0 && frac_echo <= 1.0))
        return RAZOR_EINVAL;
    for (int i = 0; i < n_heads; ++i)
        if (std::isnan(echo_host[i]) || std::isnan(induction_host[i])) return RAZOR_EINVAL;
    std::fill(mask_host, mask_host + n_heads / group, (uint8_t)0);
    std::vector<int> order(n_heads);
    const auto protect = [&](const float *score, double frac) {
        const int count = (int)std::floor(frac * n_heads + 0.5);
        for (int i = 0; i < n_heads; ++i) order[i] = i;
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return score[a] > score[b]; });
        for (int k = 0; k < count; ++k) mask_host[order[k] / group] = 1;   // OR over the group
    };
    protect(induction_host, frac_induction);
    protect(echo_host, frac_echo);
    return RAZOR_OK;
}

extern "C" const char *razor_strerror(int status)
{
    switch (status) {
    case RAZOR_OK: return "ok";
    case RAZOR_EINVAL: return "invalid argument";
    case RAZOR_ECAPACITY: return razor::g_capacity_text;
    case RAZOR_EHIP: return razor::g_hip_error_text;
    default: return "unknown status";
    }
}
