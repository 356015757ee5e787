// Shared host-side definitions of the razor library (not part of the public ABI).
#ifndef RAZOR_INTERNAL_H
#define RAZOR_INTERNAL_H

#include <cstddef>
#include <cstdint>
#include <vector>

#include "razor.h"

namespace razor {

constexpr int kBlockRows = RAZOR_BLOCK_ROWS;  // K rows per arena block
// razor_compress: a copy workgroup moves kGroupBlocks 16-row blocks of a head, a summing
// workgroup adds up kSumBlocks blocks of its dropped rows.  Each summing workgroup (and, when the
// caller brings column sums, each copy workgroup of a head that dropped rows) leaves one partial
// column sum behind the fixed part of the compress workspace.
constexpr int kGroupBlocks = 4;
#ifndef RAZOR_SUM_BLOCKS
#define RAZOR_SUM_BLOCKS 32
#endif
constexpr int kSumBlocks = RAZOR_SUM_BLOCKS;
constexpr int kMinBlocksPerWorker = 2;        // never split a decode finer than this

inline int elem_size(int dtype) { return dtype == RAZOR_F32 ? 4 : 2; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Where the pieces of the caller's workspace sit.  Decode and compress reuse the
// same buffer; both layouts start at offset 0.
struct DecodeWorkspace {
    size_t prefix_off;  // int32[n_heads + 2]: block prefix sums, then blocks-per-worker
    size_t nd_off;      // int32[n_heads]: N_d of every head as it counts for this step
    size_t ml_off;      // float[slots][g][2]: running max (log2 domain) and denominator
    size_t acc_off;     // float[slots][g][head_dim]: unnormalised output
    size_t bytes;
    int slots;
};
// `workers`: wavefronts the launch is split over; the caller-provided workspace is sized for the
// largest count a launch may use.
DecodeWorkspace decode_workspace(const razor_params &p, int workers = RAZOR_MAX_WORKERS);

struct CompressWorkspace {
    size_t prefix_off;   // int32[n_heads + 2]: first partial sum of every head (razor_compress), or block
                         // prefix sums and blocks per worker (razor_column_sums)
    size_t partial_off;  // float[slots][2][head_dim]: column sums per (worker, head) segment (razor_column_sums)
    size_t desc_off;     // razor_head_desc[n_heads]: private table of razor_column_sums
    size_t bytes;
};
CompressWorkspace compress_workspace(const razor_params &p);

// Wavefronts a streaming launch is split over on the current device (one per SIMD).
int auto_workers(int *out);

// Validates p; returns RAZOR_OK or RAZOR_EINVAL.
int check_params(const razor_params *p);

// Fills desc (size batch * n_kv_heads); returns RAZOR_OK / RAZOR_EINVAL.
int build_plan(const razor_params &p, const int32_t *seq_lens, const uint8_t *mask,
               std::vector<razor_head_desc> &desc, razor_sizes &sizes, int &max_dropped,
               size_t *partial_sum_bytes = nullptr);

// Remembers `what` + the HIP error text for razor_strerror; returns RAZOR_EHIP.
int hip_failure(const char *what, int hip_error);

// Remembers which buffer was too small for razor_strerror; returns RAZOR_ECAPACITY.
int capacity_failure(const char *what);

#ifdef RAZOR_TIMELINE
// Debug build: where the streaming waves leave their clock stamps, in floats from the start of
// the partial outputs of the decode workspace.
constexpr size_t timeline_floats(int n_heads, int g, int head_dim)
{
    return (size_t)(RAZOR_MAX_WORKERS / 2 + n_heads) * g * head_dim;
}
#endif

}  // namespace razor
#endif
