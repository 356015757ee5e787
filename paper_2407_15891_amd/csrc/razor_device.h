// Device-side helpers shared by the streaming kernels: the ragged per-head length table
// flattened into one axis of 16-row blocks, cut into equal ranges, one per wavefront.
// Every wave derives its range from the descriptor table alone (one coalesced load per 64
// heads plus wave scans), so no launch has to precede the streaming kernels.
#ifndef RAZOR_DEVICE_H
#define RAZOR_DEVICE_H

#include <hip/hip_runtime.h>

#include <cstddef>

#include "razor_internal.h"

namespace razor {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// {rows, cap, n_dropped, flags} of a table entry travel as one aligned 128-bit load, the buffer
// length as a separate word: the entry is 48 bytes and the table 16-byte aligned (checked by
// every entry point that takes one).
static_assert(sizeof(razor_head_desc) == 48, "table entries must keep 16-byte alignment");
static_assert(offsetof(razor_head_desc, rows) == 16 && offsetof(razor_head_desc, cap) == 20 &&
              offsetof(razor_head_desc, n_dropped) == 24 && offsetof(razor_head_desc, flags) == 28,
              "desc_counts() reads these four as one int4");
__device__ __forceinline__ int4 desc_counts(const razor_head_desc *__restrict__ desc, int idx)
{
    return *reinterpret_cast<const int4 *>(&desc[idx].rows);   // {rows, cap, n_dropped, flags}
}

// Cache and source rows are read once per pass and not again before everything else has
// gone by: non-temporal loads keep them from displacing each other in L2 and measurably
// raise the streaming rate.
template <typename T>
__device__ __forceinline__ T stream_load(const T *p) { return __builtin_nontemporal_load(p); }

__device__ __forceinline__ int wave_sum(int v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Inclusive prefix sum over the 64 lanes with data-parallel-primitive moves (shifts inside rows
// of 16 lanes, then the last lane of a row broadcast to the rows after it): six vector
// instructions, where a scan built on __shfl_up is six dependent trips through the LDS crossbar.
__device__ __forceinline__ int wave_inclusive_scan(int v, int /*lane*/)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
    return v;
}

// How many 16-row blocks a head contributes to the axis being streamed.
struct CachedBlocks {   // rows held this decode step (the token being appended included)
    int has_new;        // a token is appended this step
    int sliding;        // params.sliding
    int n_sink;

    // In sliding mode a non-retrieval head that already holds n_sink + window rows keeps that
    // count: the new token overwrites its oldest window row.
    __device__ __forceinline__ bool slides(int rows, uint32_t flags, int window) const
    {
        return has_new && sliding && !(flags & RAZOR_HEAD_RETRIEVAL) && rows >= n_sink + window;
    }
    __device__ __forceinline__ int rows_of(int rows, int cap, uint32_t flags, int window) const
    {
        if (!has_new || slides(rows, flags, window)) return rows;
        return rows < cap ? rows + 1 : rows;   // an append to a full head is skipped
    }
    __device__ __forceinline__ int operator()(const razor_head_desc *__restrict__ desc, int idx) const
    {
        const int4 f = desc_counts(desc, idx);
        const int window = desc[idx].window;
        return (rows_of(f.x, f.y, (uint32_t)f.w, window) + kBlockRows - 1) / kBlockRows;
    }
    // N_d as it counts for this step (the row a sliding head evicts already included)
    __device__ __forceinline__ int step_n_dropped(const razor_head_desc *__restrict__ desc, int idx) const
    {
        const int4 f = desc_counts(desc, idx);
        const int window = desc[idx].window;
        return f.z + (slides(f.x, (uint32_t)f.w, window) ? 1 : 0);
    }
};
// Row sets a streaming column sum can run over: n(e) source rows per head, the t-th of which is
// source row row(t, e, n_sink).
struct DroppedRows {      // the set D of Eq.(4)
    static __device__ __forceinline__ int n(int rows, int n_dropped) { return n_dropped; }
    static __device__ __forceinline__ int64_t row(int t, int rows, int n_dropped, int n_sink) { return (int64_t)n_sink + t; }
};
struct AllRows {          // every valid row of the sequence
    static __device__ __forceinline__ int n(int rows, int n_dropped) { return rows + n_dropped; }
    static __device__ __forceinline__ int64_t row(int t, int rows, int n_dropped, int n_sink) { return t; }
};
template <class ROWS>
struct RowSetBlocks {     // 16-row blocks of such a set
    __device__ __forceinline__ int operator()(const razor_head_desc *__restrict__ desc, int idx) const
    {
        const int4 f = desc_counts(desc, idx);
        return (ROWS::n(f.x, f.z) + kBlockRows - 1) / kBlockRows;
    }
};

// The flattened axis cut into n_workers equal ranges.
__device__ __forceinline__ int blocks_per_worker(int total, int n_workers)
{
    const int per = (total + n_workers - 1) / n_workers;
    return per < kMinBlocksPerWorker ? kMinBlocksPerWorker : per;
}

// Wave-cooperative.  Length of the axis.
template <class F>
__device__ __forceinline__ int total_blocks(F count, const razor_head_desc *__restrict__ desc,
                                            int n_heads, int lane)
{
    int acc = 0;
    for (int base = 0; base < n_heads; base += 64)
        if (base + lane < n_heads) acc += count(desc, base + lane);
    return wave_sum(acc);
}

// Wave-cooperative.  The head that owns flattened block `blk` (< total) and the flattened
// index of that head's first block.
template <class F>
__device__ __forceinline__ void locate_block(F count, const razor_head_desc *__restrict__ desc,
                                             int n_heads, int lane, int blk, int &head, int &first)
{
    int carry = 0;
    head = 0;
    first = 0;
    for (int base = 0; base < n_heads; base += 64) {
        const int nb = base + lane < n_heads ? count(desc, base + lane) : 0;
        const int end = carry + wave_inclusive_scan(nb, lane);   // flattened end of head base + lane
        const int c = __popcll(__ballot(end <= blk));             // ends are non-decreasing
        if (c < 64) {
            head = base + c;
            first = c == 0 ? carry : __shfl(end, c - 1);
            return;
        }
        carry = __shfl(end, 63);
    }
}

// Wave-cooperative.  Everything a worker needs in one go: the length of the axis, the blocks
// per worker, this worker's range [lo, hi) and, if that range is not empty, the head that owns
// block lo with the flattened index of its first block.  With at most 64 heads (the usual
// case) one load and one scan serve all of it; up to 256 heads the loads of the table go out
// together (a loop of dependent load + scan rounds cost a microsecond per round).
template <class F>
__device__ __forceinline__ void plan_range(F count, const razor_head_desc *__restrict__ desc,
                                           int n_heads, int n_workers, int w, int lane, int &total,
                                           int &per, int &lo, int &hi, int &head, int &first)
{
    if (n_heads <= 64) {
        const int nb = lane < n_heads ? count(desc, lane) : 0;
        const int end = wave_inclusive_scan(nb, lane);
        total = __shfl(end, 63);
        per = blocks_per_worker(total, n_workers);
        lo = w * per;
        hi = lo + per < total ? lo + per : total;
        const int c = __popcll(__ballot(end <= lo));
        head = c;
        first = c == 0 ? 0 : __shfl(end, c - 1);
        return;
    }
    if (n_heads <= 256) {   // four loads issued together, four scans, the rest from registers
        int nb[4], end[4], carry = 0;
#pragma unroll
        for (int t = 0; t < 4; ++t) nb[t] = t * 64 + lane < n_heads ? count(desc, t * 64 + lane) : 0;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            end[t] = carry;
            if (t * 64 < n_heads) {   // uniform: tiles past the table cost nothing
                end[t] = carry + wave_inclusive_scan(nb[t], lane);
                carry = __builtin_amdgcn_readlane(end[t], 63);
            }
        }
        total = carry;
        per = blocks_per_worker(total, n_workers);
        lo = w * per;
        hi = lo + per < total ? lo + per : total;
        head = first = 0;
        if (lo < hi) {   // ends are non-decreasing; lanes past n_heads hold `total` > lo
            int c = 0;
#pragma unroll
            for (int t = 0; t < 4; ++t) c += __popcll(__ballot(end[t] <= lo));
            head = c;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int v = __shfl(end[t], (c - 1) & 63);
                if (c > 0 && ((c - 1) >> 6) == t) first = v;
            }
        }
        return;
    }
    total = total_blocks(count, desc, n_heads, lane);
    per = blocks_per_worker(total, n_workers);
    lo = w * per;
    hi = lo + per < total ? lo + per : total;
    head = first = 0;
    if (lo < hi) locate_block(count, desc, n_heads, lane, lo, head, first);
}

// Wave-cooperative.  prefix[i] = flattened index of head i's first block, prefix[n_heads] =
// length of the axis, prefix[n_heads + 1] = blocks per worker: what a later kernel needs to
// find the partial results of a head (segment of worker w in head i -> slot w + i).
template <class F>
__device__ __forceinline__ void write_prefix(F count, const razor_head_desc *__restrict__ desc,
                                             int n_heads, int lane, int per,
                                             int32_t *__restrict__ prefix)
{
    int carry = 0;
    for (int base = 0; base < n_heads; base += 64) {
        const int nb = base + lane < n_heads ? count(desc, base + lane) : 0;
        const int incl = wave_inclusive_scan(nb, lane);
        if (base + lane < n_heads) prefix[base + lane + 1] = carry + incl;
        carry += __shfl(incl, 63);
    }
    if (lane == 0) {
        prefix[0] = 0;
        prefix[n_heads + 1] = per;
    }
}

}  // namespace razor
#endif
