// razor_compress: prefill-time pass that turns a full K/V cache into the per-head
// heterogeneous cache (Algorithm 1 steps 1-4, Eq.(4)).  Three kinds of work:
//   mean   column sums of the dropped rows [n_sink, N - window) -> khat, vhat (fp32)
//   copy   kept rows (sinks + window, or everything) -> arena; K re-tiled through LDS
//   index  kept positions as int32 (optional)
// All of it is HBM streaming: every source row is read once, kept rows written once.
// Given the column sums over the whole sequence (razor_column_sums, or a prefill epilogue) the
// dropped rows are not read: the copy adds up the kept rows it moves and the mean is taken
// from the difference.
//
// Launches of one call, by the number of (sequence, KV head) pairs:
//   up to 64    sum_dropped_kernel, compress_kernel -- the table travels as a kernel argument of
//               both, and the second level of Eq.(4) rides in the first grid row of the copy
//   up to 256   upload_desc_kernel (one per 64 pairs) first; the rest as above
//   beyond      upload, compress_kernel (copy and first-level sums in one launch), mean_final_kernel
//   column sums given   upload, compress_kernel (copy + sums of the kept rows), mean_final_kernel
//   nothing dropped anywhere   (upload,) compress_kernel
// plus kept_index_kernel when the caller asks for the positions.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <vector>

#include "razor_device.h"
#include "razor_internal.h"

namespace razor {
namespace {

#ifndef RAZOR_LDS_PAD
#define RAZOR_LDS_PAD 0
#endif
constexpr int kDescPerLaunch = 64;
constexpr int kStagedSums = 12;   // partial sums a wave of sum_dropped_kernel parks in LDS before it writes them out
struct DescBatch {
    razor_head_desc d[kDescPerLaunch];
    int32_t sum_prefix[kDescPerLaunch];   // first partial-sum slot of each head (see compress_kernel)
};

// The table is tiny and known on the host; it travels as a kernel argument so that no
// host buffer has to outlive the call and no copy has to be waited for.  Together with it goes
// the running count of partial column sums the heads before each one own; entry n_heads of that
// list (the total) comes with the last batch.
__global__ void upload_desc_kernel(DescBatch batch, int first, int count, int total_after,
                                   razor_head_desc *desc, int32_t *sum_prefix)
{
    int t = threadIdx.x;
    if (t < count) {
        desc[first + t] = batch.d[t];
        if (sum_prefix) sum_prefix[first + t] = batch.sum_prefix[t];
    }
    if (t == 0 && sum_prefix && total_after >= 0) sum_prefix[first + count] = total_after;
}

// Source rows are read exactly once: non-temporal loads.
__device__ __forceinline__ uint4 stream_load16(const char *p)
{
    const u32x4 v = stream_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
}

// The arena rows written here are next read by the first decode step, long after they have left
// the caches: store them non-temporally (measured on a plain copy: 6.2 against 5.7 TB/s).
__device__ __forceinline__ void stream_store16(char *p, const uint4 v)
{
    __builtin_nontemporal_store(u32x4{v.x, v.y, v.z, v.w}, reinterpret_cast<u32x4 *>(p));
}

// Adds the elements of one 16-byte piece to acc[0..NE).
template <int DTYPE>
__device__ __forceinline__ void accumulate_piece(const uint4 &v, float *acc)
{
    if constexpr (DTYPE == RAZOR_F32) {
        acc[0] += __uint_as_float(v.x);
        acc[1] += __uint_as_float(v.y);
        acc[2] += __uint_as_float(v.z);
        acc[3] += __uint_as_float(v.w);
    } else {   // bf16 pair per dword: low half shifted up, high half masked
        acc[0] += __uint_as_float(v.x << 16);
        acc[1] += __uint_as_float(v.x & 0xffff0000u);
        acc[2] += __uint_as_float(v.y << 16);
        acc[3] += __uint_as_float(v.y & 0xffff0000u);
        acc[4] += __uint_as_float(v.z << 16);
        acc[5] += __uint_as_float(v.z & 0xffff0000u);
        acc[6] += __uint_as_float(v.w << 16);
        acc[7] += __uint_as_float(v.w & 0xffff0000u);
    }
}

// One wavefront adds up source rows: lane (prow, piece) owns the 16-byte piece `piece` of rows
// prow, prow + RPI, ... of every 16-row block and keeps fp32 column sums of K and of V.
//   run     streams blocks [t0, t1) of a row set (row idx of the set = source row first_row +
//           idx, idx < n_rows), two blocks in flight, fixed order
//   reduce  adds the row groups with shuffles: afterwards the lanes with prow == 0 hold the
//           sums of their piece's columns
template <int DTYPE, int D>
struct RowSummer {
    static constexpr int ES = DTYPE == RAZOR_F32 ? 4 : 2;
    static constexpr int NE = 16 / ES;        // elements per piece
    static constexpr int LPR = D * ES / 16;   // lanes per row
    static constexpr int RPI = 64 / LPR;      // rows one wave-wide load covers
    static constexpr int NI = kBlockRows / RPI;
    float ak[NE], av[NE];

    __device__ __forceinline__ RowSummer() { clear(); }
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int c = 0; c < NE; ++c) ak[c] = av[c] = 0.f;
    }
    // Issues the loads of block t of the row set and nothing else: no loaded value is used here, so
    // nothing waits before all of them are on their way.  Rows past n_rows (only a set's last block
    // has any) re-read the last row; add_block leaves them out.
    static __device__ __forceinline__ void load_block(const char *__restrict__ K, const char *__restrict__ V,
                                                      int64_t base, int64_t row_bytes, int64_t first_row, int n_rows,
                                                      int t, int prow, uint4 (&k)[NI], uint4 (&v)[NI])
    {
#pragma unroll
        for (int r = 0; r < NI; ++r) {
            const int idx = t * kBlockRows + r * RPI + prow;
            const int64_t row = first_row + (idx < n_rows ? idx : n_rows - 1);
            k[r] = stream_load16(K + base + row * row_bytes);
            v[r] = stream_load16(V + base + row * row_bytes);
        }
    }
    // n_valid: rows of the block that belong to the set (>= 16 for every block but the last)
    __device__ __forceinline__ void add_block(const uint4 (&k)[NI], const uint4 (&v)[NI], int n_valid, int prow)
    {
#pragma unroll
        for (int r = 0; r < NI; ++r) {
            if (r * RPI + prow < n_valid) {
                accumulate_piece<DTYPE>(k[r], ak);
                accumulate_piece<DTYPE>(v[r], av);
            }
        }
    }
    __device__ __forceinline__ void run(const char *__restrict__ K, const char *__restrict__ V, int64_t base,
                                        int64_t row_bytes, int64_t first_row, int n_rows, int t0, int t1, int prow)
    {
        uint4 kb[2][NI], vb[2][NI];
#pragma unroll
        for (int u = 0; u < 2; ++u)
            if (t0 + u < t1) load_block(K, V, base, row_bytes, first_row, n_rows, t0 + u, prow, kb[u], vb[u]);
        for (int t = t0; t < t1; t += 2) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                if (t + u < t1) {
                    add_block(kb[u], vb[u], n_rows - (t + u) * kBlockRows, prow);
                    if (t + u + 2 < t1)
                        load_block(K, V, base, row_bytes, first_row, n_rows, t + u + 2, prow, kb[u], vb[u]);
                }
            }
        }
    }
    // the lanes with prow == 0 store the column sums of their piece (call reduce() first)
    __device__ __forceinline__ void store(float *__restrict__ dst, int piece) const
    {
#pragma unroll
        for (int c = 0; c < NE; ++c) {
            dst[piece * NE + c] = ak[c];
            dst[D + piece * NE + c] = av[c];
        }
    }
    __device__ __forceinline__ void reduce()
    {
#pragma unroll
        for (int c = 0; c < NE; ++c) {
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) {
                ak[c] += __shfl_xor(ak[c], o);
                av[c] += __shfl_xor(av[c], o);
            }
        }
    }
};

// Column sums of every row of every head (razor_column_sums, the stand-in for a prefill
// epilogue), first level.  The rows form one axis of 16-row blocks, cut into equal ranges, one
// per wavefront (same scheme as the decode kernel); a wave streams its rows once and stores
// one partial sum per head segment into slot wave + head.  Fixed order throughout.
template <int DTYPE, int D, class ROWS>
__global__ __launch_bounds__(256) void mean_stream_kernel(
    const char *__restrict__ K, const char *__restrict__ V, int64_t stride_b, int64_t stride_h,
    int64_t stride_n, const razor_head_desc *__restrict__ desc, int n_heads, int n_kv_heads,
    int n_sink, int n_workers, int32_t *__restrict__ prefix, float *__restrict__ partial)
{
    using Summer = RowSummer<DTYPE, D>;
    constexpr int ES = Summer::ES, NE = Summer::NE, LPR = Summer::LPR;
    const int lane = threadIdx.x & 63;
    const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int prow = lane / LPR, piece = lane % LPR;
    const RowSetBlocks<ROWS> count;
    int total, per, lo, hi, i, first;
    plan_range(count, desc, n_heads, n_workers, w, lane, total, per, lo, hi, i, first);
    if (w == 0) write_prefix(count, desc, n_heads, lane, per, prefix);
    if (lo >= hi) return;

    while (lo < hi) {
        razor_head_desc e = desc[i];
        while (first + (ROWS::n(e.rows, e.n_dropped) + kBlockRows - 1) / kBlockRows <= lo) {
            first += (ROWS::n(e.rows, e.n_dropped) + kBlockRows - 1) / kBlockRows;
            e = desc[++i];
        }
        const int n_rows = ROWS::n(e.rows, e.n_dropped);
        const int head_end = first + (n_rows + kBlockRows - 1) / kBlockRows;
        const int seg_end = hi < head_end ? hi : head_end;
        const int b = i / n_kv_heads, h = i % n_kv_heads;
        const int64_t base = (b * stride_b + h * stride_h) * ES + piece * 16;

        Summer sum;
        sum.run(K, V, base, stride_n * ES, ROWS::row(0, e.rows, e.n_dropped, n_sink), n_rows, lo - first,
                seg_end - first, prow);
        sum.reduce();
        if (prow == 0) {
            float *dst = partial + (size_t)(w + i) * 2 * D + piece * NE;
#pragma unroll
            for (int c = 0; c < NE; ++c) {
                dst[c] = sum.ak[c];
                dst[D + c] = sum.av[c];
            }
        }
        lo = seg_end;
    }
}

// Second level of razor_column_sums: add the segment sums of a head (four interleaved groups,
// each in slot order, then the groups in order; double keeps the result independent of how the
// rows were cut).  blockDim = (2 * D, 4).
template <int D, class ROWS>
__global__ void segment_sum_kernel(const razor_head_desc *__restrict__ desc, int n_heads,
                                   const int32_t *__restrict__ prefix,
                                   const float *__restrict__ partial, float *__restrict__ sums)
{
    __shared__ double red[4][2 * D];
    const int head = blockIdx.x, t = threadIdx.x, grp = threadIdx.y;
    const razor_head_desc e = desc[head];
    double s = 0.0;
    if (ROWS::n(e.rows, e.n_dropped) > 0) {
        const int first = prefix[head], last = prefix[head + 1], per = prefix[n_heads + 1];
        const int w0 = first / per, n_slots = (last - 1) / per - w0 + 1;
        for (int k = grp; k < n_slots; k += 4)
            s += (double)partial[(size_t)(w0 + k + head) * 2 * D + t];
    }
    red[grp][t] = s;
    __syncthreads();
    if (grp == 0) sums[(size_t)head * 2 * D + t] = (float)(((red[0][t] + red[1][t]) + red[2][t]) + red[3][t]);
}

// Eq.(4), first level, for up to 64 * TILES heads.  The dropped rows of all heads form one axis of
// 16-row blocks.  That axis is cut into n_workers * chunks_per_worker chunks of (nearly) equal
// length -- chunk c covers blocks [c T / M, (c + 1) T / M), T blocks in all, M chunks -- and
// wavefront w streams chunks w, w + n_workers, w + 2 n_workers, ...: every wave moves the same
// number of bytes to within one block per chunk, one wave per SIMD keeps the memory system at its
// best streaming rate, and at any moment the whole chip reads inside one moving window of the
// source.  The last point matters right after a prefill: the last 256 MB that were written are
// still dirty in the memory-side cache, reading them forces their write-back, and they come back
// about a quarter slower (non-temporal traffic in between does not displace them; plain loads of
// other data do).  With one contiguous range per wave the waves that own such rows finish last
// (measured 278 us instead of 197 us for the sums of the 128K benchmark layer); interleaved, the
// inherited write-back costs every wave the same little (about 225 us).
// Two blocks stay in flight across chunk and head boundaries.  The head table is held in
// registers (one entry per lane and tile), so finding the head of a block is a few ballots.
// A chunk's rows of head i go to partial sum c + i (unique, ascending inside a head).
template <int DTYPE, int D, int TILES, bool ARGS>   // ARGS: the table comes with the launch (batch), not from memory
__global__ __launch_bounds__(256) void sum_dropped_kernel(
    const char *__restrict__ K, const char *__restrict__ V, int64_t stride_b_bytes, int64_t stride_h_bytes,
    int64_t stride_n_bytes, const DescBatch batch, const razor_head_desc *__restrict__ desc, int n_heads,
    int n_kv_heads, int n_sink, int n_workers, int chunks_per_worker, int32_t *__restrict__ prefix,
    float *__restrict__ partial)
{
    static_assert(!ARGS || TILES == 1, "a launch carries at most 64 table entries");
    using Summer = RowSummer<DTYPE, D>;
    constexpr int LPR = Summer::LPR, NI = Summer::NI;
    const int lane = threadIdx.x & 63;
    const int w = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: so is all that follows from it
    const int prow = lane / LPR, piece = lane % LPR;

    // dropped blocks of every head: end[t] = flattened end of head 64 t + lane, nd[t] = its N_d
    int end[TILES], nd[TILES], carry = 0;
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
        const int idx = t * 64 + lane;
        if constexpr (ARGS) nd[t] = idx < n_heads ? batch.d[idx].n_dropped : 0;
        else nd[t] = idx < n_heads ? desc_counts(desc, idx).z : 0;
        end[t] = carry + wave_inclusive_scan((nd[t] + kBlockRows - 1) / kBlockRows, lane);
        carry = __shfl(end[t], 63);
    }
    const int64_t T = carry, M = (int64_t)n_workers * chunks_per_worker;
    if (w == 0) {   // what the second level needs to find a head's partial sums
#pragma unroll
        for (int t = 0; t < TILES; ++t)
            if (t * 64 + lane < n_heads) prefix[t * 64 + lane + 1] = end[t];
        if (lane == 0) {
            prefix[0] = 0;
            prefix[n_heads + 1] = (int32_t)M;
        }
    }
    if (w >= n_workers) return;   // the last workgroup may hold waves beyond the count
    auto pick = [&](const int (&arr)[TILES], int idx) {   // arr of head idx (idx is wave-uniform)
        int r = 0;
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            const int v = __builtin_amdgcn_readlane(arr[t], idx & 63);
            r = (idx >> 6) == t ? v : r;
        }
        return r;
    };

    // the wave's blocks in order: chunk ordinal j, block g of the axis, hi = end of the chunk.  The
    // chunk bounds floor(c T / M) and floor((c + 1) T / M) are carried as quotient and remainder and
    // advanced by n_workers chunks at a time with additions only (a 64-bit division per chunk costs
    // a wave about a microsecond).
    const int64_t step_q = (int64_t)n_workers * T / M, step_r = (int64_t)n_workers * T % M;
    int64_t lo_q = (int64_t)w * T / M, lo_r = (int64_t)w * T % M;             // chunk w
    int64_t hi_q = ((int64_t)w + 1) * T / M, hi_r = ((int64_t)w + 1) * T % M;
    int j = -1;
    int64_t g = 0, hi = 0;
    auto next_block = [&]() -> bool {   // moves to the next block; false when the wave is done
        ++g;
        while (g >= hi) {
            if (++j >= chunks_per_worker) return false;
            g = lo_q;
            hi = hi_q;
            lo_q += step_q; lo_r += step_r;
            if (lo_r >= M) { lo_r -= M; ++lo_q; }
            hi_q += step_q; hi_r += step_r;
            if (hi_r >= M) { hi_r -= M; ++hi_q; }
        }
        return true;
    };
    struct Meta { bool valid; int slot, n_valid; };
    Meta meta[2];
    uint4 kb[2][NI], vb[2][NI];
    bool more = T > 0;
    g = -1;
    // the head that owns block g: looked up only when g leaves the blocks [h_first, h_end) of the last one
    int head = 0, h_first = 0, h_end = 0, h_rows = 0;
    int64_t h_base = 0;
    auto fetch = [&](Meta &m, uint4(&k)[NI], uint4(&v)[NI]) {
        more = more && next_block();
        m.valid = more;
        if (!more) return;
        if (g >= h_end) {   // blocks only move forward
            head = 0;
#pragma unroll
            for (int t = 0; t < TILES; ++t) head += __popcll(__ballot(end[t] <= (int)g));
            head = __builtin_amdgcn_readfirstlane(head);
            h_first = head == 0 ? 0 : pick(end, head - 1);
            h_end = pick(end, head);
            h_rows = pick(nd, head);
            h_base = (int64_t)(head / n_kv_heads) * stride_b_bytes + (int64_t)(head % n_kv_heads) * stride_h_bytes +
                     piece * 16;
        }
        Summer::load_block(K, V, h_base, stride_n_bytes, n_sink, h_rows, (int)g - h_first, prow, k, v);
        m.slot = (int)(w + (int64_t)j * n_workers) + head;
        m.n_valid = h_rows - ((int)g - h_first) * kBlockRows;
    };
    fetch(meta[0], kb[0], vb[0]);
    fetch(meta[1], kb[1], vb[1]);

    // Partial sums wait in LDS until the wave has issued its last load: a store in the middle of the
    // stream sits in the same in-order counter as the loads behind it, so the wave would wait for
    // its write acknowledgement before it could use those loads (measured: 2 us per chunk).
    __shared__ float staged[4][kStagedSums][2 * D];
    __shared__ int staged_slot[4][kStagedSums];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int n_staged = 0;
    auto drain = [&]() {   // LDS -> partial sums, 16 bytes per lane and step
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        for (int i = 0; i < n_staged; ++i) {
            float *dst = partial + (size_t)staged_slot[wave][i] * 2 * D;
            for (int c = lane * 4; c < 2 * D; c += 256)
                *reinterpret_cast<float4 *>(dst + c) = *reinterpret_cast<const float4 *>(&staged[wave][i][c]);
        }
        __builtin_amdgcn_wave_barrier();
        n_staged = 0;
    };
    Summer sum;
    int open_slot = -1;
    auto flush = [&]() {
        sum.reduce();
        if (n_staged == kStagedSums) drain();
        if (prow == 0) sum.store(staged[wave][n_staged], piece);
        if (lane == 0) staged_slot[wave][n_staged] = open_slot;
        ++n_staged;
        sum.clear();
    };
    while (meta[0].valid) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (meta[u].valid) {
                if (meta[u].slot != open_slot) {
                    if (open_slot >= 0) flush();
                    open_slot = meta[u].slot;
                }
                sum.add_block(kb[u], vb[u], meta[u].n_valid, prow);
                fetch(meta[u], kb[u], vb[u]);
            }
        }
    }
    if (open_slot >= 0) flush();
    drain();
}

// Cache row t of a head sits at source position t (sinks, or nothing dropped) or
// t + n_dropped (window part).
__device__ __forceinline__ int64_t source_row(int t, const razor_head_desc &e, int n_sink)
{
    return (e.n_dropped > 0 && t >= n_sink) ? (int64_t)t + e.n_dropped : (int64_t)t;
}

// What the compression kernel adds up besides moving rows.
enum {
    kSumNothing = 0,   // nothing was dropped anywhere
    kSumDropped = 1,   // Eq.(4) as it stands: the dropped rows of every head
    kSumKept = 2,      // the caller brought column sums over all rows: the kept rows (complement)
    kSumStreamed = 3   // second level only: the dropped rows were added up by sum_dropped_kernel
};

// Eq.(4), second level: add the partial sums of a head (interleaved chains, each in index
// order, then the chains in order, in double) and divide by N_d.  Called by a whole workgroup.
//   kSumDropped  comp = sum / N_d               (the partial sums cover the dropped rows)
//   kSumKept     comp = (col_sums - sum) / N_d  (they cover the kept rows: Eq.(4) by complement)
//   kSumStreamed like kSumDropped, the partial sums being those of sum_dropped_kernel: sum_prefix
//                then holds the heads' dropped-block prefix and the number of chunks M, and head i
//                owns the slots c + i of the chunks c that overlap its blocks
//   kSumNothing  comp = 0
// comp_lo (sliding mode: low-order parts of the running means) starts at zero.
template <int D, int MODE>
__device__ __forceinline__ void finalize_head(const razor_head_desc &e, int head, int n_heads,
                                              const int32_t *__restrict__ sum_prefix,
                                              const float *__restrict__ sums, const float *__restrict__ col_sums,
                                              float *__restrict__ comp, float *__restrict__ comp_lo,
                                              double *red, int t, int n_threads)
{
    // the workgroup's threads: 2 D columns x (n_threads / 2 D) chains; chain c adds the partial sums
    // first + c, first + c + chains, ... in that order, eight loads at a time
    constexpr int COLS = 2 * D;
    const int chains = n_threads / COLS, col = t % COLS, grp = t / COLS;
    double s = 0.0;
    if constexpr (MODE != kSumNothing) {
        int first = sum_prefix[head], last = sum_prefix[head + 1];
        if constexpr (MODE == kSumStreamed) {
            // blocks [lo, hi) of the axis; chunk of block g: the largest c with c T / M <= g
            const int64_t lo = first, hi = last, T = sum_prefix[n_heads], M = sum_prefix[n_heads + 1];
            first = hi > lo ? (int)(((lo + 1) * M - 1) / T) + head : 0;
            last = hi > lo ? (int)((hi * M - 1) / T) + head + 1 : 0;
        }
        int k = first + grp;
        for (; k + 7 * chains < last; k += 8 * chains) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = sums[(size_t)(k + chains * u) * COLS + col];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += (double)v[u];
        }
        for (; k < last; k += chains) s += (double)sums[(size_t)k * COLS + col];
    }
    red[t] = s;
    __syncthreads();
    if (grp == 0) {
        double sum = red[col];
        for (int c = 1; c < chains; ++c) sum += red[c * COLS + col];
        float out = 0.f;
        if ((MODE == kSumDropped || MODE == kSumStreamed) && e.n_dropped > 0) out = (float)(sum / (double)e.n_dropped);
        if (MODE == kSumKept && e.n_dropped > 0)
            out = (float)(((double)col_sums[(size_t)head * COLS + col] - sum) / (double)e.n_dropped);
        comp[(size_t)head * COLS + col] = out;
        if (comp_lo) comp_lo[(size_t)head * COLS + col] = 0.f;
    }
}

// The second level as a launch of its own (the partial sums come from the launch before it).
constexpr int kFinalThreads = 1024;
template <int D, int MODE>
__global__ __launch_bounds__(kFinalThreads) void mean_final_kernel(
    const razor_head_desc *__restrict__ desc, int n_heads, const int32_t *__restrict__ sum_prefix,
    const float *__restrict__ sums, const float *__restrict__ col_sums, float *__restrict__ comp,
    float *__restrict__ comp_lo)
{
    __shared__ double red[kFinalThreads];
    finalize_head<D, MODE>(desc[blockIdx.x], (int)blockIdx.x, n_heads, sum_prefix, sums, col_sums, comp, comp_lo,
                           red, (int)threadIdx.x, kFinalThreads);
}

// The whole pass over the source cache in one launch (Algorithm 1 steps 3-4): every valid source
// row is read once.  Workgroup (x, head) is one of two kinds.
//
//   sum   (kSumDropped, x < chunks of the head)  adds up kSumBlocks 16-row blocks of the head's
//         dropped rows, four per wavefront: fp32 column sums per lane, row groups by shuffles,
//         the four waves in order through LDS; one partial sum per workgroup (Eq.(4), first level).
//   copy  moves four 16-row destination blocks of the head, one per wavefront: V rows are copied
//         as they are; K rows are read row-major (coalesced), staged in wave-private LDS and
//         written back piece-major, the layout the decode kernel loads straight into matrix-core
//         operands.  Rows past `rows` inside a head's last block are written as zeros.  With
//         kSumKept a head that dropped rows also gets the column sums of its kept rows, which
//         this workgroup holds in registers anyway: one partial sum per workgroup.
//
// A head's sum workgroups come first, so its source rows are visited in address order; the
// partial sums of head i are slots sum_prefix[i] .. sum_prefix[i + 1] - 1.  Workgroups are small
// and handed out in (x, head) order as earlier ones retire: at any moment the chip works inside
// one moving window of each plane (measured 15 % faster for read + write traffic than a private
// contiguous range per wave), and rows that cost more to fetch -- the last 256 MB a prefill
// kernel wrote are still dirty in the memory-side cache; reading them forces their write-back
// and they come back a quarter slower -- delay only the workgroups that meet them instead of
// becoming the tail of a statically cut launch.
//
// FINAL >= 0 (a final mode of finalize_head; the partial sums it needs are complete before this
// launch): the second level of Eq.(4) rides along.  The grid has one more row, dispatched first;
// workgroup (x, 0) finishes head x while the others copy, so neither a launch nor its few
// microseconds of latency-bound additions are left on the critical path.  ARGS (with FINAL; at most
// 64 heads): the table comes with the launch instead of from memory, and those workgroups also
// store it for the decode calls to come -- no launch for the table either.
template <int RB, int DTYPE, int MODE, int FINAL, bool ARGS>   // RB: bytes per row
__global__ __launch_bounds__(256) void compress_kernel(
    const char *__restrict__ K, const char *__restrict__ V, int64_t stride_b_bytes,
    int64_t stride_h_bytes, int64_t stride_n_bytes, const DescBatch batch, razor_head_desc *__restrict__ desc,
    int n_heads, int n_kv_heads, int n_sink, char *__restrict__ arena, const int32_t *__restrict__ sum_prefix,
    float *__restrict__ sums, float *__restrict__ comp, float *__restrict__ comp_lo)
{
    constexpr int ES = DTYPE == RAZOR_F32 ? 4 : 2;
    constexpr int D = RB / ES;
    using Summer = RowSummer<DTYPE, D>;
    constexpr int LPR = Summer::LPR, RPI = Summer::RPI, NI = Summer::NI, NE = Summer::NE;
    static_assert(!ARGS || FINAL >= 0, "the table is stored by the workgroups that finish the means");
    static_assert(2 * D <= 256, "finalize_head needs a thread per column");
    __shared__ uint4 stage[4][kBlockRows * LPR];
    __shared__ float wave_sums[MODE != kSumNothing ? 4 : 1][MODE != kSumNothing ? 2 * D : 1];
    __shared__ double red[FINAL >= 0 ? 256 : 1];
    int head = blockIdx.y;
    if constexpr (FINAL >= 0) {
        if (head == 0) {   // the row that finishes Eq.(4): one workgroup per head
            const int hd = blockIdx.x;
            if (hd >= n_heads) return;
            razor_head_desc entry;
            if constexpr (ARGS) {
                entry = batch.d[hd];
                if (threadIdx.x == 0) desc[hd] = entry;
            } else {
                entry = desc[hd];
            }
            finalize_head<D, FINAL>(entry, hd, n_heads, sum_prefix, sums, nullptr, comp, comp_lo, red,
                                    (int)threadIdx.x, 256);
            return;
        }
        head -= 1;
    }
    razor_head_desc e;
    if constexpr (ARGS) e = batch.d[head];
    else e = desc[head];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int prow = lane / LPR, piece = lane % LPR;
    const int b = head / n_kv_heads, h = head % n_kv_heads;
    const int64_t src_base = b * stride_b_bytes + h * stride_h_bytes + piece * 16;
    const int n_blocks = (e.rows + kBlockRows - 1) / kBlockRows;
    int x = blockIdx.x;

    // stores the workgroup's sum (its four waves in order) as partial sum `slot`
    auto store_partial = [&](Summer &sum, int slot) {
        if constexpr (MODE != kSumNothing) {
            sum.reduce();
            if (prow == 0) {
#pragma unroll
                for (int c = 0; c < NE; ++c) {
                    wave_sums[wave][piece * NE + c] = sum.ak[c];
                    wave_sums[wave][D + piece * NE + c] = sum.av[c];
                }
            }
            __syncthreads();
            float *dst = sums + (size_t)slot * 2 * D;
            for (int t = threadIdx.x; t < 2 * D; t += 256)
                dst[t] = ((wave_sums[0][t] + wave_sums[1][t]) + wave_sums[2][t]) + wave_sums[3][t];
        }
    };

    if constexpr (MODE == kSumDropped) {
        const int d_blocks = (e.n_dropped + kBlockRows - 1) / kBlockRows;
        const int chunks = (d_blocks + kSumBlocks - 1) / kSumBlocks;
        if (x < chunks) {
            constexpr int kPerWave = kSumBlocks / 4;
            const int t0 = x * kSumBlocks + wave * kPerWave;
            const int t1 = t0 + kPerWave < d_blocks ? t0 + kPerWave : d_blocks;
            Summer sum;
            sum.run(K, V, src_base, stride_n_bytes, n_sink, e.n_dropped, t0, t1, prow);   // empty when t0 >= t1
            store_partial(sum, sum_prefix[head] + x);
            return;
        }
        x -= chunks;
    }

    const int blk = x * kGroupBlocks + wave;
    const bool summing = MODE == kSumKept && e.n_dropped > 0;
    // the copy is wave-private work; only a summing workgroup meets at a barrier, so its idle
    // waves stay until then
    if (x * kGroupBlocks >= n_blocks || (!summing && blk >= n_blocks)) return;
    Summer sum;
    if (blk < n_blocks) {
        char *kplane = arena + e.row_off * 2 * RB;
        char *vplane = kplane + (int64_t)e.cap * RB;

        uint4 kv[NI], vv[NI];
#pragma unroll
        for (int r = 0; r < NI; ++r) {   // loads only: nothing waits before all of them are issued
            const int t = blk * kBlockRows + r * RPI + prow;   // cache row
            const int64_t off = src_base + source_row(t < e.rows ? t : e.rows - 1, e, n_sink) * stride_n_bytes;
            kv[r] = stream_load16(K + off);
            vv[r] = stream_load16(V + off);
        }
#pragma unroll
        for (int r = 0; r < NI; ++r)
            if (blk * kBlockRows + r * RPI + prow >= e.rows) kv[r] = vv[r] = make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < NI; ++r) {
            const int row = r * RPI + prow;
            stream_store16(vplane + (int64_t)(blk * kBlockRows + row) * RB + piece * 16, vv[r]);
            stage[wave][row * LPR + (piece ^ (row % LPR))] = kv[r];   // xor: conflict-free column reads
            if (summing) {
                accumulate_piece<DTYPE>(kv[r], sum.ak);
                accumulate_piece<DTYPE>(vv[r], sum.av);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        char *kblock = kplane + (int64_t)blk * kBlockRows * RB;
#pragma unroll
        for (int s = 0; s < NI; ++s) {
            const int pos = s * 64 + lane;                // 16-byte slot inside the block
            const int c = pos / 16, r = pos % 16;         // piece-major: slot = c * 16 + r
            stream_store16(kblock + (int64_t)pos * 16, stage[wave][r * LPR + (c ^ (r % LPR))]);
        }
    }
    if constexpr (MODE == kSumKept) {
        if (summing) store_partial(sum, sum_prefix[head] + x);   // uniform over the workgroup
    }
}

__global__ void kept_index_kernel(const razor_head_desc *__restrict__ desc, int n_sink,
                                  int32_t *__restrict__ kept_idx)
{
    const razor_head_desc e = desc[blockIdx.y];
    for (int t = blockIdx.x * blockDim.x + threadIdx.x; t < e.rows; t += gridDim.x * blockDim.x)
        kept_idx[e.kept_off + t] = (int32_t)source_row(t, e, n_sink);
}

#define RAZOR_HIP_CHECK(expr)                                              \
    do {                                                                   \
        hipError_t err__ = (expr);                                         \
        if (err__ != hipSuccess) return hip_failure(#expr, (int)err__);    \
    } while (0)

// Copy workgroups / summing workgroups a head needs in compress_kernel.
inline int copy_groups(const razor_head_desc &e)
{
    return ((e.rows + kBlockRows - 1) / kBlockRows + kGroupBlocks - 1) / kGroupBlocks;
}
inline int sum_chunks(const razor_head_desc &e)
{
    return ((e.n_dropped + kBlockRows - 1) / kBlockRows + kSumBlocks - 1) / kSumBlocks;
}

// One batch of the table (entries first .. first + 63) with, for `mode`, the partial-sum slots
// every head owns; `running` carries the slot count across batches.
DescBatch make_batch(const std::vector<razor_head_desc> &desc, int first, int mode, int32_t &running)
{
    DescBatch batch;
    const int count = std::min(kDescPerLaunch, (int)desc.size() - first);
    for (int i = 0; i < kDescPerLaunch; ++i) {
        batch.d[i] = i < count ? desc[(size_t)first + i] : razor_head_desc{};
        batch.sum_prefix[i] = running;
        if (i < count && batch.d[i].n_dropped > 0)
            running += mode == kSumDropped ? sum_chunks(batch.d[i]) : mode == kSumKept ? copy_groups(batch.d[i]) : 0;
    }
    return batch;
}

// Sends the table (and, with `mode`, the partial-sum slots every head owns) to the device.
void upload_table(const std::vector<razor_head_desc> &desc, int mode, razor_head_desc *desc_dev,
                  int32_t *sum_prefix, hipStream_t stream)
{
    const int n_heads = (int)desc.size();
    int32_t running = 0;
    for (int first = 0; first < n_heads; first += kDescPerLaunch) {
        const DescBatch batch = make_batch(desc, first, mode, running);
        const int count = std::min(kDescPerLaunch, n_heads - first);
        hipLaunchKernelGGL(upload_desc_kernel, dim3(1), dim3(kDescPerLaunch), 0, stream, batch, first, count,
                           first + count == n_heads ? running : -1, desc_dev,
                           mode == kSumNothing ? nullptr : sum_prefix);
    }
}

template <int DTYPE, int D>
int launch_compress(const razor_params &p, const char *K, const char *V, int64_t stride_b,
                    int64_t stride_h, int64_t stride_n, const std::vector<razor_head_desc> &desc,
                    int max_dropped, char *arena, float *comp, razor_head_desc *desc_dev,
                    int32_t *kept_idx_dev, const float *col_sums, int32_t *sum_prefix, float *sums,
                    int workers, hipStream_t stream)
{
    constexpr int ES = DTYPE == RAZOR_F32 ? 4 : 2;
    constexpr int RB = D * ES;
    const int n_heads = (int)desc.size();
    float *comp_lo = p.sliding ? comp + (size_t)n_heads * 2 * D : nullptr;
    const int mode = max_dropped == 0 ? kSumNothing : col_sums ? kSumKept : kSumDropped;
    // Eq.(4) as it stands, up to 256 heads: the dropped rows are streamed by persistent waves, the
    // copy is a launch of its own and finishes the means on the side; beyond that one launch of small
    // workgroups sums and copies.  Up to 64 heads the table travels with those launches.
    const bool streamed = mode == kSumDropped && n_heads <= 256;
    const bool folded = (streamed || mode == kSumNothing) && n_heads <= 256;
    const bool by_args = folded && n_heads <= kDescPerLaunch;
    int max_rows = 0, grid_x = 0;
    int64_t dropped_blocks = 0;
    for (const razor_head_desc &e : desc) {
        max_rows = std::max(max_rows, e.rows);
        grid_x = std::max(grid_x, copy_groups(e) + (mode == kSumDropped && !streamed ? sum_chunks(e) : 0));
        dropped_blocks += (e.n_dropped + kBlockRows - 1) / kBlockRows;
    }
    int32_t running = 0;
    const DescBatch batch = by_args ? make_batch(desc, 0, kSumNothing, running) : DescBatch{};
    if (!by_args) upload_table(desc, streamed ? kSumNothing : mode, desc_dev, sum_prefix, stream);

    const int64_t sb = stride_b * ES, sh = stride_h * ES, sn = stride_n * ES;
    if (streamed) {
        // chunks of about kSumBlocks blocks or more, never more chunks than that: their partial sums
        // (chunks + heads slots) then fit what razor_plan reserved
        const int w = (int)std::max<int64_t>(1, std::min<int64_t>(workers, dropped_blocks / kSumBlocks));
        const int per_worker = (int)std::max<int64_t>(1, std::min<int64_t>(dropped_blocks / ((int64_t)w * kSumBlocks), 64));
        const dim3 sgrid((w + 3) / 4);
#define RAZOR_SUM(TILES, ARGS)                                                                                 \
        hipLaunchKernelGGL((sum_dropped_kernel<DTYPE, D, TILES, ARGS>), sgrid, dim3(256), 0, stream, K, V, sb, sh, \
                           sn, batch, desc_dev, n_heads, p.n_kv_heads, p.n_sink, w, per_worker, sum_prefix, sums)
        if (by_args) RAZOR_SUM(1, true);
        else if (n_heads <= 64) RAZOR_SUM(1, false);
        else if (n_heads <= 128) RAZOR_SUM(2, false);
        else RAZOR_SUM(4, false);
#undef RAZOR_SUM
    }
    // the copy (with the sums it may have to take along), then the second level of Eq.(4) unless it rode along
#define RAZOR_COPY(MODE, FINAL, ARGS, GX, GY)                                                                  \
    hipLaunchKernelGGL((compress_kernel<RB, DTYPE, MODE, FINAL, ARGS>), dim3(GX, GY), dim3(256), RAZOR_LDS_PAD, \
                       stream, K, V, sb, sh, sn, batch, desc_dev, n_heads, p.n_kv_heads, p.n_sink, arena,      \
                       sum_prefix, sums, comp, comp_lo)
#define RAZOR_FINAL(FINAL)                                                                                     \
    hipLaunchKernelGGL((mean_final_kernel<D, FINAL>), dim3(n_heads), dim3(kFinalThreads), 0, stream, desc_dev, \
                       n_heads, sum_prefix, sums, col_sums, comp, comp_lo)
    if (folded) {
        const int gx = std::max(grid_x, n_heads), gy = n_heads + 1;   // row 0 finishes the means
        if (streamed && by_args) RAZOR_COPY(kSumNothing, kSumStreamed, true, gx, gy);
        else if (streamed) RAZOR_COPY(kSumNothing, kSumStreamed, false, gx, gy);
        else if (by_args) RAZOR_COPY(kSumNothing, kSumNothing, true, gx, gy);
        else RAZOR_COPY(kSumNothing, kSumNothing, false, gx, gy);
    } else if (mode == kSumDropped) {
        if (grid_x > 0) RAZOR_COPY(kSumDropped, -1, false, grid_x, n_heads);
        RAZOR_FINAL(kSumDropped);
    } else if (mode == kSumKept) {
        if (grid_x > 0) RAZOR_COPY(kSumKept, -1, false, grid_x, n_heads);
        RAZOR_FINAL(kSumKept);
    } else {
        if (grid_x > 0) RAZOR_COPY(kSumNothing, -1, false, grid_x, n_heads);
        RAZOR_FINAL(kSumNothing);
    }
#undef RAZOR_COPY
#undef RAZOR_FINAL
    if (kept_idx_dev && max_rows > 0) {
        const int gx = std::min((max_rows + 255) / 256, 64);
        hipLaunchKernelGGL(kept_index_kernel, dim3(gx, n_heads), dim3(256), 0, stream, desc_dev,
                           p.n_sink, kept_idx_dev);
    }
    RAZOR_HIP_CHECK(hipGetLastError());
    return RAZOR_OK;
}

template <int DTYPE, int D>
int launch_column_sums(const razor_params &p, const char *K, const char *V, int64_t stride_b,
                       int64_t stride_h, int64_t stride_n, const std::vector<razor_head_desc> &desc,
                       razor_head_desc *desc_dev, float *sums, int32_t *prefix, float *partial,
                       int workers, hipStream_t stream)
{
    const int n_heads = (int)desc.size();
    upload_table(desc, kSumNothing, desc_dev, nullptr, stream);
    hipLaunchKernelGGL((mean_stream_kernel<DTYPE, D, AllRows>), dim3((workers + 3) / 4), dim3(256), 0,
                       stream, K, V, stride_b, stride_h, stride_n, desc_dev, n_heads, p.n_kv_heads,
                       p.n_sink, workers, prefix, partial);
    hipLaunchKernelGGL((segment_sum_kernel<D, AllRows>), dim3(n_heads), dim3(2 * D, 4), 0, stream,
                       desc_dev, n_heads, prefix, partial, sums);
    RAZOR_HIP_CHECK(hipGetLastError());
    return RAZOR_OK;
}

// Wavefronts a pass over the source cache is split over.
int stream_workers(const razor_params *p, int *out)
{
    int workers = p->n_workers;
    if (workers == 0) {
        const int rc = auto_workers(&workers);
        if (rc != RAZOR_OK) return rc;
        // 128-byte rows: a wave has half the bytes in flight, two waves per SIMD make up for it
        // (column sums of a 2.1 GB cache: 415 us with one wave per SIMD)
        if (p->head_dim * elem_size(p->dtype) == 128) workers *= 2;
    }
    *out = std::max(4, std::min(workers, RAZOR_MAX_WORKERS));
    return RAZOR_OK;
}

// Shared argument checks of the two entry points that read the full cache.
int check_source(const razor_params *p, const void *K, const void *V, int64_t stride_b,
                 int64_t stride_h, int64_t stride_n)
{
    if (check_params(p) != RAZOR_OK) return RAZOR_EINVAL;
    if (!K || !V) return RAZOR_EINVAL;
    const int64_t align = 16 / elem_size(p->dtype);   // rows must start on 16-byte boundaries
    if (stride_n < p->head_dim || stride_n % align || stride_h % align || stride_b % align)
        return RAZOR_EINVAL;
    if (stride_b < 0 || stride_h < 0) return RAZOR_EINVAL;
    if (((uintptr_t)K | (uintptr_t)V) & 15) return RAZOR_EINVAL;
    return RAZOR_OK;
}

}  // namespace
}  // namespace razor

extern "C" int razor_column_sums(const razor_params *p, const void *K, const void *V,
                                 int64_t stride_b, int64_t stride_h, int64_t stride_n,
                                 const int32_t *seq_lens_host, float *col_sums, void *workspace,
                                 size_t workspace_bytes, void *stream)
{
    using namespace razor;
    if (check_source(p, K, V, stride_b, stride_h, stride_n) != RAZOR_OK) return RAZOR_EINVAL;
    if (!seq_lens_host || !col_sums || ((uintptr_t)col_sums & 15)) return RAZOR_EINVAL;
    // every head keeps everything: rows = seq_len, which is all AllRows needs from the table
    std::vector<uint8_t> all(p->n_kv_heads, 1);
    std::vector<razor_head_desc> desc;
    razor_sizes sizes;
    int max_dropped = 0;
    int rc = build_plan(*p, seq_lens_host, all.data(), desc, sizes, max_dropped);
    if (rc != RAZOR_OK) return rc;
    const CompressWorkspace ws = compress_workspace(*p);
    if (!workspace || workspace_bytes < ws.bytes)
        return capacity_failure("razor_column_sums: workspace smaller than razor_plan reported");
    int workers = 0;
    rc = stream_workers(p, &workers);
    if (rc != RAZOR_OK) return rc;
    char *wsb = static_cast<char *>(workspace);
    int32_t *prefix = reinterpret_cast<int32_t *>(wsb + ws.prefix_off);
    float *partial = reinterpret_cast<float *>(wsb + ws.partial_off);
    razor_head_desc *desc_dev = reinterpret_cast<razor_head_desc *>(wsb + ws.desc_off);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const char *k = static_cast<const char *>(K), *v = static_cast<const char *>(V);
#define RAZOR_DISPATCH(DT, DD)                                                                      \
    return launch_column_sums<DT, DD>(*p, k, v, stride_b, stride_h, stride_n, desc, desc_dev,       \
                                      col_sums, prefix, partial, workers, s)
    if (p->dtype == RAZOR_BF16 && p->head_dim == 128) RAZOR_DISPATCH(RAZOR_BF16, 128);
    if (p->dtype == RAZOR_BF16 && p->head_dim == 64) RAZOR_DISPATCH(RAZOR_BF16, 64);
    if (p->dtype == RAZOR_F32 && p->head_dim == 128) RAZOR_DISPATCH(RAZOR_F32, 128);
    if (p->dtype == RAZOR_F32 && p->head_dim == 64) RAZOR_DISPATCH(RAZOR_F32, 64);
#undef RAZOR_DISPATCH
    return RAZOR_EINVAL;
}

extern "C" int razor_compress(const razor_params *p, const void *K, const void *V,
                              int64_t stride_b, int64_t stride_h, int64_t stride_n,
                              const int32_t *seq_lens_host, const uint8_t *retrieval_mask_host,
                              void *arena, float *comp, razor_head_desc *desc_dev,
                              int32_t *kept_idx_dev, const float *col_sums, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    using namespace razor;
    if (check_source(p, K, V, stride_b, stride_h, stride_n) != RAZOR_OK) return RAZOR_EINVAL;
    if (!seq_lens_host || !retrieval_mask_host || !comp || !desc_dev) return RAZOR_EINVAL;
    if (((uintptr_t)arena | (uintptr_t)comp | (uintptr_t)col_sums | (uintptr_t)desc_dev | (uintptr_t)workspace) & 15)
        return RAZOR_EINVAL;
    if ((uintptr_t)kept_idx_dev & 3) return RAZOR_EINVAL;

    std::vector<razor_head_desc> desc;
    razor_sizes sizes;
    int max_dropped = 0;
    size_t sum_bytes = 0;   // partial column sums: behind the fixed part of the workspace
    int rc = build_plan(*p, seq_lens_host, retrieval_mask_host, desc, sizes, max_dropped, &sum_bytes);
    if (rc != RAZOR_OK) return rc;
    if (sizes.arena_bytes > 0 && !arena) return RAZOR_EINVAL;
    const CompressWorkspace ws = compress_workspace(*p);
    if (!workspace || workspace_bytes < ws.bytes + sum_bytes)
        return capacity_failure("razor_compress: workspace smaller than razor_plan reported");
    float *sums = reinterpret_cast<float *>(static_cast<char *>(workspace) + ws.bytes);

    hipStream_t s = static_cast<hipStream_t>(stream);
    const char *k = static_cast<const char *>(K), *v = static_cast<const char *>(V);
    char *a = static_cast<char *>(arena);
    int32_t *sum_prefix = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + ws.prefix_off);
    int workers = 0;
    rc = stream_workers(p, &workers);
    if (rc != RAZOR_OK) return rc;
#define RAZOR_DISPATCH(DT, DD)                                                                    \
    return launch_compress<DT, DD>(*p, k, v, stride_b, stride_h, stride_n, desc, max_dropped, a,  \
                                   comp, desc_dev, kept_idx_dev, col_sums, sum_prefix, sums, workers, s)
    if (p->dtype == RAZOR_BF16 && p->head_dim == 128) RAZOR_DISPATCH(RAZOR_BF16, 128);
    if (p->dtype == RAZOR_BF16 && p->head_dim == 64) RAZOR_DISPATCH(RAZOR_BF16, 64);
    if (p->dtype == RAZOR_F32 && p->head_dim == 128) RAZOR_DISPATCH(RAZOR_F32, 128);
    if (p->dtype == RAZOR_F32 && p->head_dim == 64) RAZOR_DISPATCH(RAZOR_F32, 64);
#undef RAZOR_DISPATCH
    return RAZOR_EINVAL;
}
