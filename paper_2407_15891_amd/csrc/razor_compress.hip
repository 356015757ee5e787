// razor_compress: prefill-time pass that turns a full K/V cache into the per-head
// heterogeneous cache (Algorithm 1 steps 1-4, Eq.(4)).  Three kinds of work:
//   mean   column sums of the dropped rows [n_sink, N - window) -> khat, vhat (fp32)
//   copy   kept rows (sinks + window, or everything) -> arena; K re-tiled through LDS
//   index  kept positions as int32 (optional)
// All of it is HBM streaming: every source row is read once, kept rows written once.
// Given the column sums over the whole sequence (razor_column_sums, or a prefill epilogue) the
// dropped rows are not read: the copy adds up the kept rows it moves and the mean is taken
// from the difference.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <vector>

#include "razor_device.h"
#include "razor_internal.h"

namespace razor {
namespace {

constexpr int kDescPerLaunch = 64;
struct DescBatch {
    razor_head_desc d[kDescPerLaunch];
};

// The table is tiny and known on the host; it travels as a kernel argument so that no
// host buffer has to outlive the call and no copy has to be waited for.
__global__ void upload_desc_kernel(DescBatch batch, int first, int count, razor_head_desc *desc)
{
    int t = threadIdx.x;
    if (t < count) desc[first + t] = batch.d[t];
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

// Eq.(4), first level.  The rows to be summed (ROWS: the dropped set of every head, or every
// row) form one axis of 16-row blocks, cut into
// equal ranges, one per wavefront (same scheme as the decode kernel).  A wave streams its
// rows once -- lane (prow, piece) owns one 16-byte piece of rows prow, prow + RPI, ... of
// every block -- keeps fp32 column sums of K and V, adds the row groups with shuffles and
// stores one partial sum per head segment into slot wave + head.  Fixed order throughout.
template <int DTYPE, int D, class ROWS>
__global__ __launch_bounds__(256) void mean_stream_kernel(
    const char *__restrict__ K, const char *__restrict__ V, int64_t stride_b, int64_t stride_h,
    int64_t stride_n, const razor_head_desc *__restrict__ desc, int n_heads, int n_kv_heads,
    int n_sink, int n_workers, int32_t *__restrict__ prefix, float *__restrict__ partial)
{
    constexpr int ES = DTYPE == RAZOR_F32 ? 4 : 2;
    constexpr int NE = 16 / ES;        // elements per piece
    constexpr int LPR = D * ES / 16;   // lanes per row
    constexpr int RPI = 64 / LPR;      // rows one wave-wide load covers
    constexpr int NI = kBlockRows / RPI;
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
        const int64_t row_bytes = stride_n * ES;

        float ak[NE], av[NE];
#pragma unroll
        for (int c = 0; c < NE; ++c) ak[c] = av[c] = 0.f;
        uint4 kb[2][NI], vb[2][NI];
        auto load_block = [&](int t, uint4(&k)[NI], uint4(&v)[NI]) {
#pragma unroll
            for (int r = 0; r < NI; ++r) {
                const int idx = t * kBlockRows + r * RPI + prow;
                const bool valid = idx < n_rows;
                const int64_t row = ROWS::row(valid ? idx : n_rows - 1, e.rows, e.n_dropped, n_sink);
                k[r] = stream_load16(K + base + row * row_bytes);
                v[r] = stream_load16(V + base + row * row_bytes);
                if (!valid) k[r] = v[r] = make_uint4(0, 0, 0, 0);   // +0.0 in either format
            }
        };
        auto add_block = [&](const uint4(&k)[NI], const uint4(&v)[NI]) {
#pragma unroll
            for (int r = 0; r < NI; ++r) {
                accumulate_piece<DTYPE>(k[r], ak);
                accumulate_piece<DTYPE>(v[r], av);
            }
        };
        const int t0 = lo - first, t1 = seg_end - first;
#pragma unroll
        for (int u = 0; u < 2; ++u)
            if (t0 + u < t1) load_block(t0 + u, kb[u], vb[u]);
        for (int t = t0; t < t1; t += 2) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                if (t + u < t1) {
                    add_block(kb[u], vb[u]);
                    if (t + u + 2 < t1) load_block(t + u + 2, kb[u], vb[u]);
                }
            }
        }
#pragma unroll
        for (int c = 0; c < NE; ++c) {
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) {
                ak[c] += __shfl_xor(ak[c], o);
                av[c] += __shfl_xor(av[c], o);
            }
        }
        if (prow == 0) {
            float *dst = partial + (size_t)(w + i) * 2 * D + piece * NE;
#pragma unroll
            for (int c = 0; c < NE; ++c) {
                dst[c] = ak[c];
                dst[D + c] = av[c];
            }
        }
        lo = seg_end;
    }
}

// Eq.(4), second level: add the segment sums of a head (four interleaved groups, each in
// slot order, then the groups in order; double keeps the result independent of how the rows
// were cut).  blockDim = (2 * D, 4).
//   kFinalMean  comp = sum / N_d   (the streamed rows were the dropped set)
//   kFinalSum   comp = sum         (plain column sums)
enum { kFinalMean = 0, kFinalSum = 2 };

template <int D, int MODE, class ROWS>
__global__ void mean_final_kernel(const razor_head_desc *__restrict__ desc, int n_heads,
                                  const int32_t *__restrict__ prefix,
                                  const float *__restrict__ partial, float *__restrict__ comp,
                                  float *__restrict__ comp_lo)
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
    if (grp == 0) {
        const double sum = ((red[0][t] + red[1][t]) + red[2][t]) + red[3][t];
        float out;
        if (MODE == kFinalSum) out = (float)sum;
        else if (e.n_dropped <= 0) out = 0.f;
        else out = (float)(sum / (double)e.n_dropped);
        comp[(size_t)head * 2 * D + t] = out;
        if (comp_lo) comp_lo[(size_t)head * 2 * D + t] = 0.f;   // low-order parts of the sliding-mode means
    }
}

// Cache row t of a head sits at source position t (sinks, or nothing dropped) or
// t + n_dropped (window part).
__device__ __forceinline__ int64_t source_row(int t, const razor_head_desc &e, int n_sink)
{
    return (e.n_dropped > 0 && t >= n_sink) ? (int64_t)t + e.n_dropped : (int64_t)t;
}

// Compaction (Algorithm 1 step 3).  Workgroup (x, head) moves four 16-row destination blocks
// of that head, one per wavefront: V rows are copied as they are; K rows are read row-major
// (coalesced), staged in wave-private LDS and written back piece-major, the layout the decode
// kernel loads straight into matrix-core operands.  Rows past `rows` inside a head's last
// block are written as zeros.  Workgroups are dispatched in (x, head) order, so at any moment
// the chip reads and writes one moving window of each plane: measured 15 % faster for this
// read + write traffic than giving every wave a private contiguous range.
//
// SUMS (razor_compress given column sums): a head that dropped rows also needs the column sums
// of its kept rows, and this kernel has them in registers anyway.  Each wave adds up its block,
// the workgroup adds its four waves in order through LDS and stores one partial sum; the
// workgroups of head i own the partial sums group_prefix[i] .. group_prefix[i + 1] - 1.
template <int RB, int DTYPE, bool SUMS>   // RB: bytes per row
__global__ __launch_bounds__(256) void compact_kernel(
    const char *__restrict__ K, const char *__restrict__ V, int64_t stride_b_bytes,
    int64_t stride_h_bytes, int64_t stride_n_bytes, const razor_head_desc *__restrict__ desc,
    int n_kv_heads, int n_sink, char *__restrict__ arena, const int32_t *__restrict__ group_prefix,
    float *__restrict__ group_sums)
{
    constexpr int LPR = RB / 16;       // 16-byte pieces per row
    constexpr int RPI = 64 / LPR;      // rows one wave-wide load covers
    constexpr int NI = kBlockRows / RPI;
    constexpr int ES = DTYPE == RAZOR_F32 ? 4 : 2;
    constexpr int NE = 16 / ES, D = RB / ES;
    __shared__ uint4 stage[4][kBlockRows * LPR];
    __shared__ float wave_sums[SUMS ? 4 : 1][SUMS ? 2 * D : 1];
    const int head = blockIdx.y;
    const razor_head_desc e = desc[head];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int blk = blockIdx.x * 4 + wave;
    const int n_blocks = (e.rows + kBlockRows - 1) / kBlockRows;
    const bool summing = SUMS && e.n_dropped > 0;
    // the copy is wave-private work; only a summing workgroup meets at a barrier, so its idle
    // waves stay until then
    if (blockIdx.x * 4 >= n_blocks || (!summing && blk >= n_blocks)) return;
    const int prow = lane / LPR, piece = lane % LPR;
    float ak[NE], av[NE];
#pragma unroll
    for (int c = 0; c < NE; ++c) ak[c] = av[c] = 0.f;

    if (blk < n_blocks) {
        const int b = head / n_kv_heads, h = head % n_kv_heads;
        const int64_t src_base = b * stride_b_bytes + h * stride_h_bytes + piece * 16;
        char *kplane = arena + e.row_off * 2 * RB;
        char *vplane = kplane + (int64_t)e.cap * RB;

        uint4 kv[NI], vv[NI];
#pragma unroll
        for (int r = 0; r < NI; ++r) {
            const int t = blk * kBlockRows + r * RPI + prow;   // cache row
            const bool valid = t < e.rows;
            const int64_t off = src_base + source_row(valid ? t : e.rows - 1, e, n_sink) * stride_n_bytes;
            kv[r] = stream_load16(K + off);
            vv[r] = stream_load16(V + off);
            if (!valid) kv[r] = vv[r] = make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < NI; ++r) {
            const int row = r * RPI + prow;
            stream_store16(vplane + (int64_t)(blk * kBlockRows + row) * RB + piece * 16, vv[r]);
            stage[wave][row * LPR + (piece ^ (row % LPR))] = kv[r];   // xor: conflict-free column reads
            if (summing) {
                accumulate_piece<DTYPE>(kv[r], ak);
                accumulate_piece<DTYPE>(vv[r], av);
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
    if constexpr (SUMS) {
        if (!summing) return;                             // uniform over the workgroup
#pragma unroll
        for (int c = 0; c < NE; ++c) {
#pragma unroll
            for (int o = LPR; o < 64; o <<= 1) {
                ak[c] += __shfl_xor(ak[c], o);
                av[c] += __shfl_xor(av[c], o);
            }
        }
        if (prow == 0) {
#pragma unroll
            for (int c = 0; c < NE; ++c) {
                wave_sums[wave][piece * NE + c] = ak[c];
                wave_sums[wave][D + piece * NE + c] = av[c];
            }
        }
        __syncthreads();
        float *dst = group_sums + (size_t)(group_prefix[head] + blockIdx.x) * 2 * D;
        for (int t = threadIdx.x; t < 2 * D; t += 256)
            dst[t] = ((wave_sums[0][t] + wave_sums[1][t]) + wave_sums[2][t]) + wave_sums[3][t];
    }
}

// Workgroups of the compaction kernel that hold kept rows of a head that dropped something.
struct KeptGroupsOfCompressedHeads {
    __device__ __forceinline__ int operator()(const razor_head_desc *__restrict__ desc, int idx) const
    {
        const int4 f = desc_counts(desc, idx);
        const int blocks = f.z > 0 ? (f.x + kBlockRows - 1) / kBlockRows : 0;
        return (blocks + kGroupBlocks - 1) / kGroupBlocks;
    }
};

__global__ __launch_bounds__(64) void group_prefix_kernel(const razor_head_desc *__restrict__ desc, int n_heads,
                                                          int32_t *__restrict__ prefix)
{
    write_prefix(KeptGroupsOfCompressedHeads{}, desc, n_heads, (int)threadIdx.x, 0, prefix);
}

// Eq.(4) by complement: comp = (col_sums - sum over the head's kept rows) / N_d, the kept rows
// given as the partial sums of the compaction kernel (four interleaved chains, each in index
// order, then the chains in order, in double).  blockDim = (2 * D, 4).
template <int D>
__global__ void complement_final_kernel(const razor_head_desc *__restrict__ desc,
                                        const int32_t *__restrict__ group_prefix,
                                        const float *__restrict__ group_sums,
                                        const float *__restrict__ col_sums, float *__restrict__ comp,
                                        float *__restrict__ comp_lo)
{
    __shared__ double red[4][2 * D];
    const int head = blockIdx.x, t = threadIdx.x, grp = threadIdx.y;
    const razor_head_desc e = desc[head];
    double s = 0.0;
    // chain grp takes the partial sums first + grp, first + grp + 4, ...; eight loads are issued
    // together, the additions keep their order
    const int first = group_prefix[head], last = group_prefix[head + 1];
    int k = first + grp;
    for (; k + 28 < last; k += 32) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = group_sums[(size_t)(k + 4 * u) * 2 * D + t];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += (double)v[u];
    }
    for (; k < last; k += 4) s += (double)group_sums[(size_t)k * 2 * D + t];
    red[grp][t] = s;
    __syncthreads();
    if (grp == 0) {
        const double kept = ((red[0][t] + red[1][t]) + red[2][t]) + red[3][t];
        comp[(size_t)head * 2 * D + t] =
            e.n_dropped > 0 ? (float)(((double)col_sums[(size_t)head * 2 * D + t] - kept) / (double)e.n_dropped) : 0.f;
        if (comp_lo) comp_lo[(size_t)head * 2 * D + t] = 0.f;
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

template <int DTYPE, int D>
int launch_compress(const razor_params &p, const char *K, const char *V, int64_t stride_b,
                    int64_t stride_h, int64_t stride_n, const std::vector<razor_head_desc> &desc,
                    int max_dropped, char *arena, float *comp, razor_head_desc *desc_dev,
                    int32_t *kept_idx_dev, const float *col_sums, int32_t *prefix, float *partial,
                    float *group_sums, int workers, hipStream_t stream)
{
    constexpr int ES = DTYPE == RAZOR_F32 ? 4 : 2;
    const int n_heads = (int)desc.size();
    float *comp_lo = p.sliding ? comp + (size_t)n_heads * 2 * D : nullptr;
    for (int first = 0; first < n_heads; first += kDescPerLaunch) {
        DescBatch batch;
        const int count = std::min(kDescPerLaunch, n_heads - first);
        for (int i = 0; i < count; ++i) batch.d[i] = desc[(size_t)first + i];
        for (int i = count; i < kDescPerLaunch; ++i) batch.d[i] = razor_head_desc{};
        hipLaunchKernelGGL(upload_desc_kernel, dim3(1), dim3(kDescPerLaunch), 0, stream, batch,
                           first, count, desc_dev);
    }
    int max_rows = 0;
    for (const razor_head_desc &e : desc) max_rows = std::max(max_rows, e.rows);
    const dim3 grid((workers + 3) / 4);
    if (max_dropped > 0 && !col_sums) {
        // Eq.(4) as it stands: stream the dropped rows
        hipLaunchKernelGGL((mean_stream_kernel<DTYPE, D, DroppedRows>), grid, dim3(256), 0, stream, K, V,
                           stride_b, stride_h, stride_n, desc_dev, n_heads, p.n_kv_heads, p.n_sink,
                           workers, prefix, partial);
        hipLaunchKernelGGL((mean_final_kernel<D, kFinalMean, DroppedRows>), dim3(n_heads), dim3(2 * D, 4), 0,
                           stream, desc_dev, n_heads, prefix, partial, comp, comp_lo);
    } else if (max_dropped == 0) {
        hipLaunchKernelGGL((mean_final_kernel<D, kFinalMean, DroppedRows>), dim3(n_heads), dim3(2 * D, 4), 0,
                           stream, desc_dev, n_heads, prefix, partial, comp, comp_lo);
    }
    const int groups = ((max_rows + kBlockRows - 1) / kBlockRows + kGroupBlocks - 1) / kGroupBlocks;
    if (max_dropped > 0 && col_sums) {
        // the caller already holds the column sums over the whole sequence (a prefill epilogue can
        // accumulate them for free): the dropped rows are not read at all; the compaction kernel
        // adds up the kept rows it moves anyway and Eq.(4) is taken as the complement
        hipLaunchKernelGGL(group_prefix_kernel, dim3(1), dim3(64), 0, stream, desc_dev, n_heads, prefix);
        if (max_rows > 0)   // no head keeps a row (no sinks, no window): comp = col_sums / N_d below
            hipLaunchKernelGGL((compact_kernel<D * ES, DTYPE, true>), dim3(groups, n_heads), dim3(256), 0, stream, K, V,
                               stride_b * ES, stride_h * ES, stride_n * ES, desc_dev, p.n_kv_heads, p.n_sink, arena,
                               prefix, group_sums);
        hipLaunchKernelGGL((complement_final_kernel<D>), dim3(n_heads), dim3(2 * D, 4), 0, stream, desc_dev,
                           prefix, group_sums, col_sums, comp, comp_lo);
    } else if (max_rows > 0) {
        hipLaunchKernelGGL((compact_kernel<D * ES, DTYPE, false>), dim3(groups, n_heads), dim3(256), 0, stream, K, V,
                           stride_b * ES, stride_h * ES, stride_n * ES, desc_dev, p.n_kv_heads, p.n_sink, arena,
                           nullptr, nullptr);
    }
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
    for (int first = 0; first < n_heads; first += kDescPerLaunch) {
        DescBatch batch;
        const int count = std::min(kDescPerLaunch, n_heads - first);
        for (int i = 0; i < count; ++i) batch.d[i] = desc[(size_t)first + i];
        for (int i = count; i < kDescPerLaunch; ++i) batch.d[i] = razor_head_desc{};
        hipLaunchKernelGGL(upload_desc_kernel, dim3(1), dim3(kDescPerLaunch), 0, stream, batch,
                           first, count, desc_dev);
    }
    hipLaunchKernelGGL((mean_stream_kernel<DTYPE, D, AllRows>), dim3((workers + 3) / 4), dim3(256), 0,
                       stream, K, V, stride_b, stride_h, stride_n, desc_dev, n_heads, p.n_kv_heads,
                       p.n_sink, workers, prefix, partial);
    hipLaunchKernelGGL((mean_final_kernel<D, kFinalSum, AllRows>), dim3(n_heads), dim3(2 * D, 4), 0, stream,
                       desc_dev, n_heads, prefix, partial, sums, nullptr);
    RAZOR_HIP_CHECK(hipGetLastError());
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
    int workers = p->n_workers;
    if (workers == 0) {
        rc = auto_workers(&workers);
        if (rc != RAZOR_OK) return rc;
        // 128-byte rows: a wave has half the bytes in flight, two waves per SIMD make up for it
        // (column sums of a 2.1 GB cache: 415 us with one wave per SIMD)
        if (p->head_dim * elem_size(p->dtype) == 128) workers *= 2;
    }
    workers = std::max(4, std::min(workers, RAZOR_MAX_WORKERS));
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
    size_t group_bytes = 0;
    int rc = build_plan(*p, seq_lens_host, retrieval_mask_host, desc, sizes, max_dropped, &group_bytes);
    if (rc != RAZOR_OK) return rc;
    if (sizes.arena_bytes > 0 && !arena) return RAZOR_EINVAL;
    const CompressWorkspace ws = compress_workspace(*p);
    if (!workspace || workspace_bytes < ws.bytes + (col_sums ? group_bytes : 0))
        return capacity_failure("razor_compress: workspace smaller than razor_plan reported");
    float *group_sums = reinterpret_cast<float *>(static_cast<char *>(workspace) + ws.bytes);

    hipStream_t s = static_cast<hipStream_t>(stream);
    const char *k = static_cast<const char *>(K), *v = static_cast<const char *>(V);
    char *a = static_cast<char *>(arena);
    int32_t *prefix = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + ws.prefix_off);
    float *partial = reinterpret_cast<float *>(static_cast<char *>(workspace) + ws.partial_off);
    int workers = p->n_workers;
    if (workers == 0) {
        rc = auto_workers(&workers);
        if (rc != RAZOR_OK) return rc;
        // 128-byte rows: a wave has half the bytes in flight, two waves per SIMD make up for it
        // (column sums of a 2.1 GB cache: 415 us with one wave per SIMD)
        if (p->head_dim * elem_size(p->dtype) == 128) workers *= 2;
    }
    workers = std::max(4, std::min(workers, RAZOR_MAX_WORKERS));
#define RAZOR_DISPATCH(DT, DD)                                                                    \
    return launch_compress<DT, DD>(*p, k, v, stride_b, stride_h, stride_n, desc, max_dropped, a,  \
                                   comp, desc_dev, kept_idx_dev, col_sums, prefix, partial, group_sums, workers, s)
    if (p->dtype == RAZOR_BF16 && p->head_dim == 128) RAZOR_DISPATCH(RAZOR_BF16, 128);
    if (p->dtype == RAZOR_BF16 && p->head_dim == 64) RAZOR_DISPATCH(RAZOR_BF16, 64);
    if (p->dtype == RAZOR_F32 && p->head_dim == 128) RAZOR_DISPATCH(RAZOR_F32, 128);
    if (p->dtype == RAZOR_F32 && p->head_dim == 64) RAZOR_DISPATCH(RAZOR_F32, 64);
#undef RAZOR_DISPATCH
    return RAZOR_EINVAL;
}
