// razor_compress: prefill-time pass that turns a full K/V cache into the per-head
// heterogeneous cache (Algorithm 1 steps 1-4, Eq.(4)).  Three kinds of work:
//   mean   column sums of the dropped rows [n_sink, N - window) -> khat, vhat (fp32)
//   copy   kept rows (sinks + window, or everything) -> arena; K re-tiled through LDS
//   index  kept positions as int32 (optional)
// All of it is HBM streaming: every source row is read once, kept rows written once.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <vector>

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

__device__ __forceinline__ float bf16_bits_to_float(uint32_t lo16)
{
    return __uint_as_float(lo16 << 16);
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
    } else {
        acc[0] += bf16_bits_to_float(v.x & 0xffffu);
        acc[1] += __uint_as_float(v.x & 0xffff0000u);
        acc[2] += bf16_bits_to_float(v.y & 0xffffu);
        acc[3] += __uint_as_float(v.y & 0xffff0000u);
        acc[4] += bf16_bits_to_float(v.z & 0xffffu);
        acc[5] += __uint_as_float(v.z & 0xffff0000u);
        acc[6] += bf16_bits_to_float(v.w & 0xffffu);
        acc[7] += __uint_as_float(v.w & 0xffff0000u);
    }
}

// Eq.(4), first level.  Workgroup (slab, head) sums up to kMeanSlabRows dropped rows of
// K and of V column-wise.  Thread t owns the 16-byte piece t % LPR of rows
// t / LPR, t / LPR + RPP, ...; the row groups are then added in a fixed order.
template <int DTYPE, int D>
__global__ __launch_bounds__(256) void mean_partial_kernel(
    const char *__restrict__ K, const char *__restrict__ V, int64_t stride_b, int64_t stride_h,
    int64_t stride_n, const razor_head_desc *__restrict__ desc, int n_kv_heads, int n_sink,
    int max_slabs, float *__restrict__ partial)
{
    constexpr int ES = DTYPE == RAZOR_F32 ? 4 : 2;
    constexpr int NE = 16 / ES;        // elements per piece
    constexpr int LPR = D * ES / 16;   // pieces (threads) per row
    constexpr int RPP = 256 / LPR;     // rows per pass of the workgroup
    const int head = blockIdx.y, slab = blockIdx.x;
    const razor_head_desc e = desc[head];
    const int64_t lo = (int64_t)n_sink + (int64_t)slab * kMeanSlabRows;
    const int64_t d_hi = (int64_t)n_sink + e.n_dropped;
    if (e.n_dropped <= 0 || lo >= d_hi) return;
    const int64_t hi = lo + kMeanSlabRows < d_hi ? lo + kMeanSlabRows : d_hi;
    const int b = head / n_kv_heads, h = head % n_kv_heads;
    const int64_t base = (b * stride_b + h * stride_h) * ES;
    const int piece = threadIdx.x % LPR, rgrp = threadIdx.x / LPR;

    float ak[NE], av[NE];
#pragma unroll
    for (int i = 0; i < NE; ++i) ak[i] = av[i] = 0.f;
    int64_t r = lo + rgrp;
    for (; r + 3 * RPP < hi; r += 4 * RPP) {   // four rows in flight per thread
        uint4 k4[4], v4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t off = base + (r + u * RPP) * stride_n * ES + piece * 16;
            k4[u] = *reinterpret_cast<const uint4 *>(K + off);
            v4[u] = *reinterpret_cast<const uint4 *>(V + off);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            accumulate_piece<DTYPE>(k4[u], ak);
            accumulate_piece<DTYPE>(v4[u], av);
        }
    }
    for (; r < hi; r += RPP) {
        const int64_t off = base + r * stride_n * ES + piece * 16;
        accumulate_piece<DTYPE>(*reinterpret_cast<const uint4 *>(K + off), ak);
        accumulate_piece<DTYPE>(*reinterpret_cast<const uint4 *>(V + off), av);
    }

    __shared__ float red[2][RPP][D + 4];
#pragma unroll
    for (int i = 0; i < NE; ++i) {
        red[0][rgrp][piece * NE + i] = ak[i];
        red[1][rgrp][piece * NE + i] = av[i];
    }
    __syncthreads();
    for (int t = threadIdx.x; t < 2 * D; t += 256) {
        const int which = t / D, c = t % D;
        float s = 0.f;
        for (int g = 0; g < RPP; ++g) s += red[which][g][c];
        partial[(((size_t)head * max_slabs + slab) * 2 + which) * D + c] = s;
    }
}

// Eq.(4), second level: add the slab sums in order (double keeps the tail exact enough
// that the result does not depend on the slab size) and divide by N_d.
template <int D>
__global__ void mean_final_kernel(const razor_head_desc *__restrict__ desc, int max_slabs,
                                  const float *__restrict__ partial, float *__restrict__ comp)
{
    const int head = blockIdx.x;
    const razor_head_desc e = desc[head];
    for (int t = threadIdx.x; t < 2 * D; t += blockDim.x) {
        float out = 0.f;
        if (e.n_dropped > 0) {
            const int slabs = (e.n_dropped + kMeanSlabRows - 1) / kMeanSlabRows;
            double s = 0.0;
            for (int k = 0; k < slabs; ++k)
                s += (double)partial[((size_t)head * max_slabs + k) * 2 * D + t];
            out = (float)(s / (double)e.n_dropped);
        }
        comp[(size_t)head * 2 * D + t] = out;
    }
}

// Cache row t of a head sits at source position t (sinks, or nothing dropped) or
// t + n_dropped (window part).
__device__ __forceinline__ int64_t source_row(int t, const razor_head_desc &e, int n_sink)
{
    return (e.n_dropped > 0 && t >= n_sink) ? (int64_t)t + e.n_dropped : (int64_t)t;
}

// Compaction (Algorithm 1 step 3).  One wavefront moves one 16-row block: V rows are
// copied as they are; K rows are read row-major (coalesced), staged in LDS and written
// back piece-major, the layout the decode kernel loads straight into matrix-core operands.
// Rows past `rows` inside the last block are written as zeros.
template <int RB>   // bytes per row
__global__ __launch_bounds__(256) void compact_kernel(
    const char *__restrict__ K, const char *__restrict__ V, int64_t stride_b_bytes,
    int64_t stride_h_bytes, int64_t stride_n_bytes, const razor_head_desc *__restrict__ desc,
    int n_kv_heads, int n_sink, char *__restrict__ arena)
{
    constexpr int LPR = RB / 16;       // 16-byte pieces per row
    constexpr int RPI = 64 / LPR;      // rows one wave-wide load covers
    constexpr int NI = 16 / RPI;       // loads per block
    const int head = blockIdx.y;
    const razor_head_desc e = desc[head];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int blk = blockIdx.x * 4 + wave;
    const int n_blocks = (e.rows + kBlockRows - 1) / kBlockRows;
    if (blk >= n_blocks) return;       // wave-private work below: no workgroup barrier
    const int b = head / n_kv_heads, h = head % n_kv_heads;
    const int64_t src_base = b * stride_b_bytes + h * stride_h_bytes;
    char *kplane = arena + e.row_off * 2 * RB;
    char *vplane = kplane + (int64_t)e.cap * RB;

    __shared__ uint4 stage[4][16 * LPR];
    const int prow = lane / LPR, piece = lane % LPR;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int r = i * RPI + prow;                 // row inside the block
        const int t = blk * kBlockRows + r;           // cache row
        uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
        if (t < e.rows) {
            const int64_t off = src_base + source_row(t, e, n_sink) * stride_n_bytes + piece * 16;
            kv = *reinterpret_cast<const uint4 *>(K + off);
            vv = *reinterpret_cast<const uint4 *>(V + off);
        }
        *reinterpret_cast<uint4 *>(vplane + (int64_t)t * RB + piece * 16) = vv;
        stage[wave][r * LPR + (piece ^ (r % LPR))] = kv;   // xor keeps the column reads conflict-free
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    char *kblock = kplane + (int64_t)blk * kBlockRows * RB;
#pragma unroll
    for (int s = 0; s < NI; ++s) {
        const int pos = s * 64 + lane;                // 16-byte slot inside the block
        const int c = pos / 16, r = pos % 16;         // piece-major: slot = c * 16 + r
        *reinterpret_cast<uint4 *>(kblock + (int64_t)pos * 16) = stage[wave][r * LPR + (c ^ (r % LPR))];
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
                    int32_t *kept_idx_dev, float *partial, hipStream_t stream)
{
    constexpr int ES = DTYPE == RAZOR_F32 ? 4 : 2;
    constexpr int RB = D * ES;
    const int n_heads = (int)desc.size();
    for (int first = 0; first < n_heads; first += kDescPerLaunch) {
        DescBatch batch;
        const int count = std::min(kDescPerLaunch, n_heads - first);
        for (int i = 0; i < count; ++i) batch.d[i] = desc[(size_t)first + i];
        for (int i = count; i < kDescPerLaunch; ++i) batch.d[i] = razor_head_desc{};
        hipLaunchKernelGGL(upload_desc_kernel, dim3(1), dim3(kDescPerLaunch), 0, stream, batch,
                           first, count, desc_dev);
    }
    const int max_slabs = compress_workspace(p, max_dropped).max_slabs;
    if (max_slabs > 0) {
        hipLaunchKernelGGL((mean_partial_kernel<DTYPE, D>), dim3(max_slabs, n_heads), dim3(256), 0,
                           stream, K, V, stride_b, stride_h, stride_n, desc_dev, p.n_kv_heads,
                           p.n_sink, max_slabs, partial);
    }
    hipLaunchKernelGGL((mean_final_kernel<D>), dim3(n_heads), dim3(2 * D), 0, stream, desc_dev,
                       max_slabs, partial, comp);
    int max_blocks = 0, max_rows = 0;
    for (const razor_head_desc &e : desc) {
        max_rows = std::max(max_rows, e.rows);
        max_blocks = std::max(max_blocks, (e.rows + kBlockRows - 1) / kBlockRows);
    }
    if (max_blocks > 0) {
        hipLaunchKernelGGL((compact_kernel<RB>), dim3((max_blocks + 3) / 4, n_heads), dim3(256), 0,
                           stream, K, V, stride_b * ES, stride_h * ES, stride_n * ES, desc_dev,
                           p.n_kv_heads, p.n_sink, arena);
        if (kept_idx_dev) {
            const int gx = std::min((max_rows + 255) / 256, 64);
            hipLaunchKernelGGL(kept_index_kernel, dim3(gx, n_heads), dim3(256), 0, stream, desc_dev,
                               p.n_sink, kept_idx_dev);
        }
    }
    RAZOR_HIP_CHECK(hipGetLastError());
    return RAZOR_OK;
}

}  // namespace
}  // namespace razor

extern "C" int razor_compress(const razor_params *p, const void *K, const void *V,
                              int64_t stride_b, int64_t stride_h, int64_t stride_n,
                              const int32_t *seq_lens_host, const uint8_t *retrieval_mask_host,
                              void *arena, float *comp, razor_head_desc *desc_dev,
                              int32_t *kept_idx_dev, void *workspace, size_t workspace_bytes,
                              void *stream)
{
    using namespace razor;
    if (check_params(p) != RAZOR_OK) return RAZOR_EINVAL;
    if (!K || !V || !seq_lens_host || !retrieval_mask_host || !comp || !desc_dev) return RAZOR_EINVAL;
    const int es = elem_size(p->dtype);
    const int64_t align = 16 / es;   // rows must start on 16-byte boundaries
    if (stride_n < p->head_dim || stride_n % align || stride_h % align || stride_b % align)
        return RAZOR_EINVAL;
    if (stride_b < 0 || stride_h < 0) return RAZOR_EINVAL;
    if (((uintptr_t)K | (uintptr_t)V | (uintptr_t)arena | (uintptr_t)comp) & 15) return RAZOR_EINVAL;

    std::vector<razor_head_desc> desc;
    razor_sizes sizes;
    int max_dropped = 0;
    int rc = build_plan(*p, seq_lens_host, retrieval_mask_host, desc, sizes, max_dropped);
    if (rc != RAZOR_OK) return rc;
    if (sizes.arena_bytes > 0 && !arena) return RAZOR_EINVAL;
    const CompressWorkspace ws = compress_workspace(*p, max_dropped);
    if (ws.bytes > 0 && (!workspace || workspace_bytes < ws.bytes)) return RAZOR_ECAPACITY;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const char *k = static_cast<const char *>(K), *v = static_cast<const char *>(V);
    char *a = static_cast<char *>(arena);
    float *partial = reinterpret_cast<float *>(static_cast<char *>(workspace) + ws.partial_off);
#define RAZOR_DISPATCH(DT, DD)                                                                    \
    return launch_compress<DT, DD>(*p, k, v, stride_b, stride_h, stride_n, desc, max_dropped, a,  \
                                   comp, desc_dev, kept_idx_dev, partial, s)
    if (p->dtype == RAZOR_BF16 && p->head_dim == 128) RAZOR_DISPATCH(RAZOR_BF16, 128);
    if (p->dtype == RAZOR_BF16 && p->head_dim == 64) RAZOR_DISPATCH(RAZOR_BF16, 64);
    if (p->dtype == RAZOR_F32 && p->head_dim == 128) RAZOR_DISPATCH(RAZOR_F32, 128);
    if (p->dtype == RAZOR_F32 && p->head_dim == 64) RAZOR_DISPATCH(RAZOR_F32, 64);
#undef RAZOR_DISPATCH
    return RAZOR_EINVAL;
}
