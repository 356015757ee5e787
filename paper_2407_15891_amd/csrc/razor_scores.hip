// Head scoring for the identification of retrieval heads (Sec. 3.3): echo and induction
// score of every query head on a prompt of `period` random tokens repeated to n_tokens.
//
// The score of a head is the mean, over the positions m that have a previous copy, of one or
// two entries of its causal attention map.  The map is never formed: per query row only the
// softmax denominator is needed (a dense Q K^T contraction on the matrix cores with an online
// maximum / sum, the first half of a fused attention kernel) plus the logits of the few target
// positions, which are plain dot products.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <type_traits>

#include "razor.h"
#include "razor_device.h"

namespace razor {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kQueriesPerWave = 32;                       // two 16-query operand tiles
constexpr int kQueryTiles = kQueriesPerWave / 16;
constexpr int kQueriesPerGroup = 4 * kQueriesPerWave;     // one workgroup of four wavefronts
constexpr int kStageKeys = 64;                            // keys staged in LDS per step
constexpr int kStepKeys = 32;                             // keys per pipeline step
constexpr int kStepTiles = kStepKeys / 16;
constexpr float kLowest = -1.0e30f;                       // finite "no key seen yet"
constexpr float kMinusInf = -__builtin_huge_valf();

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
// max(a, b) as the median of (a, b, +inf): one instruction, no NaN quieting of the operands
__device__ __forceinline__ float max_of(float a, float b) { return __builtin_amdgcn_fmed3f(a, b, __builtin_huge_valf()); }

// Dot product of two 16-byte pieces of bf16 (fp32 products and sums, element order).
__device__ __forceinline__ float dot_piece(const uint4 a, const uint4 b, float acc)
{
    const uint32_t x[4] = {a.x, a.y, a.z, a.w}, y[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        acc = fmaf(__uint_as_float(x[i] << 16), __uint_as_float(y[i] << 16), acc);
        acc = fmaf(__uint_as_float(x[i] & 0xffff0000u), __uint_as_float(y[i] & 0xffff0000u), acc);
    }
    return acc;
}

// Workgroup (tile, head): 256 consecutive query rows of one head, 64 per wavefront, against
// keys 0 .. last query of the tile in stages of 64 keys.
//
// Lane l = 16 * kg + n.  A stage of keys is staged in LDS piece-major per 16-key tile (16-byte
// piece c of key r at slot c * 16 + (r ^ c): the xor spreads the row-major global loads over
// the banks, and a wave still reads one contiguous kilobyte per matrix-core operand).
//   S^T[key][query] = K[key][:] . Q[query][:]   v_mfma_f32_16x16x32_bf16, A = key tile, B = Q
//   lane (kg, n) gets query n of the tile and keys 4 kg .. 4 kg + 3: the running maximum and
//   sum of a query stay inside a lane until the four key groups are merged at the very end.
// Stages right of the diagonal are skipped, the diagonal stage is masked per element.
template <int D>
__global__ __launch_bounds__(256, 3) void head_scores_kernel(
    const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, int64_t q_stride_h,
    int64_t q_stride_n, int64_t k_stride_h, int64_t k_stride_n, int n_tokens, int group,
    int period, int all_copies, float scale_log2e, int n_tiles, float *__restrict__ partial)
{
    constexpr int NS = D / 32;        // contraction steps of 32 columns
    constexpr int LPR = D / 8;        // 16-byte pieces per row
    constexpr int STAGE = kStageKeys * LPR;          // pieces per stage
    constexpr int LOADS = STAGE / 256;               // pieces per thread per stage
    __shared__ uint4 stage[2][STAGE];

    const int tile = n_tiles - 1 - (int)blockIdx.x;   // longest rows first
    const int head = blockIdx.y;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int kg = lane >> 4, n = lane & 15;
    const int q0 = tile * kQueriesPerGroup;           // first query of the workgroup
    const int qw0 = q0 + wave * kQueriesPerWave;      // first query of this wave
    const uint16_t *Qh = Q + (int64_t)head * q_stride_h;
    const uint16_t *Kh = K + (int64_t)(head / group) * k_stride_h;
    const int last = n_tokens - 1;

    // B operands: the wave's 64 queries, 16 per tile (rows past the prompt repeat the last one)
    bf16x8 qreg[kQueryTiles][NS];
#pragma unroll
    for (int qt = 0; qt < kQueryTiles; ++qt) {
        const int row = min(qw0 + qt * 16 + n, last);
#pragma unroll
        for (int s = 0; s < NS; ++s)
            qreg[qt][s] = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const uint4 *>(Qh + (int64_t)row * q_stride_n + (4 * s + kg) * 8));
    }

    // running maximum (already times scale * log2 e) and sum of 2^(logit - maximum), per query tile
    float m[kQueryTiles], l[kQueryTiles];
#pragma unroll
    for (int qt = 0; qt < kQueryTiles; ++qt) {
        m[qt] = kLowest;
        l[qt] = 0.f;
    }

    const int n_stages = (min(q0 + kQueriesPerGroup, n_tokens) + kStageKeys - 1) / kStageKeys;
    static_assert(LOADS == 2 || LOADS == 4, "a thread moves two or four pieces per stage");
    // Staging: thread t moves pieces t, t + 256, ... of a stage (row-major, coalesced).  The
    // source pointers advance by one stage per step; rows past the prompt read its last row.
    const int64_t stage_elems = (int64_t)kStageKeys * k_stride_n;
    const uint16_t *src[LOADS], *tail[LOADS];
    int src_row[LOADS], dst[LOADS];
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        const int idx = j * 256 + (int)threadIdx.x;
        const int row = idx / LPR, c = idx % LPR;
        src_row[j] = row;
        src[j] = Kh + (int64_t)row * k_stride_n + c * 8;
        tail[j] = Kh + (int64_t)last * k_stride_n + c * 8;
        dst[j] = ((row >> 4) * LPR + c) * 16 + ((row & 15) ^ c);
    }
    // Named registers, not an array: the loads stay in registers across the barrier.
    uint4 hold0, hold1, hold2 = {}, hold3 = {};
    auto fetch_piece = [&](int st, int j) {
        const uint16_t *from = st * kStageKeys + src_row[j] > last ? tail[j] : src[j] + st * stage_elems;
        return *reinterpret_cast<const uint4 *>(from);
    };
    auto fetch = [&](int st) {
        hold0 = fetch_piece(st, 0);
        hold1 = fetch_piece(st, 1);
        if constexpr (LOADS == 4) {
            hold2 = fetch_piece(st, 2);
            hold3 = fetch_piece(st, 3);
        }
    };
    auto deposit = [&](int buf) {
        stage[buf][dst[0]] = hold0;
        stage[buf][dst[1]] = hold1;
        if constexpr (LOADS == 4) {
            stage[buf][dst[2]] = hold2;
            stage[buf][dst[3]] = hold3;
        }
    };

    // One pipeline step covers 32 keys (two key tiles) against the wave's 64 queries.
    auto products = [&](int u, f32x4(&S)[kQueryTiles][kStepTiles]) {
        const uint4 *buf = stage[(u >> 1) & 1];
#pragma unroll
        for (int kt = 0; kt < kStepTiles; ++kt) {
            const int tile = (u & 1) * kStepTiles + kt;
            bf16x8 a[NS];
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const int c = 4 * s + kg;
                a[s] = __builtin_bit_cast(bf16x8, buf[(tile * LPR + c) * 16 + (n ^ c)]);
            }
#pragma unroll
            for (int qt = 0; qt < kQueryTiles; ++qt) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < NS; ++s)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[s], qreg[qt][s], acc, 0, 0, 0);
                S[qt][kt] = acc;
            }
        }
    };
    auto absorb = [&](int u, f32x4(&S)[kQueryTiles][kStepTiles], auto masked) {
        const int k0 = u * kStepKeys;
#pragma unroll
        for (int qt = 0; qt < kQueryTiles; ++qt) {
            if (masked) {                      // key k0 + 16 kt + 4 kg + r against query qw0 + 16 qt + n
#pragma unroll
                for (int kt = 0; kt < kStepTiles; ++kt)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (k0 + kt * 16 + 4 * kg + r > qw0 + qt * 16 + n) S[qt][kt][r] = kMinusInf;
            }
            float raw = kMinusInf;
#pragma unroll
            for (int kt = 0; kt < kStepTiles; ++kt)
#pragma unroll
                for (int r = 0; r < 4; ++r) raw = max_of(raw, S[qt][kt][r]);
            const float top = max_of(m[qt], raw * scale_log2e);   // stays finite: m starts finite
            float sum = l[qt] * exp2_fast(m[qt] - top);
#pragma unroll
            for (int kt = 0; kt < kStepTiles; ++kt)
#pragma unroll
                for (int r = 0; r < 4; ++r) sum += exp2_fast(fmaf(S[qt][kt][r], scale_log2e, -top));
            m[qt] = top;
            l[qt] = sum;
        }
    };
    // A step in the interior of the causal region: the maximum / sum update of its logits (`cur`)
    // is issued together with the products of the next step (`nxt`) in one straight block, so
    // that the vector unit and the matrix cores of a SIMD work at the same time.
    auto plain_step = [&](int u, f32x4(&cur)[kQueryTiles][kStepTiles], f32x4(&nxt)[kQueryTiles][kStepTiles]) {
        __builtin_amdgcn_sched_barrier(0);                          // a scheduling region of its own
        products(u + 1, nxt);
        absorb(u, cur, std::false_type{});
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * NS, 0);     // LDS reads of the key tiles
        __builtin_amdgcn_sched_group_barrier(0x002, 10, 0);         // vector work while they land
#pragma unroll
        for (int i = 0; i < kQueryTiles * kStepTiles * NS; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // one matrix instruction
            __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);      // three vector instructions
            __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);      // one exp2
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // Stage `diag` holds the wave's own keys (masked per element); the stages before it are
    // interior, the stages after it lie right of the diagonal and only need this wave's share of
    // the staging.  Three loops instead of one loop with branches: no register shuffling where
    // control flow would merge.  Every wave passes the same number of barriers.
    const int diag = qw0 / kStageKeys;
    const bool active = diag < n_stages;               // false: the wave lies past the prompt
    const int interior = active ? diag : 0;
    f32x4 S0[kQueryTiles][kStepTiles], S1[kQueryTiles][kStepTiles];
    fetch(0);
    deposit(0);
    __syncthreads();
    if (active) products(0, S0);
    int st = 0;
    for (; st < interior; ++st) {
        fetch(st + 1);                            // st + 1 <= diag < n_stages
        plain_step(2 * st, S0, S1);
        deposit((st + 1) & 1);
        __syncthreads();
        plain_step(2 * st + 1, S1, S0);                 // its products read the stage deposited just now
    }
    if (active) {
        // the last stage of the workgroup fetches itself again and parks it in the idle buffer
        fetch(min(st + 1, n_stages - 1));
        products(2 * st + 1, S1);
        absorb(2 * st, S0, std::true_type{});
        deposit((st + 1) & 1);
        __syncthreads();
        absorb(2 * st + 1, S1, std::true_type{});
        ++st;
    }
    for (; st < n_stages; ++st) {
        fetch(min(st + 1, n_stages - 1));
        deposit((st + 1) & 1);
        __syncthreads();
    }

    // Denominators: merge the four key groups of every query; log2 of the row sum, relative to 0.
    float echo = 0.f, induction = 0.f;
#pragma unroll
    for (int qt = 0; qt < kQueryTiles; ++qt) {
        float mm = m[qt], ll = l[qt];
#pragma unroll
        for (int o = 16; o < 64; o <<= 1) {
            const float mo = __shfl_xor(mm, o), lo = __shfl_xor(ll, o);
            const float top = fmaxf(mm, mo);
            ll = ll * exp2_fast(mm - top) + lo * exp2_fast(mo - top);
            mm = top;
        }
        const float lse2 = mm + __log2f(ll);
        // Target logits: lane (kg, n) holds pieces 4 s + kg of query n and takes the same pieces
        // of the target key; the four key groups then add up.
        const int q = qw0 + qt * 16 + n;
        const bool valid = q < n_tokens && q >= period;
        int prev = q - period;
        bool live = valid;
        while (__any(live)) {
            float de = 0.f, di = 0.f;
            if (live) {
                const uint16_t *ke = Kh + (int64_t)prev * k_stride_n;
                const uint16_t *ki = ke + k_stride_n;            // prev + 1 <= q since period >= 1
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    const uint4 qv = __builtin_bit_cast(uint4, qreg[qt][s]);
                    de = dot_piece(qv, *reinterpret_cast<const uint4 *>(ke + (4 * s + kg) * 8), de);
                    di = dot_piece(qv, *reinterpret_cast<const uint4 *>(ki + (4 * s + kg) * 8), di);
                }
            }
#pragma unroll
            for (int o = 16; o < 64; o <<= 1) {
                de += __shfl_xor(de, o);
                di += __shfl_xor(di, o);
            }
            if (live && kg == 0) {
                echo += exp2_fast(fmaf(de, scale_log2e, -lse2));
                induction += exp2_fast(fmaf(di, scale_log2e, -lse2));
            }
            prev -= period;
            live = live && all_copies && prev >= 0;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        echo += __shfl_xor(echo, o);
        induction += __shfl_xor(induction, o);
    }
    if (lane == 0) {
        float *dst = partial + (((int64_t)head * n_tiles + tile) * 4 + wave) * 2;
        dst[0] = echo;
        dst[1] = induction;
    }
}

// Adds a head's per-wave sums in index order (double) and divides by the number of scored rows.
__global__ void head_scores_reduce_kernel(const float *__restrict__ partial, int n_heads, int per_head,
                                          double inv_rows, float *__restrict__ echo,
                                          float *__restrict__ induction)
{
    const int head = blockIdx.x * blockDim.x + threadIdx.x;
    if (head >= n_heads) return;
    const float *src = partial + (int64_t)head * per_head * 2;
    double e = 0.0, i = 0.0;
    for (int k = 0; k < per_head; ++k) {
        e += (double)src[2 * k];
        i += (double)src[2 * k + 1];
    }
    echo[head] = (float)(e * inv_rows);
    induction[head] = (float)(i * inv_rows);
}

}  // namespace
}  // namespace razor

extern "C" size_t razor_head_scores_workspace(int n_q_heads, int n_tokens)
{
    using namespace razor;
    if (n_q_heads <= 0 || n_tokens <= 0) return 0;
    const size_t tiles = ((size_t)n_tokens + kQueriesPerGroup - 1) / kQueriesPerGroup;
    return (size_t)n_q_heads * tiles * 4 * 2 * sizeof(float);
}

extern "C" int razor_head_scores(const void *Q, const void *K, int dtype, int n_q_heads, int n_kv_heads,
                                 int head_dim, int n_tokens, int64_t q_stride_h, int64_t q_stride_n,
                                 int64_t k_stride_h, int64_t k_stride_n, float scale, int period,
                                 int all_copies, float *echo, float *induction, void *workspace,
                                 size_t workspace_bytes, void *stream)
{
    using namespace razor;
    if (!Q || !K || !echo || !induction) return RAZOR_EINVAL;
    if (dtype != RAZOR_BF16) return RAZOR_EINVAL;                 // matrix-core path only
    if (head_dim != 64 && head_dim != 128) return RAZOR_EINVAL;
    if (n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads || n_q_heads > 65535) return RAZOR_EINVAL;
    if (n_tokens < 2 || period < 1 || period >= n_tokens) return RAZOR_EINVAL;
    if (!(scale > 0.f) || !std::isfinite(scale)) return RAZOR_EINVAL;
    if (q_stride_n < head_dim || k_stride_n < head_dim || q_stride_h < 0 || k_stride_h < 0) return RAZOR_EINVAL;
    if ((q_stride_n | q_stride_h | k_stride_n | k_stride_h) % 8) return RAZOR_EINVAL;   // 16-byte rows
    if (((uintptr_t)Q | (uintptr_t)K) & 15) return RAZOR_EINVAL;
    const size_t need = razor_head_scores_workspace(n_q_heads, n_tokens);
    if (!workspace || workspace_bytes < need) return RAZOR_ECAPACITY;

    const int n_tiles = (n_tokens + kQueriesPerGroup - 1) / kQueriesPerGroup;
    const float scale_log2e = scale * 1.4426950408889634f;
    float *partial = static_cast<float *>(workspace);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint16_t *q = static_cast<const uint16_t *>(Q), *k = static_cast<const uint16_t *>(K);
    const dim3 grid(n_tiles, n_q_heads);
    if (head_dim == 128)
        hipLaunchKernelGGL((head_scores_kernel<128>), grid, dim3(256), 0, s, q, k, q_stride_h, q_stride_n,
                           k_stride_h, k_stride_n, n_tokens, n_q_heads / n_kv_heads, period, all_copies,
                           scale_log2e, n_tiles, partial);
    else
        hipLaunchKernelGGL((head_scores_kernel<64>), grid, dim3(256), 0, s, q, k, q_stride_h, q_stride_n,
                           k_stride_h, k_stride_n, n_tokens, n_q_heads / n_kv_heads, period, all_copies,
                           scale_log2e, n_tiles, partial);
    hipLaunchKernelGGL(head_scores_reduce_kernel, dim3((n_q_heads + 255) / 256), dim3(256), 0, s, partial,
                       n_q_heads, n_tiles * 4, 1.0 / (double)(n_tokens - period), echo, induction);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return hip_failure("razor_head_scores launch", (int)err);
    return RAZOR_OK;
}
