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
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kQueriesPerWave = 32;                       // one 32-query operand tile
constexpr int kQueriesPerGroup = 4 * kQueriesPerWave;     // one workgroup of four wavefronts
constexpr int kStageKeys = 64;                            // keys staged in LDS per barrier
constexpr int kStepKeys = 32;                             // keys per pipeline step: one 32-key tile
constexpr float kLowest = -1.0e30f;                       // finite "no key seen yet"
constexpr float kMinusInf = -__builtin_huge_valf();
constexpr float kRenormalise = 0x1p100f;                  // running sums above this are rebased on the maximum

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
// max(a, b) as the median of (a, b, +inf): no NaN quieting of the operands, and the compiler
// pairs two of them into one three-operand maximum
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

// Workgroup (tile, head): 128 consecutive query rows of one head, 32 per wavefront, against
// keys 0 .. last query of the tile in stages of 64 keys.
//
// Lane l = 32 * g + r.  A stage of keys is staged in LDS piece-major per 32-key tile (16-byte
// piece c of key j at slot c * 32 + (j ^ c): the xor spreads the row-major global loads over
// the banks, and a wave still reads one contiguous kilobyte per matrix-core operand).
//   S^T[key][query] = K[key][:] . Q[query][:]   v_mfma_f32_32x32x16_bf16, A = key tile, B = Q
//   lane (g, r) gets query r of the wave and, in accumulator register v, key
//   8 (v / 4) + 4 g + v % 4 of the tile: the running reference and sum of a query stay inside
//   a lane until the two key halves are merged at the very end.
// The 32x32 shape halves the matrix instructions per logit against 16x16x32; what bounds this
// kernel is the vector unit (one fma, one exp2, one add per logit), and every matrix
// instruction costs it about two issue slots whatever its size.
// Stages right of the diagonal are skipped, the diagonal stage is masked per element.
template <int D>
__global__ __launch_bounds__(256, 3) void head_scores_kernel(
    const uint16_t *__restrict__ Q, const uint16_t *__restrict__ K, int64_t q_stride_h,
    int64_t q_stride_n, int64_t k_stride_h, int64_t k_stride_n, int n_tokens, int group,
    int period, int all_copies, float scale_log2e, int n_tiles, float *__restrict__ partial)
{
    constexpr int NS = D / 16;        // contraction steps of 16 columns
    constexpr int LPR = D / 8;        // 16-byte pieces per row
    constexpr int STAGE = kStageKeys * LPR;          // pieces per stage
    constexpr int LOADS = STAGE / 256;               // pieces per thread per stage
    __shared__ uint4 stage[2][STAGE];

    const int tile = n_tiles - 1 - (int)blockIdx.x;   // longest rows first
    const int head = blockIdx.y;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int g = lane >> 5, r = lane & 31;
    const int q0 = tile * kQueriesPerGroup;           // first query of the workgroup
    const int qw0 = q0 + wave * kQueriesPerWave;      // first query of this wave
    const uint16_t *Qh = Q + (int64_t)head * q_stride_h;
    const uint16_t *Kh = K + (int64_t)(head / group) * k_stride_h;
    const int last = n_tokens - 1;

    // B operands: the wave's 32 queries (rows past the prompt repeat the last one); lane (g, r)
    // holds pieces g, 2 + g, 4 + g, ... of query r
    bf16x8 qreg[NS];
    {
        const int row = min(qw0 + r, last);
#pragma unroll
        for (int s = 0; s < NS; ++s)
            qreg[s] = __builtin_bit_cast(
                bf16x8, *reinterpret_cast<const uint4 *>(Qh + (int64_t)row * q_stride_n + (2 * s + g) * 8));
    }

    // reference point (a scaled logit already seen, or the start value) and the sum of
    // 2^(scale * log2 e * logit - reference) over the keys absorbed so far
    float m = kLowest, l = 0.f;

    const int n_stages = (min(q0 + kQueriesPerGroup, n_tokens) + kStageKeys - 1) / kStageKeys;
    static_assert(LOADS == 2 || LOADS == 4, "a thread moves two or four pieces per stage");
    // Staging: thread t moves pieces t, t + 256, ... of a stage (row-major, coalesced); piece j
    // of a thread sits 256 / LPR rows below piece j - 1, in the same column.  Per thread: one
    // running source pointer (advanced by a stage per fetch), and the LDS slots of its pieces.
    constexpr int ROWS_PER_LOAD = 256 / LPR;
    const int64_t stage_elems = (int64_t)kStageKeys * k_stride_n;
    const int64_t load_elems = (int64_t)ROWS_PER_LOAD * k_stride_n;
    const int row0 = (int)threadIdx.x / LPR, col = (int)threadIdx.x % LPR;
    const uint16_t *src = Kh + (int64_t)row0 * k_stride_n + col * 8;     // this thread's first piece of stage 0
    const uint16_t *tail = Kh + (int64_t)last * k_stride_n + col * 8;    // same column of the last row
    int slot_of[LOADS];
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
        const int row = row0 + j * ROWS_PER_LOAD;
        slot_of[j] = ((row >> 5) * LPR + col) * 32 + ((row & 31) ^ col);
    }
    uint4 hold0, hold1, hold2 = {}, hold3 = {};   // named registers: they stay in registers across the barrier
    // a stage that ends inside the prompt: no row needs clamping
    auto fetch_inside = [&](int st) {
        const uint16_t *from = src + st * stage_elems;
        hold0 = *reinterpret_cast<const uint4 *>(from);
        hold1 = *reinterpret_cast<const uint4 *>(from + load_elems);
        if constexpr (LOADS == 4) {
            hold2 = *reinterpret_cast<const uint4 *>(from + 2 * load_elems);
            hold3 = *reinterpret_cast<const uint4 *>(from + 3 * load_elems);
        }
    };
    // any stage: rows past the prompt read its last row
    auto fetch_piece = [&](int st, int j) {
        const uint16_t *from = st * kStageKeys + row0 + j * ROWS_PER_LOAD > last ? tail
                                                                                  : src + st * stage_elems + j * load_elems;
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
        uint4 *to = stage[buf];
        to[slot_of[0]] = hold0;
        to[slot_of[1]] = hold1;
        if constexpr (LOADS == 4) {
            to[slot_of[2]] = hold2;
            to[slot_of[3]] = hold3;
        }
    };

    // One pipeline step covers one 32-key tile against the wave's 32 queries.  The LDS slot of
    // piece 2 s + g of key r inside a tile is kept per lane; buffer and tile are compile-time
    // constants of a step, so they end up in the offset field of the LDS reads.
    int slot[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) slot[s] = (2 * s + g) * 32 + (r ^ (2 * s + g));
    auto products = [&](auto buf_tile, f32x16 &S) {       // buf_tile: 2 * buffer + tile of the stage
        constexpr int BT = decltype(buf_tile)::value;
        const uint4 *base = &stage[BT >> 1][(BT & 1) * LPR * 32];
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, base[slot[s]]), qreg[s], acc, 0, 0, 0);
        S = acc;
    };
    // Exact update: m becomes the maximum of everything seen, l the sum relative to it.
    auto absorb_exact = [&](int u, f32x16 &S, float l_before, auto masked) {
        if (masked) {                          // key k0 + 8 (v / 4) + 4 g + v % 4 against query qw0 + r
            const int k0 = u * kStepKeys;
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (k0 + 8 * (v / 4) + 4 * g + v % 4 > qw0 + r) S[v] = kMinusInf;
        }
        float raw = kMinusInf;
#pragma unroll
        for (int v = 0; v < 16; ++v) raw = max_of(raw, S[v]);
        const float top = max_of(m, raw * scale_log2e);   // stays finite: m starts finite
        // all exponents, then all exp2, then a tree of adds: independent instructions back to back
        float p[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) p[v] = fmaf(S[v], scale_log2e, -top);
#pragma unroll
        for (int v = 0; v < 16; ++v) p[v] = exp2_fast(p[v]);
        const float keep = l_before * exp2_fast(m - top);
#pragma unroll
        for (int w = 8; w > 0; w >>= 1)
#pragma unroll
            for (int v = 0; v < w; ++v) p[v] += p[v + w];
        m = top;
        l = keep + p[0];
    };
    // Interior update.  m only has to be some logit already seen (a reference point, not the
    // maximum) as long as the sum stays inside the fp32 range: the exponents are taken against
    // the old m right away and the maximum is computed only on the rare step where the sum
    // passes 2^100 or overflows (the very first step, where m is still the start value, is one).
    // Terms that underflow against m are below 2^-126 of a term already in the sum.
    auto absorb_fast = [&](int u, f32x16 &S) {
        float p[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) p[v] = fmaf(S[v], scale_log2e, -m);
#pragma unroll
        for (int v = 0; v < 16; ++v) p[v] = exp2_fast(p[v]);
#pragma unroll
        for (int w = 8; w > 0; w >>= 1)
#pragma unroll
            for (int v = 0; v < w; ++v) p[v] += p[v + w];
        const float l_before = l;
        l = l_before + p[0];
        if (__any(!(l < kRenormalise))) absorb_exact(u, S, l_before, std::false_type{});
    };
    // A step in the interior of the causal region: the products of the next step (`nxt`) are
    // issued first, the maximum / sum update of this step's logits (`cur`) follows while the
    // matrix cores work.
    auto plain_step = [&](int u, auto next_buf_tile, f32x16 &cur, f32x16 &nxt) {
        products(next_buf_tile, nxt);
        absorb_fast(u, cur);
    };
    using BT0 = std::integral_constant<int, 0>;    // as argument of products: buffer 0, tile 0;
    using BT1 = std::integral_constant<int, 1>;    // as argument of the stage lambdas: buffer 0 / 1

    // Stage `diag` holds the wave's own keys (masked per element); the stages before it are
    // interior, the stages after it lie right of the diagonal and only need this wave's share of
    // the staging.  Separate loops instead of one loop with branches: no register shuffling
    // where control flow would merge.  Every wave passes the same number of barriers.
    const int diag = qw0 / kStageKeys;
    const bool active = diag < n_stages;               // false: the wave lies past the prompt
    const int interior = active ? diag : 0;
    f32x16 S0, S1;
    fetch(0);
    deposit(0);
    __syncthreads();
    if (active) products(BT0{}, S0);
    // an interior stage in buffer B: tile 1 of the stage, then (after the barrier that publishes
    // the next stage in the other buffer) tile 0 of that one
    auto interior_stage = [&](int st, auto buffer, auto next_inside) {
        constexpr int B = decltype(buffer)::value;
        if (next_inside) fetch_inside(st + 1);          // st + 1 <= diag < n_stages
        else fetch(st + 1);
        plain_step(2 * st, std::integral_constant<int, 2 * B + 1>{}, S0, S1);
        deposit(B ^ 1);
        __syncthreads();
        plain_step(2 * st + 1, std::integral_constant<int, 2 * (B ^ 1)>{}, S1, S0);
    };
    auto diagonal_stage = [&](int st, auto buffer) {
        constexpr int B = decltype(buffer)::value;
        // the last stage of the workgroup fetches itself again and parks it in the idle buffer
        fetch(min(st + 1, n_stages - 1));
        const bool second = qw0 % kStageKeys != 0;      // else the stage's second tile lies right of every query
        if (second) products(std::integral_constant<int, 2 * B + 1>{}, S1);
        absorb_exact(2 * st, S0, l, std::true_type{});
        deposit(B ^ 1);
        __syncthreads();
        if (second) absorb_exact(2 * st + 1, S1, l, std::true_type{});
    };
    // Every stage but the workgroup's last one ends inside the prompt and is fetched without
    // clamping; that covers all interior stages except possibly a wave's last one.
    const int unclamped = min(interior, n_stages - 2);  // stages st < unclamped have st + 1 <= n_stages - 2
    int st = 0;
    for (; st + 1 < unclamped; st += 2) {
        interior_stage(st, BT0{}, std::true_type{});
        interior_stage(st + 1, BT1{}, std::true_type{});
    }
    if (st < interior) {                                // at most two interior stages are left
        interior_stage(st, BT0{}, std::false_type{});
        ++st;
        if (st < interior) {
            interior_stage(st, BT1{}, std::false_type{});
            ++st;
        }
    }
    if (active) {
        if (st & 1) diagonal_stage(st, BT1{});
        else diagonal_stage(st, BT0{});
        ++st;
    }
    for (; st < n_stages; ++st) {
        fetch(min(st + 1, n_stages - 1));
        deposit((st + 1) & 1);
        __syncthreads();
    }

    // Denominator: merge the two key halves of every query; log2 of the row sum, relative to 0.
    float echo = 0.f, induction = 0.f;
    {
        const float mo = __shfl_xor(m, 32), lo = __shfl_xor(l, 32);
        const float top = fmaxf(m, mo);
        const float ll = l * exp2_fast(m - top) + lo * exp2_fast(mo - top);
        const float lse2 = top + __log2f(ll);
        // Target logits: lane (g, r) holds pieces 2 s + g of query r and takes the same pieces of
        // the target key; the two halves then add up.
        const int q = qw0 + r;
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
                    const uint4 qv = __builtin_bit_cast(uint4, qreg[s]);
                    de = dot_piece(qv, *reinterpret_cast<const uint4 *>(ke + (2 * s + g) * 8), de);
                    di = dot_piece(qv, *reinterpret_cast<const uint4 *>(ki + (2 * s + g) * 8), di);
                }
            }
            de += __shfl_xor(de, 32);
            di += __shfl_xor(di, 32);
            if (live && g == 0) {
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
        float *out = partial + (((int64_t)head * n_tiles + tile) * 4 + wave) * 2;
        out[0] = echo;
        out[1] = induction;
    }
}

// One wavefront per head: lane i adds the per-wave sums i, i + 64, ... in double, then the lanes
// are folded in a fixed butterfly; divides by the number of scored rows.
__global__ __launch_bounds__(64) void head_scores_reduce_kernel(const float *__restrict__ partial, int per_head,
                                                                double inv_rows, float *__restrict__ echo,
                                                                float *__restrict__ induction)
{
    const int head = blockIdx.x, lane = threadIdx.x;
    const float2 *src = reinterpret_cast<const float2 *>(partial) + (int64_t)head * per_head;
    double e = 0.0, i = 0.0;
    for (int k = lane; k < per_head; k += 64) {
        const float2 v = src[k];
        e += (double)v.x;
        i += (double)v.y;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        e += __shfl_xor(e, o);
        i += __shfl_xor(i, o);
    }
    if (lane == 0) {
        echo[head] = (float)(e * inv_rows);
        induction[head] = (float)(i * inv_rows);
    }
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
    if (!workspace || workspace_bytes < need)
        return capacity_failure("razor_head_scores: workspace smaller than razor_head_scores_workspace reported");

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
    hipLaunchKernelGGL(head_scores_reduce_kernel, dim3(n_q_heads), dim3(64), 0, s, partial, n_tiles * 4,
                       1.0 / (double)(n_tokens - period), echo, induction);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return hip_failure("razor_head_scores launch", (int)err);
    return RAZOR_OK;
}
