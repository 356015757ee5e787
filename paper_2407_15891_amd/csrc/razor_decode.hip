// razor_decode_attn: one decode step over the per-head heterogeneous cache
// (Algorithm 1 step 5, Eq.(5)).  Two launches on the caller's stream:
//
//   partial   the ragged per-head length table is flattened into one axis of 16-row
//             blocks, and that axis is cut into equal ranges, one per wavefront (every
//             wave derives the cut itself from the descriptor table).  A wavefront
//             streams the K and V blocks of its range once from HBM with 128-bit
//             non-temporal loads held in registers several blocks ahead, keeps an online
//             softmax state (running max, denominator, unnormalised output) for the
//             whole query group of the KV head, and stores one partial state per head
//             segment it touched.  Long retrieval heads and short compressed heads cost
//             exactly their bytes; no wavefront idles behind another, and waves never
//             synchronise with each other.  The wave that owns the block a new token
//             falls into stores that token first (the append).
//   combine   merges the partial states of each query head in a fixed order, folds
//             in the compensation token with weight N_d (logit + ln N_d), normalises,
//             and makes the append permanent (rows += 1).
//
// Both products run on the matrix cores (the query group is padded to the 16-wide
// operand): v_mfma_f32_16x16x32_bf16 for bf16 caches, v_mfma_f32_16x16x4_f32 for fp32.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <mutex>
#include <type_traits>

#include "razor_bench.h"
#include "razor_device.h"
#include "razor_internal.h"

namespace razor {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr float kNegInf = -__builtin_huge_valf();

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Debug builds (-DRAZOR_TIMELINE) stamp the 100 MHz wall clock at a few points of every
// streaming wave and drop the stamps into the unused upper half of the partial-output slots
// (such builds run at most RAZOR_MAX_WORKERS / 2 waves); off in the product.
#ifdef RAZOR_TIMELINE
#define RAZOR_STAMP(k) long long stamp_##k = wall_clock64()
#define RAZOR_STAMP_SEG() ++stamp_segments
#define RAZOR_STAMP_FLUSH()                                                                        \
    if (lane == 0) {                                                                               \
        long long *dst = reinterpret_cast<long long *>(part_acc + timeline_floats(n_heads, g, D)) + (size_t)w * 4; \
        dst[0] = stamp_0; dst[1] = stamp_1; dst[2] = stamp_2; dst[3] = stamp_segments;             \
    }
#else
#define RAZOR_STAMP(k)
#define RAZOR_STAMP_SEG()
#define RAZOR_STAMP_FLUSH()
#endif

// The new token of head `head` goes to row e.rows of its planes (K piece-major inside its
// block, V row-major).  Called by the one wave whose range holds that row's block.
template <int RB>
__device__ __forceinline__ void append_row(const razor_head_desc &e, int head, char *kplane, char *vplane,
                                           const char *__restrict__ k_new,
                                           const char *__restrict__ v_new, int lane)
{
    constexpr int LPR = RB / 16;
    const int t = e.rows;
    if (lane < LPR) {
        const uint4 v = *reinterpret_cast<const uint4 *>(k_new + (int64_t)head * RB + lane * 16);
        char *blk = kplane + (int64_t)(t / kBlockRows) * kBlockRows * RB;
        *reinterpret_cast<uint4 *>(blk + (lane * 16 + t % kBlockRows) * 16) = v;
    } else if (lane >= 32 && lane < 32 + LPR) {
        const int piece = lane - 32;
        const uint4 v = *reinterpret_cast<const uint4 *>(v_new + (int64_t)head * RB + piece * 16);
        *reinterpret_cast<uint4 *>(vplane + (int64_t)t * RB + piece * 16) = v;
    }
    // Only this wave reads the row again in this launch: the store has to be complete before
    // those loads are issued, nothing has to be made visible to other compute units.
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
}

// Sliding mode, head full: row `slot` (the oldest window row) first moves into the
// compensation token -- khat += (k - khat) / (N_d + 1), likewise vhat: Eq.(4) over the
// dropped set enlarged by that row -- and is then overwritten by the new token.  Lanes
// 0..LPR-1 handle the K pieces, lanes 32..32+LPR-1 the V pieces.  Called by the one wave whose
// range holds the row's block; comp is not read by anyone else before the combine kernel.
//
// The mean is carried as an unevaluated fp32 pair hi + lo (hi in comp, lo in comp_lo): the
// increment is added with an error-free transformation, so what each addition rounds away
// stays in lo instead of piling up.  A plain fp32 update drifts like the square root of the
// number of steps (about 40 ulp of the mean after a million evictions); the pair stays within
// an ulp of the exact mean of Eq.(4) for generations of any length.
template <int RB, int DTYPE>
__device__ __forceinline__ void evict_row(const razor_head_desc &e, int head, int slot, char *kplane,
                                          char *vplane, const char *__restrict__ k_new,
                                          const char *__restrict__ v_new, float *__restrict__ comp,
                                          float *__restrict__ comp_lo, int lane)
{
    constexpr int LPR = RB / 16;
    constexpr int ES = DTYPE == RAZOR_F32 ? 4 : 2;
    constexpr int NE = 16 / ES, D = RB / ES;
    const int which = lane >> 5, piece = lane & 31;
    if (piece < LPR) {
        char *pos = which ? vplane + (int64_t)slot * RB + piece * 16
                          : kplane + (int64_t)(slot / kBlockRows) * kBlockRows * RB +
                                (piece * 16 + slot % kBlockRows) * 16;
        const uint4 old = *reinterpret_cast<const uint4 *>(pos);
        float x[NE];
        if constexpr (DTYPE == RAZOR_F32) {
            x[0] = __uint_as_float(old.x); x[1] = __uint_as_float(old.y);
            x[2] = __uint_as_float(old.z); x[3] = __uint_as_float(old.w);
        } else {
            x[0] = __uint_as_float(old.x << 16); x[1] = __uint_as_float(old.x & 0xffff0000u);
            x[2] = __uint_as_float(old.y << 16); x[3] = __uint_as_float(old.y & 0xffff0000u);
            x[4] = __uint_as_float(old.z << 16); x[5] = __uint_as_float(old.z & 0xffff0000u);
            x[6] = __uint_as_float(old.w << 16); x[7] = __uint_as_float(old.w & 0xffff0000u);
        }
        const size_t at = ((size_t)head * 2 + which) * D + piece * NE;
        float *hi = comp + at, *lo = comp_lo + at;
        const float inv = 1.f / (float)(e.n_dropped + 1);
#pragma unroll
        for (int k = 0; k < NE; ++k) {
            const float h = hi[k], l = lo[k];
            const float y = ((x[k] - h) - l) * inv + l;   // increment plus what earlier additions lost
            const float t = h + y;
            const float bb = t - h;
            lo[k] = (h - (t - bb)) + (y - bb);            // h + y = t + this, exactly
            hi[k] = t;
        }
        *reinterpret_cast<uint4 *>(pos) =
            *reinterpret_cast<const uint4 *>((which ? v_new : k_new) + (int64_t)head * RB + piece * 16);
    }
    // Only this wave reads the row again in this launch (comp is read by the next kernel).
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
}

// ALiBi (Eq.(1)): how far behind the query (the newest token) cache row `row` lies.
// Sinks keep their prefill position; window rows are in order until the head starts to
// overwrite them (sliding mode), after which they form a ring whose newest row is known.
struct RowDistance {
    int n_sink, rows, total, newest, window;   // newest < 0: rows still in order
    __device__ __forceinline__ RowDistance(const razor_head_desc &e, int rows_now, bool slides, int n_sink_)
    {
        const int evicted = e.evicted + (slides ? 1 : 0);
        n_sink = n_sink_;
        rows = rows_now;
        total = rows_now + e.n_dropped + (slides ? 1 : 0);   // tokens seen so far
        window = e.window;
        newest = evicted > 0 ? n_sink_ + (evicted - 1) % e.window : -1;
    }
    __device__ __forceinline__ float operator()(int row) const
    {
        int dist;
        if (row < n_sink) dist = total - 1 - row;
        else if (newest >= 0) dist = newest - row + (newest < row ? window : 0);
        else dist = rows - 1 - row;
        return (float)dist;
    }
    // Most blocks lie on one straight piece of that map: distance(row) = A - row for every row
    // of block t (no sink row, not the block where the ring wraps).  Returns false otherwise.
    __device__ __forceinline__ bool linear(int t, int &A) const
    {
        const int lo = t * kBlockRows, hi = lo + kBlockRows - 1;
        if (lo < n_sink) return false;
        if (newest < 0) { A = rows - 1; return true; }
        if (hi <= newest) { A = newest; return true; }
        if (lo > newest) { A = newest + window; return true; }
        return false;
    }
};

// ---------------------------------------------------------------- partial, bf16 / matrix cores
//
// Lane l = 16 * kg + n.  For one 16-row block:
//   S[row][head]  = K[row][:] . Q[head][:]    v_mfma_f32_16x16x32_bf16, A = K block, B = Q
//                   lane (kg, n) ends up with head n, rows 4*kg .. 4*kg+3
//   P             = exp2(S - max), split into a bf16 pair hi + lo, still in those lanes: it
//                   is already the B operand of the second product
//   O^T[col][head] += V^T[col][row] . P[row][head]   v_mfma_f32_16x16x32_bf16, A = V^T twice
//                   lane (kg, n) loads 16 bytes of rows 4*kg .. 4*kg+3 (coalesced), and a
//                   4-row in-lane transpose (v_perm_b32) yields A for one column phase e
//                   lane (kg, n) accumulates head n, columns 4*VE*kg .. 4*VE*kg + 4*VE-1
// The K plane is stored piece-major per block, so the A operand of the first product is
// one contiguous 1 KB load per 32 columns.  A single bf16 P (2^-9 per weight) would miss
// the 2e-3 absolute bound on caches with large-magnitude value channels; hi + lo does not.
template <int D, int PF>
__global__ __launch_bounds__(256, 2) void decode_partial_bf16_kernel(
    const uint16_t *__restrict__ Q, char *__restrict__ arena,
    const razor_head_desc *__restrict__ desc, const char *__restrict__ k_new,
    const char *__restrict__ v_new, float *__restrict__ comp, int32_t *__restrict__ prefix,
    int32_t *__restrict__ nd_step, float *__restrict__ part_ml, float *__restrict__ part_acc,
    int n_heads, int n_kv_heads, int g, int n_workers, int sliding, int n_sink,
    const float *__restrict__ slopes, float scale_log2e)
{
    constexpr int RB = D * 2;     // bytes per row
    constexpr int NS = D / 32;    // K loads (= first-product steps) per block
    constexpr int VE = D / 16;    // V elements per lane per row
    using VT = typename std::conditional<VE == 8, u32x4, u32x2>::type;

    const int lane = threadIdx.x & 63;
    const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int kg = lane >> 4, n = lane & 15;
    const int has_new = k_new != nullptr;
#ifdef RAZOR_TIMELINE
    long long stamp_segments = 0;
#endif
    RAZOR_STAMP(0);
    const CachedBlocks count{has_new, sliding, n_sink};
    int total, per, lo, hi, i, first;
    plan_range(count, desc, n_heads, n_workers, w, lane, total, per, lo, hi, i, first);
    if (w == 0) {   // what the combine kernel needs, taken before anything is committed
        write_prefix(count, desc, n_heads, lane, per, prefix);
        for (int idx = lane; idx < n_heads; idx += 64) nd_step[idx] = count.step_n_dropped(desc, idx);
    }
    if (lo >= hi) return;
    RAZOR_STAMP(1);

    // The query group of head `head` as B operand of the first product (zero rows pad the group).
    auto load_query = [&](int head, bf16x8(&q)[NS]) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            uint4 qv = make_uint4(0, 0, 0, 0);
            if (n < g)
                qv = *reinterpret_cast<const uint4 *>(Q + ((int64_t)head * g + n) * D + (4 * s + kg) * 8);
            q[s] = __builtin_bit_cast(bf16x8, qv);
        }
    };
    razor_head_desc e = desc[i];   // head i owns block lo (locate_block never returns an empty head)
    bf16x8 qreg[NS];
    load_query(i, qreg);

    while (lo < hi) {
        const int rows = count.rows_of(e.rows, e.cap, e.flags, e.window);
        const int head_end = first + (rows + kBlockRows - 1) / kBlockRows;
        const int seg_end = hi < head_end ? hi : head_end;
        // A range that runs past this head continues in the next one: fetch that head's entry and
        // query group now, so that the switch does not wait for them.
        const bool more = seg_end < hi;
        razor_head_desc e_next = e;
        bf16x8 q_next[NS];
        if (more) {
            e_next = desc[i + 1];
            load_query(i + 1, q_next);
        }
        const int h = i % n_kv_heads;
        char *kplane = arena + e.row_off * 2 * RB;
        char *vplane = kplane + (int64_t)e.cap * RB;
        if (has_new) {   // the wave that owns the block of the row the new token goes to stores it
            const bool slides = count.slides(e.rows, e.flags, e.window);
            const int slot = slides ? n_sink + e.evicted % e.window : e.rows;
            if ((slides || rows > e.rows) && slot / kBlockRows >= lo - first && slot / kBlockRows < seg_end - first) {
                if (slides) evict_row<RB, RAZOR_BF16>(e, i, slot, kplane, vplane, k_new, v_new, comp, comp + (size_t)n_heads * 2 * D, lane);
                else append_row<RB>(e, i, kplane, vplane, k_new, v_new, lane);
            }
        }

        const bool slides_now = count.slides(e.rows, e.flags, e.window);
        const RowDistance distance(e, rows, slides_now, n_sink);
        const float slope_l2e = (slopes && n < g) ? slopes[h * g + n] * 1.4426950408889634f : 0.f;

        float m = kNegInf, l = 0.f;
        f32x4 acc[VE];
#pragma unroll
        for (int c = 0; c < VE; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};

        u32x4 kb[PF][NS];
        VT vb[PF][4];
        auto load_block = [&](int t, u32x4(&k)[NS], VT(&v)[4]) {
            const u32x4 *kp = reinterpret_cast<const u32x4 *>(kplane + (int64_t)t * kBlockRows * RB) + lane;
#pragma unroll
            for (int s = 0; s < NS; ++s) k[s] = stream_load(kp + s * 64);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                int row = t * kBlockRows + 4 * kg + r;
                row = row < rows ? row : rows - 1;   // stay on initialised, finite rows
                v[r] = stream_load(reinterpret_cast<const VT *>(vplane + (int64_t)row * RB) + n);
            }
        };
        auto compute_block = [&](int t, const u32x4(&k)[NS], const VT(&v)[4]) {
            f32x4 S = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < NS; ++s)
                S = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k[s]), qreg[s], S, 0, 0, 0);
            float sv[4];
            const int row0 = t * kBlockRows + 4 * kg;
            float bmax = kNegInf;
#pragma unroll
            for (int r = 0; r < 4; ++r) sv[r] = S[r] * scale_log2e;
            if (slopes) {   // Eq.(1): minus slope * distance to the query
                int A;
                if (distance.linear(t, A)) {
                    const float c0 = slope_l2e * (float)(A - row0);
#pragma unroll
                    for (int r = 0; r < 4; ++r) sv[r] -= c0 - slope_l2e * (float)r;
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) sv[r] -= slope_l2e * distance(row0 + r);
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                sv[r] = row0 + r < rows ? sv[r] : kNegInf;
                bmax = fmaxf(bmax, sv[r]);
            }
            bmax = fmaxf(bmax, __shfl_xor(bmax, 16));
            bmax = fmaxf(bmax, __shfl_xor(bmax, 32));
            const float m_new = fmaxf(m, bmax);     // finite: every block holds a valid row
            const float alpha = fast_exp2(m - m_new);
            m = m_new;
            // P goes to the matrix core as a bf16 pair hi + lo (p = hi + lo to 2^-17), stacked along
            // the contraction axis against two copies of the V rows, so one 16x16x32 product
            // accumulates V^T.(P_hi + P_lo); the denominator sums the fp32 p.
            bf16x8 pk;
            float psum = 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float pr = fast_exp2(sv[r] - m_new);
                const __bf16 hi = (__bf16)pr;
                pk[r] = hi;
                pk[4 + r] = (__bf16)(pr - (float)hi);
                psum += pr;
            }
            l = l * alpha + psum;
#pragma unroll
            for (int c = 0; c < VE; ++c) {
                const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
                const uint32_t w0 = reinterpret_cast<const uint32_t *>(&v[0])[c >> 1];
                const uint32_t w1 = reinterpret_cast<const uint32_t *>(&v[1])[c >> 1];
                const uint32_t w2 = reinterpret_cast<const uint32_t *>(&v[2])[c >> 1];
                const uint32_t w3 = reinterpret_cast<const uint32_t *>(&v[3])[c >> 1];
                u32x4 packed;
                packed.x = __builtin_amdgcn_perm(w1, w0, sel);   // rows 4kg, 4kg+1 of column phase c
                packed.y = __builtin_amdgcn_perm(w3, w2, sel);   // rows 4kg+2, 4kg+3
                packed.z = packed.x;
                packed.w = packed.y;
                acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                    __builtin_bit_cast(bf16x8, packed), pk, acc[c] * alpha, 0, 0, 0);
            }
        };

        const int t0 = lo - first, t1 = seg_end - first;
#pragma unroll
        for (int u = 0; u < PF; ++u)
            if (t0 + u < t1) load_block(t0 + u, kb[u], vb[u]);
        for (int t = t0; t < t1; t += PF) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                if (t + u < t1) {
                    compute_block(t + u, kb[u], vb[u]);
                    if (t + u + PF < t1) load_block(t + u + PF, kb[u], vb[u]);
                }
            }
        }

        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (n < g) {
            const size_t slot = (size_t)(w + i) * g + n;
            float *pa = part_acc + slot * D + 4 * VE * kg;
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < VE; c += 4)
                    *reinterpret_cast<float4 *>(pa + VE * r + c) =
                        make_float4(acc[c][r], acc[c + 1][r], acc[c + 2][r], acc[c + 3][r]);
            if (kg == 0) {
                part_ml[slot * 2] = m;
                part_ml[slot * 2 + 1] = l;
            }
        }
        lo = seg_end;
        RAZOR_STAMP_SEG();
        if (more) {
            first = head_end;
            e = e_next;
            ++i;
#pragma unroll
            for (int s = 0; s < NS; ++s) qreg[s] = q_next[s];
            while (count.rows_of(e.rows, e.cap, e.flags, e.window) == 0) {   // heads that hold no row
                e = desc[++i];
                load_query(i, qreg);
            }
        }
    }
    RAZOR_STAMP(2);
    RAZOR_STAMP_FLUSH();
}

// ---------------------------------------------------------------- partial, fp32 / matrix cores
//
// Same scheme as the bf16 kernel with v_mfma_f32_16x16x4_f32 (one float of A and of B per lane,
// contraction length 4).  Lane l = 16 * kg + n.  For one 16-row block:
//   S[row][head] = K[row][:] . Q[head][:]   lane (kg, n) loads 16 bytes = columns
//                  16 s + 4 kg .. + 3 of row n (the piece-major K plane makes that one contiguous
//                  kilobyte per load) and feeds them to four products in turn, against the same
//                  four columns of query n; the order of the contraction is immaterial as long as
//                  A and B agree.  The lane ends up with head n, rows 4 kg .. 4 kg + 3.
//   O^T[col][head] += V^T[col][row] . P[row][head]   lane (kg, n) loads columns 64 q + 4 n .. + 3
//                  of rows 4 kg .. 4 kg + 3 (coalesced: 256 contiguous bytes per row), one product
//                  per loaded element and row; its exp2 values are already the B operand.
//                  Accumulator (q, e) of lane (kg, n) holds head n, columns 64 q + 16 kg + 4 j + e.
// 64 matrix instructions per 16-row block (D = 128) at 32 cycles each: about half of the time the
// block's 16 KB take to arrive at this SIMD's share of the HBM rate.  Two blocks in flight, the
// query group of this head and of the next and the accumulators need more than 256 registers:
// one wavefront per SIMD, which is how the kernel is launched anyway.
template <int D, int PF>
__global__ __launch_bounds__(256, 1) void decode_partial_f32_kernel(
    const float *__restrict__ Q, char *__restrict__ arena,
    const razor_head_desc *__restrict__ desc, const char *__restrict__ k_new,
    const char *__restrict__ v_new, float *__restrict__ comp, int32_t *__restrict__ prefix,
    int32_t *__restrict__ nd_step, float *__restrict__ part_ml, float *__restrict__ part_acc,
    int n_heads, int n_kv_heads, int g, int n_workers, int sliding, int n_sink,
    const float *__restrict__ slopes, float scale_log2e)
{
    constexpr int RB = D * 4;     // bytes per row
    constexpr int NS = D / 16;    // K loads per block, four first-product steps each
    constexpr int VQ = D / 64;    // V loads per lane per row
    constexpr int VE = 4 * VQ;    // V elements per lane per row = accumulators

    const int lane = threadIdx.x & 63;
    const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int kg = lane >> 4, n = lane & 15;
    const int has_new = k_new != nullptr;
#ifdef RAZOR_TIMELINE
    long long stamp_segments = 0;
#endif
    RAZOR_STAMP(0);
    const CachedBlocks count{has_new, sliding, n_sink};
    int total, per, lo, hi, i, first;
    plan_range(count, desc, n_heads, n_workers, w, lane, total, per, lo, hi, i, first);
    if (w == 0) {   // what the combine kernel needs, taken before anything is committed
        write_prefix(count, desc, n_heads, lane, per, prefix);
        for (int idx = lane; idx < n_heads; idx += 64) nd_step[idx] = count.step_n_dropped(desc, idx);
    }
    if (lo >= hi) return;
    RAZOR_STAMP(1);

    // The query group of head `head` as B operand of the first product (zero rows pad the group).
    auto load_query = [&](int head, f32x4(&q)[NS]) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            q[s] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (n < g) q[s] = *reinterpret_cast<const f32x4 *>(Q + ((int64_t)head * g + n) * D + (4 * s + kg) * 4);
        }
    };
    razor_head_desc e = desc[i];   // head i owns block lo (locate_block never returns an empty head)
    f32x4 qreg[NS];
    load_query(i, qreg);

    while (lo < hi) {
        const int rows = count.rows_of(e.rows, e.cap, e.flags, e.window);
        const int head_end = first + (rows + kBlockRows - 1) / kBlockRows;
        const int seg_end = hi < head_end ? hi : head_end;
        // A range that runs past this head continues in the next one: fetch that head's entry and
        // query group now, so that the switch does not wait for them.
        const bool more = seg_end < hi;
        razor_head_desc e_next = e;
        f32x4 q_next[NS];
        if (more) {
            e_next = desc[i + 1];
            load_query(i + 1, q_next);
        }
        const int h = i % n_kv_heads;
        char *kplane = arena + e.row_off * 2 * RB;
        char *vplane = kplane + (int64_t)e.cap * RB;
        if (has_new) {   // the wave that owns the block of the row the new token goes to stores it
            const bool slides = count.slides(e.rows, e.flags, e.window);
            const int slot = slides ? n_sink + e.evicted % e.window : e.rows;
            if ((slides || rows > e.rows) && slot / kBlockRows >= lo - first && slot / kBlockRows < seg_end - first) {
                if (slides) evict_row<RB, RAZOR_F32>(e, i, slot, kplane, vplane, k_new, v_new, comp, comp + (size_t)n_heads * 2 * D, lane);
                else append_row<RB>(e, i, kplane, vplane, k_new, v_new, lane);
            }
        }

        const bool slides_now = count.slides(e.rows, e.flags, e.window);
        const RowDistance distance(e, rows, slides_now, n_sink);
        const float slope_l2e = (slopes && n < g) ? slopes[h * g + n] * 1.4426950408889634f : 0.f;

        float m = kNegInf, l = 0.f;
        f32x4 acc[VE];
#pragma unroll
        for (int c = 0; c < VE; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};

        f32x4 kb[PF][NS], vb[PF][4][VQ];
        auto load_block = [&](int t, f32x4(&k)[NS], f32x4(&v)[4][VQ]) {
            const f32x4 *kp = reinterpret_cast<const f32x4 *>(kplane + (int64_t)t * kBlockRows * RB) + lane;
#pragma unroll
            for (int s = 0; s < NS; ++s) k[s] = stream_load(kp + s * 64);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                int row = t * kBlockRows + 4 * kg + r;
                row = row < rows ? row : rows - 1;   // stay on initialised, finite rows
#pragma unroll
                for (int q = 0; q < VQ; ++q)
                    v[r][q] = stream_load(reinterpret_cast<const f32x4 *>(vplane + (int64_t)row * RB) + 16 * q + n);
            }
        };
        auto compute_block = [&](int t, const f32x4(&k)[NS], const f32x4(&v)[4][VQ]) {
            f32x4 S = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < NS; ++s)
#pragma unroll
                for (int j = 0; j < 4; ++j) S = __builtin_amdgcn_mfma_f32_16x16x4f32(k[s][j], qreg[s][j], S, 0, 0, 0);
            float sv[4];
            const int row0 = t * kBlockRows + 4 * kg;
            float bmax = kNegInf;
#pragma unroll
            for (int r = 0; r < 4; ++r) sv[r] = S[r] * scale_log2e;
            if (slopes) {   // Eq.(1): minus slope * distance to the query
                int A;
                if (distance.linear(t, A)) {
                    const float c0 = slope_l2e * (float)(A - row0);
#pragma unroll
                    for (int r = 0; r < 4; ++r) sv[r] -= c0 - slope_l2e * (float)r;
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) sv[r] -= slope_l2e * distance(row0 + r);
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                sv[r] = row0 + r < rows ? sv[r] : kNegInf;
                bmax = fmaxf(bmax, sv[r]);
            }
            bmax = fmaxf(bmax, __shfl_xor(bmax, 16));
            bmax = fmaxf(bmax, __shfl_xor(bmax, 32));
            const float m_new = fmaxf(m, bmax);     // finite: every block holds a valid row
            const float alpha = fast_exp2(m - m_new);
            m = m_new;
            float pr[4], psum = 0.f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                pr[r] = fast_exp2(sv[r] - m_new);
                psum += pr[r];
            }
            l = l * alpha + psum;
#pragma unroll
            for (int q = 0; q < VQ; ++q)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    f32x4 o = acc[4 * q + c] * alpha;
#pragma unroll
                    for (int r = 0; r < 4; ++r) o = __builtin_amdgcn_mfma_f32_16x16x4f32(v[r][q][c], pr[r], o, 0, 0, 0);
                    acc[4 * q + c] = o;
                }
        };

        const int t0 = lo - first, t1 = seg_end - first;
#pragma unroll
        for (int u = 0; u < PF; ++u)
            if (t0 + u < t1) load_block(t0 + u, kb[u], vb[u]);
        for (int t = t0; t < t1; t += PF) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                if (t + u < t1) {
                    compute_block(t + u, kb[u], vb[u]);
                    if (t + u + PF < t1) load_block(t + u + PF, kb[u], vb[u]);
                }
            }
        }

        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (n < g) {
            const size_t slot = (size_t)(w + i) * g + n;
            float *pa = part_acc + slot * D + 16 * kg;
#pragma unroll
            for (int q = 0; q < VQ; ++q)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    *reinterpret_cast<float4 *>(pa + 64 * q + 4 * j) =
                        make_float4(acc[4 * q][j], acc[4 * q + 1][j], acc[4 * q + 2][j], acc[4 * q + 3][j]);
            if (kg == 0) {
                part_ml[slot * 2] = m;
                part_ml[slot * 2 + 1] = l;
            }
        }
        lo = seg_end;
        RAZOR_STAMP_SEG();
        if (more) {
            first = head_end;
            e = e_next;
            ++i;
#pragma unroll
            for (int s = 0; s < NS; ++s) qreg[s] = q_next[s];
            while (count.rows_of(e.rows, e.cap, e.flags, e.window) == 0) {   // heads that hold no row
                e = desc[++i];
                load_query(i, qreg);
            }
        }
    }
    RAZOR_STAMP(2);
    RAZOR_STAMP_FLUSH();
}

// ---------------------------------------------------------------- combine
__device__ __forceinline__ float load_q(const void *Q, int dtype, int64_t idx)
{
    if (dtype == RAZOR_F32) return static_cast<const float *>(Q)[idx];
    return __uint_as_float((uint32_t) static_cast<const uint16_t *>(Q)[idx] << 16);
}

// One workgroup per query head.  Eq.(5): the compensation token is one more softmax entry with
// logit scale * q.khat + ln N_d and value vhat.  The partial states of the head's segments are
// merged in one pass: the workgroup's threads form GR slot groups x D / 4 columns (GR = 32 with
// 1024 threads; launches with many query heads use 256 threads, GR = 8, so that all workgroups
// are resident at once); each group folds its slots (in slot order) into a running state, the GR
// states are merged around their common maximum in group order.
constexpr int kCombineThreads = 1024;
constexpr int kCombineAhead = 4;   // partial states a thread fetches at a time
#ifndef RAZOR_COMBINE_WIDE_UP_TO
#define RAZOR_COMBINE_WIDE_UP_TO 256
#endif
constexpr int kCombineWideUpTo = RAZOR_COMBINE_WIDE_UP_TO;   // query heads up to which a workgroup gets 1024 threads

template <int D>
__global__ __launch_bounds__(kCombineThreads) void combine_kernel(
    const void *__restrict__ Q, int q_dtype, const float *__restrict__ comp,
    razor_head_desc *__restrict__ desc, const int32_t *__restrict__ prefix,
    const int32_t *__restrict__ nd_step, const float *__restrict__ part_ml,
    const float *__restrict__ part_acc, void *__restrict__ O, int out_dtype, int n_heads,
    int n_kv_heads, int g, int has_new, int use_comp, int sliding, int n_sink, float scale_log2e)
{
    constexpr int C4 = D / 4;                      // float4 columns
    constexpr int NG = kCombineThreads / C4;       // most slot groups a workgroup can have
    __shared__ float s_comp;
    __shared__ float s_m[NG], s_l[NG];
    __shared__ float4 s_acc[NG][C4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int GR = blockDim.x / C4;                // slot groups working in parallel
    const int n_q_heads = n_kv_heads * g;
    const int bj = blockIdx.x, b = bj / n_q_heads, j = bj % n_q_heads;
    const int h = j / g, n = j % g, i = b * n_kv_heads + h;
    const razor_head_desc e = desc[i];
    const int n_dropped = nd_step[i];   // N_d of this step (a row evicted this step included)
    const bool has_comp = use_comp && n_dropped > 0;
    const int first = prefix[i], last = prefix[i + 1], per = prefix[n_heads + 1];
    const int w0 = first / per;
    const int n_slots = last > first ? (last - 1) / per - w0 + 1 : 0;

    // wave 0 starts q . khat; its loads travel together with the partial states below
    float dot = 0.f;
    if (wave == 0 && has_comp)
        for (int c = lane; c < D; c += 64)
            dot += load_q(Q, q_dtype, (int64_t)bj * D + c) * comp[(size_t)i * 2 * D + c];

    // vhat is needed last; its load goes out with the others instead of after the barrier
    const int col = tid % C4, grp = tid / C4;
    float4 vhat = make_float4(0.f, 0.f, 0.f, 0.f);
    if (has_comp && grp == 0) vhat = *reinterpret_cast<const float4 *>(comp + ((size_t)i * 2 + 1) * D + 4 * col);

    // every slot group folds its share of the head's partial states into one running state: slots
    // grp, grp + GR, ... in that order; the loads of kCombineAhead slots are issued together so
    // that a long head costs a few memory round trips, not one per slot
    float mg = kNegInf, lg = 0.f;
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s0 = grp; s0 < n_slots; s0 += kCombineAhead * GR) {
        float2 ml[kCombineAhead];
        float4 v[kCombineAhead];
#pragma unroll
        for (int u = 0; u < kCombineAhead; ++u) {
            const int s = s0 + u * GR < n_slots ? s0 + u * GR : s0;   // past the end: a valid slot, not used
            const size_t slot = (size_t)(w0 + s + i) * g + n;
            ml[u] = *reinterpret_cast<const float2 *>(part_ml + slot * 2);
            v[u] = *reinterpret_cast<const float4 *>(part_acc + slot * D + 4 * col);
        }
#pragma unroll
        for (int u = 0; u < kCombineAhead; ++u) {
            if (s0 + u * GR < n_slots) {
                const float m_new = fmaxf(mg, ml[u].x);
                const float so = fast_exp2(mg - m_new), sn = fast_exp2(ml[u].x - m_new);   // mg = -inf gives 0
                a.x = a.x * so + v[u].x * sn; a.y = a.y * so + v[u].y * sn;
                a.z = a.z * so + v[u].z * sn; a.w = a.w * so + v[u].w * sn;
                lg = lg * so + ml[u].y * sn;
                mg = m_new;
            }
        }
    }
    if (wave == 0) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) dot += __shfl_xor(dot, o);
        if (lane == 0) s_comp = dot;
    }
    s_acc[grp][col] = a;
    if (col == 0) {
        s_m[grp] = mg;
        s_l[grp] = lg;
    }
    __syncthreads();
    if (grp == 0) {
        // Eq.(5): the compensation token is one more entry, logit scale * q.khat + ln N_d, value vhat
        const float m_comp = has_comp ? s_comp * scale_log2e + log2f((float)n_dropped) : kNegInf;
        float M = m_comp;
        for (int k = 0; k < GR; ++k) M = fmaxf(M, s_m[k]);
        float den = 0.f;
        float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
        if (M > kNegInf) {
            for (int k = 0; k < GR; ++k) {
                const float wgt = fast_exp2(s_m[k] - M);   // empty groups: exp2(-inf) = 0
                const float4 v = s_acc[k][col];
                num.x += wgt * v.x; num.y += wgt * v.y; num.z += wgt * v.z; num.w += wgt * v.w;
                den += wgt * s_l[k];
            }
            if (has_comp) {
                const float wgt = fast_exp2(m_comp - M);
                num.x += wgt * vhat.x; num.y += wgt * vhat.y; num.z += wgt * vhat.z; num.w += wgt * vhat.w;
                den += wgt;
            }
        }
        const float inv = den > 0.f ? 1.f / den : 0.f;   // a head with no entry at all gives zeros
        num.x *= inv; num.y *= inv; num.z *= inv; num.w *= inv;
        if (out_dtype == RAZOR_F32) {
            *reinterpret_cast<float4 *>(static_cast<float *>(O) + (int64_t)bj * D + 4 * col) = num;
        } else {
            const __bf16 o0 = (__bf16)num.x, o1 = (__bf16)num.y, o2 = (__bf16)num.z, o3 = (__bf16)num.w;
            uint2 pk;
            pk.x = (uint32_t)__builtin_bit_cast(uint16_t, o0) | ((uint32_t)__builtin_bit_cast(uint16_t, o1) << 16);
            pk.y = (uint32_t)__builtin_bit_cast(uint16_t, o2) | ((uint32_t)__builtin_bit_cast(uint16_t, o3) << 16);
            *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(O) + (int64_t)bj * D + 4 * col) = pk;
        }
    }
    // The step is over for this head: make the append permanent.  No other workgroup of this
    // kernel reads what changes here (block positions come from `prefix`, N_d from `nd_step`).
    if (has_new && n == 0 && tid == 0) {
        const CachedBlocks count{has_new, sliding, n_sink};
        if (count.slides(e.rows, e.flags, e.window)) {
            desc[i].n_dropped = e.n_dropped + 1;
            desc[i].evicted = e.evicted + 1;
            desc[i].flags = e.flags | RAZOR_HEAD_COMP;
        } else if (e.rows < e.cap) {
            desc[i].rows = e.rows + 1;
        } else {
            desc[i].flags = e.flags | RAZOR_HEAD_OVERFLOW;
        }
    }
}

#define RAZOR_HIP_CHECK(expr)                                              \
    do {                                                                   \
        hipError_t err__ = (expr);                                         \
        if (err__ != hipSuccess) return hip_failure(#expr, (int)err__);    \
    } while (0)

thread_local hipEvent_t g_profile_start = nullptr, g_profile_stop = nullptr;

// Argument checks shared by the decode entry points (everything but the workspace).
int check_decode_args(const razor_params *p, const void *Q, const void *k_new, const void *v_new,
                      const void *arena, const float *comp, const razor_head_desc *desc_dev, const void *O)
{
    if (check_params(p) != RAZOR_OK) return RAZOR_EINVAL;
    if (!Q || !arena || !comp || !desc_dev || !O) return RAZOR_EINVAL;
    if ((k_new == nullptr) != (v_new == nullptr)) return RAZOR_EINVAL;
    if (((uintptr_t)Q | (uintptr_t)arena | (uintptr_t)comp | (uintptr_t)O | (uintptr_t)desc_dev |
         (uintptr_t)k_new | (uintptr_t)v_new) & 15)
        return RAZOR_EINVAL;
    if ((uintptr_t)p->alibi_slopes & 3) return RAZOR_EINVAL;
    return RAZOR_OK;
}

// Wavefronts the streaming kernel is split over.
int decode_workers(const razor_params *p, int *out)
{
    int workers = p->n_workers;
    if (workers == 0) {
        int rc = auto_workers(&workers);
        if (rc != RAZOR_OK) return rc;
        // A 16-row block of 128-byte rows (bf16, head_dim 64) is only 4 KB, and the chain of
        // dependent steps per block costs a wave as long as for 8 KB: a second wave per SIMD
        // hides it (859 MB cache: 4.4 TB/s with one wave per SIMD, 6.4 with two; every other
        // row size is at its best with one).
        if (p->dtype == RAZOR_BF16 && p->head_dim == 64) workers *= 2;
    }
    *out = std::max(4, std::min(workers, RAZOR_MAX_WORKERS));
    return RAZOR_OK;
}

// The two launches of a decode step; `scratch` holds the layout `ws` (caller's workspace or the
// library's static array).
int launch_decode(const razor_params *p, const void *Q, const void *k_new, const void *v_new, void *arena,
                  float *comp, razor_head_desc *desc_dev, void *O, void *scratch, const DecodeWorkspace &ws,
                  int workers, void *stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int n_heads = p->batch * p->n_kv_heads, g = p->n_q_heads / p->n_kv_heads;
    const int D = p->head_dim, has_new = k_new != nullptr;
    char *wsb = static_cast<char *>(scratch);
    int32_t *prefix = reinterpret_cast<int32_t *>(wsb + ws.prefix_off);
    int32_t *nd = reinterpret_cast<int32_t *>(wsb + ws.nd_off);
    float *ml = reinterpret_cast<float *>(wsb + ws.ml_off);
    float *acc = reinterpret_cast<float *>(wsb + ws.acc_off);
    char *a = static_cast<char *>(arena);
    const char *kn = static_cast<const char *>(k_new), *vn = static_cast<const char *>(v_new);
    const float sl2e = p->scale * 1.4426950408889634f;

    const dim3 grid((workers + 3) / 4);
    if (g_profile_start) RAZOR_HIP_CHECK(hipEventRecord(g_profile_start, s));
    if (p->dtype == RAZOR_BF16) {
        const uint16_t *q = static_cast<const uint16_t *>(Q);
        if (D == 128)
            hipLaunchKernelGGL((decode_partial_bf16_kernel<128, 2>), grid, dim3(256), 0, s, q, a, desc_dev,
                               kn, vn, comp, prefix, nd, ml, acc, n_heads, p->n_kv_heads, g, workers,
                               p->sliding, p->n_sink, p->alibi_slopes, sl2e);
        else
            hipLaunchKernelGGL((decode_partial_bf16_kernel<64, 2>), grid, dim3(256), 0, s, q, a, desc_dev,
                               kn, vn, comp, prefix, nd, ml, acc, n_heads, p->n_kv_heads, g, workers,
                               p->sliding, p->n_sink, p->alibi_slopes, sl2e);
    } else {
        const float *q = static_cast<const float *>(Q);
        if (D == 128)
            hipLaunchKernelGGL((decode_partial_f32_kernel<128, 2>), grid, dim3(256), 0, s, q, a, desc_dev,
                               kn, vn, comp, prefix, nd, ml, acc, n_heads, p->n_kv_heads, g, workers,
                               p->sliding, p->n_sink, p->alibi_slopes, sl2e);
        else
            hipLaunchKernelGGL((decode_partial_f32_kernel<64, 2>), grid, dim3(256), 0, s, q, a, desc_dev,
                               kn, vn, comp, prefix, nd, ml, acc, n_heads, p->n_kv_heads, g, workers,
                               p->sliding, p->n_sink, p->alibi_slopes, sl2e);
    }
    if (g_profile_stop) RAZOR_HIP_CHECK(hipEventRecord(g_profile_stop, s));

    // 1024 threads per query head while those fit the chip in one go, else 256
    const dim3 cgrid(p->batch * p->n_q_heads), cblock(p->batch * p->n_q_heads <= kCombineWideUpTo ? kCombineThreads : 256);
    if (D == 128)
        hipLaunchKernelGGL((combine_kernel<128>), cgrid, cblock, 0, s, Q, p->dtype, comp,
                           desc_dev, prefix, nd, ml, acc, O, p->out_dtype, n_heads, p->n_kv_heads, g, has_new,
                           p->use_comp, p->sliding, p->n_sink, sl2e);
    else
        hipLaunchKernelGGL((combine_kernel<64>), cgrid, cblock, 0, s, Q, p->dtype, comp,
                           desc_dev, prefix, nd, ml, acc, O, p->out_dtype, n_heads, p->n_kv_heads, g, has_new,
                           p->use_comp, p->sliding, p->n_sink, sl2e);
    RAZOR_HIP_CHECK(hipGetLastError());
    return RAZOR_OK;
}

// ---------------------------------------------------------------- scratch owned by the library
//
// razor_decode_attn_static keeps the split-K scratch of a step (block-prefix table, per-step N_d,
// partial softmax states) in this array instead of a caller-provided workspace.  Every device
// the library runs on holds its own copy at its own address until the process ends; the host
// learns that address once per device and passes it to the kernels like any other buffer.
static __device__ __align__(256) unsigned char scratch[RAZOR_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device.
int static_scratch(void **out)
{
    int dev = 0;
    RAZOR_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return RAZOR_EINVAL;
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        ptr = g_scratch_ptr[dev].load(std::memory_order_relaxed);
        if (!ptr) {
            RAZOR_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
            if (!ptr) return hip_failure("hipGetSymbolAddress(scratch) returned NULL", (int)hipErrorInvalidSymbol);
            g_scratch_ptr[dev].store(ptr, std::memory_order_release);
        }
    }
    *out = ptr;
    return RAZOR_OK;
}

}  // namespace
}  // namespace razor

extern "C" int razor_decode_attn(const razor_params *p, const void *Q, const void *k_new,
                                 const void *v_new, void *arena, float *comp,
                                 razor_head_desc *desc_dev, void *O, void *workspace,
                                 size_t workspace_bytes, void *stream)
{
    using namespace razor;
    int rc = check_decode_args(p, Q, k_new, v_new, arena, comp, desc_dev, O);
    if (rc != RAZOR_OK) return rc;
    if (!workspace || ((uintptr_t)workspace & 15)) return RAZOR_EINVAL;
    const DecodeWorkspace ws = decode_workspace(*p);
    if (workspace_bytes < ws.bytes)
        return capacity_failure("razor_decode_attn: workspace smaller than razor_plan reported");
    int workers = 0;
    rc = decode_workers(p, &workers);
    if (rc != RAZOR_OK) return rc;
    return launch_decode(p, Q, k_new, v_new, arena, comp, desc_dev, O, workspace, ws, workers, stream);
}

extern "C" int razor_decode_attn_static(const razor_params *p, const void *Q, const void *k_new,
                                        const void *v_new, void *arena, float *comp,
                                        razor_head_desc *desc_dev, void *O, void *stream)
{
    using namespace razor;
    int rc = check_decode_args(p, Q, k_new, v_new, arena, comp, desc_dev, O);
    if (rc != RAZOR_OK) return rc;
    int workers = 0;
    rc = decode_workers(p, &workers);
    if (rc != RAZOR_OK) return rc;
    // the layout is cut for the wavefronts this launch really uses, not for the largest count
    const DecodeWorkspace ws = decode_workspace(*p, workers);
    if (ws.bytes > (size_t)RAZOR_STATIC_SCRATCH_BYTES)
        return capacity_failure("razor_decode_attn_static: this step needs more split-K scratch than "
                                "RAZOR_STATIC_SCRATCH_BYTES; lower n_workers or call razor_decode_attn");
    void *ptr = nullptr;
    rc = static_scratch(&ptr);
    if (rc != RAZOR_OK) return rc;
    return launch_decode(p, Q, k_new, v_new, arena, comp, desc_dev, O, ptr, ws, workers, stream);
}

#ifdef RAZOR_TIMELINE
// Debug build only: byte offset inside the decode workspace of the per-wave clock stamps
// (four int64 per wave: start, range located, end, head segments crossed).
extern "C" RAZOR_API uint64_t razor_timeline_offset(const razor_params *p)
{
    using namespace razor;
    if (check_params(p) != RAZOR_OK) return 0;
    const int g = p->n_q_heads / p->n_kv_heads;
    return decode_workspace(*p).acc_off + timeline_floats(p->batch * p->n_kv_heads, g, p->head_dim) * sizeof(float);
}
#endif

extern "C" int razor_profile_events(void *ev_start, void *ev_stop)
{
    razor::g_profile_start = static_cast<hipEvent_t>(ev_start);
    razor::g_profile_stop = static_cast<hipEvent_t>(ev_stop);
    return RAZOR_OK;
}
