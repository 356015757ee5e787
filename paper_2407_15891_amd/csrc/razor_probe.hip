// Measurement hooks: what the device's memory system gives kernels that only move bytes.  A read
// stream and a copy, 128-bit accesses in 4 KB wave-wide pieces, with the hand-out of pieces to
// wavefronts, the number of pieces in flight and the cache hints as parameters, so that the
// streaming kernels' own choices can be held against the alternatives on the same device.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "razor_bench.h"
#include "razor_device.h"

namespace razor {
namespace {

constexpr int kPieceBytes = 4096;   // one wave-wide step: 4 loads of 16 bytes per lane

template <bool NT>
__device__ __forceinline__ u32x4 probe_load(const u32x4 *p)
{
    if constexpr (NT) return stream_load(p);
    return *p;
}

template <bool NT>
__device__ __forceinline__ void probe_store(u32x4 *p, const u32x4 v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// Piece k of wavefront w.  chunk = 0, group = 0: its own contiguous range [w * per, ...).
// chunk = n: interleaved in chunks of n pieces -- the pieces of chunks w, w + n_waves, w + 2 n_waves, ...
// group = G: the wavefronts form groups of G; a group owns one contiguous range and its G waves
// take that range's pieces in turn (wave j of the group: pieces j, j + G, j + 2 G, ... of it).
struct PieceMap {
    int64_t n_pieces, per, n_waves;
    int chunk, group;
    __device__ __forceinline__ void group_range(int64_t w, int64_t &lo, int64_t &hi) const
    {
        const int64_t n_groups = (n_waves + group - 1) / group, per_group = (n_pieces + n_groups - 1) / n_groups;
        lo = w / group * per_group;
        hi = lo + per_group < n_pieces ? lo + per_group : n_pieces;
    }
    __device__ __forceinline__ int64_t count(int64_t w) const
    {
        if (group) {
            int64_t lo, hi;
            group_range(w, lo, hi);
            const int64_t j = w % group;
            return hi - lo > j ? (hi - lo - j + group - 1) / group : 0;
        }
        if (chunk) {
            const int64_t n_chunks = (n_pieces + chunk - 1) / chunk;
            if (w >= n_chunks) return 0;
            const int64_t mine = (n_chunks - w + n_waves - 1) / n_waves;             // chunks of this wave
            const int64_t last = w + (mine - 1) * n_waves;                            // its last chunk
            const int64_t tail = last == n_chunks - 1 ? n_pieces - last * chunk : chunk;   // pieces in it
            return (mine - 1) * chunk + tail;
        }
        const int64_t lo = w * per, hi = lo + per < n_pieces ? lo + per : n_pieces;
        return hi > lo ? hi - lo : 0;
    }
    // piece k of wavefront w = start + (k / run) * jump + k % run for every hand-out: `run` consecutive
    // pieces, then a jump (contiguous: one run; grouped: runs of one piece, G apart)
    __device__ __forceinline__ void walk(int64_t w, int64_t &start, int &run, int64_t &jump) const
    {
        if (group) {
            int64_t lo, hi;
            group_range(w, lo, hi);
            start = lo + w % group;
            run = 1;
            jump = group;
        } else if (chunk) {
            start = w * chunk;
            run = chunk;
            jump = n_waves * chunk;
        } else {
            start = w * per;
            run = 0x7fffffff;
            jump = 0;
        }
    }
};

// The pieces of one wavefront in order, without a division per piece.
struct PieceWalk {
    int64_t at, jump;
    int run, left;
    __device__ __forceinline__ PieceWalk(const PieceMap &map, int64_t w)
    {
        map.walk(w, at, run, jump);
        left = run;
    }
    __device__ __forceinline__ int64_t next()   // the current piece; moves on
    {
        const int64_t p = at;
        if (--left == 0) {
            at += jump - (run - 1);
            left = run;
        } else {
            ++at;
        }
        return p;
    }
};

template <int DEPTH, bool NT>
__global__ __launch_bounds__(256) void read_stream_kernel(const u32x4 *__restrict__ p, PieceMap map,
                                                          uint32_t *__restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t n = map.count(w);
    uint32_t acc = 0;
    PieceWalk walk(map, w);
    int64_t piece = 0;
    for (int64_t k = 0; k < n; k += DEPTH) {
        u32x4 v[DEPTH][4];
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
            if (k + u < n) piece = walk.next();   // past the end: the last piece once more
            const u32x4 *q = p + piece * (kPieceBytes / 16) + lane;
#pragma unroll
            for (int s = 0; s < 4; ++s) v[u][s] = probe_load<NT>(q + s * 64);
        }
#pragma unroll
        for (int u = 0; u < DEPTH; ++u)
#pragma unroll
            for (int s = 0; s < 4; ++s) acc += v[u][s].x ^ v[u][s].y ^ v[u][s].z ^ v[u][s].w;
    }
    if (acc == 0x9e3779b9u) sink[w] = acc;   // keeps the loads alive; practically never taken
}

template <bool NT_LOAD, bool NT_STORE>
__global__ __launch_bounds__(256) void copy_stream_kernel(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src,
                                                          PieceMap map)
{
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t n = map.count(w);
    PieceWalk walk(map, w);
    for (int64_t k = 0; k < n; k += 2) {
        u32x4 v[2][4];
        int64_t piece[2] = {0, 0};
        const int m = k + 1 < n ? 2 : 1;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (u < m) {
                piece[u] = walk.next();
                const u32x4 *q = src + piece[u] * (kPieceBytes / 16) + lane;
#pragma unroll
                for (int s = 0; s < 4; ++s) v[u][s] = probe_load<NT_LOAD>(q + s * 64);
            }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (u < m) {
                u32x4 *q = dst + piece[u] * (kPieceBytes / 16) + lane;
#pragma unroll
                for (int s = 0; s < 4; ++s) probe_store<NT_STORE>(q + s * 64, v[u][s]);
            }
        }
    }
}

// Shared argument handling: wavefront count (multiple of 4) and the piece map.
int probe_setup(size_t bytes, int n_workers, int pattern, int &workers, PieceMap &map)
{
    if (bytes < (size_t)kPieceBytes || n_workers < 0 || n_workers > RAZOR_MAX_WORKERS) return RAZOR_EINVAL;
    if (pattern < -RAZOR_MAX_WORKERS || pattern > 65536) return RAZOR_EINVAL;
    workers = n_workers;
    if (workers == 0) {
        const int rc = auto_workers(&workers);
        if (rc != RAZOR_OK) return rc;
    }
    workers = std::max(4, std::min(workers, RAZOR_MAX_WORKERS)) / 4 * 4;
    map.n_pieces = (int64_t)(bytes / kPieceBytes);        // a tail shorter than a piece is not touched
    map.per = (map.n_pieces + workers - 1) / workers;
    map.n_waves = workers;
    map.chunk = pattern > 0 ? pattern : 0;
    map.group = pattern < 0 ? std::min(-pattern, workers) : 0;
    while (map.group > 1 && workers % map.group) --map.group;   // whole groups only
    return RAZOR_OK;
}

}  // namespace
}  // namespace razor

extern "C" int razor_probe_read_stream(const void *buf, size_t bytes, int n_workers, int pattern, int depth,
                                       int nontemporal, void *sink, void *stream)
{
    using namespace razor;
    if (!buf || !sink || ((uintptr_t)buf & 15) || ((uintptr_t)sink & 3)) return RAZOR_EINVAL;
    if (depth != 1 && depth != 2 && depth != 4 && depth != 8) return RAZOR_EINVAL;
    int workers = 0;
    PieceMap map{};
    const int rc = probe_setup(bytes, n_workers, pattern, workers, map);
    if (rc != RAZOR_OK) return rc;
    const dim3 grid(workers / 4), block(256);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const u32x4 *p = static_cast<const u32x4 *>(buf);
    uint32_t *out = static_cast<uint32_t *>(sink);
#define RAZOR_PROBE(DEPTH)                                                                              \
    if (nontemporal) hipLaunchKernelGGL((read_stream_kernel<DEPTH, true>), grid, block, 0, s, p, map, out); \
    else hipLaunchKernelGGL((read_stream_kernel<DEPTH, false>), grid, block, 0, s, p, map, out)
    if (depth == 1) { RAZOR_PROBE(1); }
    else if (depth == 2) { RAZOR_PROBE(2); }
    else if (depth == 4) { RAZOR_PROBE(4); }
    else { RAZOR_PROBE(8); }
#undef RAZOR_PROBE
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return hip_failure("razor_probe_read_stream launch", (int)err);
    return RAZOR_OK;
}

extern "C" int razor_probe_copy(void *dst, const void *src, size_t bytes, int n_workers, int pattern,
                                int nontemporal, void *stream)
{
    using namespace razor;
    if (!dst || !src || (((uintptr_t)dst | (uintptr_t)src) & 15) || nontemporal < 0 || nontemporal > 3)
        return RAZOR_EINVAL;
    const uintptr_t d = (uintptr_t)dst, s0 = (uintptr_t)src;
    if (d < s0 + bytes && s0 < d + bytes) return RAZOR_EINVAL;   // overlapping ranges
    int workers = 0;
    PieceMap map{};
    const int rc = probe_setup(bytes, n_workers, pattern, workers, map);
    if (rc != RAZOR_OK) return rc;
    const dim3 grid(workers / 4), block(256);
    hipStream_t s = static_cast<hipStream_t>(stream);
    u32x4 *out = static_cast<u32x4 *>(dst);
    const u32x4 *in = static_cast<const u32x4 *>(src);
    switch (nontemporal) {
    case 0: hipLaunchKernelGGL((copy_stream_kernel<false, false>), grid, block, 0, s, out, in, map); break;
    case 1: hipLaunchKernelGGL((copy_stream_kernel<true, false>), grid, block, 0, s, out, in, map); break;
    case 2: hipLaunchKernelGGL((copy_stream_kernel<false, true>), grid, block, 0, s, out, in, map); break;
    default: hipLaunchKernelGGL((copy_stream_kernel<true, true>), grid, block, 0, s, out, in, map); break;
    }
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return hip_failure("razor_probe_copy launch", (int)err);
    return RAZOR_OK;
}
