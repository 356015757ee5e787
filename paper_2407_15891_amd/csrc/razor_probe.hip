// Measurement hook: the read-stream ceiling of the device, taken with the access pattern of the
// streaming kernels (one contiguous range per wavefront, 128-bit non-temporal loads, two 4 KB
// pieces in flight per wave) and no arithmetic worth the name.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "razor_device.h"

namespace razor {
namespace {

constexpr int kPieceBytes = 4096;   // one wave-wide step: 4 loads of 16 bytes per lane

__global__ __launch_bounds__(256) void read_stream_kernel(const u32x4 *__restrict__ p, int64_t n_pieces,
                                                          int64_t per, uint32_t *__restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t lo = w * per, hi = lo + per < n_pieces ? lo + per : n_pieces;
    uint32_t acc = 0;
    for (int64_t k = lo; k < hi; k += 2) {
        u32x4 v[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int64_t piece = k + u < hi ? k + u : hi - 1;
            const u32x4 *q = p + piece * (kPieceBytes / 16) + lane;
#pragma unroll
            for (int s = 0; s < 4; ++s) v[u][s] = stream_load(q + s * 64);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int s = 0; s < 4; ++s) acc += v[u][s].x ^ v[u][s].y ^ v[u][s].z ^ v[u][s].w;
    }
    if (acc == 0x9e3779b9u) sink[w] = acc;   // keeps the loads alive; practically never taken
}

}  // namespace
}  // namespace razor

extern "C" int razor_probe_read_stream(const void *buf, size_t bytes, int n_workers, void *sink, void *stream)
{
    using namespace razor;
    if (!buf || !sink || ((uintptr_t)buf & 15) || ((uintptr_t)sink & 3) || bytes < (size_t)kPieceBytes)
        return RAZOR_EINVAL;
    int workers = n_workers;
    if (workers == 0) {
        const int rc = auto_workers(&workers);
        if (rc != RAZOR_OK) return rc;
    }
    if (workers < 0) return RAZOR_EINVAL;
    workers = std::max(4, std::min(workers, RAZOR_MAX_WORKERS)) / 4 * 4;
    const int64_t n_pieces = (int64_t)(bytes / kPieceBytes);        // a tail shorter than a piece is not read
    const int64_t per = (n_pieces + workers - 1) / workers;
    hipLaunchKernelGGL(read_stream_kernel, dim3(workers / 4), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4 *>(buf), n_pieces, per, static_cast<uint32_t *>(sink));
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return hip_failure("razor_probe_read_stream launch", (int)err);
    return RAZOR_OK;
}
