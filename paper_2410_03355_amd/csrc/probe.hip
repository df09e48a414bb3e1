// Measurement aid, not part of the method: a plain streaming read with the access pattern of the
// verification kernel (one 256-thread workgroup per 64 KiB, sixteen 16-byte non-temporal loads per
// thread, all issued before any is used), to put the device's reachable read rate beside the
// verification kernel's.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_utils.h"
#include "lantern.h"
#include "verify_common.h"

namespace lantern {

__global__ __launch_bounds__(NT) void stream_read_kernel(const uint4* src_a, const uint4* src_b, unsigned chunks,
                                                         uint32_t* sink) {
    const uint4* q = blockIdx.x < chunks ? src_a + (size_t)blockIdx.x * (16 * NT)
                                         : src_b + (size_t)(blockIdx.x - chunks) * (16 * NT);
    uint4 v[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) v[c] = load_stream16(q + c * NT + threadIdx.x);
    uint32_t a = 0;
#pragma unroll
    for (int c = 0; c < 16; ++c) a ^= v[c].x ^ v[c].y ^ v[c].z ^ v[c].w;
    if (a == 0x9E3779B9u) sink[0] = a;   // keeps the loads alive; practically never taken
}

}  // namespace lantern

extern "C" int lantern_probe_stream_read(const void* src_a, const void* src_b, size_t bytes, uint32_t* sink,
                                         void* hip_stream) {
    if (!src_a || !sink) return LANTERN_E_NULL;
    if (((reinterpret_cast<uintptr_t>(src_a) | reinterpret_cast<uintptr_t>(src_b)) & 15) != 0) return LANTERN_E_SHAPE;
    const size_t chunks = bytes / 65536;      // whole 64 KiB chunks only
    if (chunks == 0) return LANTERN_OK;
    if (chunks > 0x3FFFFFFF) return LANTERN_E_SHAPE;
    const unsigned grid = (unsigned)chunks * (src_b ? 2u : 1u);
    hipLaunchKernelGGL(lantern::stream_read_kernel, dim3(grid), dim3(lantern::NT), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const uint4*>(src_a),
                       static_cast<const uint4*>(src_b), (unsigned)chunks, sink);
    return hipGetLastError() == hipSuccess ? LANTERN_OK : LANTERN_E_DEVICE;
}
