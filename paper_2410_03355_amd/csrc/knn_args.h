// Argument block and host entry of the neighbour-table build.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace lantern {

struct KnnArgs {
    const void* codebook;  // [V, d]
    int cb_dtype;          // 0 fp32, 1 bf16
    int V;
    int d;
    int k;
    int metric;            // 0 squared l2, 1 cosine
    int32_t* out;          // [V, k]
    void* workspace;
};

size_t knn_workspace_bytes(int V, int d, int k, int cb_dtype);
hipError_t launch_build_knn(const KnnArgs& a, hipStream_t stream);

// The build on the library's static device scratch (no workspace from the caller, nothing
// allocated).  knn_static_fits: whether a codebook of V codes is within what that scratch serves.
bool knn_static_fits(int V);
hipError_t launch_build_knn_static(const KnnArgs& a, int32_t* exact_rows, hipStream_t stream);

// Random table of k <= RANDOM_MAX_K entries per row; t0: first threshold on the 32-bit keys, in [1, 2^32].
constexpr int RANDOM_MAX_K = 4096;
hipError_t launch_build_random(int V, int k, uint64_t seed, uint64_t t0, int32_t* out, hipStream_t stream);

}  // namespace lantern
