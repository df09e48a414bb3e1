// Walk of drafted chains (Algorithm 1, the loop over the L candidates of a
// chain): drafts are kept while they are accepted; the first candidate that
// is not accepted ends the chain with its resampled token.
// Integer work on the outputs of lantern_verify; one wavefront per chain (or tree).
#include <hip/hip_runtime.h>
#include <limits.h>
#include <stdint.h>

#include "device_utils.h"
#include "tree_walk.h"

namespace lantern {

__global__ __launch_bounds__(NT) void accept_chains_kernel(const int32_t* accept, const int32_t* resample,
                                                           int B, int L, int32_t* out_len, int32_t* out_next) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int chain = blockIdx.x * NW + (threadIdx.x >> 6);
    if (chain >= B) return;   // uniform per wavefront
    const int32_t* acc = accept + (int64_t)chain * L;
    const int32_t* res = resample + (int64_t)chain * L;
    int first = L;            // position of the first candidate that is not accepted
    for (int base = 0; base < L; base += WAVE) {
        const int t = base + lane;
        const bool stop = (t < L) && (acc[t] != 1);
        const unsigned long long m = __ballot(stop);
        if (m) {
            first = base + __ffsll((long long)m) - 1;
            break;
        }
    }
    if (lane == 0) {
        out_len[chain] = first;
        int next = -1;
        if (first < L) next = (acc[first] == 0) ? res[first] : -2;
        out_next[chain] = next;
    }
}

// Walk of drafted trees, one wavefront per tree: tree b owns nodes b*M .. b*M+M-1.
__global__ __launch_bounds__(NT) void accept_trees_kernel(const int32_t* accept, const int32_t* resample,
                                                          const int32_t* parent, int B, int M, int32_t* out_len,
                                                          int32_t* out_path, int32_t* out_next) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int tree = blockIdx.x * NW + (threadIdx.x >> 6);
    if (tree >= B) return;    // uniform per wavefront
    int32_t* path = out_path + (int64_t)tree * M;
    int len;
    const int next = walk_tree(accept + (int64_t)tree * M, resample ? resample + (int64_t)tree * M : nullptr,
                               parent + (int64_t)tree * M, M, tree, path, &len);
    for (int j = len + lane; j < M; j += WAVE) path[j] = -1;
    if (lane == 0) {
        out_len[tree] = len;
        out_next[tree] = next;
    }
}

// Makes the runtime load this file's kernels on the current device (it defers that to a kernel's
// first use), so that their first launch can be recorded into a graph.
hipError_t prepare_walks() {
    hipFuncAttributes attr;
    return hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(&accept_chains_kernel));
}

hipError_t launch_accept_trees(const int32_t* accept, const int32_t* resample, const int32_t* parent, int B,
                               int M, int32_t* out_len, int32_t* out_path, int32_t* out_next,
                               hipStream_t stream) {
    hipLaunchKernelGGL(accept_trees_kernel, dim3((B + NW - 1) / NW), dim3(NT), 0, stream, accept, resample,
                       parent, B, M, out_len, out_path, out_next);
    return hipGetLastError();
}

hipError_t launch_accept_chains(const int32_t* accept, const int32_t* resample, int B, int L,
                                int32_t* out_len, int32_t* out_next, hipStream_t stream) {
    hipLaunchKernelGGL(accept_chains_kernel, dim3((B + NW - 1) / NW), dim3(NT), 0, stream, accept, resample, B,
                       L, out_len, out_next);
    return hipGetLastError();
}

}  // namespace lantern
