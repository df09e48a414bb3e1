// Walk of drafted chains (Algorithm 1, the loop over the L candidates of a
// chain): drafts are kept while they are accepted; the first candidate that
// is not accepted ends the chain with its resampled token.
// Integer work on the outputs of lantern_verify; one wavefront per chain (or tree).
#include <hip/hip_runtime.h>
#include <limits.h>
#include <stdint.h>

#include "device_utils.h"

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

// Walk of drafted trees: tree b owns nodes b*M .. b*M+M-1 in drafting order, parent[i] < i
// (-1: the node follows the committed prefix).  Standing at a node, its children are tried in
// index order and the first accepted one is taken; Algorithm 1 is the case of one child per node.
// One wavefront per tree; every step scans the nodes after the current one, 64 at a time.
// Without resampled tokens (resample null) the walk reports, in place of the token, which
// verification (tree * M + node) has to be resampled.
constexpr int CACHED = 4;   // nodes per lane that the walk keeps in registers: trees of up to 256 nodes
__global__ __launch_bounds__(NT) void accept_trees_kernel(const int32_t* accept, const int32_t* resample,
                                                          const int32_t* parent, int B, int M, int32_t* out_len,
                                                          int32_t* out_path, int32_t* out_next) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int tree = blockIdx.x * NW + (threadIdx.x >> 6);
    if (tree >= B) return;    // uniform per wavefront
    const int32_t* acc = accept + (int64_t)tree * M;
    const int32_t* res = resample + (int64_t)tree * M;
    const int32_t* par = parent + (int64_t)tree * M;
    int32_t* path = out_path + (int64_t)tree * M;

    int malformed = 0;
    for (int i = lane; i < M; i += WAVE)
        if (par[i] < -1 || par[i] >= i) malformed = 1;
    malformed = wave_or(malformed);

    int cur = -1, len = 0, next = -1;
    if (malformed) {
        next = -3;
    } else if (M <= CACHED * WAVE) {
        // small trees (the usual case): every lane keeps its nodes' parent and decision in registers,
        // node i in slot i / 64 of lane i % 64, so a step of the walk touches no memory
        int cp[CACHED], ca[CACHED];
#pragma unroll
        for (int q = 0; q < CACHED; ++q) {
            const int i = q * WAVE + lane;
            cp[q] = i < M ? par[i] : INT_MIN;
            ca[q] = i < M ? acc[i] : 0;
        }
        for (;;) {            // cur grows with every step: at most M steps
            int first_child = -1, decisive = -1, decisive_acc = 0;
#pragma unroll
            for (int q = 0; q < CACHED; ++q) {
                if (decisive >= 0) continue;
                const bool child = cp[q] == cur;
                const unsigned long long cm = __ballot(child);
                const unsigned long long dm = __ballot(child && ca[q] != 0);
                if (first_child < 0 && cm) first_child = q * WAVE + __ffsll((long long)cm) - 1;
                if (dm) {
                    const int l = __ffsll((long long)dm) - 1;
                    decisive = q * WAVE + l;
                    decisive_acc = __builtin_amdgcn_readlane(ca[q], l);
                }
            }
            if (decisive >= 0 && decisive_acc == 1) {
                if (lane == 0) path[len] = decisive;
                ++len;
                cur = decisive;
                continue;
            }
            if (decisive >= 0) next = -2;
            else if (first_child >= 0) next = resample ? res[first_child] : tree * M + first_child;
            else next = -1;
            break;
        }
    } else {
        for (;;) {            // cur grows with every step: at most M steps
            int first_child = -1, decisive = -1;
            for (int base = cur + 1; base < M; base += WAVE) {
                const int i = base + lane;
                const bool child = (i < M) && (par[i] == cur);
                const unsigned long long cm = __ballot(child);
                const unsigned long long dm = __ballot(child && acc[i] != 0);
                if (first_child < 0 && cm) first_child = base + __ffsll((long long)cm) - 1;
                if (dm) {
                    decisive = base + __ffsll((long long)dm) - 1;
                    break;
                }
            }
            if (decisive >= 0 && acc[decisive] == 1) {
                if (lane == 0) path[len] = decisive;
                ++len;
                cur = decisive;
                continue;
            }
            if (decisive >= 0) next = -2;                     // an unusable row ends the walk
            else if (first_child >= 0)                        // every child was rejected
                next = resample ? res[first_child] : tree * M + first_child;
            else next = -1;                                   // a leaf: every draft on the branch accepted
            break;
        }
    }
    for (int j = len + lane; j < M; j += WAVE) path[j] = -1;
    if (lane == 0) {
        out_len[tree] = len;
        out_next[tree] = next;
    }
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
