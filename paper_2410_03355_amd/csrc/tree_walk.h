// Walk of a drafted tree by one wavefront (Algorithm 1 along a branch): nodes in drafting order,
// parent[i] < i (-1: the node follows the committed prefix).  Standing at a node, its children are
// tried in index order and the first accepted one is taken; Algorithm 1 is the case of one child
// per node.
#pragma once

#include <hip/hip_runtime.h>
#include <limits.h>
#include <stdint.h>

#include "device_utils.h"

namespace lantern {

constexpr int CACHED = 4;   // nodes per lane that the walk keeps in registers: trees of up to 256 nodes

// acc, res, par: the tree's M decisions, resampled tokens (or null) and parents; path: its M path
// slots, of which the first *len_out are written (by lane 0).  Returns what follows the accepted
// nodes: the resampled token of the first child when every child of the last node was rejected
// (without resampled tokens, res null: the verification tree * M + node whose token that is), -1 at
// a leaf, -2 when an unusable child was met first, -3 for a malformed parent array (nothing walked).
__device__ __forceinline__ int walk_tree(const int32_t* acc, const int32_t* res, const int32_t* par, int M, int tree,
                                         int32_t* path, int* len_out) {
    const int lane = threadIdx.x & (WAVE - 1);
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
            else if (first_child >= 0) next = res ? res[first_child] : tree * M + first_child;
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
                next = res ? res[first_child] : tree * M + first_child;
            else next = -1;                                   // a leaf: every draft on the branch accepted
            break;
        }
    }
    *len_out = len;
    return next;
}

}  // namespace lantern
