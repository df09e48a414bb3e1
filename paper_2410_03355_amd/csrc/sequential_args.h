// Argument block of the tree walk under the sequential-residual sibling rule.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lantern {

struct SequentialArgs {
    const void* target;        // [R, stride] logits of the target model
    const void* draft;         // [R, stride] logits of the drafter
    int R;
    int V;
    int64_t stride;            // elements between rows
    const int32_t* row_index;  // [B*M] logit row of every candidate, or null: candidate i reads row i
    const int32_t* parent;     // [B*M]
    int B;
    int M;
    const int32_t* tokens;     // [B*M] draft tokens
    const int32_t* knn;        // [V, k] neighbour table
    int k;
    int divergence;            // bound on A: 0 total variation distance, 1 Jensen-Shannon divergence
    float delta;
    const float* uniforms;     // [B*M, 2]
    const int32_t* accept;     // [B*M] decisions of the plain verification of every candidate (1, 0, -1)
    int32_t* out_len;          // [B]
    int32_t* out_path;         // [B*M]
    int32_t* out_next;         // [B]
    double* work;              // [B, 2, V] current target and drafter distribution of every tree
    int cur_in_lds;            // set by the launch: the current target lives in LDS (V doubles fit)
};

// One workgroup per tree.  logits_dtype: 0 fp32, 1 bf16.
hipError_t launch_trees_sequential(const SequentialArgs& a, int logits_dtype, hipStream_t stream);

// Loads the kernels on the current device and raises their LDS limit for this vocabulary size.
hipError_t prepare_sequential(int logits_dtype, int V);

}  // namespace lantern
