// Argument block passed by value to the verification kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lantern {

// VERIFY_FULL: decision, and the resampled token of every rejected row.
// VERIFY_DECIDE: decision only; out_resample is not touched (rejections settle in fp32 as well).
// VERIFY_SELECTED: workgroup i evaluates verification select[i] in fp64 and writes only
//   out_resample[i]: the resampled token, -1 if that verification is accepted, -2 if it is
//   unusable or out of range; a negative select[i] is copied through.
enum { VERIFY_FULL = 0, VERIFY_DECIDE = 1, VERIFY_SELECTED = 2 };

struct VerifyArgs {
    const void* target;       // [R, stride] logits of the target model
    const void* draft;        // [R, stride] logits of the drafter
    int N;                    // verifications
    int R;                    // logit rows (N without an index array)
    const int32_t* row_index; // [N] logit row of every verification, or null: row i
    int V;
    int64_t stride;           // elements between rows
    const int32_t* tokens;    // [N] draft tokens
    const int32_t* knn;       // [V, k] neighbour table
    int k;
    int divergence;           // bound on A: 0 total variation distance, 1 Jensen-Shannon divergence
    int mode;                 // VERIFY_FULL, VERIFY_DECIDE or VERIFY_SELECTED
    const int32_t* select;    // VERIFY_SELECTED: [n_sel] verification per workgroup (negative: passed through)
    int n_sel;
    int stage_rows;           // VERIFY_SELECTED: both logit rows fit into LDS beside the exact path's data
    float delta;
    const float* uniforms;    // [N, 2]
    int32_t* out_accept;      // [N]
    int32_t* out_resample;    // [N]
    float* out_prob;          // optional diagnostics, may be null
    float* out_mass;
    float* out_gtok;
    int32_t* out_asize;
    int32_t* out_path;
};

// Enqueues the fp32 pass and the fp64 pass on the stream.  logits_dtype: 0 fp32, 1 bf16.
hipError_t launch_verify(const VerifyArgs& a, int logits_dtype, hipStream_t stream);

// VERIFY_SELECTED: one workgroup per entry of a.select.
hipError_t launch_resample_selected(const VerifyArgs& a, int logits_dtype, hipStream_t stream);

// Second half of a tree step, one workgroup per tree (a.n_sel trees of M nodes): the walk over the
// decisions in a.out_accept, then the residual draw it asks for into a.out_resample[tree].
hipError_t launch_tree_finish(const VerifyArgs& a, const int32_t* parent, int M, int32_t* out_len, int32_t* out_path,
                              int logits_dtype, hipStream_t stream);

// Raises the dynamic-LDS limits of every kernel the calls above can launch for this logit type,
// vocabulary size and table width on the current device; enqueues nothing.
hipError_t prepare_verify(int logits_dtype, int V, int k);

}  // namespace lantern

namespace lantern {

// Greedy-decoding variant: target logits only, no random draws.
struct GreedyArgs {
    const void* target;       // [R, stride] logits of the target model
    int N;                    // verifications
    int R;                    // logit rows (N without an index array)
    const int32_t* row_index; // [N] logit row of every verification, or null: row i
    int V;
    int64_t stride;
    const int32_t* tokens;    // [N] draft tokens
    const int32_t* knn;       // [V, k] neighbour table
    int k;
    float delta;
    int32_t* out_accept;      // [N]
    int32_t* out_token;       // [N]
    int32_t* out_path;        // optional, may be null
};

hipError_t launch_verify_greedy(const GreedyArgs& a, int logits_dtype, hipStream_t stream);
hipError_t prepare_greedy(int logits_dtype, int V, int k);

}  // namespace lantern

namespace lantern {

hipError_t prepare_walks();   // loads the walk kernels on the current device

hipError_t launch_accept_chains(const int32_t* accept, const int32_t* resample, int B, int L,
                                int32_t* out_len, int32_t* out_next, hipStream_t stream);

hipError_t launch_accept_trees(const int32_t* accept, const int32_t* resample, const int32_t* parent, int B,
                               int M, int32_t* out_len, int32_t* out_path, int32_t* out_next,
                               hipStream_t stream);

}  // namespace lantern
