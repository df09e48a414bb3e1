// C ABI of the library: argument validation on the host, then kernel launches.
#include <hip/hip_runtime.h>
#include <limits.h>
#include <math.h>
#include <stdint.h>

#include "knn_args.h"
#include "lantern.h"
#include "sequential_args.h"
#include "verify_args.h"

namespace {

bool dtype_ok(int dt) { return dt == LANTERN_F32 || dt == LANTERN_BF16; }

// What the second half of a tree step needs besides the verification arguments.
struct TreeFinish {
    const int32_t* parent;
    int M;
    int32_t* out_len;
    int32_t* out_path;
};

// R, row_index: number of logit rows and the row every verification reads; without an index
// array (row_index null) verification i reads row i and R is N.
int verify_impl(const void* target_logits, const void* draft_logits, int logits_dtype, int R,
                const int32_t* row_index, int N, int V,
                int64_t row_stride_elems, const int32_t* draft_tokens, const int32_t* knn, int k,
                int divergence, float delta, const float* uniforms, int32_t* out_accept, int32_t* out_resample,
                float* out_accept_prob, float* out_mass, float* out_g_tok, int32_t* out_a_size,
                int32_t* out_path, void* hip_stream, int mode = lantern::VERIFY_FULL,
                const int32_t* select = nullptr, int n_sel = 0, const TreeFinish* tree = nullptr) {
    if (!dtype_ok(logits_dtype)) return LANTERN_E_DTYPE;
    if (N < 0 || R < 0 || V < 1 || V > LANTERN_MAX_VOCAB || k < 1 || k > V || row_stride_elems < V)
        return LANTERN_E_SHAPE;
    if (N > 0 && R < 1) return LANTERN_E_SHAPE;
    if (divergence != LANTERN_DIV_TVD && divergence != LANTERN_DIV_JSD) return LANTERN_E_SHAPE;
    if (!(delta >= 0.0f)) return LANTERN_E_DELTA;  // also rejects NaN
    if (n_sel < 0 || (n_sel > 0 && N == 0)) return LANTERN_E_SHAPE;
    if (mode == lantern::VERIFY_SELECTED ? n_sel == 0 : N == 0) return LANTERN_OK;
    if (!target_logits || !draft_logits || !draft_tokens || !knn || !uniforms) return LANTERN_E_NULL;
    if (mode != lantern::VERIFY_SELECTED && !out_accept) return LANTERN_E_NULL;
    if (mode != lantern::VERIFY_DECIDE && !out_resample) return LANTERN_E_NULL;
    if (mode == lantern::VERIFY_SELECTED && !select && !tree) return LANTERN_E_NULL;
    lantern::VerifyArgs a;
    a.target = target_logits;
    a.draft = draft_logits;
    a.N = N;
    a.R = R;
    a.row_index = row_index;
    a.V = V;
    a.stride = row_stride_elems;
    a.tokens = draft_tokens;
    a.knn = knn;
    a.k = k;
    a.divergence = divergence;
    a.mode = mode;
    a.select = select;
    a.n_sel = n_sel;
    a.stage_rows = 0;
    a.delta = delta;
    a.uniforms = uniforms;
    a.out_accept = out_accept;
    a.out_resample = out_resample;
    a.out_prob = out_accept_prob;
    a.out_mass = out_mass;
    a.out_gtok = out_g_tok;
    a.out_asize = out_a_size;
    a.out_path = out_path;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e;
    if (tree)   // one workgroup per tree: the walk over out_accept, then the residual draw it asks for
        e = lantern::launch_tree_finish(a, tree->parent, tree->M, tree->out_len, tree->out_path, logits_dtype, stream);
    else if (mode == lantern::VERIFY_SELECTED)
        e = lantern::launch_resample_selected(a, logits_dtype, stream);
    else
        e = lantern::launch_verify(a, logits_dtype, stream);
    return e == hipSuccess ? LANTERN_OK : LANTERN_E_DEVICE;
}

}  // namespace

extern "C" {

int lantern_verify(const void* target_logits, const void* draft_logits, lantern_dtype logits_dtype,
                   int N, int V, int64_t row_stride_elems, const int32_t* draft_tokens,
                   const int32_t* knn, int k, float delta, const float* uniforms,
                   int32_t* out_accept, int32_t* out_resample, void* hip_stream) {
    return verify_impl(target_logits, draft_logits, (int)logits_dtype, N, nullptr, N, V, row_stride_elems,
                       draft_tokens, knn, k, LANTERN_DIV_TVD, delta, uniforms, out_accept, out_resample, nullptr,
                       nullptr, nullptr, nullptr, nullptr, hip_stream);
}

int lantern_verify_ex(const void* target_logits, const void* draft_logits,
                      lantern_dtype logits_dtype, int N, int V, int64_t row_stride_elems,
                      const int32_t* draft_tokens, const int32_t* knn, int k, float delta,
                      const float* uniforms, int32_t* out_accept, int32_t* out_resample,
                      float* out_accept_prob, float* out_mass, float* out_g_tok,
                      int32_t* out_a_size, int32_t* out_path, void* hip_stream) {
    return verify_impl(target_logits, draft_logits, (int)logits_dtype, N, nullptr, N, V, row_stride_elems,
                       draft_tokens, knn, k, LANTERN_DIV_TVD, delta, uniforms, out_accept, out_resample,
                       out_accept_prob, out_mass, out_g_tok, out_a_size, out_path, hip_stream);
}

int lantern_verify_divergence(const void* target_logits, const void* draft_logits,
                              lantern_dtype logits_dtype, int N, int V, int64_t row_stride_elems,
                              const int32_t* draft_tokens, const int32_t* knn, int k, int divergence,
                              float delta, const float* uniforms, int32_t* out_accept, int32_t* out_resample,
                              float* out_accept_prob, float* out_mass, float* out_g_tok,
                              int32_t* out_a_size, int32_t* out_path, void* hip_stream) {
    return verify_impl(target_logits, draft_logits, (int)logits_dtype, N, nullptr, N, V, row_stride_elems,
                       draft_tokens, knn, k, divergence, delta, uniforms, out_accept, out_resample,
                       out_accept_prob, out_mass, out_g_tok, out_a_size, out_path, hip_stream);
}

int lantern_verify_rows(const void* target_logits, const void* draft_logits, lantern_dtype logits_dtype,
                        int R, int V, int64_t row_stride_elems, const int32_t* row_index, int N,
                        const int32_t* draft_tokens, const int32_t* knn, int k, int divergence, float delta,
                        const float* uniforms, int32_t* out_accept, int32_t* out_resample, void* hip_stream) {
    if (N > 0 && !row_index) return LANTERN_E_NULL;
    return verify_impl(target_logits, draft_logits, (int)logits_dtype, R, row_index, N, V, row_stride_elems,
                       draft_tokens, knn, k, divergence, delta, uniforms, out_accept, out_resample, nullptr,
                       nullptr, nullptr, nullptr, nullptr, hip_stream);
}

int lantern_decide_rows(const void* target_logits, const void* draft_logits, lantern_dtype logits_dtype,
                        int R, int V, int64_t row_stride_elems, const int32_t* row_index, int N,
                        const int32_t* draft_tokens, const int32_t* knn, int k, int divergence, float delta,
                        const float* uniforms, int32_t* out_accept, int32_t* out_path, void* hip_stream) {
    if (!row_index && R != N) return LANTERN_E_SHAPE;   // without an index array row i belongs to verification i
    return verify_impl(target_logits, draft_logits, (int)logits_dtype, R, row_index, N, V, row_stride_elems,
                       draft_tokens, knn, k, divergence, delta, uniforms, out_accept, nullptr, nullptr,
                       nullptr, nullptr, nullptr, out_path, hip_stream, lantern::VERIFY_DECIDE);
}

int lantern_resample_selected(const void* target_logits, const void* draft_logits, lantern_dtype logits_dtype,
                              int R, int V, int64_t row_stride_elems, const int32_t* row_index, int N,
                              const int32_t* draft_tokens, const int32_t* knn, int k, int divergence,
                              float delta, const float* uniforms, const int32_t* select, int n_sel,
                              int32_t* out_token, void* hip_stream) {
    if (!row_index && R != N) return LANTERN_E_SHAPE;
    return verify_impl(target_logits, draft_logits, (int)logits_dtype, R, row_index, N, V, row_stride_elems,
                       draft_tokens, knn, k, divergence, delta, uniforms, nullptr, out_token, nullptr,
                       nullptr, nullptr, nullptr, nullptr, hip_stream, lantern::VERIFY_SELECTED, select, n_sel);
}

namespace {

int greedy_impl(const void* target_logits, int logits_dtype, int R, const int32_t* row_index, int N, int V,
                int64_t row_stride_elems, const int32_t* draft_tokens, const int32_t* knn, int k,
                float delta, int32_t* out_accept, int32_t* out_token, int32_t* out_path,
                void* hip_stream) {
    if (!dtype_ok(logits_dtype)) return LANTERN_E_DTYPE;
    if (N < 0 || R < 0 || V < 1 || V > LANTERN_MAX_VOCAB || k < 1 || k > V || row_stride_elems < V)
        return LANTERN_E_SHAPE;
    if (N > 0 && R < 1) return LANTERN_E_SHAPE;
    if (!(delta >= 0.0f)) return LANTERN_E_DELTA;
    if (N == 0) return LANTERN_OK;
    if (!target_logits || !draft_tokens || !knn || !out_accept || !out_token) return LANTERN_E_NULL;
    lantern::GreedyArgs a;
    a.target = target_logits;
    a.N = N;
    a.R = R;
    a.row_index = row_index;
    a.V = V;
    a.stride = row_stride_elems;
    a.tokens = draft_tokens;
    a.knn = knn;
    a.k = k;
    a.delta = delta;
    a.out_accept = out_accept;
    a.out_token = out_token;
    a.out_path = out_path;
    const hipError_t e = lantern::launch_verify_greedy(a, logits_dtype, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? LANTERN_OK : LANTERN_E_DEVICE;
}

}  // namespace

int lantern_verify_greedy(const void* target_logits, lantern_dtype logits_dtype, int N, int V,
                          int64_t row_stride_elems, const int32_t* draft_tokens, const int32_t* knn, int k,
                          float delta, int32_t* out_accept, int32_t* out_token, int32_t* out_path,
                          void* hip_stream) {
    return greedy_impl(target_logits, (int)logits_dtype, N, nullptr, N, V, row_stride_elems, draft_tokens, knn,
                       k, delta, out_accept, out_token, out_path, hip_stream);
}

int lantern_verify_greedy_rows(const void* target_logits, lantern_dtype logits_dtype, int R, int V,
                               int64_t row_stride_elems, const int32_t* row_index, int N,
                               const int32_t* draft_tokens, const int32_t* knn, int k, float delta,
                               int32_t* out_accept, int32_t* out_token, void* hip_stream) {
    if (N > 0 && !row_index) return LANTERN_E_NULL;
    return greedy_impl(target_logits, (int)logits_dtype, R, row_index, N, V, row_stride_elems, draft_tokens,
                       knn, k, delta, out_accept, out_token, nullptr, hip_stream);
}

int lantern_accept_trees(const int32_t* accept, const int32_t* resample, const int32_t* parent, int B, int M,
                         int32_t* out_len, int32_t* out_path, int32_t* out_next, void* hip_stream) {
    if (B < 0 || M < 1) return LANTERN_E_SHAPE;
    if (B == 0) return LANTERN_OK;
    if (!accept || !parent || !out_len || !out_path || !out_next) return LANTERN_E_NULL;   // resample may be null
    const hipError_t e = lantern::launch_accept_trees(accept, resample, parent, B, M, out_len, out_path,
                                                      out_next, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? LANTERN_OK : LANTERN_E_DEVICE;
}

int lantern_accept_chains(const int32_t* accept, const int32_t* resample, int B, int L, int32_t* out_len,
                          int32_t* out_next, void* hip_stream) {
    if (B < 0 || L < 1) return LANTERN_E_SHAPE;
    if (B == 0) return LANTERN_OK;
    if (!accept || !resample || !out_len || !out_next) return LANTERN_E_NULL;
    const hipError_t e = lantern::launch_accept_chains(accept, resample, B, L, out_len, out_next,
                                                       static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? LANTERN_OK : LANTERN_E_DEVICE;
}

size_t lantern_build_knn_workspace_bytes(lantern_dtype cb_dtype, int V, int d, int k) {
    if (!dtype_ok((int)cb_dtype) || V < 1 || d < 1 || k < 1 || k > V) return 0;
    return lantern::knn_workspace_bytes(V, d, k, (int)cb_dtype);
}

int lantern_build_knn_metric(const void* codebook, lantern_dtype cb_dtype, int V, int d, int k,
                             int metric, int32_t* out_knn, void* workspace, size_t workspace_bytes,
                             void* hip_stream) {
    if (!dtype_ok((int)cb_dtype)) return LANTERN_E_DTYPE;
    if (V < 1 || d < 1 || k < 1 || k > V) return LANTERN_E_SHAPE;
    if (metric != LANTERN_METRIC_L2 && metric != LANTERN_METRIC_COSINE) return LANTERN_E_SHAPE;
    if (!codebook || !out_knn) return LANTERN_E_NULL;
    const size_t need = lantern::knn_workspace_bytes(V, d, k, (int)cb_dtype);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
        return LANTERN_E_WORKSPACE;
    lantern::KnnArgs a;
    a.codebook = codebook;
    a.cb_dtype = (int)cb_dtype;
    a.V = V;
    a.d = d;
    a.k = k;
    a.metric = metric;
    a.out = out_knn;
    a.workspace = workspace;
    const hipError_t e = lantern::launch_build_knn(a, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? LANTERN_OK : LANTERN_E_DEVICE;
}

int lantern_build_knn_static(const void* codebook, lantern_dtype cb_dtype, int V, int d, int k, int metric,
                             int32_t* out_knn, int32_t* out_exact_rows, void* hip_stream) {
    if (!dtype_ok((int)cb_dtype)) return LANTERN_E_DTYPE;
    if (V < 1 || d < 1 || k < 1 || k > V) return LANTERN_E_SHAPE;
    if (metric != LANTERN_METRIC_L2 && metric != LANTERN_METRIC_COSINE) return LANTERN_E_SHAPE;
    if (!codebook || !out_knn) return LANTERN_E_NULL;
    if (V > LANTERN_STATIC_MAX_V || !lantern::knn_static_fits(V)) return LANTERN_E_WORKSPACE;
    lantern::KnnArgs a;
    a.codebook = codebook;
    a.cb_dtype = (int)cb_dtype;
    a.V = V;
    a.d = d;
    a.k = k;
    a.metric = metric;
    a.out = out_knn;
    a.workspace = nullptr;
    const hipError_t e = lantern::launch_build_knn_static(a, out_exact_rows, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? LANTERN_OK : LANTERN_E_DEVICE;
}

int lantern_build_knn(const void* codebook, lantern_dtype cb_dtype, int V, int d, int k,
                      int32_t* out_knn, void* workspace, size_t workspace_bytes, void* hip_stream) {
    return lantern_build_knn_metric(codebook, cb_dtype, V, d, k, LANTERN_METRIC_L2, out_knn,
                                    workspace, workspace_bytes, hip_stream);
}

int lantern_build_random(int V, int k, uint64_t seed, int32_t* out_knn, void* hip_stream) {
    if (V < 1 || V > LANTERN_MAX_VOCAB || k < 1 || k > V || k > LANTERN_RANDOM_MAX_K) return LANTERN_E_SHAPE;
    if (!out_knn) return LANTERN_E_NULL;
    static_assert(LANTERN_RANDOM_MAX_K == lantern::RANDOM_MAX_K, "limits of the header and the kernel differ");
    // keys are uniform on [0, 2^32): the k-1 smallest of V-1 lie below this with about three
    // standard deviations to spare (the kernel moves the threshold when they do not)
    uint64_t t0 = 1ull << 32;
    if (V > 1) {
        const double need = (double)(k - 1);
        const double frac = (need + 3.0 * sqrt(need) + 8.0) / (double)(V - 1);
        if (frac < 1.0) t0 = (uint64_t)ceil(frac * 4294967296.0);
        if (t0 < 1) t0 = 1;
    }
    const hipError_t e = lantern::launch_build_random(V, k, seed, t0, out_knn, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? LANTERN_OK : LANTERN_E_DEVICE;
}

int lantern_verify_trees(const void* target_logits, const void* draft_logits, lantern_dtype logits_dtype,
                         int R, int V, int64_t row_stride_elems, const int32_t* row_index,
                         const int32_t* parent, int B, int M, const int32_t* draft_tokens, const int32_t* knn,
                         int k, int divergence, float delta, const float* uniforms, int32_t* out_accept,
                         int32_t* out_len, int32_t* out_path, int32_t* out_next, void* hip_stream) {
    if (B < 0 || M < 1 || (int64_t)B * M > INT_MAX) return LANTERN_E_SHAPE;
    const int N = B * M;
    if (B > 0 && (!parent || !out_len || !out_path || !out_next)) return LANTERN_E_NULL;
    if (!row_index && R != N) return LANTERN_E_SHAPE;   // without an index array candidate i reads row i
    // decisions of all candidates; then, one workgroup per tree, the walk and the residual draw of the
    // one candidate it asks for
    const int rc = lantern_decide_rows(target_logits, draft_logits, logits_dtype, R, V, row_stride_elems, row_index,
                                       N, draft_tokens, knn, k, divergence, delta, uniforms, out_accept, nullptr,
                                       hip_stream);
    if (rc != LANTERN_OK || B == 0) return rc;
    const TreeFinish tree{parent, M, out_len, out_path};
    return verify_impl(target_logits, draft_logits, (int)logits_dtype, R, row_index, N, V, row_stride_elems,
                       draft_tokens, knn, k, divergence, delta, uniforms, out_accept, out_next, nullptr, nullptr,
                       nullptr, nullptr, nullptr, hip_stream, lantern::VERIFY_SELECTED, nullptr, B, &tree);
}

int lantern_verify_trees_greedy(const void* target_logits, lantern_dtype logits_dtype, int R, int V,
                                int64_t row_stride_elems, const int32_t* row_index, const int32_t* parent, int B,
                                int M, const int32_t* draft_tokens, const int32_t* knn, int k, float delta,
                                int32_t* out_accept, int32_t* out_token, int32_t* out_len, int32_t* out_path,
                                int32_t* out_next, void* hip_stream) {
    if (B < 0 || M < 1 || (int64_t)B * M > INT_MAX) return LANTERN_E_SHAPE;
    const int N = B * M;
    if (B > 0 && (!parent || !out_len || !out_path || !out_next)) return LANTERN_E_NULL;
    if (!row_index && R != N) return LANTERN_E_SHAPE;
    const int rc = greedy_impl(target_logits, (int)logits_dtype, R, row_index, N, V, row_stride_elems, draft_tokens,
                               knn, k, delta, out_accept, out_token, nullptr, hip_stream);
    if (rc != LANTERN_OK || B == 0) return rc;
    return lantern_accept_trees(out_accept, out_token, parent, B, M, out_len, out_path, out_next, hip_stream);
}

size_t lantern_verify_trees_sequential_workspace_bytes(int B, int M, int V) {
    if (B < 0 || M < 1 || V < 1 || V > LANTERN_MAX_VOCAB || (int64_t)B * M > INT_MAX) return 0;
    // per tree the current target and the drafter's distribution (fp64); then one decision per candidate
    const size_t vectors = (size_t)B * 2 * (size_t)V * sizeof(double);
    const size_t decisions = (((size_t)B * M * sizeof(int32_t)) + 255) & ~size_t(255);
    return B == 0 ? 0 : vectors + decisions;
}

int lantern_verify_trees_sequential(const void* target_logits, const void* draft_logits, lantern_dtype logits_dtype,
                                    int R, int V, int64_t row_stride_elems, const int32_t* row_index,
                                    const int32_t* parent, int B, int M, const int32_t* draft_tokens,
                                    const int32_t* knn, int k, int divergence, float delta, const float* uniforms,
                                    int32_t* out_len, int32_t* out_path, int32_t* out_next, void* workspace,
                                    size_t workspace_bytes, void* hip_stream) {
    if (!dtype_ok((int)logits_dtype)) return LANTERN_E_DTYPE;
    if (B < 0 || M < 1 || (int64_t)B * M > INT_MAX) return LANTERN_E_SHAPE;
    if (R < 0 || V < 1 || V > LANTERN_MAX_VOCAB || k < 1 || k > V || row_stride_elems < V) return LANTERN_E_SHAPE;
    if (divergence != LANTERN_DIV_TVD && divergence != LANTERN_DIV_JSD) return LANTERN_E_SHAPE;
    if (B > 0 && R < 1) return LANTERN_E_SHAPE;
    if (!(delta >= 0.0f)) return LANTERN_E_DELTA;
    if (B == 0) return LANTERN_OK;
    if (!row_index && R != B * M) return LANTERN_E_SHAPE;   // without an index array candidate i reads row i
    if (!target_logits || !draft_logits || !parent || !draft_tokens || !knn || !uniforms || !out_len || !out_path ||
        !out_next)
        return LANTERN_E_NULL;
    if (!workspace || ((uintptr_t)workspace & 255) != 0 ||
        workspace_bytes < lantern_verify_trees_sequential_workspace_bytes(B, M, V))
        return LANTERN_E_WORKSPACE;
    // the plain verification of every candidate decides the first child of every sibling group
    int32_t* decisions = reinterpret_cast<int32_t*>(static_cast<unsigned char*>(workspace) +
                                                    (size_t)B * 2 * (size_t)V * sizeof(double));
    const int rc = lantern_decide_rows(target_logits, draft_logits, logits_dtype, R, V, row_stride_elems, row_index,
                                       B * M, draft_tokens, knn, k, divergence, delta, uniforms, decisions, nullptr,
                                       hip_stream);
    if (rc != LANTERN_OK) return rc;
    lantern::SequentialArgs a;
    a.accept = decisions;
    a.target = target_logits;
    a.draft = draft_logits;
    a.R = R;
    a.V = V;
    a.stride = row_stride_elems;
    a.row_index = row_index;
    a.parent = parent;
    a.B = B;
    a.M = M;
    a.tokens = draft_tokens;
    a.knn = knn;
    a.k = k;
    a.divergence = divergence;
    a.delta = delta;
    a.uniforms = uniforms;
    a.out_len = out_len;
    a.out_path = out_path;
    a.out_next = out_next;
    a.work = static_cast<double*>(workspace);
    const hipError_t e = lantern::launch_trees_sequential(a, (int)logits_dtype, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? LANTERN_OK : LANTERN_E_DEVICE;
}

int lantern_prepare(lantern_dtype logits_dtype, int V, int k) {
    if (!dtype_ok((int)logits_dtype)) return LANTERN_E_DTYPE;
    if (V < 1 || V > LANTERN_MAX_VOCAB || k < 1 || k > V) return LANTERN_E_SHAPE;
    hipError_t e = lantern::prepare_verify((int)logits_dtype, V, k);
    if (e == hipSuccess) e = lantern::prepare_greedy((int)logits_dtype, V, k);
    if (e == hipSuccess) e = lantern::prepare_walks();
    if (e == hipSuccess) e = lantern::prepare_sequential((int)logits_dtype, V);
    return e == hipSuccess ? LANTERN_OK : LANTERN_E_DEVICE;
}

const char* lantern_status_string(int status) {
    switch (status) {
        case LANTERN_OK: return "ok";
        case LANTERN_E_NULL: return "null pointer argument";
        case LANTERN_E_SHAPE: return "invalid shape argument";
        case LANTERN_E_DTYPE: return "unsupported dtype";
        case LANTERN_E_DELTA: return "delta is NaN or negative";
        case LANTERN_E_TOKEN: return "unusable verification: token, table entry or row index out of range, or unusable logits";
        case LANTERN_E_WORKSPACE: return "workspace missing, misaligned or too small";
        case LANTERN_E_DEVICE: return "HIP call failed";
        default: return "unknown status";
    }
}

int lantern_version(void) { return 227; }

}  // extern "C"
