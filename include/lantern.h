/*
 * lantern.h - C ABI of the MI355X (gfx950) library for LANTERN's relaxed
 * speculative-decoding verification (arXiv 2410.03355).
 *
 * The two operations of the method:
 *   lantern_build_knn  the latent-space neighbour table B_k of the VQ codebook
 *                      (Section 4.2; Algorithm 2, precompute part)
 *   lantern_verify     one relaxed verification per row: TVD-bounded
 *                      neighbourhood A_{k,delta}, acceptance test, residual
 *                      resampling (Section 4.3; Algorithm 2, inference part;
 *                      Algorithm 1, the accept / resample branch)
 * and what the paper builds around them:
 *   lantern_build_knn_metric, lantern_build_random   the cosine and random
 *                      neighbourhoods of the ablation (Section 5.3.1)
 *   lantern_verify_divergence   the Jensen-Shannon bound (Section 5.3.2)
 *   lantern_verify_greedy       greedy decoding (Section 4.3, last sentence)
 *   lantern_accept_chains, lantern_accept_trees   the loop of Algorithm 1
 *                      over a drafted chain / along the branches of a tree
 *   lantern_verify_rows, lantern_verify_greedy_rows   candidates that share
 *                      logit rows (siblings of a draft tree)
 *   lantern_decide_rows, lantern_resample_selected, lantern_verify_trees
 *                      decisions for all candidates, the residual draw only
 *                      where Algorithm 1 uses it
 *   lantern_verify_trees_greedy   the tree step under greedy decoding
 *   lantern_verify_trees_sequential   the tree step with siblings verified one
 *                      after the other against the residual of those before
 *
 * Naming.  The paper writes p for the drafter and q for the target model.
 * Other texts use the letters the other way round, so this header uses
 * neither: arguments are called target_* and draft_*.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller and must stay
 *     valid until the work enqueued on the stream has finished.  The library
 *     allocates nothing, frees nothing and keeps no state between calls that
 *     a result could depend on.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default
 *     stream).  Calls only enqueue kernels; they do not synchronise.  The
 *     current HIP device must be the one that owns the pointers and the
 *     stream.  Calls may come from several host threads.
 *   - One exception to "only enqueue": the first time a kernel needs more
 *     than 64 KiB of LDS on a device, its limit is raised with a runtime call
 *     (hipFuncSetAttribute), and the runtime loads a kernel on its first use.
 *     Neither belongs inside a stream capture: call lantern_prepare for the
 *     shape beforehand, or make one call of the shape outside the capture.
 *   - The return value is a lantern_status.  Argument errors are found on the
 *     host before anything is launched; then nothing is written.
 *   - Row-level problems that only the device can see (see lantern_verify) are
 *     reported per row through sentinel outputs, not through the status.
 */
#ifndef LANTERN_H
#define LANTERN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LANTERN_F32 = 0,  /* IEEE binary32                       */
    LANTERN_BF16 = 1  /* bfloat16 (upper 16 bits of binary32) */
} lantern_dtype;

typedef enum {
    LANTERN_OK = 0,
    LANTERN_E_NULL = -1,      /* a required pointer is NULL                           */
    LANTERN_E_SHAPE = -2,     /* V<1, d<1, N<0, k<1, k>V, row stride < V, V too large  */
    LANTERN_E_DTYPE = -3,     /* dtype is not one of lantern_dtype                     */
    LANTERN_E_DELTA = -4,     /* delta is NaN or negative                              */
    LANTERN_E_TOKEN = -5,     /* a verification was unusable (see below); never returned
                                 by the calls here, which are asynchronous: raised by the
                                 Python binding's checked mode after it has synchronised */
    LANTERN_E_WORKSPACE = -6, /* workspace missing, misaligned or too small            */
    LANTERN_E_DEVICE = -7     /* a HIP call failed (launch error, no device)           */
} lantern_status;

typedef enum {
    LANTERN_METRIC_L2 = 0,    /* squared l2 distance, the paper's choice (Section 5.1) */
    LANTERN_METRIC_COSINE = 1 /* cosine similarity (ablation, Section 5.3.1)           */
} lantern_metric;

typedef enum {
    LANTERN_DIV_TVD = 0,      /* total variation distance, the paper's choice (Section 4.3) */
    LANTERN_DIV_JSD = 1       /* Jensen-Shannon divergence, natural logarithm (ablation, Section 5.3.2) */
} lantern_divergence;

/* Largest vocabulary lantern_verify accepts (a bitmask of one row and its partial sums must fit in LDS). */
#define LANTERN_MAX_VOCAB (1 << 19)

/*
 * Bytes of device workspace lantern_build_knn needs for this problem, or 0 if
 * the arguments are invalid.  The workspace holds, for a block of query rows,
 * either candidate lists and the rows' approximate distances to a sample of
 * the codebook, or their approximate distances to every token (which of the
 * two depends on V and k alone); its contents are scratch.  Sized for few,
 * large launches: up to about 850 MiB (V = 65536, k = 1000), 528 MiB for
 * V = 16384, k = 1000.
 */
size_t lantern_build_knn_workspace_bytes(lantern_dtype cb_dtype, int V, int d, int k);

/*
 * Neighbour table of the codebook: row x lists x and the k-1 codes closest to
 * it in latent space (B_k of Section 4.2; Algorithm 2, precompute part).
 *
 *   codebook   [V, d] row-major, dtype cb_dtype, device memory, 16-byte aligned
 *   out_knn    [V, k] row-major int32, device memory.  Row i holds i itself in
 *              slot 0, then the k-1 other tokens in increasing distance.  The
 *              distance that decides the order is the squared l2 distance
 *              evaluated in fp64 as sum over coordinates, in index order, of
 *              (c_i[t]-c_j[t])^2 with every operation rounded separately;
 *              equal distances are ordered by the lower token index.  A
 *              distance that is not a number (infinite or NaN coordinates;
 *              under the cosine key a code of zero norm, 0/0) counts as
 *              +infinity: such a pair is the farthest possible.
 *   workspace  device memory of at least lantern_build_knn_workspace_bytes,
 *              256-byte aligned.  Scratch, except that when the work has
 *              finished its first int32 holds the number of rows whose
 *              pre-selection could not be proven complete and that were
 *              therefore ranked from all V exact distances (slow; zero for
 *              codebooks without massive exact ties).
 *
 * An approximate distance from a matrix-core contraction, and for larger k a
 * per-row threshold estimated from a sample of the codebook, only pre-select
 * candidates; the order written is always the fp64 one, and a row whose
 * pre-selection cannot be proven complete is ranked from all V distances, so
 * the result depends neither on the contraction's rounding nor on the sample.
 * Errors: E_NULL, E_SHAPE (k>V, V<1, d<1, k<1), E_DTYPE, E_WORKSPACE, E_DEVICE.
 */
int lantern_build_knn(const void* codebook, lantern_dtype cb_dtype, int V, int d, int k,
                      int32_t* out_knn, void* workspace, size_t workspace_bytes, void* hip_stream);

/* As lantern_build_knn with a choice of metric. */
int lantern_build_knn_metric(const void* codebook, lantern_dtype cb_dtype, int V, int d, int k,
                             int metric, int32_t* out_knn, void* workspace, size_t workspace_bytes,
                             void* hip_stream);

/*
 * lantern_build_knn_metric for callers that cannot allocate device memory and
 * so cannot bring a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The workspace is a static device
 * array inside the library (LANTERN_STATIC_SCRATCH_BYTES, held on every GPU
 * the library runs on until the process ends); the call allocates and frees
 * nothing.  Same table, bit for bit, as lantern_build_knn_metric.
 *
 *   out_exact_rows  device int32 or NULL: receives the number of rows ranked
 *                   by the all-pairs pass (what lantern_build_knn leaves in the
 *                   first word of its workspace)
 * Limits: V <= LANTERN_STATIC_MAX_V; beyond that E_WORKSPACE, nothing launched.
 * All calls on one GPU share that GPU's scratch (the library clears what must
 * start at zero): calls that overlap in time on one GPU - from several streams
 * or threads - race and give undefined tables; serialise them.  The first call
 * on a device looks the array's address up (a runtime call, no allocation):
 * make it outside a stream capture.  The HIP runtime places the array in device
 * memory when it loads the library's device code, which it may put off until
 * the first launch of these kernels in the process: free device memory can
 * drop by the array's size across that one call, never across a later one.
 * Errors: E_NULL, E_SHAPE, E_DTYPE, E_WORKSPACE (V over the limit), E_DEVICE.
 */
#define LANTERN_STATIC_MAX_V 32768
#define LANTERN_STATIC_SCRATCH_BYTES (40u << 20)
int lantern_build_knn_static(const void* codebook, lantern_dtype cb_dtype, int V, int d, int k, int metric,
                             int32_t* out_knn, int32_t* out_exact_rows, void* hip_stream);

/*
 * N independent relaxed verifications (Section 4.3, final rule):
 *   t = softmax(target row), g = softmax(draft row), xt = draft token
 *   walk knn[xt, 0..k) nearest first; a neighbour x != xt is taken while the
 *   total variation distance after moving t(x) onto xt stays strictly below
 *   delta; the first that does not fit ends the walk; xt is always taken
 *   mass = sum of t over the taken set A
 *   accept iff u_accept * g(xt) < mass          (i.e. u < min(1, mass/g(xt)))
 *   else resample from max(0, t_A - g) normalised, where t_A is t with mass at
 *   xt and zero on A \ {xt}: the first token, in index order, whose cumulative
 *   residual exceeds u_resample * (total residual)
 *
 *   target_logits, draft_logits  [N, V] with row_stride_elems elements between
 *                rows (>= V), dtype logits_dtype.  -inf marks a filtered token.
 *   draft_tokens [N] int32
 *   knn          [V, k] int32 neighbour table (entries of a row distinct)
 *   delta        TVD bound, >= 0.  delta = 0 or k = 1 gives standard
 *                speculative acceptance min(1, t(xt)/g(xt)).  The bound IS the
 *                binary32 number passed here, widened exactly where the rule
 *                is evaluated in fp64: a caller who writes 0.4 gets the bound
 *                0.4000000059604645 (the float nearest to 0.4), and a prefix
 *                whose TVD lies between 0.4 and that number is inside it.
 *   uniforms     [N, 2] float32 in [0,1): column 0 acceptance draw, column 1
 *                resampling draw.  The library draws no random numbers.
 *   out_accept   [N] int32: 1 accepted, 0 rejected
 *   out_resample [N] int32: resampled token when rejected, -1 when accepted
 *
 * Rows the device finds unusable - draft token outside [0,V), any of the k
 * entries of its table row outside [0,V) (all k are checked, also those the
 * walk never reaches), a NaN or +inf logit, or no finite logit - get
 * out_accept = -1 and out_resample = -1; other rows are unaffected.
 *
 * Decisions are exact with respect to fp64 evaluation of the rule above: a
 * fast fp32 pass settles every row whose comparisons clear a proven rounding
 * margin, and the remaining rows (and all rejected rows, whose inverse-CDF
 * bucket cannot be settled in fp32) are evaluated in fp64.  Two fp64
 * evaluations that add in different orders agree to about 1e-15 relative, so
 * a comparison whose sides are closer than that has no defined outcome: this
 * is so by construction for delta = 1 with a table row that lists every token
 * when t(xt) = 0, where the prefix sum equals delta in exact arithmetic.
 * A rejected row
 * therefore costs many times an accepted one (about 23 us of one compute unit
 * at V = 16384); callers that walk chains or trees and use one resampled
 * token per walk should use lantern_decide_rows / lantern_resample_selected or
 * lantern_verify_trees below.
 *
 * Errors: E_NULL, E_SHAPE (also V > LANTERN_MAX_VOCAB), E_DTYPE, E_DELTA,
 * E_DEVICE.  N = 0 is valid and does nothing.
 */
int lantern_verify(const void* target_logits, const void* draft_logits, lantern_dtype logits_dtype,
                   int N, int V, int64_t row_stride_elems, const int32_t* draft_tokens,
                   const int32_t* knn, int k, float delta, const float* uniforms,
                   int32_t* out_accept, int32_t* out_resample, void* hip_stream);

/*
 * lantern_verify plus optional per-row diagnostics (each pointer may be NULL):
 *   out_accept_prob [N] float  min(1, mass/g(xt))
 *   out_mass        [N] float  sum of t over A_{k,delta}(xt)
 *   out_g_tok       [N] float  g(xt)
 *   out_a_size      [N] int32  number of table slots taken into A
 *   out_path        [N] int32  0: settled by the fp32 pass, 1: evaluated in fp64
 * Unusable rows get NaN / -1 in the diagnostics.
 * The three probabilities are binary32 values for inspection, not inputs of
 * any decision: for a row settled by the fp32 pass they are formed from its
 * fp32 terms (about 1e-5 relative for fp32 logits, 2e-3 for bf16), and where
 * t(xt) or g(xt) lies below the smallest normal binary32 number (a token some
 * 87 nats under the row's maximum) they lose precision or read zero, and
 * out_accept_prob with them.  Decisions and out_a_size are not affected.
 */
int lantern_verify_ex(const void* target_logits, const void* draft_logits,
                      lantern_dtype logits_dtype, int N, int V, int64_t row_stride_elems,
                      const int32_t* draft_tokens, const int32_t* knn, int k, float delta,
                      const float* uniforms, int32_t* out_accept, int32_t* out_resample,
                      float* out_accept_prob, float* out_mass, float* out_g_tok,
                      int32_t* out_a_size, int32_t* out_path, void* hip_stream);

/*
 * lantern_verify_ex with a choice of the divergence that bounds the neighbourhood
 * (Section 5.3.2 compares the two): the walk takes a neighbour while the
 * divergence between the distorted target and the target, after adding it,
 * stays strictly below delta.  LANTERN_DIV_TVD is lantern_verify_ex itself.
 * For LANTERN_DIV_JSD the divergence of a prefix is
 *   1/2 [ m ln(2m/(m+t0)) + t0 ln(2 t0/(m+t0)) + (m - t0) ln 2 ],
 * t0 = t(xt), m = mass of the prefix (the entries where the two distributions
 * differ; it never exceeds ln 2).  All other arguments, outputs and errors as
 * in lantern_verify_ex; an unknown divergence is E_SHAPE.
 */
int lantern_verify_divergence(const void* target_logits, const void* draft_logits,
                              lantern_dtype logits_dtype, int N, int V, int64_t row_stride_elems,
                              const int32_t* draft_tokens, const int32_t* knn, int k, int divergence,
                              float delta, const float* uniforms, int32_t* out_accept, int32_t* out_resample,
                              float* out_accept_prob, float* out_mass, float* out_g_tok,
                              int32_t* out_a_size, int32_t* out_path, void* hip_stream);

/*
 * Greedy-decoding variant (Section 4.3, last sentence): accept the draft token
 * xt iff xt = argmax_x t_A(x), where t_A is the target distribution distorted
 * by A_{k,delta}(xt) (the mass of A at xt, zero on the rest of A, t elsewhere).
 * Equal values go to the lower token index.  No drafter logits and no random
 * draws are involved.
 *
 *   target_logits, draft_tokens, knn, k, delta   as in lantern_verify
 *   out_accept [N] int32: 1 accepted, 0 rejected
 *   out_token  [N] int32: -1 when accepted, else argmax_x t_A(x), the token
 *              greedy decoding of the distorted target emits
 *   out_path   [N] int32 or NULL: 0 settled by the fp32 pass, 1 evaluated in fp64
 * Unusable rows (see lantern_verify) get -1 in both outputs.  Decisions are
 * exact with respect to fp64 evaluation, as for lantern_verify.
 * Errors: E_NULL, E_SHAPE, E_DTYPE, E_DELTA, E_DEVICE.
 */
int lantern_verify_greedy(const void* target_logits, lantern_dtype logits_dtype, int N, int V,
                          int64_t row_stride_elems, const int32_t* draft_tokens, const int32_t* knn, int k,
                          float delta, int32_t* out_accept, int32_t* out_token, int32_t* out_path,
                          void* hip_stream);

/*
 * Walk of B drafted chains of L candidates each (Algorithm 1, the loop over
 * the drafts): chain b owns rows b*L .. b*L+L-1 of the outputs of
 * lantern_verify (or lantern_verify_greedy), in drafting order.  Drafts are
 * kept while they are accepted; the first candidate that is not accepted ends
 * the chain with its resampled token.
 *
 *   accept, resample  [B*L] int32, as written by lantern_verify
 *   out_len   [B] int32: number of drafts kept (0..L)
 *   out_next  [B] int32: the token that follows them: the resampled token of
 *             the first rejected candidate; -1 when all L were accepted (the
 *             caller then samples the extra token from the target's next row);
 *             -2 when the chain was ended by an unusable row (accept = -1)
 * Errors: E_NULL, E_SHAPE (B < 0, L < 1), E_DEVICE.  B = 0 does nothing.
 */
int lantern_accept_chains(const int32_t* accept, const int32_t* resample, int B, int L, int32_t* out_len,
                          int32_t* out_next, void* hip_stream);

/*
 * Random neighbourhood table (Section 5.3.1 and Table 3: the ablation that
 * selects the k tokens at random instead of by latent proximity).  Row x holds
 * x in slot 0 and then k-1 other tokens, a uniform sample without replacement
 * in random order, fixed by the seed: the pair (x, y) gets as key word y mod 4
 * of Philox4x32-10 at counter (y div 4, x, 0, 0) under the key (seed low word,
 * seed high word), and the row lists the other tokens by increasing
 * (key, token).  The table for a smaller k is a prefix of the one for a
 * larger k.  It feeds lantern_verify like the table of lantern_build_knn.
 *
 *   out_knn  device, [V, k] int32, written
 * Limits: k <= LANTERN_RANDOM_MAX_K.  Should more than 4096 keys of one row
 * share a 32-bit value (not with this generator), that row's slots 1..k-1
 * are written as -1, which lantern_verify reports as unusable.
 * Errors: E_SHAPE (V < 1, V > LANTERN_MAX_VOCAB, k < 1, k > V, k over the
 * limit), E_NULL, E_DEVICE.
 */
#define LANTERN_RANDOM_MAX_K 4096
int lantern_build_random(int V, int k, uint64_t seed, int32_t* out_knn, void* hip_stream);

/*
 * Verification over shared logit rows.  A draft tree holds several candidate
 * tokens for one position (the paper verifies 60 candidates per step of the
 * target model, Appendix on experimental details); the siblings are verified
 * against the same pair of distributions, the ones after their parent's
 * prefix.  Verification i reads row row_index[i] of both logit matrices; all
 * else is lantern_verify (divergence as in lantern_verify_divergence) and
 * lantern_verify_greedy.
 *
 *   target_logits, draft_logits  device, [R, V] rows of row_stride_elems
 *   row_index     device, [N] int32, values in [0, R); a value outside makes
 *                 that verification unusable (-1 in both outputs)
 *   draft_tokens, uniforms, outputs  [N], one per verification
 * Errors: as lantern_verify; E_SHAPE also for R < 1 with N > 0; E_NULL for a
 * missing row_index.  N = 0 does nothing.
 */
int lantern_verify_rows(const void* target_logits, const void* draft_logits, lantern_dtype logits_dtype,
                        int R, int V, int64_t row_stride_elems, const int32_t* row_index, int N,
                        const int32_t* draft_tokens, const int32_t* knn, int k, int divergence, float delta,
                        const float* uniforms, int32_t* out_accept, int32_t* out_resample, void* hip_stream);

int lantern_verify_greedy_rows(const void* target_logits, lantern_dtype logits_dtype, int R, int V,
                               int64_t row_stride_elems, const int32_t* row_index, int N,
                               const int32_t* draft_tokens, const int32_t* knn, int k, float delta,
                               int32_t* out_accept, int32_t* out_token, void* hip_stream);

/*
 * Walk of B drafted trees of M candidate nodes each (Algorithm 1 applied along
 * the branches).  Tree b owns rows b*M .. b*M+M-1 of accept / resample /
 * parent, in drafting order.  parent[i] is the node of the same tree whose
 * token precedes node i, or -1 when node i follows the committed prefix;
 * parent[i] < i.  The paper leaves the rule for siblings to its drafter; the
 * rule here: standing at a node (first the prefix), its children are tried in
 * index order, the first accepted one is taken and the walk goes on from it.
 * With one child per node this is lantern_accept_chains.  With more than one
 * child per node the walk does NOT preserve the target's law, not even at
 * delta = 0 or k = 1 where a chain does: every sibling is tested on its own
 * against the undistorted rows, while law-preserving multi-candidate sampling
 * would test sibling j against the residual left by siblings 1 .. j-1.
 *
 *   accept, resample  [B*M] int32, as written by lantern_verify_rows;
 *             resample may be NULL: out_next then holds, where it would hold a
 *             resampled token, the index b*M + node of the verification whose
 *             resampled token it is (for lantern_resample_selected)
 *   parent    [B*M] int32
 *   out_len   [B] int32: number of accepted nodes
 *   out_path  [B*M] int32: the accepted nodes of tree b, in order, then -1
 *   out_next  [B] int32: the token after them: when every child of the last
 *             node was rejected, the resampled token of its first child (the
 *             candidate Algorithm 1 tries at that position); -1 when the last
 *             node has no child (all drafts of the branch accepted, the caller
 *             samples the extra token); -2 when an unusable child (accept < 0)
 *             was met before an accepted one; -3, with len 0, when the tree's
 *             parent array is malformed
 * Errors: E_NULL, E_SHAPE (B < 0, M < 1), E_DEVICE.  B = 0 does nothing.
 */
int lantern_accept_trees(const int32_t* accept, const int32_t* resample, const int32_t* parent, int B, int M,
                         int32_t* out_len, int32_t* out_path, int32_t* out_next, void* hip_stream);

/*
 * The same verification split in two, for callers that need the resampled
 * token of few verifications only.  Algorithm 1 leaves its loop at the first
 * rejection: of all the candidates of a chain or tree, one residual is sampled.
 *
 * lantern_decide_rows: the decisions of lantern_verify_rows without the
 * resampled tokens (a rejection is then settled by the fp32 pass as well).
 *   row_index  may be NULL when R == N: verification i reads row i
 *   out_accept [N] int32: 1, 0, or -1 for an unusable verification; equal to
 *              what lantern_verify_rows writes
 *   out_path   [N] int32 or NULL: 0 settled by the fp32 pass, 1 evaluated in fp64
 *
 * lantern_resample_selected: for i < n_sel, the resampled token of
 * verification select[i], from the same inputs.
 *   select     device, [n_sel] int32: verification indices in [0, N); a
 *              negative entry is copied to out_token[i] unchanged (the codes of
 *              lantern_accept_trees pass through)
 *   out_token  device, [n_sel] int32: the token lantern_verify_rows would write
 *              to out_resample[select[i]] if that verification is rejected; -1
 *              if it is accepted; -2 if it is unusable or select[i] >= N.  May
 *              be the same array as select.
 * Errors: as lantern_verify_rows; E_SHAPE also for n_sel < 0, for n_sel > 0
 * with N == 0, and for a NULL row_index with R != N.
 */
int lantern_decide_rows(const void* target_logits, const void* draft_logits, lantern_dtype logits_dtype,
                        int R, int V, int64_t row_stride_elems, const int32_t* row_index, int N,
                        const int32_t* draft_tokens, const int32_t* knn, int k, int divergence, float delta,
                        const float* uniforms, int32_t* out_accept, int32_t* out_path, void* hip_stream);

int lantern_resample_selected(const void* target_logits, const void* draft_logits, lantern_dtype logits_dtype,
                              int R, int V, int64_t row_stride_elems, const int32_t* row_index, int N,
                              const int32_t* draft_tokens, const int32_t* knn, int k, int divergence,
                              float delta, const float* uniforms, const int32_t* select, int n_sel,
                              int32_t* out_token, void* hip_stream);

/*
 * One verification step over B draft trees of M candidates (Algorithm 1 along
 * the branches; rule of lantern_accept_trees): decisions of all B*M
 * candidates, the walk, and the residual draw of the one candidate per tree
 * whose token is needed.  Same results as lantern_verify_rows followed by
 * lantern_accept_trees, without the resampling work that the walk never
 * looks at.  Two launches: the decisions; then one workgroup per tree walks
 * it and draws the residual.
 *
 *   row_index, draft_tokens, uniforms, parent  [B*M], candidate i of tree b at b*M + i;
 *              row_index may be NULL when R == B*M (candidate i reads row i: drafted
 *              chains, parent[i] = i - 1, have a pair of rows per candidate)
 *   out_accept [B*M], out_len [B], out_path [B*M], out_next [B]  as in
 *              lantern_verify_rows / lantern_accept_trees
 * Errors: those of the three calls; E_SHAPE also when B*M exceeds INT_MAX.
 */
int lantern_verify_trees(const void* target_logits, const void* draft_logits, lantern_dtype logits_dtype,
                         int R, int V, int64_t row_stride_elems, const int32_t* row_index,
                         const int32_t* parent, int B, int M, const int32_t* draft_tokens, const int32_t* knn,
                         int k, int divergence, float delta, const float* uniforms, int32_t* out_accept,
                         int32_t* out_len, int32_t* out_path, int32_t* out_next, void* hip_stream);

/*
 * The tree step under greedy decoding (Section 4.3, last sentence, along the
 * branches of Algorithm 1): lantern_verify_greedy_rows for all B*M candidates,
 * then lantern_accept_trees on its outputs.  No drafter logits, no random
 * draws; the token that follows a branch is the arg-max of the distorted
 * target of the first child of its last node.
 *   row_index  may be NULL when R == B*M
 *   out_accept, out_token [B*M]; out_len [B], out_path [B*M], out_next [B]
 * Errors: those of the two calls.
 */
int lantern_verify_trees_greedy(const void* target_logits, lantern_dtype logits_dtype, int R, int V,
                                int64_t row_stride_elems, const int32_t* row_index, const int32_t* parent, int B,
                                int M, const int32_t* draft_tokens, const int32_t* knn, int k, float delta,
                                int32_t* out_accept, int32_t* out_token, int32_t* out_len, int32_t* out_path,
                                int32_t* out_next, void* hip_stream);

/*
 * The tree step under the sequential-residual sibling rule (Section 2 and
 * Algorithm 1: a rejected draft is followed by the residual distribution;
 * Section 4.3 for each candidate).  lantern_verify_trees tests every child of
 * a node against the same target, which with more than one child per node
 * does not keep the target law even at k = 1.  Here the children of a node are
 * tried one after the other, in index order, on the logit rows of the first
 * child: the first against t_1 = the target distribution of those rows; child
 * j + 1, reached when child j was rejected, against t_{j+1} = the normalised
 * residual max(0, t_{j,A} - g) / Z of child j's verification, with the
 * neighbourhood, the mass and the acceptance test of Section 4.3 all taken on
 * t_{j+1}.  The first accepted child is taken and the walk goes on from it.
 * With k = 1 or delta = 0 and tokens drawn independently from g this is
 * recursive rejection sampling, and the emitted token follows the target.
 * Two launches: the plain verification of all B*M candidates (it decides the
 * first child of every group, whose test is against t_1 itself), then one
 * workgroup per tree that walks it and evaluates the residual targets in fp64.
 *
 *   row_index, draft_tokens, uniforms, parent  [B*M] as in lantern_verify_trees
 *              (row_index may be NULL when R == B*M); each candidate owns its
 *              two draws, uniforms[2i] for the acceptance test and
 *              uniforms[2i+1] for the residual draw
 *   out_len    [B], out_path [B*M] as in lantern_accept_trees
 *   out_next   [B] int32: when every child of the last node was rejected, the
 *              token drawn from the residual of its last child; -1 when the
 *              last node has no child; -2 when a child that had to be tried is
 *              unusable (row index, token or a table entry out of range, logit
 *              rows with a NaN, a +inf or no finite entry, or a row index other
 *              than the first child's); -3, with len 0, for a malformed parent
 *              array
 *   workspace  device memory, 256-byte aligned, of at least
 *              lantern_verify_trees_sequential_workspace_bytes(B, M, V) bytes
 *              (2 V doubles per tree and 4 bytes per candidate; 0 for invalid
 *              arguments and for B = 0); owned by the
 *              caller, contents unspecified afterwards, must not be shared by
 *              calls that may overlap
 * Errors: E_DTYPE, E_SHAPE (as lantern_verify_trees, and an unknown
 * divergence), E_DELTA, E_NULL, E_WORKSPACE, E_DEVICE.  B = 0 does nothing.
 */
size_t lantern_verify_trees_sequential_workspace_bytes(int B, int M, int V);

int lantern_verify_trees_sequential(const void* target_logits, const void* draft_logits, lantern_dtype logits_dtype,
                                    int R, int V, int64_t row_stride_elems, const int32_t* row_index,
                                    const int32_t* parent, int B, int M, const int32_t* draft_tokens,
                                    const int32_t* knn, int k, int divergence, float delta, const float* uniforms,
                                    int32_t* out_len, int32_t* out_path, int32_t* out_next, void* workspace,
                                    size_t workspace_bytes, void* hip_stream);

/*
 * Measurement aid, not part of the method: reads the first bytes / 65536 whole
 * 64 KiB chunks of src_a, and of src_b when it is not NULL, once, with the
 * access pattern of the verification kernel (one workgroup per chunk, 16-byte
 * loads), and discards them.  Timed by the caller it gives the read rate the
 * device reaches for such a stream.
 *   src_a, src_b  device, 16-byte aligned;  sink  device, one uint32
 *                 (practically never written)
 * Errors: E_NULL, E_SHAPE (alignment, more than 2^30 - 1 chunks), E_DEVICE.
 */
int lantern_probe_stream_read(const void* src_a, const void* src_b, size_t bytes, uint32_t* sink,
                              void* hip_stream);

/*
 * Set-up for callers that record calls into a HIP graph (or want the first
 * call of a shape to cost what the later ones do): on the current device,
 * loads the kernels and raises the LDS limit of every kernel that the
 * verification entry points above (sampling, greedy, rows, decide, selected,
 * trees, chain and tree walks) can launch for this logit type, vocabulary size
 * and table width, whatever the alignment of the buffers turns out to be.
 * Enqueues nothing; must itself be called outside a stream capture; once per
 * device and shape is enough, repeating it is harmless.
 * Errors: E_DTYPE, E_SHAPE (V < 1, V > LANTERN_MAX_VOCAB, k < 1, k > V), E_DEVICE.
 */
int lantern_prepare(lantern_dtype logits_dtype, int V, int k);

/* Human-readable name of a status code (static string, never NULL). */
const char* lantern_status_string(int status);

/* Library version as major*10000 + minor*100 + patch. */
int lantern_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LANTERN_H */
