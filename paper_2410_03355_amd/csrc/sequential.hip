// Walk of draft trees under the sequential-residual sibling rule (Section 2, Algorithm 1 applied
// to the several candidates a tree offers for one position; Section 4.3 for each candidate).
//
// Standing at a node, its children are tried in index order on the logit rows of the first child:
//     t_1 = softmax(target row)
//     child j: the relaxed verification of Section 4.3 with t_j in place of the target;
//              accepted: the walk moves to that child;
//              rejected: t_{j+1} = max(0, t_{j,A} - g) / Z, the residual of that verification
//     every child rejected: the token that follows is drawn from the last residual.
// With k = 1 or delta = 0 this is recursive rejection sampling, which keeps the target law.
//
// The chain t_1, t_2, ... is sequential, so one workgroup of 1024 threads walks one tree and keeps
// the current target and the drafter's distribution as fp64 vectors (unnormalised terms and a
// scale each: no division per token), the drafter's in a workspace (cache resident), the current
// target in LDS when it fits and in the workspace otherwise; evaluated in fp64.  The test of a group's first child is
// the plain verification of that candidate, so its decision is read from the row-parallel pass
// (lantern_decide_rows over all candidates, launched first): only groups whose first child is
// rejected build the vectors.
#include <hip/hip_runtime.h>
#include <limits.h>
#include <stdint.h>

#include "device_utils.h"
#include "exp64.h"
#include "lds_limit.h"
#include "sequential_args.h"
#include "verify_common.h"

namespace lantern {

constexpr int SNT = 1024;
constexpr int SNW = SNT / WAVE;

// Elements a thread keeps in flight per step of a pass: the loads of a step are all issued before
// the first of them is used, so a pass pays the memory latency once per step, not once per element.
constexpr int SU = 8;

// Unnormalised softmax terms exp(l - max) of the target row and of the drafter's row into
// pt[0, V) and pg[0, V) (fp64), and their sums into *zt and *zg: the probabilities are pt[x] / *zt
// and pg[x] / *zg.  Returns false, with the outputs unspecified, if either row has a NaN, a +inf
// or no finite logit.  Ends with every thread past a barrier that follows its last write.
template <typename LT>
__device__ bool softmax_pair(const LT* trow, const LT* grow, int V, double* pt, double* pg, double* zt_out,
                             double* zg_out, ExactShared& sh, int tid) {
    using L = Lane<LT>;
    const float inf = __builtin_huge_valf();
    float mt = -inf, mg = -inf;
    int bad = 0;
    for (int xb = tid; xb < V; xb += SNT * SU) {
        float lt[SU], lg[SU];
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            const int x = xb + u * SNT;
            lt[u] = x < V ? L::glob(trow, x) : -inf;
            lg[u] = x < V ? L::glob(grow, x) : -inf;
        }
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            if (lt[u] != lt[u] || lt[u] == inf || lg[u] != lg[u] || lg[u] == inf) bad = 1;
            mt = fmaxf(mt, lt[u]);
            mg = fmaxf(mg, lg[u]);
        }
    }
    bad = block_or_i<SNW>(bad, sh.ired, tid);
    const double mxt = block_max<SNW>((double)mt, sh.red, tid);
    const double mxg = block_max<SNW>((double)mg, sh.red2, tid);
    if (bad || mxt == -__builtin_huge_val() || mxg == -__builtin_huge_val()) return false;   // uniform
    double zt = 0.0, zg = 0.0;
    for (int xb = tid; xb < V; xb += SNT * SU) {
        float lt[SU], lg[SU];
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            const int x = xb + u * SNT;
            lt[u] = x < V ? L::glob(trow, x) : -inf;
            lg[u] = x < V ? L::glob(grow, x) : -inf;
        }
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            const int x = xb + u * SNT;
            const double et = exp_nonpos((double)lt[u] - mxt);
            const double eg = exp_nonpos((double)lg[u] - mxg);
            if (x < V) {
                pt[x] = et;
                pg[x] = eg;
                zt += et;
                zg += eg;
            }
        }
    }
    *zt_out = block_sum<SNW>(zt, sh.red, tid);
    *zg_out = block_sum<SNW>(zg, sh.red2, tid);
    __syncthreads();
    return true;
}

template <typename LT>
__global__ __launch_bounds__(SNT) void trees_sequential(SequentialArgs a) {
    __shared__ ExactShared sh;
    __shared__ double s_wr[SNW];   // residual mass of every wavefront's part of the vocabulary
    __shared__ double s_wt[SNW];   // mass of the distorted target over the same part

    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1);
    const int wave = tid >> 6;
    const int b = blockIdx.x;
    const int V = a.V;
    const int k = a.k;
    const int M = a.M;
    const int32_t* par = a.parent + (int64_t)b * M;
    int32_t* path = a.out_path + (int64_t)b * M;
    // t_j and the drafter's distribution of the group, both unnormalised: t_j(x) = cur[x] * inv_st,
    // g(x) = g[x] * inv_sg.  The drafter's terms are written once per group and then only read: they
    // stay in the workspace.  t_j is read at random by the walk and rewritten for every rejected
    // child: it lives in LDS when V doubles fit beside the rest (a.cur_in_lds), else in the workspace.
    extern __shared__ __align__(16) unsigned char seq_smem[];
    double* cur = a.cur_in_lds ? reinterpret_cast<double*>(seq_smem) : a.work + (int64_t)b * 2 * V;
    double* g = a.work + (int64_t)b * 2 * V + V;
    double inv_st = 0.0, inv_sg = 0.0, st = 0.0;
    const double delta = (double)a.delta;

    // the part of the vocabulary this wavefront sums and scans: [x0, x1), in steps of 64
    const int per = (((V + SNW - 1) / SNW) + WAVE - 1) & ~(WAVE - 1);
    const int x0 = min(V, wave * per);
    const int x1 = min(V, x0 + per);

    int malformed = 0;
    for (int j = tid; j < M; j += SNT) {
        path[j] = -1;
        const int p = par[j];
        if (p < -1 || p >= j) malformed = 1;
    }
    malformed = block_or_i<SNW>(malformed, sh.ired, tid);
    if (malformed) {
        if (tid == 0) {
            a.out_len[b] = 0;
            a.out_next[b] = -3;
        }
        return;
    }

    int node = -1, len = 0, next = -1;
    for (;;) {   // one sibling group per round; every branch below is uniform over the workgroup
        next = -1;
        int taken = -1;
        int group_row = -1;
        bool have_rows = false;
        int i = node;
        for (;;) {
            // the next child: the smallest index above i whose parent is the node
            int cand = INT_MAX;
            for (int q = i + 1 + tid; q < M; q += SNT)
                if (par[q] == node) {
                    cand = q;
                    break;
                }
            i = block_min_i<SNW>(cand, sh.ired, tid);
            if (i == INT_MAX) break;
            const int64_t c = (int64_t)b * M + i;
            const int r = a.row_index ? a.row_index[c] : (int)c;
            const int xt = a.tokens[c];
            if (!have_rows) {
                // The first child is tested against t_1 = t itself, which is the plain verification the
                // row-parallel pass has already decided for every candidate: an accepted first child is
                // taken without building the group's vectors.
                const int decided = a.accept[c];
                if (decided == 1) {
                    taken = i;
                    break;
                }
                if (decided < 0) {   // unusable row, token or table entry
                    next = -2;
                    break;
                }
                // rejected: the first child brings the group's rows, and is verified again below in
                // fp64 for its distorted target and residual
                have_rows = true;
                group_row = r;
                bool ok = (r >= 0 && r < a.R);
                double sg = 0.0;
                if (ok)
                    ok = softmax_pair<LT>(reinterpret_cast<const LT*>(a.target) + (int64_t)r * a.stride,
                                          reinterpret_cast<const LT*>(a.draft) + (int64_t)r * a.stride, V, cur, g, &st,
                                          &sg, sh, tid);
                inv_st = 1.0 / st;
                inv_sg = 1.0 / sg;
                if (!ok) {
                    next = -2;
                    break;
                }
            }
            bool usable = (r == group_row) && ((unsigned)xt < (unsigned)V);
            const int32_t* nrow = a.knn + (int64_t)(usable ? xt : 0) * k;
            if (usable) {
                int off = 0;
                for (int j = tid; j < k; j += SNT)
                    if ((unsigned)nrow[j] >= (unsigned)V) off = 1;
                usable = block_or_i<SNW>(off, sh.ired, tid) == 0;
            }
            if (!usable) {
                next = -2;
                break;
            }

            // ---- nearest-first walk on t_j (Algorithm 2, inference part) ----
            const double t_tok = cur[xt] * inv_st;
            double carry = 0.0, S = 0.0;
            int a_size = k;
            for (int base = 0; base < k; base += SNT) {
                const int j = base + tid;
                const bool valid = j < k;
                const int n = valid ? nrow[j] : xt;
                const bool self = (n == xt);
                const double tj = self ? 0.0 : cur[n] * inv_st;
                double ctot;
                const double incl = carry + block_scan_incl<SNW>(tj, sh.red, tid, &ctot);
                const int fail_j =
                    (valid && !self && !(prefix_divergence64(a.divergence, t_tok, incl) < delta)) ? j : INT_MAX;
                const int first = block_min_i<SNW>(fail_j, sh.ired, tid);
                if (first != INT_MAX) {
                    a_size = first;
                    if (first == base) {
                        S = carry;
                    } else {
                        if (j == first - 1) sh.bcast[0] = incl;   // the sum before the failing slot
                        __syncthreads();
                        S = sh.bcast[0];
                    }
                    break;
                }
                carry += ctot;
                S = carry;
            }
            const double mass = t_tok + S;
            const double gx = g[xt] * inv_sg;
            const double u_acc = (double)a.uniforms[2 * c];
            const double u_res = (double)a.uniforms[2 * c + 1];
            if (u_acc * gx < mass) {
                taken = i;
                break;
            }

            // ---- rejected: distorted target in place, its residual, the draw, t_{j+1} ----
            __syncthreads();   // every read of t_j by the walk is done
            for (int j = tid; j < a_size; j += SNT) {
                const int n = nrow[j];
                if (n != xt) cur[n] = 0.0;
            }
            if (tid == 0) cur[xt] = mass * st;
            __syncthreads();
            double pr = 0.0, pt = 0.0;
            for (int xb = x0 + lane; xb < x1; xb += WAVE * SU) {
                double ta[SU], gv[SU];
#pragma unroll
                for (int u = 0; u < SU; ++u) {
                    const int x = xb + u * WAVE;
                    ta[u] = x < x1 ? cur[x] : 0.0;
                    gv[u] = x < x1 ? g[x] : 0.0;
                }
#pragma unroll
                for (int u = 0; u < SU; ++u) {
                    const double tn = ta[u] * inv_st;
                    const double d = tn - gv[u] * inv_sg;
                    pr += (d > 0.0) ? d : 0.0;
                    pt += tn;
                }
            }
            pr = wave_sum(pr);
            pt = wave_sum(pt);
            if (lane == 0) {
                s_wr[wave] = pr;
                s_wt[wave] = pt;
            }
            __syncthreads();
            double z = 0.0, zt = 0.0, base_r = 0.0, base_t = 0.0;
#pragma unroll
            for (int w = 0; w < SNW; ++w) {
                if (w < wave) {
                    base_r += s_wr[w];
                    base_t += s_wt[w];
                }
                z += s_wr[w];
                zt += s_wt[w];
            }
            const bool zero_resid = !(z > 0.0);   // the residual has no mass: the distorted target is sampled
            const double zz = zero_resid ? zt : z;
            const double edge = u_res * zz;
            double run = zero_resid ? base_t : base_r;
            int found = INT_MAX;
            for (int xb = x0; xb < x1; xb += WAVE * SU) {   // uniform per wavefront
                double rx[SU];
#pragma unroll
                for (int u = 0; u < SU; ++u) {
                    const int x = xb + u * WAVE + lane;
                    const double ta = x < x1 ? cur[x] : 0.0;
                    const double gv = (x < x1 && !zero_resid) ? g[x] : 0.0;
                    const double d = ta * inv_st - gv * inv_sg;
                    rx[u] = (d > 0.0) ? d : 0.0;
                }
#pragma unroll
                for (int u = 0; u < SU; ++u) {
                    const int x = xb + u * WAVE + lane;
                    const bool valid = x < x1;
                    const double incl = run + wave_scan_incl(rx[u]);
                    const unsigned long long m = __ballot(valid && incl > edge);
                    if (found == INT_MAX && m) found = xb + u * WAVE + __ffsll((long long)m) - 1;
                    run = lane63_d(incl);
                    if (valid) cur[x] = rx[u];   // t_{j+1}, unnormalised: its scale is zz
                }
            }
            st = zz;
            inv_st = 1.0 / zz;
            next = block_min_i<SNW>(found, sh.ired, tid);
            if (next == INT_MAX) next = -1;
            __syncthreads();   // t_{j+1} is complete
        }
        if (taken < 0) break;   // next: -1 no child, -2 unusable, else the last child's resampled token
        if (tid == 0) path[len] = taken;
        len += 1;
        node = taken;
    }
    if (tid == 0) {
        a.out_len[b] = len;
        a.out_next[b] = next;
    }
}

// LDS for the current target: V doubles when they fit beside the static arrays of the kernel.
constexpr size_t SEQ_LDS_BUDGET = 150 * 1024;
static size_t sequential_lds_bytes(int V) {
    const size_t need = (size_t)V * sizeof(double);
    return need <= SEQ_LDS_BUDGET ? need : 0;
}

template <typename LT>
static hipError_t launch_typed(SequentialArgs a, hipStream_t stream, bool launch) {
    const size_t lds = sequential_lds_bytes(a.V);
    a.cur_in_lds = lds > 0 ? 1 : 0;
    const hipError_t e = allow_lds<&trees_sequential<LT>>(lds);
    if (e != hipSuccess || !launch) return e;
    hipLaunchKernelGGL((trees_sequential<LT>), dim3(a.B), dim3(SNT), lds, stream, a);
    return hipGetLastError();
}

// Loads the kernels on the current device and raises their LDS limit for this vocabulary size.
hipError_t prepare_sequential(int logits_dtype, int V) {
    SequentialArgs a{};
    a.V = V;
    hipFuncAttributes attr;
    hipError_t e = hipFuncGetAttributes(&attr, logits_dtype == 0
                                                   ? reinterpret_cast<const void*>(&trees_sequential<float>)
                                                   : reinterpret_cast<const void*>(&trees_sequential<uint16_t>));
    if (e != hipSuccess) return e;
    return logits_dtype == 0 ? launch_typed<float>(a, nullptr, false) : launch_typed<uint16_t>(a, nullptr, false);
}

hipError_t launch_trees_sequential(const SequentialArgs& a, int logits_dtype, hipStream_t stream) {
    return logits_dtype == 0 ? launch_typed<float>(a, stream, true) : launch_typed<uint16_t>(a, stream, true);
}

}  // namespace lantern
