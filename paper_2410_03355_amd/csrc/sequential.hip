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
// the current target and the drafter's distribution as fp64 probability vectors in a workspace
// (2 V doubles per tree, cache resident), evaluated in fp64.  The test of a group's first child is
// the plain verification of that candidate, so its decision is read from the row-parallel pass
// (lantern_decide_rows over all candidates, launched first): only groups whose first child is
// rejected build the vectors.
#include <hip/hip_runtime.h>
#include <limits.h>
#include <stdint.h>

#include "device_utils.h"
#include "exp64.h"
#include "sequential_args.h"
#include "verify_common.h"

namespace lantern {

constexpr int SNT = 1024;
constexpr int SNW = SNT / WAVE;

__device__ __forceinline__ double lane63_d(double v) {
    const unsigned long long u = (unsigned long long)__double_as_longlong(v);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(u & 0xffffffffull), 63);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(u >> 32), 63);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// Elements a thread keeps in flight per step of a pass: the loads of a step are all issued before
// the first of them is used, so a pass pays the memory latency once per step, not once per element.
constexpr int SU = 8;

// softmax of the target row and of the drafter's row into pt[0, V) and pg[0, V) (fp64):
// exp(l - max) / sum for each.  Returns false, with the outputs unspecified, if either row has a
// NaN, a +inf or no finite logit.  Ends with every thread past a barrier that follows its last
// write.
template <typename LT>
__device__ bool softmax_pair(const LT* trow, const LT* grow, int V, double* pt, double* pg, ExactShared& sh, int tid) {
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
    zt = block_sum<SNW>(zt, sh.red, tid);
    zg = block_sum<SNW>(zg, sh.red2, tid);
    for (int xb = tid; xb < V; xb += SNT * SU) {   // the elements this thread wrote
        double et[SU], eg[SU];
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            const int x = xb + u * SNT;
            et[u] = x < V ? pt[x] : 0.0;
            eg[u] = x < V ? pg[x] : 0.0;
        }
#pragma unroll
        for (int u = 0; u < SU; ++u) {
            const int x = xb + u * SNT;
            if (x < V) {
                pt[x] = et[u] / zt;
                pg[x] = eg[u] / zg;
            }
        }
    }
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
    double* cur = a.work + (int64_t)b * 2 * V;   // t_j
    double* g = cur + V;                          // the drafter's distribution of the group
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
                if (ok)
                    ok = softmax_pair<LT>(reinterpret_cast<const LT*>(a.target) + (int64_t)r * a.stride,
                                          reinterpret_cast<const LT*>(a.draft) + (int64_t)r * a.stride, V, cur, g, sh, tid);
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
            const double t_tok = cur[xt];
            double carry = 0.0, S = 0.0;
            int a_size = k;
            for (int base = 0; base < k; base += SNT) {
                const int j = base + tid;
                const bool valid = j < k;
                const int n = valid ? nrow[j] : xt;
                const bool self = (n == xt);
                const double tj = self ? 0.0 : cur[n];
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
            const double gx = g[xt];
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
            if (tid == 0) cur[xt] = mass;
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
                    const double d = ta[u] - gv[u];
                    pr += (d > 0.0) ? d : 0.0;
                    pt += ta[u];
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
                    const double d = ta - gv;
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
                    if (valid) cur[x] = rx[u] / zz;
                }
            }
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

hipError_t prepare_sequential() {
    hipFuncAttributes attr;
    hipError_t e = hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(&trees_sequential<float>));
    if (e == hipSuccess) e = hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(&trees_sequential<uint16_t>));
    return e;
}

hipError_t launch_trees_sequential(const SequentialArgs& a, int logits_dtype, hipStream_t stream) {
    if (logits_dtype == 0)
        hipLaunchKernelGGL((trees_sequential<float>), dim3(a.B), dim3(SNT), 0, stream, a);
    else
        hipLaunchKernelGGL((trees_sequential<uint16_t>), dim3(a.B), dim3(SNT), 0, stream, a);
    return hipGetLastError();
}

}  // namespace lantern
