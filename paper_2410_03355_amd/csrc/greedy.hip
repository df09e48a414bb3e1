// Greedy-decoding variant of the relaxed verification (Section 4.3, last
// sentence): accept the draft token xt iff it is the arg-max of the distorted
// target t_A (the mass of A_{k,delta}(xt) at xt, zero on the rest of A, t
// elsewhere); otherwise emit that arg-max.  Ties go to the lower token index.
//
// Outside A the distorted target is t, so its arg-max there is the arg-max of
// the raw logits, an exact comparison.  Only two floating-point comparisons
// decide a row: the TVD cut and "mass of A against the largest t outside A".
// The fp32 path takes both under the rounding margin of the sampling kernel;
// rows that do not clear it are re-evaluated in fp64 by the same workgroup.
// One workgroup per row; the target row is streamed from HBM once.
#include "fast_cut.h"
#include "lds_limit.h"
#include "verify_args.h"
#include "verify_common.h"

namespace lantern {

struct GreedyShared {
    float wmax[NW];       // per-wave maxima over the sampled part of the row
    float wsum[NW];       // per-wave sums of exponentials
    float wemax[NW];      // per-wave largest exponential
    float wtot[NW];       // scan: wavefront totals
    int wbad[NW];
    float best_val[NW];   // arg-max outside A: per-wave value and lowest index
    int best_idx[NW];
    int cut_np[NW];       // per wavefront: first slot not definitely passing, first slot definitely
    int cut_df[NW];       // failing, and the sum before the former
    float cut_s[NW];
    int tail[4];          // the walk beyond slot 1024 (k > 1024): slots taken, sum, definite, bad
    // from here on the memory is reused by the exact path once the fp32 path gives up
    float gs[NT * 4];
    unsigned gskip[NT];
};
constexpr size_t GREEDY_SHARED_HEAD = offsetof(GreedyShared, gs);
constexpr size_t GREEDY_SHARED_TAIL = sizeof(GreedyShared) - GREEDY_SHARED_HEAD;
static_assert(GREEDY_SHARED_HEAD % 16 == 0, "the exact path's LDS region must be 16-byte aligned");

// LDS of the exact path: reductions and a bitmask of A (and xt) over the vocabulary.
__host__ __device__ inline size_t greedy_exact_lds_bytes(int V) {
    return ((sizeof(ExactShared) + 15) & ~size_t(15)) + (((size_t)V + 31) / 32) * 4 + 64;
}

// Lowest-index arg-max over the workgroup of per-thread (value, index) pairs; index INT_MAX = none.
__device__ __forceinline__ void block_argmax(float val, int idx, float* sval, int* sidx, float* out_val,
                                             int* out_idx) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = threadIdx.x >> 6;
    const float vmax = wave_max(val);
    const int imin = wave_min((val == vmax) ? idx : INT_MAX);
    __syncthreads();
    if (lane == 0) { sval[wave] = vmax; sidx[wave] = imin; }
    __syncthreads();
    float bv = sval[0];
    int bi = sidx[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
        const float v = sval[w];
        const int i = sidx[w];
        if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
    }
    *out_val = bv;
    *out_idx = bi;
}

// fp64 evaluation of one row by the whole workgroup.  ex: LDS region of greedy_exact_lds_bytes().
template <typename LT, bool VEC>
__device__ void greedy_exact_row(const GreedyArgs& a, int row, unsigned char* ex, const unsigned char* lds_row) {
    using L = Lane<LT>;
    constexpr int EPV = EXV;
    ExactShared& sh = *reinterpret_cast<ExactShared*>(ex);
    uint32_t* mask = reinterpret_cast<uint32_t*>(ex + ((sizeof(ExactShared) + 15) & ~size_t(15)));
    const int tid = threadIdx.x;
    const int V = a.V;
    const int k = a.k;
    const int nwords = (V + 31) >> 5;
    float* sval = reinterpret_cast<float*>(mask + nwords);
    int* sidx = reinterpret_cast<int*>(sval + NW);
    const int nvec = (V + EPV - 1) / EPV;
    const int nchunk = (nvec + NT - 1) / NT;
    bool row_ok;
    const int lrow = logit_row(a.row_index, a.R, row, &row_ok);
    const LT* trow = reinterpret_cast<const LT*>(a.target) + (int64_t)lrow * a.stride;
    const int xt = a.tokens[row];
    const double delta = (double)a.delta;

    // usability and maximum
    int bad = ((unsigned)xt < (unsigned)V) ? 0 : 1;
    const int32_t* nrow = a.knn + (int64_t)(bad ? 0 : xt) * k;
    if (!row_ok) bad = 1;
    if (!bad)
        for (int j = tid; j < k; j += NT)
            if ((unsigned)nrow[j] >= (unsigned)V) bad = 1;
    float mtf = neg_inf_f();
    for (int c = 0; c < nchunk; ++c) {
        float tf[EPV];
        VecLoad<LT, VEC>::load(trow, lds_row, c * NT + tid, V, tf);
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            if (isnan(tf[e]) || tf[e] == INFINITY) bad = 1;
            mtf = fmaxf(mtf, tf[e]);
        }
    }
    const double mt = block_max((double)mtf, sh.red, tid);
    if (mt == -INFINITY) bad = 1;
    bad = block_or_i(bad, sh.ired, tid);
    if (bad) {
        if (tid == 0) {
            a.out_accept[row] = -1;
            a.out_token[row] = -1;
            if (a.out_path) a.out_path[row] = 1;
        }
        return;
    }
    // normaliser
    double zt = 0.0;
    for (int c = 0; c < nchunk; ++c) {
        float tf[EPV];
        VecLoad<LT, VEC>::load(trow, lds_row, c * NT + tid, V, tf);
        double st = 0.0;
#pragma unroll
        for (int e = 0; e < EPV; ++e) st += exp_nonpos((double)tf[e] - mt);
        zt += st;
    }
    zt = block_sum(zt, sh.red, tid);
    // walk, mass
    int a_size;
    double S;
    const double t_tok = exp_nonpos((double)L::glob(trow, xt) - mt) / zt;
    exact_walk<LT>(trow, lds_row, nrow, k, xt, mt, zt, 0, t_tok, delta, sh, tid, &a_size, &S);
    const double mass = t_tok + S;

    // bitmask of A and of xt, then the lowest-index arg-max of the raw logits outside it
    for (int w = tid; w < nwords; w += NT) mask[w] = 0u;
    __syncthreads();
    for (int j = tid; j < a_size; j += NT) {
        const int n = nrow[j];
        atomicOr(&mask[n >> 5], 1u << (n & 31));
    }
    if (tid == 0) atomicOr(&mask[xt >> 5], 1u << (xt & 31));
    __syncthreads();
    float bv = neg_inf_f();
    int bi = INT_MAX;
    for (int c = 0; c < nchunk; ++c) {
        const int vi = c * NT + tid;
        float tf[EPV];
        VecLoad<LT, VEC>::load(trow, lds_row, vi, V, tf);
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            const int x = vi * EPV + e;
            if (x < V && !((mask[x >> 5] >> (x & 31)) & 1u) && (tf[e] > bv || bi == INT_MAX)) {
                bv = tf[e];
                bi = x;
            }
        }
    }
    float ov;
    int oi;
    block_argmax(bv, bi, sval, sidx, &ov, &oi);
    if (tid == 0) {
        bool accept = true;
        if (oi != INT_MAX) {
            const double other = exp_nonpos((double)ov - mt) / zt;
            accept = (mass > other) || (mass == other && xt < oi);
        }
        a.out_accept[row] = accept ? 1 : 0;
        a.out_token[row] = accept ? -1 : oi;
        if (a.out_path) a.out_path[row] = 1;
    }
}

// fp32 path.  FULL: the row fills all NV vector slots of every thread.  VT: the token's table row
// can be read with 16-byte loads (a kernel of its own for the other case: a load that only one of
// two paths issues makes the statically placed wait counters wait for every load).
template <typename LT, int NV, bool FULL, bool VT>
__global__ __launch_bounds__(NT) void greedy_fast(GreedyArgs a) {
    using L = Lane<LT>;
    constexpr int EPV = L::EPV;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* s_row = smem;
    const int row_bytes = (a.V * (int)sizeof(LT) + 15) & ~15;
    GreedyShared& sh = *reinterpret_cast<GreedyShared*>(smem + row_bytes);
    unsigned char* ex_lds = reinterpret_cast<unsigned char*>(sh.gs);

    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1);
    const int wave = tid >> 6;
    const int V = a.V;
    const int k = a.k;
    const int nvec = V / EPV;
    const int row = verification_of_block(blockIdx.x, a.N, a.row_index != nullptr);
    bool row_ok;
    const int lrow = logit_row(a.row_index, a.R, row, &row_ok);

    // ---- loads, the token first: its table row's address depends on it, and that dependent load
    // should be in flight together with the streamed row ----
    const int xt = a.tokens[row];
    // stream the target row: NV 16-byte loads per thread, coalesced
    uint4 T[NV];
    {
        const uint4* tv = reinterpret_cast<const uint4*>(reinterpret_cast<const LT*>(a.target) + (int64_t)lrow * a.stride);
#pragma unroll
        for (int c = 0; c < NV; ++c) {
            const int vi = c * NT + tid;
            if (FULL || vi < nvec) T[c] = load_stream16(tv + vi);
            else T[c] = make_uint4(L::NEG_INF_WORD, L::NEG_INF_WORD, L::NEG_INF_WORD, L::NEG_INF_WORD);
        }
    }
    const bool tok_ok = (unsigned)xt < (unsigned)V;
    const int xs = tok_ok ? xt : 0;
    const int32_t* nrow = a.knn + (int64_t)xs * k;
    int nb[4];   // table slots 4*tid .. 4*tid+3 (unspecified where the slot is beyond k: every use checks)
    {
        const int j0 = tid * 4;
        if (VT) {   // k a multiple of four: loaded unconditionally from a clamped slot, no branch around the load
            const int4 q = *reinterpret_cast<const int4*>(nrow + min(j0, k - 4));
            nb[0] = q.x; nb[1] = q.y; nb[2] = q.z; nb[3] = q.w;
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) nb[q] = (j0 + q < k) ? nrow[j0 + q] : 0;
        }
    }
    __builtin_amdgcn_sched_barrier(0);   // every load of the row is issued before anything waits for one

    // ---- raw row to LDS; reference = maximum over vector slot 0 of every thread ----
#pragma unroll
    for (int c = 0; c < NV; ++c) {
        const int vi = c * NT + tid;
        if (FULL || vi < nvec) reinterpret_cast<uint4*>(s_row)[vi] = T[c];
    }
    float rt = neg_inf_f();
#pragma unroll
    for (int e = 0; e < EPV; e += 2) rt = fmaxf(rt, fmaxf(L::get(T[0], e), L::get(T[0], e + 1)));
    rt = wave_max(rt);
    if (lane == 0) sh.wmax[wave] = rt;
    __syncthreads();
    rt = sh.wmax[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) rt = fmaxf(rt, sh.wmax[w]);
    if (rt == neg_inf_f()) rt = 0.f;
    const float ct = rt * LOG2E_F;

    // ---- exponentials 2^(l*log2e - c), summed; neighbour terms scanned ----
    float st = 0.f, emax = 0.f;
#pragma unroll
    for (int c = 0; c < NV; ++c) {
        float et[EPV];
#pragma unroll
        for (int e = 0; e < EPV; ++e) et[e] = hw_exp2(__builtin_fmaf(L::get(T[c], e), LOG2E_F, -ct));
#pragma unroll
        for (int e = 0; e < EPV; e += 2) emax = fmaxf(emax, fmaxf(et[e], et[e + 1]));
#pragma unroll
        for (int s = EPV / 2; s > 0; s >>= 1)
#pragma unroll
            for (int e = 0; e < s; ++e) et[e] += et[e + s];
        st += et[0];
    }
    st = wave_sum(st);
    emax = wave_max(emax);
    const SlotTerms slots = slot_terms<LT>(nb, xt, k, V, nrow, s_row, ct, sh.wtot, sh.wbad);
    if (lane == 0) { sh.wsum[wave] = st; sh.wemax[wave] = emax; }
    __syncthreads();

    // ---- every wavefront: the bound on its own slots ----
    float Zt = 0.f, Emax = 0.f, woff = 0.f, run_off = 0.f;
    int bad = (tok_ok && row_ok) ? 0 : 1;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        Zt += sh.wsum[w];
        Emax = fmaxf(Emax, sh.wemax[w]);
        if (w < wave) woff += sh.wtot[w];
        run_off += sh.wtot[w];
        bad |= sh.wbad[w];
    }
    const float e_tx = hw_exp2(__builtin_fmaf(L::lds(s_row, xs), LOG2E_F, -ct));
    SlotTest test;
    {
        const float R = a.delta * Zt;   // total variation of the prefix, times Zt, < delta * Zt
        test.divergence = 0;
        test.e_tx = e_tx;
        test.lo = R * (1.f - TAU_CUT) - ABS_SLACK;
        test.hi = R * (1.f + TAU_CUT) + ABS_SLACK;
    }
    classify_slots(slots, test, woff, WaveCut{sh.cut_np, sh.cut_df, sh.cut_s});
    __syncthreads();

    // ---- every thread: the cut and the mass (same inputs, same result) ----
    int first_np = INT_MAX, first_df = INT_MAX;
    float s_cut = 0.f;
#pragma unroll
    for (int w = NW - 1; w >= 0; --w) {
        if (sh.cut_np[w] != INT_MAX) { first_np = sh.cut_np[w]; s_cut = sh.cut_s[w]; }
        first_df = min(first_df, sh.cut_df[w]);
    }
    bool cut_definite = (first_np == INT_MAX) || (first_np == first_df);
    int a_size = (first_np == INT_MAX) ? k : first_np;
    float S = (first_np == INT_MAX) ? run_off : s_cut;
    if (first_np == INT_MAX && k > NT * 4) {   // uniform: the walk goes on beyond slot 1024
        if (wave == 0) {
            const CutResult tail = walk_tail<LT>(test, run_off, xt, xs, k, V, a.knn, s_row, ct);
            if (lane == 0) {
                sh.tail[0] = tail.a_size;
                sh.tail[1] = __float_as_int(tail.S);
                sh.tail[2] = tail.definite ? 1 : 0;
                sh.tail[3] = tail.bad;
            }
        }
        __syncthreads();
        a_size = sh.tail[0];
        S = __int_as_float(sh.tail[1]);
        cut_definite = sh.tail[2] != 0;
        bad |= sh.tail[3];
    }
    const bool sums_ok = (Zt >= 1.f) && (Zt <= Z_MAX);
    const bool cut_ok = cut_definite && !bad && sums_ok;
    const float mass_z = e_tx + S;
    if (!cut_ok) {  // uniform: the cut itself needs fp64 (or the row is unusable)
        greedy_exact_row<LT, true>(a, row, ex_lds, s_row);
        return;
    }
    // no term of the row, inside or outside A, reaches the mass of A: accepted without looking at A
    if (mass_z * (1.f - TAU_ACC) > Emax * (1.f + TAU_ACC) + ABS_SLACK) {
        if (tid == 0) {
            a.out_accept[row] = 1;
            a.out_token[row] = -1;
            if (a.out_path) a.out_path[row] = 0;
        }
        return;
    }

    // ---- remove A and xt from the LDS row, then the arg-max of what is left ----
    for (int base = 0; base < a_size; base += NT * 4) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int j = base + tid * 4 + q;
            if (j < a_size) {
                const int n = base == 0 ? nb[q] : nrow[j];
                L::lds_set_neg_inf(s_row, n);
            }
        }
    }
    if (tid == 0) L::lds_set_neg_inf(s_row, xs);
    __syncthreads();
    float bv = neg_inf_f();
    int bi = INT_MAX;
#pragma unroll
    for (int c = 0; c < NV; ++c) {
        const int vi = c * NT + tid;
        if (FULL || vi < nvec) {
            const uint4 v = reinterpret_cast<const uint4*>(s_row)[vi];
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                const float x = L::get(v, e);
                if (x > bv) { bv = x; bi = vi * EPV + e; }
            }
        }
    }
    float ov;
    int oi;
    block_argmax(bv, bi, sh.best_val, sh.best_idx, &ov, &oi);
    // mass of A against the largest remaining term, both times Z
    const float other_z = hw_exp2(__builtin_fmaf(ov, LOG2E_F, -ct));   // 0 when nothing is left
    const bool accept_def = (oi == INT_MAX) || (mass_z * (1.f - TAU_ACC) > other_z * (1.f + TAU_ACC) + ABS_SLACK);
    const bool reject_def = (oi != INT_MAX) && (other_z * (1.f - TAU_ACC) > mass_z * (1.f + TAU_ACC) + ABS_SLACK);
    if (accept_def || reject_def) {
        if (tid == 0) {
            a.out_accept[row] = accept_def ? 1 : 0;
            a.out_token[row] = accept_def ? -1 : oi;
            if (a.out_path) a.out_path[row] = 0;
        }
        return;
    }
    // too close to call in fp32 (the LDS row has been overwritten: read the row from global memory)
    __syncthreads();
    greedy_exact_row<LT, true>(a, row, ex_lds, nullptr);
}

template <typename LT>
__global__ __launch_bounds__(NT) void greedy_exact(GreedyArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    greedy_exact_row<LT, false>(a, verification_of_block(blockIdx.x, a.N, a.row_index != nullptr), smem, nullptr);
}

// launch == false: only the LDS limit is raised (lantern_prepare), nothing is enqueued.
template <typename LT, int NV>
static hipError_t launch_greedy_nv(const GreedyArgs& a, hipStream_t stream, bool launch) {
    const size_t row_bytes = ((size_t)a.V * sizeof(LT) + 15) & ~size_t(15);
    const size_t tail = greedy_exact_lds_bytes(a.V) > GREEDY_SHARED_TAIL ? greedy_exact_lds_bytes(a.V) : GREEDY_SHARED_TAIL;
    const size_t lds = row_bytes + GREEDY_SHARED_HEAD + tail;
    const bool full = a.V == NV * NT * Lane<LT>::EPV;
    const bool vt = ((a.k & 3) == 0) && ((reinterpret_cast<uintptr_t>(a.knn) & 15) == 0);
    if (!launch) {   // every instantiation may be needed later
        hipError_t e = allow_lds<&greedy_fast<LT, NV, true, true>>(lds);
        if (e == hipSuccess) e = allow_lds<&greedy_fast<LT, NV, false, true>>(lds);
        if (e == hipSuccess) e = allow_lds<&greedy_fast<LT, NV, false, false>>(lds);
        return e;
    }
    const hipError_t e = (full && vt) ? allow_lds<&greedy_fast<LT, NV, true, true>>(lds)
                         : vt         ? allow_lds<&greedy_fast<LT, NV, false, true>>(lds)
                                      : allow_lds<&greedy_fast<LT, NV, false, false>>(lds);
    if (e != hipSuccess) return e;
    if (full && vt)
        hipLaunchKernelGGL((greedy_fast<LT, NV, true, true>), dim3(a.N), dim3(NT), lds, stream, a);
    else if (vt)
        hipLaunchKernelGGL((greedy_fast<LT, NV, false, true>), dim3(a.N), dim3(NT), lds, stream, a);
    else
        hipLaunchKernelGGL((greedy_fast<LT, NV, false, false>), dim3(a.N), dim3(NT), lds, stream, a);
    return hipGetLastError();
}

template <typename LT>
static hipError_t launch_greedy_fast(const GreedyArgs& a, hipStream_t stream, bool launch) {
    const int nvec = a.V / Lane<LT>::EPV;
    const int nv = (nvec + NT - 1) / NT;
    if (nv <= 1) return launch_greedy_nv<LT, 1>(a, stream, launch);
    if (nv <= 2) return launch_greedy_nv<LT, 2>(a, stream, launch);
    if (nv <= 4) return launch_greedy_nv<LT, 4>(a, stream, launch);
    if (nv <= 8) return launch_greedy_nv<LT, 8>(a, stream, launch);
    return launch_greedy_nv<LT, 16>(a, stream, launch);
}

template <typename LT>
static bool greedy_fast_shape(int V, int k) {
    constexpr int EPV = Lane<LT>::EPV;
    return (V % EPV) == 0 && (V / EPV + NT - 1) / NT <= 16 && k <= FAST_MAX_K;
}

template <typename LT>
static hipError_t launch_greedy_typed(const GreedyArgs& a, hipStream_t stream) {
    const uintptr_t align = reinterpret_cast<uintptr_t>(a.target) | (uintptr_t)(a.stride * (int64_t)sizeof(LT));
    if ((align & 15) == 0 && greedy_fast_shape<LT>(a.V, a.k)) return launch_greedy_fast<LT>(a, stream, true);
    const size_t lds = greedy_exact_lds_bytes(a.V);
    const hipError_t e = allow_lds<&greedy_exact<LT>>(lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((greedy_exact<LT>), dim3(a.N), dim3(NT), lds, stream, a);
    return hipGetLastError();
}

template <typename LT>
static hipError_t prepare_greedy_typed(int V, int k) {
    hipFuncAttributes attr;   // loads this file's kernels on the current device
    hipError_t e = hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(&greedy_exact<LT>));
    if (e != hipSuccess) return e;
    if (greedy_fast_shape<LT>(V, k)) {
        GreedyArgs a{};
        a.V = V;
        a.k = k;
        e = launch_greedy_fast<LT>(a, nullptr, false);
    }
    if (e == hipSuccess) e = allow_lds<&greedy_exact<LT>>(greedy_exact_lds_bytes(V));
    return e;
}

hipError_t prepare_greedy(int logits_dtype, int V, int k) {
    return logits_dtype == 0 ? prepare_greedy_typed<float>(V, k) : prepare_greedy_typed<uint16_t>(V, k);
}

hipError_t launch_verify_greedy(const GreedyArgs& a, int logits_dtype, hipStream_t stream) {
    if (logits_dtype == 0) return launch_greedy_typed<float>(a, stream);
    return launch_greedy_typed<uint16_t>(a, stream);
}

}  // namespace lantern
