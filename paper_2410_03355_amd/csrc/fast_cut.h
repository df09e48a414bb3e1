// The fp32 neighbourhood walk shared by the sampling and greedy kernels
// (Algorithm 2, inference part, as a prefix scan over the k table slots).
//
// Every thread of the workgroup exponentiates its 4 consecutive slots of the
// first 1024 (gathering the raw target logits from LDS) and the wavefront scans
// the partial sums; after a barrier every wavefront adds the totals of the
// wavefronts before it, compares the inclusive sums of its own slots with
// delta * Z under the rounding margin and publishes the first slot that does
// not pass; after a second barrier every thread combines the four results.
// Slots beyond 1024 are walked by wavefront 0 alone, 1024 at a time.
#pragma once

#include "verify_common.h"

namespace lantern {

constexpr int SPL = 16;              // table slots per lane when one wavefront walks 1024 slots
constexpr int FAST_MAX_K = 8192;     // keeps the scan's summation depth inside the margin

struct CutResult {
    int a_size;      // slots taken into A
    float S;         // sum of the unnormalised terms over A without the token
    bool definite;   // every comparison up to the cut cleared the margin
    int bad;         // a table entry outside [0, V)
};

// Decides one slot of the walk from its inclusive sum I (unnormalised, like e_tx = the term of
// the token itself and Zt = the row sum).  Total variation: I against delta * Zt.  Jensen-Shannon:
// the divergence of the prefix, evaluated in fp32 on unnormalised terms (it is homogeneous of
// degree one), against delta * Zt; its error is bounded by the derivative (at most ln 2 in either
// argument) times the error of the arguments plus the rounding of the evaluation itself.
struct SlotTest {
    int divergence;
    float e_tx;
    float lo, hi;     // delta * Zt shrunk / grown by the margin
    __device__ __forceinline__ void classify(float I, bool* passes, bool* fails) const {
        if (divergence == 0) {
            *passes = I < lo;
            *fails = I > hi;
        } else if (I * 0.69314718f < lo) {
            // JSD <= ln 2 * TVD: far below the bound, no need to evaluate the divergence
            *passes = true;
            *fails = false;
        } else if (I * 0.34657359f > hi) {
            // JSD >= 1/2 ln 2 * (moved mass): far above the bound
            *passes = false;
            *fails = true;
        } else {
            const float mass = e_tx + I;
            const float mid = 0.5f * (mass + e_tx);
            // a ratio below the smallest normal number is flushed to zero and its logarithm is
            // -inf; the term x ln(x / mid) it stands for is below 1e-36 * mid: taken as zero
            const float ratio = e_tx / mid;
            const float kl_a = mass > 0.f ? mass * __logf(mass / mid) : 0.f;
            const float kl_t = ratio >= 1.1754944e-38f ? e_tx * __logf(ratio) : 0.f;
            const float J = 0.5f * kl_a + 0.5f * (kl_t + I * 0.69314718f);
            const float err = 0.7f * (8.0e-6f * I + 3.0e-6f * e_tx) + 1.0e-6f * (e_tx + I);
            *passes = J + err < lo;
            *fails = J - err > hi;
        }
    }
};

// ---- the walk with every wavefront classifying its own slots ----
// The same walk split differently: between the barrier that publishes the wavefront totals and the
// one that publishes the per-wavefront results, every wavefront compares the four slots each of its
// threads holds in registers; afterwards every thread combines the four results.  No wavefront
// waits while another one scans all 1024 slots, and the serial work no longer lands on the one
// SIMD that hosts wavefront 0 of every resident workgroup.

// What a thread keeps of its slots 4*tid .. 4*tid+3 between the halves of the walk.
struct SlotTerms {
    float incl[4];   // inclusive sums within the wavefront, lane order
    float excl;      // the sum before the thread's first slot, within the wavefront
    unsigned skip;   // bit q: slot 4*tid+q is the token itself or beyond k
};

// All threads, before the barrier that publishes wtot / wbad.
template <typename LT>
__device__ __forceinline__ SlotTerms slot_terms(const int (&nb)[4], int xt, int k, int V, const int32_t* nrow,
                                                const unsigned char* s_row, float ct, float* wtot, int* wbad) {
    using L = Lane<LT>;
    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1);
    const int wave = tid >> 6;
    SlotTerms st;
    float run = 0.f;
    st.skip = 0;
    int bad = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const bool valid = tid * 4 + q < k;
        const int n = nb[q];
        const bool inr = (unsigned)n < (unsigned)V;
        if (valid && !inr) bad = 1;
        float e = 0.f;
        if (n == xt || !valid) st.skip |= 1u << q;
        else if (inr) e = hw_exp2(__builtin_fmaf(L::lds(s_row, n), LOG2E_F, -ct));
        run += e;
        st.incl[q] = run;
    }
    for (int j = NT * 4 + tid; j < k; j += NT)     // entries the walk may never reach are range-checked too
        if ((unsigned)nrow[j] >= (unsigned)V) bad = 1;
    const float incl = wave_scan_incl(run);
    st.excl = wave_prev(incl, 0.f);
#pragma unroll
    for (int q = 0; q < 4; ++q) st.incl[q] += st.excl;
    bad = wave_or(bad);
    if (lane == WAVE - 1) wtot[wave] = incl;
    if (lane == 0) wbad[wave] = bad;
    return st;
}

// Per-wavefront results of the classification: first slot not definitely passing (and the sum
// before it), first slot definitely failing; INT_MAX when there is none.
struct WaveCut {
    int* np;
    int* df;
    float* s;
};

// All threads, after the barrier.  woff: sum of the totals of the wavefronts before this one.
__device__ __forceinline__ void classify_slots(const SlotTerms& st, const SlotTest& test, float woff,
                                               const WaveCut& out) {
    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1);
    const int wave = tid >> 6;
    int my_np = INT_MAX, my_df = INT_MAX;
    float my_s = 0.f;
    float before = woff + st.excl;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float I = woff + st.incl[q];
        if (!((st.skip >> q) & 1u)) {
            bool passes, fails;
            test.classify(I, &passes, &fails);
            if (my_np == INT_MAX && !passes) { my_np = tid * 4 + q; my_s = before; }
            if (my_df == INT_MAX && fails) my_df = tid * 4 + q;
        }
        before = I;
    }
    const int w_np = wave_min(my_np);
    const int w_df = wave_min(my_df);
    float s_cut = 0.f;
    if (w_np != INT_MAX) {
        const unsigned long long owner = __ballot(my_np == w_np);
        s_cut = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_s), __ffsll((long long)owner) - 1));
    }
    if (lane == 0) {
        out.np[wave] = w_np;
        out.df[wave] = w_df;
        out.s[wave] = s_cut;
    }
}

// Slots beyond the first 1024, walked by one wavefront 1024 at a time (k > 1024 and no cut among
// the first 1024).  carry: the sum over the first 1024 slots.  The result has the meaning of the combined per-wavefront results.
template <typename LT>
__device__ __forceinline__ CutResult walk_tail(const SlotTest& test, float carry, int xt, int xs, int k, int V,
                                               const int32_t* knn, const unsigned char* s_row, float ct) {
    using L = Lane<LT>;
    const int lane = threadIdx.x & (WAVE - 1);
    const int32_t* nrow = knn + (int64_t)xs * k;
    int first_np = INT_MAX, first_df = INT_MAX, bad = 0;
    float s_cut = 0.f;
    for (int base = NT * 4; base < k; base += WAVE * SPL) {
        const int j0 = base + lane * SPL;
        float ev[SPL];
        float run = 0.f;
        unsigned skip = 0;
#pragma unroll
        for (int q = 0; q < SPL; ++q) {
            const bool valid = j0 + q < k;
            const int n = valid ? nrow[j0 + q] : 0;
            const bool inr = (unsigned)n < (unsigned)V;
            if (valid && !inr) bad = 1;
            float e = 0.f;
            if (n == xt || !valid) skip |= 1u << q;
            else if (inr) e = hw_exp2(__builtin_fmaf(L::lds(s_row, n), LOG2E_F, -ct));
            ev[q] = e;
            run += e;
        }
        const float incl = wave_scan_incl(run);
        const float ctot = lane63_f(incl);
        float I = carry + wave_prev(incl, 0.f);
        int my_np = INT_MAX, my_df = INT_MAX;
        float my_s = 0.f;
#pragma unroll
        for (int q = 0; q < SPL; ++q) {
            const float bef = I;
            I += ev[q];
            if (!((skip >> q) & 1u)) {
                bool passes, fails;
                test.classify(I, &passes, &fails);
                if (my_np == INT_MAX && !passes) { my_np = j0 + q; my_s = bef; }
                if (my_df == INT_MAX && fails) my_df = j0 + q;
            }
        }
        const int w_np = wave_min(my_np);
        if (w_np != INT_MAX) {
            const unsigned long long owner = __ballot(my_np == w_np);
            first_np = w_np;
            first_df = wave_min(my_df);
            s_cut = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_s), __ffsll((long long)owner) - 1));
            break;
        }
        carry += ctot;
    }
    CutResult r;
    r.definite = (first_np == INT_MAX) || (first_np == first_df);
    r.a_size = (first_np == INT_MAX) ? k : first_np;
    r.S = (first_np == INT_MAX) ? carry : s_cut;
    r.bad = wave_or(bad);
    return r;
}

}  // namespace lantern
