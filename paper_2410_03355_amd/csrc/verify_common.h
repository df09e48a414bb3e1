// Pieces shared by the verification kernels (sampling and greedy variants):
// rounding margins of the fp32 paths, logit unpacking, workgroup reductions in
// fp64 and the four-logit vector loads of the exact paths.
#pragma once

#include <hip/hip_runtime.h>
#include <limits.h>
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#include "device_utils.h"
#include "exp64.h"

namespace lantern {

// Verification handled by workgroup b of N.  Without an index array every verification has logit
// rows of its own and workgroup b takes verification b.  With one, candidates that are neighbours
// in drafting order share logit rows (the siblings of a draft tree); workgroups go to the 8 XCDs
// round-robin (b mod 8) and every XCD has an L2 of its own, so XCD x is given the contiguous range
// x*N/8 .. (x+1)*N/8 of the verifications and siblings meet in one L2 instead of fetching their
// row once per XCD.
constexpr int XCDS = 8;
__device__ __forceinline__ int verification_of_block(int b, int N, bool shared_rows) {
    if (!shared_rows) return b;
    const int x = b % XCDS, slot = b / XCDS;
    const int q = N / XCDS, r = N % XCDS;
    return x * q + (x < r ? x : r) + slot;
}

// Row of the logit matrices that verification `row` reads: the row itself, or the entry of the
// caller's index array (the siblings of a draft tree share the rows of their parent's context).
// *ok is false for an entry outside [0, R); the row returned is then 0, so loads stay in bounds.
__device__ __forceinline__ int logit_row(const int32_t* row_index, int R, int row, bool* ok) {
    const int r = row_index ? row_index[row] : row;
    *ok = (unsigned)r < (unsigned)R;
    return *ok ? r : 0;
}

constexpr float LOG2E_F = 1.44269504088896340736f;

// ---- rounding margins of the fp32 pass -------------------------------------
// One unnormalised term e = 2^(l*log2e - c): the fused multiply-add rounds once,
// the constant log2e is off by 0.24 * 2^-24 relative, and v_exp_f32 is good to
// one ulp, so a term with |l - ref| <= 32 has a relative error below
// (1.24 * 32 + 2) * 2^-24 = 2.5e-6.  Terms more than 32 below the reference are
// below e^-32 each (V * 1.3e-14 relative to the sum, which is >= 1); terms more
// than 32 above it are excluded by requiring the sum to stay below 2^46.
// Sums are trees of depth <= 32 (per thread, wavefront scan, across waves),
// adding 32 * 2^-24 = 1.9e-6.  A comparison of one sum against another carries
// both bounds on both sides: at most 1.8e-5, covered by TAU_CUT and TAU_ACC.
constexpr float TAU_CUT = 2.0e-5f;
constexpr float TAU_ACC = 3.0e-5f;
// v_exp_f32 flushes results below 2^-126; absolute slack for products of such
// terms with sums bounded by V.
constexpr float ABS_SLACK = 1.0e-30f;
// The acceptance test multiplies such terms by a row sum (up to 2^46 = 7e13): every flushed term
// (below 1.18e-38: the token's own on either side, up to k - 1 of them in the sum over A) moves a
// side by less than 8.3e-25, so the absolute slack of that test grows with k.
__device__ __forceinline__ float acc_slack(int k) { return (float)(k + 2) * 8.3e-25f; }
constexpr float Z_MAX = 7.0e13f;  // just below 2^46 = e^31.9

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// 16-byte load of data that is read once: non-temporal, so the streamed rows
// do not evict the neighbour table from the caches.
__device__ __forceinline__ uint4 load_stream16(const uint4* p) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

template <typename LT>
struct Lane;

template <>
struct Lane<float> {
    static constexpr int EPV = 4;  // elements per 16-byte vector
    static constexpr uint32_t NEG_INF_WORD = 0xFF800000u;
    __device__ static __forceinline__ float get(const uint4& v, int e) {
        const uint32_t w = e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w;
        return __uint_as_float(w);
    }
    // the vector without its first two elements (the freed places read -inf)
    __device__ static __forceinline__ uint4 drop2(const uint4& v) {
        return make_uint4(v.z, v.w, NEG_INF_WORD, NEG_INF_WORD);
    }
    __device__ static __forceinline__ float lds(const unsigned char* row, int x) {
        return reinterpret_cast<const float*>(row)[x];
    }
    __device__ static __forceinline__ float glob(const void* row, int64_t x) {
        return reinterpret_cast<const float*>(row)[x];
    }
    __device__ static __forceinline__ void lds_set_neg_inf(unsigned char* row, int x) {
        reinterpret_cast<uint32_t*>(row)[x] = 0xFF800000u;
    }
};

template <>
struct Lane<uint16_t> {  // bfloat16 storage
    static constexpr int EPV = 8;
    static constexpr uint32_t NEG_INF_WORD = 0xFF80FF80u;
    __device__ static __forceinline__ float get(const uint4& v, int e) {
        const int wi = e >> 1;
        const uint32_t w = wi == 0 ? v.x : wi == 1 ? v.y : wi == 2 ? v.z : v.w;
        return __uint_as_float((e & 1) ? (w & 0xFFFF0000u) : (w << 16));
    }
    __device__ static __forceinline__ uint4 drop2(const uint4& v) {
        return make_uint4(v.y, v.z, v.w, NEG_INF_WORD);
    }
    __device__ static __forceinline__ float lds(const unsigned char* row, int x) {
        return __uint_as_float(static_cast<uint32_t>(reinterpret_cast<const uint16_t*>(row)[x]) << 16);
    }
    __device__ static __forceinline__ float glob(const void* row, int64_t x) {
        return __uint_as_float(static_cast<uint32_t>(reinterpret_cast<const uint16_t*>(row)[x]) << 16);
    }
    __device__ static __forceinline__ void lds_set_neg_inf(unsigned char* row, int x) {
        reinterpret_cast<uint16_t*>(row)[x] = 0xFF80u;
    }
};

// ---- fp64 workgroup helpers of the exact paths ----

// Sized for workgroups of up to MAXW wavefronts: the helpers below take the number of
// wavefronts of the calling workgroup as a template argument (NW unless stated).
constexpr int MAXW = 16;
struct ExactShared {
    double red[MAXW];
    double red2[MAXW];
    double bcast[4];
    int ired[MAXW];
    int ibcast[2];
};

template <int TNW = NW>
__device__ __forceinline__ double block_sum(double v, double* red, int tid) {
    v = wave_sum(v);
    __syncthreads();
    if ((tid & (WAVE - 1)) == 0) red[tid >> 6] = v;
    __syncthreads();
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < TNW; ++w) s += red[w];
    return s;
}

template <int TNW = NW>
__device__ __forceinline__ double block_max(double v, double* red, int tid) {
    v = wave_max(v);
    __syncthreads();
    if ((tid & (WAVE - 1)) == 0) red[tid >> 6] = v;
    __syncthreads();
    double s = red[0];
#pragma unroll
    for (int w = 1; w < TNW; ++w) s = fmax(s, red[w]);
    return s;
}

template <int TNW = NW>
__device__ __forceinline__ int block_min_i(int v, int* red, int tid) {
    v = wave_min(v);
    __syncthreads();
    if ((tid & (WAVE - 1)) == 0) red[tid >> 6] = v;
    __syncthreads();
    int s = red[0];
#pragma unroll
    for (int w = 1; w < TNW; ++w) s = min(s, red[w]);
    return s;
}

template <int TNW = NW>
__device__ __forceinline__ int block_or_i(int v, int* red, int tid) {
    v = wave_or(v);
    __syncthreads();
    if ((tid & (WAVE - 1)) == 0) red[tid >> 6] = v;
    __syncthreads();
    int s = 0;
#pragma unroll
    for (int w = 0; w < TNW; ++w) s |= red[w];
    return s;
}

// Inclusive prefix sum over the workgroup in thread order; *total gets the sum.
template <int TNW = NW>
__device__ __forceinline__ double block_scan_incl(double v, double* red, int tid, double* total) {
    const double incl = wave_scan_incl(v);
    __syncthreads();
    if ((tid & (WAVE - 1)) == WAVE - 1) red[tid >> 6] = incl;
    __syncthreads();
    double off = 0.0, tot = 0.0;
#pragma unroll
    for (int w = 0; w < TNW; ++w) {
        const double x = red[w];
        if (w < (tid >> 6)) off += x;
        tot += x;
    }
    *total = tot;
    return off + incl;
}

// The exact path walks a row four logits per lane at a time (8-byte loads for
// bf16, 16-byte loads for fp32): vector vi covers tokens [4 vi, 4 vi + 4).
// Tokens at or beyond V read as -inf.  With VEC the row is 16-byte aligned and
// V a multiple of four; lds, when not null, holds the same row in LDS.
constexpr int EXV = 4;

template <typename LT, bool VEC>
struct VecLoad;

template <bool VEC>
struct VecLoad<float, VEC> {
    __device__ static __forceinline__ void load(const float* row, const unsigned char* lds, int vi, int V,
                                                float (&out)[EXV]) {
        if (VEC) {
            if ((vi + 1) * EXV <= V) {
                const float4 v = lds ? reinterpret_cast<const float4*>(lds)[vi]
                                     : reinterpret_cast<const float4*>(row)[vi];
                out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
                return;
            }
#pragma unroll
            for (int e = 0; e < EXV; ++e) out[e] = neg_inf_f();
        } else {
#pragma unroll
            for (int e = 0; e < EXV; ++e) {
                const int x = vi * EXV + e;
                out[e] = x < V ? row[x] : neg_inf_f();
            }
        }
    }
};

template <bool VEC>
struct VecLoad<uint16_t, VEC> {
    __device__ static __forceinline__ void load(const uint16_t* row, const unsigned char* lds, int vi, int V,
                                                float (&out)[EXV]) {
        if (VEC) {
            if ((vi + 1) * EXV <= V) {
                const uint2 v = lds ? reinterpret_cast<const uint2*>(lds)[vi]
                                    : reinterpret_cast<const uint2*>(row)[vi];
                out[0] = __uint_as_float(v.x << 16);
                out[1] = __uint_as_float(v.x & 0xFFFF0000u);
                out[2] = __uint_as_float(v.y << 16);
                out[3] = __uint_as_float(v.y & 0xFFFF0000u);
                return;
            }
#pragma unroll
            for (int e = 0; e < EXV; ++e) out[e] = neg_inf_f();
        } else {
#pragma unroll
            for (int e = 0; e < EXV; ++e) {
                const int x = vi * EXV + e;
                out[e] = x < V ? Lane<uint16_t>::glob(row, x) : neg_inf_f();
            }
        }
    }
};

// Divergence between the distorted target of a prefix and the target, as a function of t0 = t(xt)
// and of the mass moved onto xt.  0: total variation distance, which is the moved mass itself
// (Section 4.3).  1: Jensen-Shannon divergence, natural logarithm (Section 5.3.2), from the
// entries where the two distributions differ: (mass, t0) at xt and (0, t(x)) at the other members.
__device__ __forceinline__ double prefix_divergence64(int divergence, double t0, double moved) {
    if (divergence == 0) return moved;
    const double mass = t0 + moved;
    const double mid = 0.5 * (mass + t0);
    const double kl_a = mass > 0.0 ? mass * log(mass / mid) : 0.0;
    const double kl_t = t0 > 0.0 ? t0 * log(t0 / mid) : 0.0;
    const double members = moved * log(2.0);
    // never negative by definition; the two terms at the token cancel down to their rounding
    // errors when the mass moved is around one unit in the last place of t0
    const double jsd = 0.5 * kl_a + 0.5 * (kl_t + members);
    return jsd < 0.0 ? 0.0 : jsd;
}

// Nearest-first walk of the neighbourhood in fp64 (Algorithm 2, inference part), by the
// whole workgroup (TNT threads): inclusive sums of t over the table slots, TNT slots at a time; the walk
// ends at the first slot, other than the token itself, at which the divergence of the prefix
// (a function of t_tok = t(xt) and of the inclusive sum) is not below delta.
// *a_size: slots taken; *S: sum of t over the taken slots other than the token.
// trow: the target row in global memory; lds_row: the same raw row in LDS, or null.
// tab: the exponential's table in LDS (exp_tab), or null for the table-free routine.
template <typename LT, int TNT = NT>
__device__ __forceinline__ void exact_walk(const LT* trow, const unsigned char* lds_row, const int32_t* nrow,
                                           int k, int xt, double mt, double zt, int divergence, double t_tok,
                                           double delta, ExactShared& sh, int tid, int* a_size, double* S,
                                           const double* tab = nullptr) {
    using L = Lane<LT>;
    double carry = 0.0;
    *a_size = k;
    *S = 0.0;
    bool cut_found = false;
    for (int base = 0; base < k && !cut_found; base += TNT) {
        const int j = base + tid;
        const bool valid = j < k;
        const int n = valid ? nrow[j] : xt;
        const bool self = (n == xt);
        const float ln = lds_row ? L::lds(lds_row, n) : L::glob(trow, n);
        const double dj = (double)ln - mt;
        const double tj = self ? 0.0 : (tab ? exp_tab(dj, tab) : exp_nonpos(dj)) / zt;
        double ctot;
        const double incl = carry + block_scan_incl<TNT / WAVE>(tj, sh.red, tid, &ctot);
        const int fail_j = (valid && !self && !(prefix_divergence64(divergence, t_tok, incl) < delta)) ? j : INT_MAX;
        const int first = block_min_i<TNT / WAVE>(fail_j, sh.ired, tid);
        if (first != INT_MAX) {
            cut_found = true;
            *a_size = first;
            // sum before the failing slot = inclusive sum of the slot before it
            if (first == base) {
                *S = carry;
            } else {
                if (j == first - 1) sh.bcast[0] = incl;
                __syncthreads();
                *S = sh.bcast[0];
            }
        } else {
            carry += ctot;
            *S = carry;
        }
    }
}

}  // namespace lantern
