// Wavefront- and workgroup-level helpers shared by the gfx950 kernels.
// Wavefronts are 64 lanes wide; workgroups are NT = 256 threads (4 waves).
//
// 32-bit reductions and scans use DPP (data-parallel primitives: the operand
// of a VALU instruction is taken from another lane), which costs one VALU
// issue per step instead of a round trip through the LDS crossbar:
//   row_shr:n      lane l reads lane l-n of its 16-lane row
//   row_bcast:15   lane 15 of each row is broadcast to the next row
//   row_bcast:31   lane 31 is broadcast to rows 2 and 3
//   wave_shr:1     lane l reads lane l-1 of the wavefront
// Lanes without a source keep the identity passed as the old value.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lantern {

constexpr int WAVE = 64;
constexpr int NT = 256;
constexpr int NW = NT / WAVE;

__device__ __forceinline__ float neg_inf_f() { return -__builtin_huge_valf(); }

enum : int {
    DPP_ROW_SHR1 = 0x111, DPP_ROW_SHR2 = 0x112, DPP_ROW_SHR4 = 0x114, DPP_ROW_SHR8 = 0x118,
    DPP_WAVE_SHR1 = 0x138, DPP_ROW_BCAST15 = 0x142, DPP_ROW_BCAST31 = 0x143
};

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f(float identity, float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(identity), __float_as_int(v), CTRL,
                                                      ROW_MASK, 0xF, false));
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_i(int identity, int v) {
    return __builtin_amdgcn_update_dpp(identity, v, CTRL, ROW_MASK, 0xF, false);
}

struct OpSum { __device__ static __forceinline__ float f(float a, float b) { return a + b; }
               __device__ static __forceinline__ int i(int a, int b) { return a + b; } };
struct OpMax { __device__ static __forceinline__ float f(float a, float b) { return fmaxf(a, b); }
               __device__ static __forceinline__ int i(int a, int b) { return max(a, b); } };
struct OpMin { __device__ static __forceinline__ float f(float a, float b) { return fminf(a, b); }
               __device__ static __forceinline__ int i(int a, int b) { return min(a, b); } };
struct OpOr  { __device__ static __forceinline__ int i(int a, int b) { return a | b; } };

// Inclusive scan over the 64 lanes in lane order; lane 63 ends with the reduction.
template <typename Op>
__device__ __forceinline__ float wave_scan_f(float v, float identity) {
    v = Op::f(v, dpp_f<DPP_ROW_SHR1, 0xF>(identity, v));
    v = Op::f(v, dpp_f<DPP_ROW_SHR2, 0xF>(identity, v));
    v = Op::f(v, dpp_f<DPP_ROW_SHR4, 0xF>(identity, v));
    v = Op::f(v, dpp_f<DPP_ROW_SHR8, 0xF>(identity, v));
    v = Op::f(v, dpp_f<DPP_ROW_BCAST15, 0xA>(identity, v));
    v = Op::f(v, dpp_f<DPP_ROW_BCAST31, 0xC>(identity, v));
    return v;
}
template <typename Op>
__device__ __forceinline__ int wave_scan_i(int v, int identity) {
    v = Op::i(v, dpp_i<DPP_ROW_SHR1, 0xF>(identity, v));
    v = Op::i(v, dpp_i<DPP_ROW_SHR2, 0xF>(identity, v));
    v = Op::i(v, dpp_i<DPP_ROW_SHR4, 0xF>(identity, v));
    v = Op::i(v, dpp_i<DPP_ROW_SHR8, 0xF>(identity, v));
    v = Op::i(v, dpp_i<DPP_ROW_BCAST15, 0xA>(identity, v));
    v = Op::i(v, dpp_i<DPP_ROW_BCAST31, 0xC>(identity, v));
    return v;
}

__device__ __forceinline__ float lane63_f(float v) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Reductions: the result is uniform across the wavefront.
__device__ __forceinline__ float wave_max(float v) { return lane63_f(wave_scan_f<OpMax>(v, neg_inf_f())); }
__device__ __forceinline__ float wave_sum(float v) { return lane63_f(wave_scan_f<OpSum>(v, 0.f)); }
__device__ __forceinline__ int wave_min(int v) {
    return __builtin_amdgcn_readlane(wave_scan_i<OpMin>(v, 0x7FFFFFFF), 63);
}
__device__ __forceinline__ int wave_or(int v) { return __builtin_amdgcn_readlane(wave_scan_i<OpOr>(v, 0), 63); }

// Inclusive prefix sum across the 64 lanes, lane order.
__device__ __forceinline__ float wave_scan_incl(float v) { return wave_scan_f<OpSum>(v, 0.f); }
// The value of the previous lane (identity for lane 0).
__device__ __forceinline__ float wave_prev(float v, float identity) {
    return dpp_f<DPP_WAVE_SHR1, 0xF>(identity, v);
}

// fp64 scans over the wavefront with DPP on the two halves of the value: six steps of two moves and
// one operation, no LDS traffic (a shuffle through the LDS crossbar costs two ds_bpermute per step
// and their latency, six times in a row).  Lanes without a source lane, and rows a step leaves out,
// take `old`, the operation's identity.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_d(double v, double old = 0.0) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    const unsigned long long o = (unsigned long long)__double_as_longlong(old);
    const int lo = __builtin_amdgcn_update_dpp((int)(unsigned)o, (int)(unsigned)b, CTRL, ROW_MASK, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp((int)(unsigned)(o >> 32), (int)(unsigned)(b >> 32), CTRL, ROW_MASK, 0xF, false);
    return __longlong_as_double((long long)(((unsigned long long)(unsigned)hi << 32) | (unsigned)lo));
}
__device__ __forceinline__ double lane63_d(double v) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)b, 63);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(b >> 32), 63);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}
// Inclusive prefix sum in lane order: within rows of 16 lanes, then row totals onto the rows after.
__device__ __forceinline__ double wave_scan_incl(double v) {
    v += dpp_d<DPP_ROW_SHR1, 0xF>(v);
    v += dpp_d<DPP_ROW_SHR2, 0xF>(v);
    v += dpp_d<DPP_ROW_SHR4, 0xF>(v);
    v += dpp_d<DPP_ROW_SHR8, 0xF>(v);
    v += dpp_d<DPP_ROW_BCAST15, 0xA>(v);
    v += dpp_d<DPP_ROW_BCAST31, 0xC>(v);
    return v;
}
// Sum and maximum over the wavefront; the result is uniform.
__device__ __forceinline__ double wave_sum_dpp(double v) { return lane63_d(wave_scan_incl(v)); }
__device__ __forceinline__ double wave_sum(double v) { return wave_sum_dpp(v); }
__device__ __forceinline__ double wave_max(double v) {
    const double ninf = -__builtin_huge_val();
    v = fmax(v, dpp_d<DPP_ROW_SHR1, 0xF>(v, ninf));
    v = fmax(v, dpp_d<DPP_ROW_SHR2, 0xF>(v, ninf));
    v = fmax(v, dpp_d<DPP_ROW_SHR4, 0xF>(v, ninf));
    v = fmax(v, dpp_d<DPP_ROW_SHR8, 0xF>(v, ninf));
    v = fmax(v, dpp_d<DPP_ROW_BCAST15, 0xA>(v, ninf));
    v = fmax(v, dpp_d<DPP_ROW_BCAST31, 0xC>(v, ninf));
    return lane63_d(v);
}

// v_exp_f32: 2^x, flushes denormal results to zero, 2^-inf = 0.
__device__ __forceinline__ float hw_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

}  // namespace lantern
