// Wavefront- and workgroup-level helpers shared by the gfx950 kernels.
// Wavefronts are 64 lanes wide; workgroups are NT = 256 threads (4 waves).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lantern {

constexpr int WAVE = 64;
constexpr int NT = 256;
constexpr int NW = NT / WAVE;

__device__ __forceinline__ float neg_inf_f() { return -__builtin_huge_valf(); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) v = fmaxf(v, __shfl_xor(v, s, WAVE));
    return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) v += __shfl_xor(v, s, WAVE);
    return v;
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) v += __shfl_xor(v, s, WAVE);
    return v;
}

__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) v = fmax(v, __shfl_xor(v, s, WAVE));
    return v;
}

__device__ __forceinline__ int wave_min(int v) {
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) v = min(v, __shfl_xor(v, s, WAVE));
    return v;
}

__device__ __forceinline__ int wave_or(int v) {
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) v |= __shfl_xor(v, s, WAVE);
    return v;
}

// Inclusive prefix sum across the 64 lanes, lane order.
template <typename T>
__device__ __forceinline__ T wave_scan_incl(T v) {
    const int lane = threadIdx.x & (WAVE - 1);
#pragma unroll
    for (int s = 1; s < WAVE; s <<= 1) {
        T up = __shfl_up(v, s, WAVE);
        if (lane >= s) v += up;
    }
    return v;
}

// v_exp_f32: 2^x, flushes denormal results to zero, 2^-inf = 0.
__device__ __forceinline__ float hw_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

}  // namespace lantern
