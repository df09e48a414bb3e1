// Random neighbourhood table (Section 5.3.1 and Table 3, the random-selection row of the ablation
// on latent proximity measures): row x holds x and then k-1 other tokens, a uniform sample without
// replacement in random order.  Every pair (x, y) has a 32-bit key, word y mod 4 of Philox4x32-10
// at counter (y div 4, x, 0, 0) under the key (seed low word, seed high word); the row lists the
// other tokens by increasing (key, token).
//
// One workgroup per row.  The keys are uniform, so the k-1 smallest lie below a threshold known in
// advance up to sampling noise: the workgroup counts the keys below the threshold (moving it until
// between k-1 and CAP keys are below), collects those into LDS, sorts them and writes the first
// k-1.  Keys are recomputed in every pass rather than stored: ten rounds of integer arithmetic per
// four keys cost less than a round trip through memory.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_utils.h"
#include "knn_args.h"
#include "lds_limit.h"

namespace lantern {

namespace {

constexpr int CAP = 8192;                // candidates a workgroup sorts in LDS (64 KiB)
constexpr uint64_t KEY_END = 1ull << 32; // threshold that lets every key through

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0;
        const uint32_t n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

struct RandomShared {
    int wsum[NW];
    int count;     // candidates collected
    int pad[3];
};

__device__ __forceinline__ int block_count(int v, RandomShared& sh) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = threadIdx.x >> 6;
    v = __builtin_amdgcn_readlane(wave_scan_i<OpSum>(v, 0), 63);
    __syncthreads();              // the previous round's readers are done with wsum
    if (lane == 0) sh.wsum[wave] = v;
    __syncthreads();
    int s = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) s += sh.wsum[w];
    return s;
}

__global__ __launch_bounds__(NT) void random_rows_kernel(int V, int k, uint32_t seed_lo, uint32_t seed_hi,
                                                         uint64_t t0, int32_t* out) {
    extern __shared__ __align__(16) unsigned char smem[];
    RandomShared& sh = *reinterpret_cast<RandomShared*>(smem);
    uint64_t* cand = reinterpret_cast<uint64_t*>(smem + sizeof(RandomShared));
    const int tid = threadIdx.x;
    const int x = blockIdx.x;
    const int need = k - 1;
    int32_t* orow = out + (int64_t)x * k;
    if (tid == 0) orow[0] = x;
    if (need == 0) return;
    const int groups = (V + 3) >> 2;

    // ---- threshold with need <= #{y != x : key < T} <= CAP ----
    uint64_t lo = 0, hi = KEY_END, T = t0;   // count(lo) < need <= V-1 = count(hi)
    bool found = false;
    for (int iter = 0; iter < 80; ++iter) {
        int c = 0;
        for (int g = tid; g < groups; g += NT) {
            uint32_t w[4];
            philox4x32_10((uint32_t)g, (uint32_t)x, 0u, 0u, seed_lo, seed_hi, w);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int y = 4 * g + q;
                if (y < V && y != x && (uint64_t)w[q] < T) ++c;
            }
        }
        c = block_count(c, sh);
        if (c >= need && c <= CAP) { found = true; break; }
        if (c < need) lo = T; else hi = T;
        if (hi - lo < 2) break;
        const uint64_t grown = T + (T >> 3) + 16;           // too few: a step up before bisecting
        T = (c < need && grown < hi) ? grown : lo + ((hi - lo) >> 1);
    }
    if (!found) {
        // only when more than CAP - k + 1 of the row's keys share one 32-bit value
        for (int j = 1 + tid; j < k; j += NT) orow[j] = -1;
        return;
    }

    // ---- collect (key, token) below the threshold ----
    if (tid == 0) sh.count = 0;
    __syncthreads();
    for (int g = tid; g < groups; g += NT) {
        uint32_t w[4];
        philox4x32_10((uint32_t)g, (uint32_t)x, 0u, 0u, seed_lo, seed_hi, w);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int y = 4 * g + q;
            if (y < V && y != x && (uint64_t)w[q] < T) {
                const int slot = atomicAdd(&sh.count, 1);
                cand[slot] = ((uint64_t)w[q] << 32) | (uint32_t)y;
            }
        }
    }
    __syncthreads();
    const int count = sh.count;            // the same keys as in the accepted counting pass: <= CAP
    int P = 2;
    while (P < count) P <<= 1;
    for (int s = count + tid; s < P; s += NT) cand[s] = ~0ull;

    // ---- bitonic sort ascending: the packed word orders by (key, token) ----
    for (int size = 2; size <= P; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int t = tid; t < (P >> 1); t += NT) {
                const int l = 2 * t - (t & (stride - 1));
                const int r = l + stride;
                const bool up = (l & size) == 0;
                const uint64_t a = cand[l], b = cand[r];
                if ((a > b) == up) { cand[l] = b; cand[r] = a; }
            }
        }
    }
    __syncthreads();
    for (int j = tid; j < need; j += NT) orow[1 + j] = (int32_t)(uint32_t)cand[j];
}

}  // namespace

hipError_t launch_build_random(int V, int k, uint64_t seed, uint64_t t0, int32_t* out, hipStream_t stream) {
    const size_t lds = sizeof(RandomShared) + (size_t)CAP * sizeof(uint64_t);
    const hipError_t e = allow_lds<&random_rows_kernel>(lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(random_rows_kernel, dim3(V), dim3(NT), lds, stream, V, k, (uint32_t)(seed & 0xFFFFFFFFu),
                       (uint32_t)(seed >> 32), t0, out);
    return hipGetLastError();
}

}  // namespace lantern
