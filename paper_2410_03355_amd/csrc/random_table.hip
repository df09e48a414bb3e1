// Random neighbourhood table (Section 5.3.1 and Table 3, the random-selection row of the ablation
// on latent proximity measures): row x holds x and then k-1 other tokens, a uniform sample without
// replacement in random order.  Every pair (x, y) has a 32-bit key, word y mod 4 of Philox4x32-10
// at counter (y div 4, x, 0, 0) under the key (seed low word, seed high word); the row lists the
// other tokens by increasing (key, token).
//
// One workgroup per row.  The keys are uniform, so the k-1 smallest lie below a threshold known in
// advance up to sampling noise: the workgroup counts the keys below the threshold (moving it until
// few enough keys are below), collects those into LDS, sorts them and writes the first k-1.
// Vocabularies of up to 16384 tokens (and k - 1 <= 2048) keep a row's keys in registers, 64 per
// thread: they are generated once, the threshold is moved until the keys below it fit the
// smallest power of two that holds k-1 (the count is linear in the threshold, so a step or two
// of proportional correction get there), and the sort is the one of the nearest-neighbour
// build.  Larger shapes recompute the keys in every pass rather than store them (ten rounds of
// integer arithmetic per four keys cost less than a round trip through memory) and sort up to
// 8192 candidates.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_utils.h"
#include "knn_args.h"
#include "lds_limit.h"
#include "lds_sort.h"

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

// ---- keys in registers ----
constexpr int RCAP = 2048;   // candidates sorted in LDS (16 KiB)

struct RegShared {
    RandomShared r;
    uint64_t cand[RCAP];     // indexed by lds_slot
};

// V <= NK * NT, k - 1 <= RCAP.  Key e of a thread is word e % 4 of group (e / 4) * NT + tid.
template <int NK>
__global__ __launch_bounds__(NT, NK > 32 ? 3 : 4) void random_rows_regs(int V, int k, uint32_t seed_lo,
                                                                        uint32_t seed_hi, uint64_t t0, int32_t* out) {
    static_assert(NK % 4 == 0 && NK <= 64, "one validity bit per key in a 64-bit word");
    __shared__ RegShared sh;
    const int tid = threadIdx.x;
    const int x = blockIdx.x;
    const int need = k - 1;
    int32_t* orow = out + (int64_t)x * k;
    if (tid == 0) orow[0] = x;
    if (need == 0) return;

    uint32_t keys[NK];
    uint64_t ok = 0;          // bit e: key e belongs to a token of the vocabulary other than x
#pragma unroll
    for (int g4 = 0; g4 < NK / 4; ++g4) {
        const int g = g4 * NT + tid;
        uint32_t w[4];
        philox4x32_10((uint32_t)g, (uint32_t)x, 0u, 0u, seed_lo, seed_hi, w);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int y = 4 * g + q;
            keys[4 * g4 + q] = w[q];
            ok |= (uint64_t)(y < V && y != x) << (4 * g4 + q);
        }
        __builtin_amdgcn_sched_barrier(0);   // one generator at a time: its temporaries are reused
    }
    // From here on the validity bits and the token numbers are taken from `ok` and the thread index
    // again, not from the 64 comparisons and sums above: the empty statements hide where the two
    // values come from, or the compiler keeps all of those alive in registers instead.
    uint32_t ok_lo = (uint32_t)ok, ok_hi = (uint32_t)(ok >> 32);
    int tid_again = tid;
    asm volatile("" : "+v"(ok_lo), "+v"(ok_hi), "+v"(tid_again));
    ok = ((uint64_t)ok_hi << 32) | ok_lo;

    // ---- threshold with need <= #{y != x : key < T} <= fit ----
    int fit = 4;              // the sort takes a power of two, at least four
    while (fit < need) fit <<= 1;
    const double aim = 0.5 * (double)(need + fit);
    uint64_t lo = 0, hi = KEY_END, T = t0;   // count(lo) < need <= V-1 = count(hi)
    uint64_t best_T = KEY_END;
    int best = V - 1;
    for (int iter = 0; iter < 80 && best > fit; ++iter) {
        // key < T with T up to 2^32: a 32-bit comparison, or everything
        const bool all = (T >> 32) != 0;
        const uint32_t t32 = (uint32_t)T;
        uint64_t below = 0;
#pragma unroll
        for (int e = 0; e < NK; ++e) below |= (uint64_t)(all | (keys[e] < t32)) << e;
        int c = __popcll(below & ok);
        c = block_count(c, sh.r);
        if (c >= need) {
            hi = T;
            if (c < best) { best = c; best_T = T; }
        } else {
            lo = T;
        }
        if (hi - lo < 2) break;
        // the count is linear in the threshold up to sampling noise: aim at the middle of the window;
        // every fourth step halves the interval instead, which alone ends the search
        uint64_t next = lo + ((hi - lo) >> 1);
        if (c > 0 && (iter & 3) != 3) {
            const double prop = (double)T * aim / (double)c;
            if (prop > (double)lo && prop < (double)hi) {
                const uint64_t p = (uint64_t)prop;
                if (p > lo && p < hi) next = p;
            }
        }
        T = next;
    }
    if (best > RCAP) {
        // only when well over a thousand of the row's keys share one 32-bit value
        for (int j = 1 + tid; j < k; j += NT) orow[j] = -1;
        return;
    }

    // ---- collect (key, token) below the threshold ----
    if (tid == 0) sh.r.count = 0;
    __syncthreads();
    const bool best_all = (best_T >> 32) != 0;
    const uint32_t best_t32 = (uint32_t)best_T;
#pragma unroll
    for (int e = 0; e < NK; ++e) {
        if (((ok >> e) & 1) && (best_all | (keys[e] < best_t32))) {
            const int y = 4 * ((e >> 2) * NT + tid_again) + (e & 3);
            const int slot = atomicAdd(&sh.r.count, 1);
            sh.cand[lds_slot(slot)] = ((uint64_t)keys[e] << 32) | (uint32_t)y;
        }
        if ((e & 3) == 3) __builtin_amdgcn_sched_barrier(0);   // four appends in flight, not all NK
    }
    __syncthreads();
    const int count = sh.r.count;            // == best <= RCAP
    int P = 4;
    while (P < count) P <<= 1;
    for (int s = count + tid; s < P; s += NT) sh.cand[lds_slot(s)] = ~0ull;
    // the packed word orders by (key, token)
    bitonic_sort_lds<NT, uint64_t>(
        P, tid, [&](int p) { return sh.cand[p]; }, [&](int p, uint64_t v) { sh.cand[p] = v; },
        [](uint64_t a, uint64_t b) { return a > b; }, [](bool sw, uint64_t a, uint64_t b) { return sw ? b : a; });
    for (int j = tid; j < need; j += NT) orow[1 + j] = (int32_t)(uint32_t)sh.cand[lds_slot(j)];
}

}  // namespace

hipError_t launch_build_random(int V, int k, uint64_t seed, uint64_t t0, int32_t* out, hipStream_t stream) {
    const uint32_t s_lo = (uint32_t)(seed & 0xFFFFFFFFu), s_hi = (uint32_t)(seed >> 32);
    if (k - 1 <= RCAP && V <= 64 * NT) {
        if (V <= 16 * NT) hipLaunchKernelGGL(random_rows_regs<16>, dim3(V), dim3(NT), 0, stream, V, k, s_lo, s_hi, t0, out);
        else if (V <= 32 * NT) hipLaunchKernelGGL(random_rows_regs<32>, dim3(V), dim3(NT), 0, stream, V, k, s_lo, s_hi, t0, out);
        else hipLaunchKernelGGL(random_rows_regs<64>, dim3(V), dim3(NT), 0, stream, V, k, s_lo, s_hi, t0, out);
        return hipGetLastError();
    }
    const size_t lds = sizeof(RandomShared) + (size_t)CAP * sizeof(uint64_t);
    const hipError_t e = allow_lds<&random_rows_kernel>(lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(random_rows_kernel, dim3(V), dim3(NT), lds, stream, V, k, (uint32_t)(seed & 0xFFFFFFFFu),
                       (uint32_t)(seed >> 32), t0, out);
    return hipGetLastError();
}

}  // namespace lantern
