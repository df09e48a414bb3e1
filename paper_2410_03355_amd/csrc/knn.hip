// Codebook neighbour table B_k (Section 4.2; Algorithm 2, precompute part).
//
// Pipeline per block of query rows:
//   1. approximate keys (fp32) for every pair (query i, token j) into the
//      workspace: squared l2 distance, or minus cosine similarity
//   2. per row: find a threshold with at least k-1+pad approximate keys at or below it
//      (bisection with counting passes), recompute
//      the survivors' keys in fp64 exactly as the definition states (coordinate
//      order, every operation rounded separately), sort them by (key, index)
//      and emit the first k-1 after the token itself.  A row is emitted only if
//      the approximation's error bound proves no discarded token could belong
//      to it; otherwise it is flagged.
//   3. flagged rows: fp64 keys for all V tokens and ranking by counting.
// The written order is therefore always the fp64 one.
//
// Vocabularies of 4096 tokens and more (aligned codebooks, k from about 60 to about 1000) never form the
// whole key block: a row's threshold is first estimated from the keys to a stratified sample of
// one token in eight, the contraction then runs with an epilogue that appends only the
// (key, token) pairs at or below the row's threshold to a short per-row list, and step 2 works
// on that list.  The threshold only decides how many candidates a row gets; the proof condition
// of step 2 is unchanged (every token left out has an approximate key above every key kept),
// and a row whose list came out too short or too long is flagged like any other.
#include <hip/hip_runtime.h>
#include <limits.h>
#include <math.h>
#include <stdint.h>

#include <mutex>

#include "device_utils.h"
#include "knn_args.h"
#include "lantern.h"
#include "lds_sort.h"

namespace lantern {

// Query rows per pass through the workspace: as many as give a key block of at most 512 MiB, up to
// 8192 (few, full launches: V = 8192 in one block measured 0.44 ms against 0.53 ms in four).
constexpr int ROW_BLOCK = 8192;
static int whole_row_block(int V) {
    const int64_t fit = ((int64_t)512 << 20) / (4 * (int64_t)V) / 128 * 128;
    return fit >= ROW_BLOCK ? ROW_BLOCK : (fit < 128 ? 128 : (int)fit);
}
// The same on the path that keeps candidate lists instead of whole rows: the lists are short, so a
// 16384-token vocabulary goes through in one block (measured at 2048 / 4096 / 8192 / 16384 rows per
// block: 1.10 / 0.93 / 0.82 / 0.77 ms for V = 16384, k = 1000; fewer, fuller launches).
constexpr int FILTER_ROW_BLOCK = 16384;
constexpr int CAND_CAP = 4096;    // candidate slots per row held in LDS
constexpr int SLOW_WGS = 128;     // workgroups (and fp64 row buffers) of the exact pass

__host__ __device__ inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Tails of the binomial law of n trials with success probability p, summed term by term from the
// given end (the terms fall off geometrically there): P(X >= r) and P(X <= r).
static double binomial_log_pmf(int n, double p, int x) {
    return lgamma((double)n + 1.0) - lgamma((double)x + 1.0) - lgamma((double)(n - x) + 1.0) + (double)x * log(p) +
           (double)(n - x) * log1p(-p);
}
static double binomial_upper_tail(int n, double p, int r) {
    if (r <= 0) return 1.0;
    if (r > n) return 0.0;
    double term = exp(binomial_log_pmf(n, p, r)), sum = 0.0;
    for (int x = r; x <= n && (term > 1e-300 || x < (int)(n * p)); ++x) {
        sum += term;
        term *= (double)(n - x) / (double)(x + 1) * p / (1.0 - p);
        if (x > (int)(n * p) && term < sum * 1e-17) break;
    }
    return sum;
}
static double binomial_lower_tail(int n, double p, int r) {
    if (r < 0) return 0.0;
    if (r >= n) return 1.0;
    double term = exp(binomial_log_pmf(n, p, r)), sum = 0.0;
    for (int x = r; x >= 0; --x) {
        sum += term;
        if (x == 0) break;
        term *= (double)x / (double)(n - x + 1) * (1.0 - p) / p;
        if (x < (int)(n * p) && term < sum * 1e-17) break;
    }
    return sum;
}

// Plan of the sampled-threshold path for one shape.  A row's threshold has between `rank` and
// `rank + slack` of the row's keys to `S` sampled tokens at or below it.  The row's list is too short
// (fewer than the k-1+pad candidates the selection wants) only if at least rank - 1 of the sampled
// tokens are among the row's k-2+pad nearest, and too long for its `cap` slots only if at most
// rank + slack of them are among its cap+1 nearest (the row's own token may be in the sample: hence
// the - 1).  The sample takes one token from each of S strata of the vocabulary, so the number of
// sampled tokens in a given set is a sum of independent trials, whose tails are no heavier than
// those of the binomial law with the same mean (Hoeffding): `rank` is the smallest and `cap` the
// smallest of 1024 .. 4096 for which that bound puts either miss below 1e-10 per row, whatever
// the codebook.  A row that misses all the same is flagged and ranked by the all-pairs pass.
// use == false: the shape takes the whole-key-block path.
struct FilterPlan {
    bool use;
    int S;      // sampled tokens, a multiple of 64, at most 4096
    int rank;   // the threshold has between rank and rank + slack of a row's S sample keys at or below it
    int slack;
    int cap;    // slots of a row's candidate list: 1024, 2048, 3072 or 4096
};

static FilterPlan filter_plan(int V, int d, int k, int cb_dtype) {
    FilterPlan P = {false, 0, 0, 0, 0};
    const bool vec = cb_dtype == 1 ? (d % 8) == 0 : (d % 4) == 0;   // what the matrix-core kernels need
    const int need = k - 1;
    const int want = need + 8 + need / 128;
    // 64 candidates or fewer: the lists would be several times longer than what the selection wants
    if (!vec || V < 4096 || want <= 64 || want > 1024) return P;
    int S = V / 8;
    if (S > 4096) S = 4096;
    S = S / 64 * 64;
    const double miss = 1e-10;
    const double others = (double)(V - 1);
    // too short: Binomial(S, (want - 1) / (V - 1)) >= rank - 1
    const double p_lo = (double)(want - 1) / others;
    int rank = (int)(S * p_lo) + 2;
    while (rank < S && binomial_upper_tail(S, p_lo, rank - 1) > miss) ++rank;
    if (rank >= S) return P;
    // the search for the threshold stops anywhere between rank and rank + slack (a sixteenth more)
    const int slack = rank / 16 < S - rank ? rank / 16 : S - rank;
    // too long: Binomial(S, (cap + 1) / (V - 1)) <= rank + slack
    int cap = 0;
    for (int c = 1024; c <= 4096 && cap == 0; c += 1024) {
        const double p_hi = (double)(c + 1) / others;
        if (p_hi >= 1.0 || binomial_lower_tail(S, p_hi, rank + slack) <= miss) cap = c;
    }
    if (cap == 0) return P;
    P.use = true;
    P.S = S;
    P.rank = rank;
    P.slack = slack;
    P.cap = cap;
    return P;
}

struct KnnLayout {
    size_t stats, norms, nmax, dist, flags, slow, total;
    // sampled-threshold path (filter.use): the sample's codes and norms, a row block's keys to the
    // sample, its thresholds, list lengths and candidate lists; `dist` is then not laid out
    size_t scb, snorms, skeys, thr, counts, cand;
    FilterPlan filter;
    int row_block;   // query rows per pass through the key block
    int slow_wgs;    // workgroups (and fp64 row buffers) of the exact pass
};

static KnnLayout knn_layout(int V, int d, int cb_dtype, const FilterPlan& plan, int row_block, int slow_wgs) {
    KnnLayout L;
    L.filter = plan;
    L.row_block = V < row_block ? V : row_block;
    L.slow_wgs = slow_wgs;
    size_t off = 0;
    L.stats = off; off = align_up(off + 256, 256);   // int32[0]: rows that took the exact all-pairs pass
    L.norms = off; off = align_up(off + sizeof(float) * (size_t)V, 256);
    L.nmax = off;  off = align_up(off + 256, 256);
    L.dist = L.scb = L.snorms = L.skeys = L.thr = L.counts = L.cand = off;
    if (plan.use) {
        L.scb = off;    off = align_up(off + (cb_dtype == 1 ? 2 : 4) * (size_t)plan.S * d, 256);
        L.snorms = off; off = align_up(off + sizeof(float) * (size_t)plan.S, 256);
        L.skeys = off;  off = align_up(off + sizeof(float) * (size_t)L.row_block * plan.S, 256);
        L.thr = off;    off = align_up(off + sizeof(float) * (size_t)L.row_block, 256);
        L.counts = off; off = align_up(off + sizeof(int) * (size_t)L.row_block, 256);
        L.cand = off;   off = align_up(off + sizeof(uint2) * (size_t)L.row_block * plan.cap, 256);
    } else {
        L.dist = off;   off = align_up(off + sizeof(float) * (size_t)L.row_block * V, 256);
    }
    L.flags = off; off = align_up(off + sizeof(int) * (size_t)V, 256);   // one word per row of the table
    L.slow = off;  off = align_up(off + sizeof(double) * (size_t)L.slow_wgs * V, 256);
    L.total = off;
    return L;
}

// The largest layout of the given path that fits `bytes`: as many query rows per pass as the
// rest holds (a multiple of 128, the contraction's tile).  row_block 0: nothing fits.
static KnnLayout knn_layout_within(int V, int d, int cb_dtype, const FilterPlan& plan, int slow_wgs, size_t bytes) {
    for (int rb = whole_row_block(V); rb >= 128; rb -= 128) {
        const KnnLayout L = knn_layout(V, d, cb_dtype, plan, rb, slow_wgs);
        if (L.total <= bytes) return L;
    }
    KnnLayout none = knn_layout(V, d, cb_dtype, plan, 128, slow_wgs);
    none.row_block = 0;
    return none;
}

static const FilterPlan NO_FILTER = {false, 0, 0, 0, 0};

// What lantern_build_knn asks of its caller: the layout of the path the shape takes.  A codebook
// that turns out not to be 16-byte aligned falls back to whole key blocks of as many rows as
// this size holds.
size_t knn_workspace_bytes(int V, int d, int k, int cb_dtype) {
    const FilterPlan plan = filter_plan(V, d, k, cb_dtype);
    return knn_layout(V, d, cb_dtype, plan, plan.use ? FILTER_ROW_BLOCK : whole_row_block(V), SLOW_WGS).total;
}

// ---- scratch of the entry point that allocates nothing ----
// Device memory that lives as long as the process, one copy per GPU.  Host code never uses the
// array's name as an address: it asks the runtime for the array's device address once per device
// and passes that pointer on.
constexpr size_t STATIC_SCRATCH_BYTES = LANTERN_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

// The static scratch serves the whole-key-block path with fewer exact-pass buffers and as many
// query rows per pass as fit.  row_block 0: V is beyond what the scratch can serve.
constexpr int STATIC_SLOW_WGS = 32;
static KnnLayout knn_layout_static(int V, int d, int cb_dtype) {
    return knn_layout_within(V, d, cb_dtype, NO_FILTER, STATIC_SLOW_WGS, STATIC_SCRATCH_BYTES);
}

bool knn_static_fits(int V) { return knn_layout_static(V, 4, 0).row_block > 0; }

// Device address of the static scratch on the current device (looked up once per device).
static hipError_t static_scratch_ptr(void** out) {
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static void* ptrs[MAX_DEVICES];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptrs[dev] = p;
    }
    *out = ptrs[dev];
    return hipSuccess;
}

template <typename CT> __device__ __forceinline__ float cb_f32(const CT* p, int64_t i);
template <> __device__ __forceinline__ float cb_f32<float>(const float* p, int64_t i) { return p[i]; }
template <> __device__ __forceinline__ float cb_f32<uint16_t>(const uint16_t* p, int64_t i) {
    return __uint_as_float(static_cast<uint32_t>(p[i]) << 16);
}

// order-preserving map float -> uint32 (ascending)
__device__ __forceinline__ uint32_t ord_key(float f) {
    const uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float ord_inv(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

// ---- exact fp64 key of the pair (i, j): the definition, operation by operation ----
// Four consecutive coordinates of a code as floats (one 16-byte or 8-byte load); the caller
// guarantees t + 3 < d and 16-byte aligned rows.
__device__ __forceinline__ void cb_load4(const float* p, int t, float (&o)[4]) {
    const float4 v = *reinterpret_cast<const float4*>(p + t);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
}
__device__ __forceinline__ void cb_load4(const uint16_t* p, int t, float (&o)[4]) {
    const uint2 v = *reinterpret_cast<const uint2*>(p + t);
    o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xFFFF0000u);
    o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xFFFF0000u);
}

// vec4: rows are 16-byte aligned and d is a multiple of 4, so coordinates are fetched four at
// a time; the arithmetic is the same sequence of separately rounded operations either way.
template <typename CT>
__device__ double exact_key(const CT* cb, int d, int i, int j, int metric, bool vec4) {
#pragma clang fp contract(off)
    const CT* ci = cb + (int64_t)i * d;
    const CT* cj = cb + (int64_t)j * d;
    if (metric == 0) {
        double acc = 0.0;
        if (vec4) {
#pragma unroll 4   // the loads of four groups are in flight together; the sum keeps its order
            for (int t = 0; t < d; t += 4) {
                float x[4], y[4];
                cb_load4(ci, t, x);
                cb_load4(cj, t, y);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const double diff = (double)x[e] - (double)y[e];
                    const double sq = diff * diff;
                    acc = acc + sq;
                }
            }
        } else {
            for (int t = 0; t < d; ++t) {
                const double diff = (double)cb_f32<CT>(ci, t) - (double)cb_f32<CT>(cj, t);
                const double sq = diff * diff;
                acc = acc + sq;
            }
        }
        return acc == acc ? acc : (double)INFINITY;
    }
    double ni = 0.0, nj = 0.0, dot = 0.0;
    for (int t = 0; t < d; ++t) {
        const double x = (double)cb_f32<CT>(ci, t);
        const double y = (double)cb_f32<CT>(cj, t);
        const double xx = x * x;
        const double yy = y * y;
        const double xy = x * y;
        ni = ni + xx;
        nj = nj + yy;
        dot = dot + xy;
    }
    ni = sqrt(ni);
    nj = sqrt(nj);
    const double den = ni * nj;
    const double key = -(dot / den);
    return key == key ? key : (double)INFINITY;   // no similarity (a code of zero norm): the farthest
}

template <typename CT>
__global__ __launch_bounds__(NT) void knn_dist_direct(const CT* cb, int V, int d, int r0, int metric,
                                                      float* dist) {
    const int row = blockIdx.y;
    const int i = r0 + row;
    const int j = blockIdx.x * NT + threadIdx.x;
    if (j >= V) return;
    const CT* ci = cb + (int64_t)i * d;
    const CT* cj = cb + (int64_t)j * d;
    float key;
    if (metric == 0) {
        float acc = 0.f;
        for (int t = 0; t < d; ++t) {
            const float diff = cb_f32<CT>(ci, t) - cb_f32<CT>(cj, t);
            acc = fmaf(diff, diff, acc);
        }
        key = acc;
    } else {
        float ni = 0.f, nj = 0.f, dot = 0.f;
        for (int t = 0; t < d; ++t) {
            const float x = cb_f32<CT>(ci, t), y = cb_f32<CT>(cj, t);
            ni = fmaf(x, x, ni);
            nj = fmaf(y, y, nj);
            dot = fmaf(x, y, dot);
        }
        key = -dot / sqrtf(ni * nj);
    }
    dist[(int64_t)row * V + j] = key;
}


// ---- stage 1 (aligned shapes): approximate keys from a matrix-core contraction ----
// G = C C^T on MFMA 32x32 tiles with fp32 accumulation; squared l2 key
// n_i + n_j - 2 G_ij, cosine key -G_ij / sqrt(n_i n_j).  One wavefront owns a
// 64x64 block of the key matrix (2x2 MFMA tiles); a workgroup of 4 wavefronts
// owns 128x128.  Operand fragments are read straight from the codebook, which
// stays cache-resident (at most a few MB).
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Sum of the squares of the coordinates held in 16 bytes of a row.
template <typename CT> __device__ __forceinline__ float sum_squares(const uint4& v, float n);
template <> __device__ __forceinline__ float sum_squares<float>(const uint4& v, float n) {
    const float x0 = __uint_as_float(v.x), x1 = __uint_as_float(v.y), x2 = __uint_as_float(v.z), x3 = __uint_as_float(v.w);
    return fmaf(x3, x3, fmaf(x2, x2, fmaf(x1, x1, fmaf(x0, x0, n))));
}
template <> __device__ __forceinline__ float sum_squares<uint16_t>(const uint4& v, float n) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float lo = __uint_as_float(w[q] << 16), hi = __uint_as_float(w[q] & 0xFFFF0000u);
        n = fmaf(hi, hi, fmaf(lo, lo, n));
    }
    return n;
}

// Squared norms of the rows and their maximum, for rows that are whole 16-byte vectors at 16-byte
// aligned addresses.  *nmax is cleared beforehand; a norm is never below +0, so the bit patterns
// order like the values and an unsigned maximum collects it, asked for only by a workgroup that
// sees a smaller value there (a NaN norm is stored but left out of the maximum).  Rows of 256 bytes
// or more take a wavefront each, NORM_ROWS rows per workgroup with the loads of all of a
// wavefront's rows in flight together (index clamped, bits masked: no branch around a load);
// shorter rows take a thread each.
constexpr int NORM_ROWS = 32;
constexpr int NORM_WAVE_VECS = 16;
template <typename CT>
__global__ __launch_bounds__(NT) void knn_norms(const CT* cb, int V, int d, float* norms, float* nmax) {
    __shared__ float red[NW];
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x >> 6;
    const int vecs = d * (int)sizeof(CT) / 16;   // 16-byte vectors per row
    const uint4* cbv = reinterpret_cast<const uint4*>(cb);
    float m = 0.f;
    if (vecs >= NORM_WAVE_VECS) {
        constexpr int RPW = NORM_ROWS / NW;
        float n[RPW];
#pragma unroll
        for (int q = 0; q < RPW; ++q) n[q] = 0.f;
        for (int c0 = 0; c0 < vecs; c0 += WAVE) {
            const int c = c0 + lane;
            const uint32_t mask = c < vecs ? 0xFFFFFFFFu : 0u;
            const int cc = c < vecs ? c : vecs - 1;
#pragma unroll
            for (int q = 0; q < RPW; ++q) {
                const int i = blockIdx.x * NORM_ROWS + q * NW + w;
                uint4 v = cbv[(int64_t)(i < V ? i : V - 1) * vecs + cc];
                v.x &= mask; v.y &= mask; v.z &= mask; v.w &= mask;
                n[q] = sum_squares<CT>(v, n[q]);
            }
        }
#pragma unroll
        for (int q = 0; q < RPW; ++q) {
            const int i = blockIdx.x * NORM_ROWS + q * NW + w;
            const float t = wave_sum(n[q]);
            if (i < V) {
                if (lane == 0) norms[i] = t;
                m = fmaxf(m, t);
            }
        }
    } else {
        const int i = blockIdx.x * NT + threadIdx.x;
        if (i < V) {
            float n = 0.f;
            for (int c = 0; c < vecs; ++c) n = sum_squares<CT>(cbv[(int64_t)i * vecs + c], n);
            norms[i] = n;
            m = fmaxf(m, n);
        }
    }
    m = fmaxf(wave_max(m), 0.f);
    if (lane == 0) red[w] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        float r = red[0];
        for (int v = 1; v < NW; ++v) r = fmaxf(r, red[v]);
        unsigned int* target = reinterpret_cast<unsigned int*>(nmax);
        const unsigned int bits = __float_as_uint(r);
        if (__hip_atomic_load(target, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < bits) atomicMax(target, bits);
    }
}

// Accumulator element r of lane l of a 32x32 MFMA tile is row 8*(r/4) + 4*(l/32) + r%4,
// column l%32 (rows come from the A operand, columns from the B operand).
__device__ __forceinline__ float approx_key(float g, float ni, float nj, int metric) {
    return metric == 0 ? (ni + nj) - 2.f * g : -g * rsqrtf(ni * nj);
}

// Columns are the VB tokens of the column operand (the codebook itself, or a sample of it) with
// norms nb; a row of dist holds VB keys.
__device__ __forceinline__ void store_tile(const f32x16& acc, int i0, int j0, int lane, int r0, int rows,
                                           int VB, int metric, const float* norms, const float* nb, float* dist) {
    const int j = j0 + (lane & 31);
    if (j >= VB) return;
    const float nj = nb[j];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int i = i0 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (i < r0 + rows) dist[(int64_t)(i - r0) * VB + j] = approx_key(acc[r], norms[i], nj, metric);
    }
}

// 64x64 block of G = A B^T for one wavefront: rows arow[0], arow[1] (32 each, one per lane & 31),
// columns brow[0], brow[1]; acc[a][b] is the 32x32 tile of row strip a and column strip b.
//
// bf16 codebook, d a multiple of 8: v_mfma_f32_32x32x16_bf16, 16 coordinates per step
// (lanes 0-31 carry coordinates k0..k0+7 of their row, lanes 32-63 k0+8..k0+15).
__device__ __forceinline__ void contract_block(const uint16_t* const (&arow)[2], const uint16_t* const (&brow)[2],
                                               int d, int lane, f32x16 (&acc)[2][2]) {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    const int kh = 8 * (lane >> 5);
    for (int k0 = 0; k0 < d; k0 += 16) {
        const int kk = k0 + kh;
        uint4 fa[2], fb[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            if (kk < d) {
                fa[t] = *reinterpret_cast<const uint4*>(arow[t] + kk);
                fb[t] = *reinterpret_cast<const uint4*>(brow[t] + kk);
            } else {
                fa[t] = make_uint4(0, 0, 0, 0);
                fb[t] = fa[t];
            }
        }
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8, fa[a]), __builtin_bit_cast(bf16x8, fb[b]), acc[a][b], 0, 0, 0);
    }
}

// fp32 codebook, d a multiple of 4: v_mfma_f32_32x32x2_f32, 2 coordinates per step
// (lanes 0-31 carry coordinate k, lanes 32-63 coordinate k+1); rows are read 8 floats at a time.
__device__ __forceinline__ void contract_block(const float* const (&arow)[2], const float* const (&brow)[2], int d,
                                               int lane, f32x16 (&acc)[2][2]) {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    const bool hi = (lane >> 5) != 0;
    for (int k0 = 0; k0 < d; k0 += 8) {
        float4 fa[2][2], fb[2][2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (k0 + 4 * h < d) {
                    fa[t][h] = *reinterpret_cast<const float4*>(arow[t] + k0 + 4 * h);
                    fb[t][h] = *reinterpret_cast<const float4*>(brow[t] + k0 + 4 * h);
                } else {
                    fa[t][h] = make_float4(0.f, 0.f, 0.f, 0.f);
                    fb[t][h] = fa[t][h];
                }
            }
#pragma unroll
        for (int s = 0; s < 4; ++s) {  // coordinates k0+2s, k0+2s+1
            float va[2], vb[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const float4 qa = fa[t][s >> 1], qb = fb[t][s >> 1];
                va[t] = (s & 1) ? (hi ? qa.w : qa.z) : (hi ? qa.y : qa.x);
                vb[t] = (s & 1) ? (hi ? qb.w : qb.z) : (hi ? qb.y : qb.x);
            }
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(va[a], vb[b], acc[a][b], 0, 0, 0);
        }
    }
}

// All keys of rows [r0, r0 + rows) of the codebook cb (V tokens, norms `norms`) against the VB
// tokens of the column operand cbB (norms nb: the codebook itself, or a sample of it) into dist.
// blockIdx = (column tile, row tile).
template <typename CT>
__global__ __launch_bounds__(NT) void knn_dist_mfma(const CT* cb, const CT* cbB, const float* norms, const float* nb,
                                                    int V, int VB, int d, int r0, int rows, int metric, float* dist) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int wave = threadIdx.x >> 6;
    const int i_base = r0 + blockIdx.y * 128 + (wave >> 1) * 64;
    const int j_base = blockIdx.x * 128 + (wave & 1) * 64;
    if (i_base >= r0 + rows || j_base >= VB) return;
    const CT* arow[2];
    const CT* brow[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        arow[t] = cb + (int64_t)min(i_base + t * 32 + (lane & 31), V - 1) * d;
        brow[t] = cbB + (int64_t)min(j_base + t * 32 + (lane & 31), VB - 1) * d;
    }
    f32x16 acc[2][2];
    contract_block(arow, brow, d, lane, acc);
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
            store_tile(acc[a][b], i_base + a * 32, j_base + b * 32, lane, r0, rows, VB, metric, norms, nb, dist);
}

// Where the filtering contraction leaves a row block's candidates.
struct FilterOut {
    const float* thr;   // [rows] threshold of each row of the block
    int* counts;        // [rows] keys at or below the threshold so far (may pass cap: the list is then cut)
    uint2* cand;        // [rows, cap] (order-preserving key, token), in no particular order
    int cap;
};

// LDS of the filtering contraction: per row of the workgroup's 128 its threshold, its norm and a
// counter (pass 1: keys kept; pass 2: next free slot of the row's list).
struct FilterShared {
    float thr[128];
    float norm[128];
    int slots[128];
};

// One 32-row strip of a wavefront's 64x64 block in the filtering contraction, columns j0..j0+63
// (tiles acc0, acc1); l0: the strip's first row within the workgroup's 128, i0 its token.  A key
// stays if it is at or below its row's threshold (NaN for rows beyond the block) and is not the
// row's own token.  Element r of lanes 0-31 belongs to one row and of lanes 32-63 to another, so
// each half of the wavefront adds its number of kept keys to its row's counter with one LDS
// atomic; WRITE: what the atomic returns is the first of the half's slots in the row's list, and
// the keys are placed by their lane rank.
template <bool WRITE, int METRIC>
__device__ __forceinline__ void filter_strip(const f32x16& acc0, const f32x16& acc1, int l0, int i0, int j0, int lane,
                                             int il_wg, int V, const float* norms, FilterShared& sh,
                                             const FilterOut& f) {
    const int half = lane >> 5;
    const int hl = lane & 31;
    const int ja = j0 + hl, jb = j0 + 32 + hl;
    const bool va = ja < V, vb = jb < V;
    const float na = norms[va ? ja : V - 1], nb = norms[vb ? jb : V - 1];
    const uint32_t below = (1u << hl) - 1u;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int l = l0 + 8 * (r >> 2) + 4 * half + (r & 3);
        const int i = i0 + 8 * (r >> 2) + 4 * half + (r & 3);
        const float ni = sh.norm[l];
        const float t = sh.thr[l];
        const float ka = approx_key(acc0[r], ni, na, METRIC), kb = approx_key(acc1[r], ni, nb, METRIC);
        const bool pa = va && ja != i && ka <= t;
        const bool pb = vb && jb != i && kb <= t;
        const uint64_t ma = __ballot(pa), mb = __ballot(pb);
        const uint32_t ha = (uint32_t)(half ? ma >> 32 : ma), hb = (uint32_t)(half ? mb >> 32 : mb);
        const int n = __popc(ha) + __popc(hb);
        if (!WRITE) {
            if (hl == 0 && n > 0) atomicAdd(&sh.slots[l], n);
        } else {
            int first = 0;
            if (hl == 0 && n > 0) first = atomicAdd(&sh.slots[l], n);
            const int b0 = __builtin_amdgcn_readlane(first, 0), b1 = __builtin_amdgcn_readlane(first, 32);
            first = half ? b1 : b0;
            uint2* list = f.cand + (int64_t)(il_wg + l) * f.cap;   // only dereferenced for rows of the block
            const int sa = first + __popc(ha & below);
            const int sb = first + __popc(ha) + __popc(hb & below);
            if (pa && sa < f.cap) list[sa] = make_uint2(min(ord_key(ka), 0xFFFFFFFEu), (uint32_t)ja);
            if (pb && sb < f.cap) list[sb] = make_uint2(min(ord_key(kb), 0xFFFFFFFEu), (uint32_t)jb);
        }
        if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);   // four rows in flight: keeps the register count down
    }
}

// Filtering contraction: rows [r0, r0 + rows) against the whole codebook, keeping for every row
// only the (key, token) pairs at or below the row's threshold.  A workgroup owns a tile of 128
// rows by 128 tokens.  It contracts, counts the kept keys per row in LDS, reserves each row's
// slots in its list with one atomic add per row, and then places the keys (the accumulators stay
// in registers meanwhile).
// Grid: one-dimensional, 8 * ceil(row tiles / 8) * column tiles workgroups, dealt so that all
// column tiles of a row strip run on one XCD (workgroups go to the eight XCDs in turn) and a
// row's list and counter stay in that XCD's L2.
template <typename CT, int METRIC>
__global__ __launch_bounds__(NT, 2) void knn_filter_mfma(const CT* cb, const float* norms, int V, int d, int r0,
                                                         int rows, FilterOut f) {
    __shared__ FilterShared sh;
    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1);
    const int wave = tid >> 6;
    const int nct = (V + 127) / 128, nrt = (rows + 127) / 128;
    const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
    const int ti = (q / nct) * 8 + xcd;
    const int tj = q % nct;
    if (ti >= nrt) return;   // the whole workgroup
    const int il_wg = ti * 128;        // first row of the workgroup within the block
    const int l_base = (wave >> 1) * 64;
    const int i_base = r0 + il_wg + l_base;
    const int j_base = tj * 128 + (wave & 1) * 64;
    const bool live = j_base < V;      // rows beyond the block are kept out by their thresholds (NaN)
    if (tid < 128) {
        const bool row_ok = il_wg + tid < rows;
        // rows beyond the block: no key compares at or below NaN (a threshold of -inf would let the
        // cosine key -g / sqrt(0 n_j) = -inf through), and the norm is kept away from zero
        sh.thr[tid] = row_ok ? f.thr[il_wg + tid] : NAN;
        sh.norm[tid] = row_ok ? norms[r0 + il_wg + tid] : 1.f;
        sh.slots[tid] = 0;
    }
    __syncthreads();
    f32x16 acc[2][2];
    if (live) {
        const CT* arow[2];
        const CT* brow[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            arow[t] = cb + (int64_t)min(i_base + t * 32 + (lane & 31), V - 1) * d;
            brow[t] = cb + (int64_t)min(j_base + t * 32 + (lane & 31), V - 1) * d;
        }
        contract_block(arow, brow, d, lane, acc);
#pragma unroll
        for (int a = 0; a < 2; ++a)
            filter_strip<false, METRIC>(acc[a][0], acc[a][1], l_base + a * 32, i_base + a * 32, j_base, lane, il_wg, V,
                                        norms, sh, f);
    }
    __syncthreads();
    if (tid < 128) {
        const int n = sh.slots[tid];   // n > 0 only for rows of the block
        sh.slots[tid] = (n > 0 && il_wg + tid < rows) ? atomicAdd(f.counts + il_wg + tid, n) : 0;
    }
    __syncthreads();
    if (live) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
            filter_strip<true, METRIC>(acc[a][0], acc[a][1], l_base + a * 32, i_base + a * 32, j_base, lane, il_wg, V,
                                       norms, sh, f);
    }
}

// ---- sampled thresholds ----
// Token of sample slot s: one token out of each of S equal strata of the vocabulary, at a hashed
// place inside the stratum.
__host__ __device__ inline int sample_token(int s, int S, int V) {
    const uint32_t h = ((uint32_t)s * 2654435761u) >> 16;   // 16 hashed bits
    const int64_t j = ((int64_t)s * V + (((int64_t)h * V) >> 16)) / S;
    return j < V ? (int)j : V - 1;
}

template <typename CT>
__global__ __launch_bounds__(NT) void knn_gather_sample(const CT* cb, const float* norms, int V, int d, int S,
                                                        CT* scb, float* snorms) {
    const int64_t t = (int64_t)blockIdx.x * NT + threadIdx.x;
    if (t >= (int64_t)S * d) return;
    const int s = (int)(t / d), c = (int)(t % d);
    const int j = sample_token(s, S, V);
    scb[t] = cb[(int64_t)j * d + c];
    if (c == 0) snorms[s] = norms[j];
}

// One wavefront per row: a value with between rank and rank + slack of the row's S <= 64 * NS keys
// to the sample at or below it (bisection over the integer range of the keys, each step one
// count) becomes the row's threshold; the row's list length is cleared.
// (At most four wavefronts per SIMD are aimed at: with more as its goal the compiler's scheduler
// keeps the register count down by waiting for each of the 64 loads of the largest variant in turn.)
template <int NS>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(1, NS > 32 ? 4 : 8))) void knn_sample_rank(const float* skeys, int S, int rows, int rank, int slack,
                                                      float* thr, int* counts) {
    const int lane = threadIdx.x & (WAVE - 1);
    const int row = blockIdx.x * NW + (threadIdx.x >> 6);
    if (row >= rows) return;   // whole wavefronts leave; no workgroup barrier below
    const float* krow = skeys + (int64_t)row * S;
    uint32_t keys[NS];
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
    for (int e = 0; e < NS; ++e) {
        const int sidx = e * WAVE + lane;
        // no branch and no select on the loaded value, so that all loads are in flight together:
        // beyond the sample the index is clamped and the key forced to all ones by a mask
        const uint32_t beyond = (uint32_t)((S - 1 - sidx) >> 31);
        const float v = krow[min(sidx, S - 1)];
        keys[e] = min(ord_key(v), 0xFFFFFFFEu) | beyond;
        kmin = min(kmin, keys[e]);
        kmax = max(kmax, keys[e] & ~beyond);
    }
    kmin = (uint32_t)__builtin_amdgcn_readlane(wave_scan_i<OpMin>((int)(kmin ^ 0x80000000u), INT_MAX), 63) ^ 0x80000000u;
    kmax = (uint32_t)__builtin_amdgcn_readlane(wave_scan_i<OpMax>((int)(kmax ^ 0x80000000u), INT_MIN), 63) ^ 0x80000000u;
    // count(lo) < rank <= count(hi)
    int64_t lo = (int64_t)kmin - 1, hi = (int64_t)kmax;
    while (hi - lo > 1) {
        const int64_t mid64 = lo + ((hi - lo) >> 1);
        const uint32_t mid = (uint32_t)mid64;
        int c = 0;
#pragma unroll
        for (int e = 0; e < NS; ++e) c += keys[e] <= mid ? 1 : 0;
        c = __builtin_amdgcn_readlane(wave_scan_i<OpSum>(c, 0), 63);
        if (c < rank) {
            lo = mid64;
        } else {
            hi = mid64;
            if (c <= rank + slack) break;
        }
    }
    if (lane == 0) {
        thr[row] = ord_inv((uint32_t)hi);
        counts[row] = 0;
    }
}

// ---- stage 2: select, re-rank exactly, emit ----
constexpr int SEL_MAXW = 8;   // wavefronts of the largest selection workgroup (512 threads)
template <int CAP>
struct SelectShared {
    static_assert(CAP % 128 == 0, "lds_slot permutes blocks of 128 slots");
    double key[CAP];   // both indexed by lds_slot
    int idx[CAP];
    unsigned red_u[2 * SEL_MAXW];
    int red_c[2][SEL_MAXW];   // per-wavefront counts of a counting pass, double-buffered
};

// Error model of the approximate keys:
//   |approximate - exact| <= err_rel * |exact| + err_abs + err_norm * (norm_i + max norm)
// (the last term applies when norms is not null: keys formed as n_i + n_j - 2 G_ij).
//
// NK > 0: the row's V <= NK * TNT approximate keys (TNT threads per row) are held in registers as order-preserving
// unsigned integers; NK == 0: they are re-read from the workspace in every pass.
// A threshold with between k-1+pad and `fit` keys at or below it is found by bisection over the
// keys' integer range, every step one counting pass over the registers (compare, add, one
// reduction): no sorting network or histogram over all V keys is needed to pick candidates.
// Runs body(e) for every key slot of a thread: fully unrolled when the keys sit in registers.
template <int NK, typename F>
__device__ __forceinline__ void for_keys(int npt, F body) {
    if (NK > 0) {
#pragma unroll
        for (int e = 0; e < NK; ++e) body(e);
    } else {
        for (int e = 0; e < npt; ++e) body(e);
    }
}

//
// LIST: the row's keys are not a row of the key block but its candidate list of the filtering
// contraction, list.counts[row] pairs (key, token) with NK * TNT >= list.cap; every token not on
// the list has an approximate key above every key on it, so the proof below reads the same.  A
// list that was cut at its capacity, or is shorter than the selection wants, flags the row.
template <typename CT, int NK, int CAP, int TNT, bool LIST>
__global__ __launch_bounds__(TNT, (LIST || NK < 64) ? 8 : 4) void knn_select(const CT* cb, int V, int d, int k, int metric, int r0,
                                                 const float* dist, FilterOut list, float err_rel, float err_abs,
                                                 float err_norm, const float* norms, const float* nmax,
                                                 int32_t* out, int* flags) {
    static_assert(!LIST || NK > 0, "a candidate list is held in registers");
    constexpr int TNW = TNT / WAVE;
    __shared__ SelectShared<CAP> sh;
    const int row = blockIdx.x;
    const int i = r0 + row;
    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1);
    const int wave = tid >> 6;
    const float* drow = LIST ? nullptr : dist + (int64_t)row * V;
    int32_t* orow = out + (int64_t)i * k;
    const int need = k - 1;
    // rows of four-coordinate groups, each group one aligned load (16 bytes fp32, 8 bytes bf16)
    const bool vec4 = (d % 4 == 0) && ((reinterpret_cast<uintptr_t>(cb) & 15) == 0);
    if (tid == 0) {
        orow[0] = i;
        flags[row] = 0;
    }
    if (need == 0) return;
    const int pad = 8 + need / 128;
    const int want = min(V - 1, need + pad);
    if (want > CAP) {
        if (tid == 0) flags[row] = 1;
        return;
    }

    constexpr int NKR = NK > 0 ? NK : 1;
    uint32_t keys[NKR];
    uint32_t toks[LIST ? NKR : 1];
    const int npt = NK > 0 ? NK : (V + TNT - 1) / TNT;   // keys per thread
    const int listed = LIST ? list.counts[row] : 0;
    if (LIST && (listed > list.cap || listed < want)) {
        if (tid == 0) flags[row] = 1;
        return;
    }
    // Token of element e of this thread.  Keys in registers: groups of four consecutive tokens per
    // thread, (e / 4) * TNT + tid being the group, so that a group is one 16-byte load; else e * TNT + tid.
    auto token_of = [&](int e) -> int {
        if (LIST) return (int)toks[e];
        return NK > 0 ? (((e >> 2) * TNT + tid) << 2) + (e & 3) : e * TNT + tid;
    };
    // key of element e; 0xFFFFFFFF for the row's own token and padding
    auto key_at = [&](int e) -> uint32_t {
        if (NK > 0) return keys[e];
        const int j = e * TNT + tid;
        return (j < V && j != i) ? min(ord_key(drow[j]), 0xFFFFFFFEu) : 0xFFFFFFFFu;
    };
    if (LIST) {
        const uint2* lrow = list.cand + (int64_t)row * list.cap;
#pragma unroll
        for (int e = 0; e < NKR; ++e) {
            const int slot = e * TNT + tid;
            const uint2 q = lrow[slot < listed ? slot : listed - 1];   // no branch: all loads in flight together (listed >= 1)
            keys[e] = slot < listed ? q.x : 0xFFFFFFFFu;
            toks[e] = q.y;
        }
    } else if (NK > 0) {
        if ((V & 3) == 0) {   // every row of the key block starts 16-byte aligned and ends with a whole group
            // No branch and no select on a loaded value, so that all the row's loads are in flight
            // together: a group beyond the row re-reads the last one, and its keys, like the row's own
            // token's, are forced to all ones by a mask.
            float4 q[NKR / 4 > 0 ? NKR / 4 : 1];
#pragma unroll
            for (int g = 0; g < NKR / 4; ++g)
                q[g] = *reinterpret_cast<const float4*>(drow + min((g * TNT + tid) << 2, V - 4));
#pragma unroll
            for (int g = 0; g < NKR / 4; ++g) {
                const int j0 = (g * TNT + tid) << 2;
                const float f[4] = {q[g].x, q[g].y, q[g].z, q[g].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int j = j0 + e;
                    const uint32_t out = (uint32_t)((V - 1 - j) >> 31) | (uint32_t)(-(int)(j == i));
                    keys[4 * g + e] = min(ord_key(f[e]), 0xFFFFFFFEu) | out;
                }
            }
        } else {
#pragma unroll
            for (int g = 0; g < NKR / 4; ++g) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int j = ((g * TNT + tid) << 2) + e;
                    const float f = j < V ? drow[j] : 0.f;
                    keys[4 * g + e] = (j < V && j != i) ? min(ord_key(f), 0xFFFFFFFEu) : 0xFFFFFFFFu;
                }
            }
        }
    }

    // range of the keys
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
    for_keys<NK>(npt, [&](int e) {
        const uint32_t key = key_at(e);
        if (key != 0xFFFFFFFFu) { kmin = min(kmin, key); kmax = max(kmax, key); }
    });
    // unsigned order through signed scans: flip the top bit
    kmin = (uint32_t)__builtin_amdgcn_readlane(wave_scan_i<OpMin>((int)(kmin ^ 0x80000000u), INT_MAX), 63) ^ 0x80000000u;
    kmax = (uint32_t)__builtin_amdgcn_readlane(wave_scan_i<OpMax>((int)(kmax ^ 0x80000000u), INT_MIN), 63) ^ 0x80000000u;
    if (lane == 0) { sh.red_u[wave] = kmin; sh.red_u[TNW + wave] = kmax; }
    __syncthreads();
    kmin = sh.red_u[0]; kmax = sh.red_u[TNW];
#pragma unroll
    for (int w = 1; w < TNW; ++w) { kmin = min(kmin, sh.red_u[w]); kmax = max(kmax, sh.red_u[TNW + w]); }

    // the sort works on a power of two: aim at the smallest one that holds `want`
    int fit = 1;
    while (fit < want) fit <<= 1;
    if (fit > CAP) fit = CAP;
    // Bisection over [kmin - 1, kmax] (as 64-bit integers): count(lo) < want <= count(hi).  The best
    // threshold seen is kept: the one with the fewest keys at or below it that still has `want` and
    // fits the LDS; the search stops as soon as that number fits the aimed-at power of two.
    int64_t lo = (int64_t)kmin - 1, hi = (int64_t)kmax;
    uint32_t thr_key = kmax;
    int best = LIST ? listed : V - 1;   // count(kmax): every listed token, every other token
    for (int pass = 0; pass < 40 && best > fit && hi - lo > 1; ++pass) {
        const int64_t mid64 = lo + ((hi - lo) >> 1);
        const uint32_t mid = (uint32_t)mid64;
        int c = 0;
        for_keys<NK>(npt, [&](int e) { c += key_at(e) <= mid ? 1 : 0; });   // own token and padding: 0xFFFFFFFF > mid
        c = __builtin_amdgcn_readlane(wave_scan_i<OpSum>(c, 0), 63);
        if (lane == 0) sh.red_c[pass & 1][wave] = c;
        __syncthreads();         // one barrier per pass: the buffers alternate
        c = 0;
#pragma unroll
        for (int w = 0; w < TNW; ++w) c += sh.red_c[pass & 1][w];
        if (c < want) {
            lo = mid64;
        } else {   // counts grow with the threshold: c <= best = count(hi)
            hi = mid64;
            best = c;
            thr_key = mid;
        }
    }
    if (best > CAP) {            // more (nearly) equal keys around the threshold than the LDS holds
        if (tid == 0) flags[row] = 1;
        return;
    }

    // compaction of every j != i with approximate key <= threshold, in thread order: every thread
    // counts its own, a scan over the workgroup gives its first slot; the largest such key
    int mine = 0;
    uint32_t my_max = 0u;
    for_keys<NK>(npt, [&](int e) {
        const uint32_t key = key_at(e);
        if (key <= thr_key) {   // the row's own token and padding carry 0xFFFFFFFF > thr_key
            ++mine;
            my_max = max(my_max, key);
        }
    });
    const int incl = wave_scan_i<OpSum>(mine, 0);
    my_max = (uint32_t)__builtin_amdgcn_readlane(wave_scan_i<OpMax>((int)(my_max ^ 0x80000000u), INT_MIN), 63) ^ 0x80000000u;
    __syncthreads();             // the counting passes are done with red_u / red_c
    if (lane == WAVE - 1) { sh.red_c[0][wave] = incl; sh.red_u[wave] = my_max; }
    __syncthreads();
    int slot = incl - mine;
    int count = 0;
    uint32_t thr_max = 0u;
#pragma unroll
    for (int w = 0; w < TNW; ++w) {
        if (w < wave) slot += sh.red_c[0][w];
        count += sh.red_c[0][w];
        thr_max = max(thr_max, sh.red_u[w]);
    }
    if (count > CAP) {  // more equal keys at the threshold than the LDS holds
        if (tid == 0) flags[row] = 1;
        return;
    }
    for_keys<NK>(npt, [&](int e) {
        if (key_at(e) <= thr_key) sh.idx[lds_slot(slot++)] = token_of(e);
    });
    __syncthreads();
    const float thr = ord_inv(thr_max);   // every discarded token has an approximate key above this
    int P = 4;   // the sort takes four elements per thread
    while (P < count) P <<= 1;
    for (int c = tid; c < P; c += TNT) {
        if (c < count) {
            sh.key[lds_slot(c)] = exact_key<CT>(cb, d, i, sh.idx[lds_slot(c)], metric, vec4);
        } else {
            sh.key[lds_slot(c)] = INFINITY;
            sh.idx[lds_slot(c)] = INT_MAX;
        }
    }
    // ascending by (key, idx)
    struct Cand {
        double key;
        int idx;
    };
    bitonic_sort_lds<TNT, Cand>(
        P, tid, [&](int p) { return Cand{sh.key[p], sh.idx[p]}; },
        [&](int p, const Cand& c) { sh.key[p] = c.key; sh.idx[p] = c.idx; },
        [](const Cand& a, const Cand& b) { return (a.key > b.key) | ((a.key == b.key) & (a.idx > b.idx)); },
        [](bool sw, const Cand& a, const Cand& b) { return Cand{sw ? b.key : a.key, sw ? b.idx : a.idx}; });
    // proof that no discarded token belongs to the row: every discarded j has an
    // approximate key above thr, hence an exact key above thr - err; the last
    // token taken must lie at or below that.
    bool ok = true;
    if (LIST || count < V - 1) {
        const double last = sh.key[lds_slot(need - 1)];
        double eabs = (double)err_abs;
        if (norms) {
            // Squared l2: the error of a key grows with the norms of its two codes, and the bound needs the
            // largest norm a discarded token can have.  A token with norm n_j > 4 (n_i + last) is further
            // away than the last one taken whatever its approximate key says, since |c_i - c_j|^2 >=
            // (sqrt n_j - sqrt n_i)^2 > (2 sqrt(n_i + last) - sqrt n_i)^2 >= last; so only norms up to that
            // (taken a thousandth larger, for the rounding of the fp32 norms) have to be covered.  A few
            // codes of very large norm then no longer send every row to the all-pairs pass.
            const double ni = (double)norms[i];
            const double far = 4.004 * (ni + last);
            const double nbound = far < (double)*nmax ? far : (double)*nmax;   // far may be inf or NaN: then the maximum
            eabs += (double)err_norm * (ni + nbound);
        }
        const double num = (double)thr - eabs;
        const double floor_discarded = num - 1.01 * (double)err_rel * fabs(num);
        ok = count >= need && last <= floor_discarded;
    }
    if (!ok) {
        if (tid == 0) flags[row] = 1;
        return;
    }
    for (int s = tid; s < need; s += TNT) orow[1 + s] = sh.idx[lds_slot(s)];
}

// ---- stage 3: flagged rows, all V keys in fp64, rank by counting ----
template <typename CT>
__global__ __launch_bounds__(NT) void knn_exact_rows(const CT* cb, int V, int d, int k, int metric,
                                                     const int* flags, double* bufs, int32_t* out, int* stats) {
    const int tid = threadIdx.x;
    double* buf = bufs + (int64_t)blockIdx.x * V;
    const int need = k - 1;
    // the workgroup's rows are blockIdx.x, blockIdx.x + gridDim.x, ...: all their flags are looked at
    // at once first, and a workgroup with none set is done
    int any = 0;
    for (int row = blockIdx.x + tid * gridDim.x; row < V; row += NT * gridDim.x) any |= flags[row];
    if (!__syncthreads_or(any)) return;
    for (int i = blockIdx.x; i < V; i += gridDim.x) {
        if (!flags[i]) continue;  // uniform
        if (tid == 0) atomicAdd(stats, 1);
        __syncthreads();
        for (int j = tid; j < V; j += NT)
            buf[j] = (j == i) ? NAN : exact_key<CT>(cb, d, i, j, metric, false);   // NaN: counted by no comparison below
        __threadfence_block();
        __syncthreads();
        int32_t* orow = out + (int64_t)i * k;
        for (int j = tid; j < V; j += NT) {
            if (j == i) continue;
            const double kj = buf[j];
            int rank = 0;
            for (int o = 0; o < V; ++o) {
                const double ko = buf[o];
                rank += (ko < kj || (ko == kj && o < j)) ? 1 : 0;
            }
            if (rank < need) orow[1 + rank] = j;
        }
    }
}

__global__ void knn_clear_stats(int* stats, float* nmax) {
    stats[threadIdx.x] = 0;
    if (threadIdx.x == 0) *nmax = 0.f;
}
__global__ void knn_copy_stats(const int* stats, int32_t* out) { *out = stats[0]; }

template <int NS>
static void launch_sample_rank(const float* skeys, const FilterPlan& plan, int rows, float* thr, int* counts,
                               hipStream_t stream) {
    hipLaunchKernelGGL((knn_sample_rank<NS>), dim3((rows + NW - 1) / NW), dim3(NT), 0, stream, skeys, plan.S, rows,
                       plan.rank, plan.slack, thr, counts);
}

template <typename CT>
static hipError_t build_typed(const KnnArgs& a, const KnnLayout& L, hipStream_t stream) {
    unsigned char* ws = static_cast<unsigned char*>(a.workspace);
    float* dist = reinterpret_cast<float*>(ws + L.dist);
    int* flags = reinterpret_cast<int*>(ws + L.flags);
    double* slow = reinterpret_cast<double*>(ws + L.slow);
    const CT* cb = static_cast<const CT*>(a.codebook);
    int* stats = reinterpret_cast<int*>(ws + L.stats);
    float* norms = reinterpret_cast<float*>(ws + L.norms);
    float* nmax = reinterpret_cast<float*>(ws + L.nmax);
    hipLaunchKernelGGL(knn_clear_stats, dim3(1), dim3(64), 0, stream, stats, nmax);
    // matrix-core path: rows 16-byte aligned and coordinates in whole vectors
    const bool aligned = (reinterpret_cast<uintptr_t>(a.codebook) & 15) == 0;
    const bool mfma = aligned && (sizeof(CT) == 2 ? (a.d % 8) == 0 : (a.d % 4) == 0) && a.V >= 32;
    const FilterPlan& plan = L.filter;   // the caller lays the filtering path out only for an aligned codebook
    // one rounding is at most 2^-23 relative here (twice the fp32 unit, to cover a
    // contraction that truncates); a d-term sum takes d + 8 of them
    const float gamma = (float)(a.d + 8) * 1.1920929e-7f;
    float err_rel, err_abs, err_norm;
    if (mfma) {
        const int per_wg = a.d * (int)sizeof(CT) / 16 >= NORM_WAVE_VECS ? NORM_ROWS : NT;
        hipLaunchKernelGGL((knn_norms<CT>), dim3((a.V + per_wg - 1) / per_wg), dim3(NT), 0, stream, cb, a.V, a.d, norms,
                           nmax);
        // n_i + n_j - 2 G: errors of the two norms and of G are each below gamma (n_i + n_j) / 2 ... gamma (n_i + n_j)
        err_rel = 0.f;
        err_abs = a.metric == 0 ? 0.f : 4.f * gamma;
        err_norm = a.metric == 0 ? 2.f * gamma : 0.f;
    } else {
        // direct evaluation: relative to the key for squared l2 (a sum of squares);
        // absolute, against |cos| <= 1, for the cosine key
        err_rel = a.metric == 0 ? gamma : 0.f;
        err_abs = a.metric == 0 ? 0.f : 2.f * gamma;
        err_norm = 0.f;
    }
    CT* scb = reinterpret_cast<CT*>(ws + L.scb);
    float* snorms = reinterpret_cast<float*>(ws + L.snorms);
    float* skeys = reinterpret_cast<float*>(ws + L.skeys);
    FilterOut fo;
    fo.thr = reinterpret_cast<float*>(ws + L.thr);
    fo.counts = reinterpret_cast<int*>(ws + L.counts);
    fo.cand = reinterpret_cast<uint2*>(ws + L.cand);
    fo.cap = plan.cap;
    const FilterOut no_list = {nullptr, nullptr, nullptr, 0};
    if (plan.use) {
        if (!mfma) return hipErrorInvalidValue;
        const int64_t elems = (int64_t)plan.S * a.d;
        hipLaunchKernelGGL((knn_gather_sample<CT>), dim3((unsigned)((elems + NT - 1) / NT)), dim3(NT), 0, stream, cb,
                           norms, a.V, a.d, plan.S, scb, snorms);
    }
    // all keys of rows [r0, r0 + rows) against the tokens of cbB
    auto contract = [&](const CT* cbB, const float* nb, int VB, int r0, int rows, float* keys) {
        hipLaunchKernelGGL((knn_dist_mfma<CT>), dim3((VB + 127) / 128, (rows + 127) / 128), dim3(NT), 0, stream, cb,
                           cbB, norms, nb, a.V, VB, a.d, r0, rows, a.metric, keys);
    };
    auto filter = [&](int r0, int rows) {
        const int nct = (a.V + 127) / 128, nrt = (rows + 127) / 128;
        const dim3 grid((unsigned)((nrt + 7) / 8 * 8 * nct));
        if (a.metric == 0)
            hipLaunchKernelGGL((knn_filter_mfma<CT, 0>), grid, dim3(NT), 0, stream, cb, norms, a.V, a.d, r0, rows, fo);
        else
            hipLaunchKernelGGL((knn_filter_mfma<CT, 1>), grid, dim3(NT), 0, stream, cb, norms, a.V, a.d, r0, rows, fo);
    };
    for (int r0 = 0; r0 < a.V; r0 += L.row_block) {
        const int rows = (a.V - r0) < L.row_block ? (a.V - r0) : L.row_block;
        const float* nsel = mfma && a.metric == 0 ? norms : nullptr;
        // candidate capacity: the smallest of 256 / 1024 / 2048 / 4096 slots that holds k-1+pad.  The
        // selection is bound by the latency of its many short phases, so its throughput is the number
        // of workgroups a compute unit holds at once, and that number is set by this LDS footprint
        // (12 bytes a slot).
        const int want_slots = (a.k - 1) + 8 + (a.k - 1) / 128;
#define LANTERN_LAUNCH_SELECT(NKV, CAPV, TNTV, LISTV)                                                       \
        hipLaunchKernelGGL((knn_select<CT, NKV, CAPV, TNTV, LISTV>), dim3(rows), dim3(TNTV), 0, stream, cb, \
                           a.V, a.d, a.k, a.metric, r0, dist, LISTV ? fo : no_list, err_rel, err_abs,       \
                           err_norm, nsel, nmax, a.out, flags + r0)
        if (plan.use) {
            // thresholds from the sample, then the contraction that keeps what lies below them
            contract(scb, snorms, plan.S, r0, rows, skeys);
            if (plan.S <= 8 * WAVE) launch_sample_rank<8>(skeys, plan, rows, const_cast<float*>(fo.thr), fo.counts, stream);
            else if (plan.S <= 16 * WAVE) launch_sample_rank<16>(skeys, plan, rows, const_cast<float*>(fo.thr), fo.counts, stream);
            else if (plan.S <= 32 * WAVE) launch_sample_rank<32>(skeys, plan, rows, const_cast<float*>(fo.thr), fo.counts, stream);
            else launch_sample_rank<64>(skeys, plan, rows, const_cast<float*>(fo.thr), fo.counts, stream);
            filter(r0, rows);
            // a list of cap slots on 256 threads: cap / 256 pairs per thread; 64 < want_slots <= 1024
            if (want_slots <= 256) {
                if (plan.cap <= 4 * NT) LANTERN_LAUNCH_SELECT(4, 256, NT, true);
                else LANTERN_LAUNCH_SELECT(8, 256, NT, true);
            } else if (plan.cap <= 8 * NT) LANTERN_LAUNCH_SELECT(8, 1024, NT, true);
            else if (plan.cap <= 12 * NT) LANTERN_LAUNCH_SELECT(12, 1024, NT, true);
            else LANTERN_LAUNCH_SELECT(16, 1024, NT, true);
        } else {
            if (mfma) contract(cb, norms, a.V, r0, rows, dist);
            else
                hipLaunchKernelGGL((knn_dist_direct<CT>), dim3((a.V + NT - 1) / NT, rows), dim3(NT), 0, stream,
                                   cb, a.V, a.d, r0, a.metric, dist);
#define LANTERN_LAUNCH_SELECT_NK(NKV, TNTV)                                                                 \
            do {                                                                                            \
                if (want_slots <= 256) LANTERN_LAUNCH_SELECT(NKV, 256, TNTV, false);                        \
                else if (want_slots <= 1024) LANTERN_LAUNCH_SELECT(NKV, 1024, TNTV, false);                 \
                else if (want_slots <= 2048) LANTERN_LAUNCH_SELECT(NKV, 2048, TNTV, false);                 \
                else LANTERN_LAUNCH_SELECT(NKV, CAND_CAP, TNTV, false);                                     \
            } while (0)
            // threads per row and keys per thread: up to 64 keys per thread in registers; vocabularies
            // beyond 64 x 256 tokens take 512 threads per row (32 keys per thread on 512 threads measured
            // the same as 64 on 256 at V = 16384); beyond 64 x 512 the keys are re-read in every pass
            if (a.V <= 8 * NT) LANTERN_LAUNCH_SELECT_NK(8, NT);
            else if (a.V <= 32 * NT) LANTERN_LAUNCH_SELECT_NK(32, NT);
            else if (a.V <= 64 * NT) LANTERN_LAUNCH_SELECT_NK(64, NT);
            else if (a.V <= 64 * 512) LANTERN_LAUNCH_SELECT_NK(64, 512);
            else LANTERN_LAUNCH_SELECT_NK(0, NT);
#undef LANTERN_LAUNCH_SELECT_NK
        }
#undef LANTERN_LAUNCH_SELECT
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // flagged rows of the whole table
    const int wgs = a.V < L.slow_wgs ? a.V : L.slow_wgs;
    hipLaunchKernelGGL((knn_exact_rows<CT>), dim3(wgs), dim3(NT), 0, stream, cb, a.V, a.d, a.k, a.metric, flags,
                       slow, a.out, stats);
    return hipGetLastError();
}

hipError_t launch_build_knn(const KnnArgs& a, hipStream_t stream) {
    // The workspace has the size of the shape's own layout.  A codebook that is not 16-byte aligned
    // cannot take the filtering path: it gets whole key blocks of as many rows as that size holds.
    FilterPlan plan = filter_plan(a.V, a.d, a.k, a.cb_dtype);
    KnnLayout L = knn_layout(a.V, a.d, a.cb_dtype, plan, plan.use ? FILTER_ROW_BLOCK : whole_row_block(a.V), SLOW_WGS);
    if (plan.use && (reinterpret_cast<uintptr_t>(a.codebook) & 15) != 0) {
        L = knn_layout_within(a.V, a.d, a.cb_dtype, NO_FILTER, SLOW_WGS, L.total);
        if (L.row_block == 0) return hipErrorInvalidValue;
    }
    if (a.cb_dtype == 0) return build_typed<float>(a, L, stream);
    return build_typed<uint16_t>(a, L, stream);
}

// The same build with the library's static scratch as workspace; a.workspace is ignored.
// exact_rows: device int32 that receives the number of rows ranked by the all-pairs pass, or null.
hipError_t launch_build_knn_static(const KnnArgs& a_in, int32_t* exact_rows, hipStream_t stream) {
    const KnnLayout L = knn_layout_static(a_in.V, a_in.d, a_in.cb_dtype);
    if (L.row_block == 0) return hipErrorInvalidValue;   // the host entry has checked this
    KnnArgs a = a_in;
    hipError_t e = static_scratch_ptr(&a.workspace);
    if (e != hipSuccess) return e;
    e = a.cb_dtype == 0 ? build_typed<float>(a, L, stream) : build_typed<uint16_t>(a, L, stream);
    if (e != hipSuccess) return e;
    if (exact_rows) {
        hipLaunchKernelGGL(knn_copy_stats, dim3(1), dim3(1), 0, stream,
                           reinterpret_cast<const int*>(static_cast<unsigned char*>(a.workspace) + L.stats), exact_rows);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace lantern
