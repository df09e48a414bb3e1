// Relaxed-acceptance verification (Section 4.3; Algorithm 2, inference part;
// Algorithm 1, accept / resample branch) for gfx950.
//
// One workgroup per row, two code paths inside the same launch:
//   fast path   fp32.  Streams the target and draft rows from HBM once with
//               16-byte loads, keeps the raw target row in LDS, gathers the
//               draft token's k neighbours from LDS, prefix-scans them and
//               takes the TVD cut and the acceptance test.  Each comparison
//               carries a rounding margin; a row is settled here only when
//               every comparison it took cleared its margin and it is accepted
//               (or, when only decisions are asked for, definitely rejected).
//   exact path  fp64.  The workgroup of a row the fast path did not settle
//               (ambiguous comparison, unusable input, a rejected row whose
//               resampled token is wanted) re-evaluates it: same rule, then
//               the residual and its inverse CDF.
// Shapes the fast path does not cover (rows not 16-byte aligned, V not a
// multiple of the vector width, rows beyond the register budget) run the
// exact path for every row (kernel verify_exact).
// Three modes (verify_args.h): decisions and resampled tokens; decisions only;
// the fp64 path for selected verifications in 512-thread workgroups
// (resample_selected, and tree_finish, which first walks its draft tree).
// Letters: t = target probability (the paper's q), g = drafter probability
// (the paper's p), xt = draft token.
#include <hip/hip_runtime.h>
#include <limits.h>
#include <stddef.h>
#include <math.h>
#include <stdint.h>

#include "exp_table.h"
#include "fast_cut.h"
#include "lds_limit.h"
#include "tree_walk.h"
#include "verify_args.h"
#include "verify_common.h"

namespace lantern {

// LDS layout of verify_fast after the raw row
struct FastShared {
    float wmax_t[NW], wmax_g[NW];   // per-wave maxima over the sampled part of the row
    float wsum_t[NW], wsum_g[NW];   // per-wave sums of exponentials
    float wtot[NW];                 // per-wave totals of the neighbour terms (first 1024 slots)
    int wbad[NW];                   // a table entry outside [0,V)
    int cut_np[NW];                 // per wavefront: first slot not definitely inside the bound,
    int cut_df[NW];                 //   first slot definitely outside it,
    float cut_s[NW];                //   sum before the former
    int tail[4];                    // k > 1024: the result of the walk beyond slot 1024 (a_size, S, definite, bad)
    // from here on the memory is reused by the exact path once the fp32 decision is taken
    float gs[NT * 4];               // inclusive sums of the neighbour terms within their wavefront
    unsigned gskip[NT];             // bit q: slot 4*tid+q is the token itself or beyond k
};
constexpr size_t FAST_SHARED_HEAD = offsetof(FastShared, gs);
constexpr size_t FAST_SHARED_TAIL = sizeof(FastShared) - FAST_SHARED_HEAD;
static_assert(FAST_SHARED_HEAD % 16 == 0, "the exact path's LDS region must be 16-byte aligned");

template <typename LT, bool VEC, int TNT = NT>
__device__ void exact_row(const VerifyArgs& a, int row, unsigned char* ex, const unsigned char* lds_row,
                          bool have_max, float max_t, float max_g, const unsigned char* lds_grow = nullptr);

// ---------------------------------------------------------------------------
// fp64 evaluation of a row in one pass, with what the fp32 pass already knows
// ---------------------------------------------------------------------------
// For a row the fp32 pass could not settle but found usable, with both sums in range and a
// definite cut: the decision and, on rejection, the resampled token, in fp64, in ONE pass over the
// two rows (2V exponentials instead of the 4V of the general path, no pass for the maxima).
// What makes one pass enough: the residual max(0, t_A - g) needs, token by token, the SIGN of
// t_A(x) - g(x), and the fp32 terms and sums decide that sign for all but the few tokens where
// the two probabilities agree to within the fp32 error bound.  So while the pass adds up the
// fp64 normalisers it also adds, per (vector chunk, wavefront) segment and in token order, the
// target and drafter terms of the tokens whose residual is certainly positive; tokens whose sign
// fp32 cannot tell go on a short list with their fp64 terms.  Once the normalisers are known a
// segment's residual mass is  P_t / Z_t - P_g / Z_g  plus its listed tokens, a scan over the
// (at most 64) segment masses finds the segment that holds the draw, and that segment alone is
// re-evaluated token by token.
// No global load sits inside the pass (under a saturated memory system each costs microseconds):
// the drafter's row is fetched again, all of it at once, before the pass starts (keeping it in
// registers from the fp32 pass on would cost that pass registers it does not have), the target row
// is in LDS, the first 1024 table slots in registers.
constexpr int AMB_CAP = 40;          // tokens whose residual sign fp32 leaves open (about one per row)
constexpr double TAU_SIGN = 2.0e-5;  // covers the error of ln(Z_t32 / Z_g32) in the sign test (<= 8.8e-6)

struct AmbEntry {
    double et, eg;   // unnormalised fp64 terms
    int x;           // token
    int pad;
};

// LDS of this path, in the region the neighbour scan no longer needs.
struct OnePassLayout {
    size_t mask, seg, amb_count, amb, total;
};
// The exponential's table sits at the very start of the workgroup's LDS (before the row): the
// address of a lookup is then the masked integer itself, with no base to add.
constexpr int EXP_TABLE_BYTES = 2 * EXP_TABLE_N * (int)sizeof(double);
__host__ __device__ inline OnePassLayout one_pass_layout(int V) {
    OnePassLayout L;
    size_t off = (sizeof(ExactShared) + 15) & ~size_t(15);
    L.mask = off;      off += (((size_t)V + 31) / 32) * 4;  off = (off + 15) & ~size_t(15);
    L.seg = off;       off += 16 * NW * 2 * sizeof(double);           // up to 16 vector chunks per thread
    L.amb = off;       off += AMB_CAP * sizeof(AmbEntry);
    L.amb_count = off; off += 16;
    L.total = off;
    return L;
}

// One residual term of the token-by-token evaluation: max(0, t_A(x) - g(x)), zero on A and at xt
// (the token's own residual is zero in a rejected row: u g >= mass with u < 1).
__device__ __forceinline__ double one_pass_term(float lt, float lg, bool zero, double rt, double rg, double inv_zt,
                                                double inv_zg, const double* tab) {
    const double d = exp_tab((double)lt - rt, tab) * inv_zt - exp_tab((double)lg - rg, tab) * inv_zg;
    return (!zero && d > 0.0) ? d : 0.0;
}

// What the pass does for one token: its fp64 terms into the normalisers; into the segment's sums
// when the residual is certainly positive; onto the list when that cannot be told.
// The sign test works on the exponents: t(x) > g(x) <=> (l_t - r_t) - (l_g - r_g) > ln(Z_t / Z_g),
// where only the two fp32 sums on the right carry an error (at most 4.4e-6 relative each: terms
// 2.5e-6, tree sums 1.9e-6, i.e. 8.8e-6 on the logarithm), so a margin of TAU_SIGN = 2e-5 on either
// side of ln(Z_t32 / Z_g32) makes "positive" and "not positive" certain.  floor_t, floor_g: the row's
// reference logit minus 700; logits below it (filtered tokens at -inf among them) are evaluated
// there: a term of 1e-304 of the sum either way.
// max of two floats as the one hardware instruction (fmaxf first quiets both operands, two more
// instructions per call; no NaN reaches this path).
__device__ __forceinline__ float max_f32_1(float a, float b) {
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

struct OnePassAcc {
    double zt, zg, pt, pg;
};
__device__ __forceinline__ void one_pass_token(OnePassAcc& acc, float lt, float lg, bool zero, int x, double rt,
                                               double rg, float floor_t, float floor_g, double ln_hi, double ln_lo,
                                               const unsigned char* tab, AmbEntry* amb, int* amb_count) {
    const double dt = (double)max_f32_1(lt, floor_t) - rt;
    const double dg = (double)max_f32_1(lg, floor_g) - rg;
    const double et = exp_tab_core(dt, tab);
    const double eg = exp_tab_core(dg, tab);
    acc.zt += et;
    acc.zg += eg;
    const double dd = dt - dg;                               // t(x) > g(x)  <=>  dd > ln(Z_t / Z_g)
    const bool pos = !zero && (dd > ln_hi);
    const bool neg = zero || (dd < ln_lo);
    const double m = pos ? 1.0 : 0.0;
    acc.pt = __builtin_fma(et, m, acc.pt);
    acc.pg = __builtin_fma(eg, m, acc.pg);
    if (!pos && !neg) {
        const int slot = atomicAdd(amb_count, 1);
        if (slot < AMB_CAP) {
            amb[slot].et = et;
            amb[slot].eg = eg;
            amb[slot].x = x;
        }
    }
}

// s_row: raw target row in LDS.
// nb: table slots 4*tid .. 4*tid+3.  ref_t, ref_g: the fp32 pass's reference logits; Zt32, Zg32:
// its sums; a_size: its (definite) cut.
// tab_lds: where the exponential's table goes in LDS.
template <typename LT, int NV, bool FULL>
__device__ __forceinline__ void exact_one_pass(const VerifyArgs& a, int row, int lrow,
                                               const int (&nb)[4], float ref_t, float ref_g,
                                               float Zt32, float Zg32, int a_size, int xt, float lg_tok, float u_acc32,
                                               unsigned char* tab_lds, unsigned char* ex,
                                               const unsigned char* s_row) {
    using L = Lane<LT>;
    constexpr int EPV = L::EPV;
    constexpr int NSEG = NV * NW;                            // at most 64: one wavefront scans them
    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1);
    const int wave = tid >> 6;
    const int V = a.V;
    const int k = a.k;
    const int nvec = V / EPV;
    const OnePassLayout lay = one_pass_layout(V);
    ExactShared& sh = *reinterpret_cast<ExactShared*>(ex);
    uint32_t* mask = reinterpret_cast<uint32_t*>(ex + lay.mask);
    double* seg = reinterpret_cast<double*>(ex + lay.seg);
    double* tab = reinterpret_cast<double*>(tab_lds);
    AmbEntry* amb = reinterpret_cast<AmbEntry*>(ex + lay.amb);
    int* amb_count = reinterpret_cast<int*>(ex + lay.amb_count);
    const int nwords = (V + 31) >> 5;
    const double rt = (double)ref_t, rg = (double)ref_g;
    const float u_res32 = a.uniforms[2 * (int64_t)row + 1];  // in flight during the pass
    // the drafter's row, every load issued now; it arrives while the table and the mask are set up
    const uint4* gsrc = reinterpret_cast<const uint4*>(reinterpret_cast<const LT*>(a.draft) + (int64_t)lrow * a.stride);
    uint4 G[NV];
#pragma unroll
    for (int c = 0; c < NV; ++c) {
        const int vi = c * NT + tid;
        G[c] = (FULL || vi < nvec) ? gsrc[vi]
                                   : make_uint4(L::NEG_INF_WORD, L::NEG_INF_WORD, L::NEG_INF_WORD, L::NEG_INF_WORD);
    }

    // ---- table of the exponential, empty mask, empty list ----
    tab[tid] = EXP_TABLE_HILO[tid];                          // 2 * 128 doubles, one per thread (cache-resident)
    for (int w = tid; w < nwords; w += NT) mask[w] = 0u;
    if (tid == 0) *amb_count = 0;
    __syncthreads();

    // ---- A as a bitmask, and its mass (unnormalised) ----
    double s_loc = 0.0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int n = nb[q];                                 // in range: the fp32 pass has checked all k entries
        if (tid * 4 + q < a_size && n != xt) {
            s_loc += exp_tab((double)L::lds(s_row, n) - rt, tab);
            atomicOr(&mask[n >> 5], 1u << (n & 31));
        }
    }
    if (a_size > NT * 4) {
        const int32_t* nrow = a.knn + (int64_t)xt * k;
        for (int j = NT * 4 + tid; j < a_size; j += NT) {
            const int n = nrow[j];
            if (n != xt) {
                s_loc += exp_tab((double)L::lds(s_row, n) - rt, tab);
                atomicOr(&mask[n >> 5], 1u << (n & 31));
            }
        }
    }
    const double S = block_sum<NW>(s_loc, sh.red, tid);      // its barriers also publish the mask
    const double e_tx = exp_tab((double)L::lds(s_row, xt) - rt, tab);
    const double e_gx = exp_tab((double)lg_tok - rg, tab);

    // ---- the pass: normalisers, and per segment the terms of the certainly positive residuals ----
    // Rolled loops with the vectors shifted down by one chunk / two elements per turn, so that
    // registers are indexed statically and the code stays small.
    OnePassAcc acc;
    acc.zt = 0.0;
    acc.zg = 0.0;
    const float floor_t = ref_t - 700.f, floor_g = ref_g - 700.f;
    // ln(Z_t / Z_g) from the fp32 sums (both finite and at least one).  Their terms are
    // 2^(l * LOG2E_F - c) with c = ref * LOG2E_F rounded to fp32, the fp64 terms here e^(l - ref): per
    // term the two differ by (l - ref) (LOG2E_F - log2 e), which the term's error bound holds, and by
    // the rounding of c, common to the row and known exactly (the product of two floats is exact in
    // fp64): that one is put back.
    const double LN2_D = 0.69314718055994530942;
    const double adj_t = ((double)(ref_t * LOG2E_F) - rt * (double)LOG2E_F) * LN2_D;
    const double adj_g = ((double)(ref_g * LOG2E_F) - rg * (double)LOG2E_F) * LN2_D;
    const double ln_z = log((double)Zt32 / (double)Zg32) + adj_t - adj_g;
    const double ln_hi = ln_z + TAU_SIGN, ln_lo = ln_z - TAU_SIGN;
#pragma unroll 1
    for (int c = 0; c < NV; ++c) {
        uint4 gv = G[0];
#pragma unroll
        for (int i = 0; i + 1 < NV; ++i) G[i] = G[i + 1];
        const int vi = c * NT + tid;
        const bool live = FULL || vi < nvec;
        uint4 tv = live ? reinterpret_cast<const uint4*>(s_row)[vi]
                        : make_uint4(L::NEG_INF_WORD, L::NEG_INF_WORD, L::NEG_INF_WORD, L::NEG_INF_WORD);
        const int x0 = vi * EPV;
        unsigned in_a = live ? (mask[x0 >> 5] >> (x0 & 31)) & ((1u << EPV) - 1u) : 0u;   // EPV divides 32
        acc.pt = 0.0;
        acc.pg = 0.0;
#pragma unroll 1
        for (int e = 0; e < EPV; e += 2) {
            const float lt0 = L::get(tv, 0), lt1 = L::get(tv, 1), lg0 = L::get(gv, 0), lg1 = L::get(gv, 1);
            // t_A is zero on A without the token, the token's own residual is zero in a rejected row,
            // and a filtered target token has t = 0
            const bool zero0 = (in_a & 1u) || (x0 + e == xt) || lt0 == neg_inf_f();
            const bool zero1 = (in_a & 2u) || (x0 + e + 1 == xt) || lt1 == neg_inf_f();
            one_pass_token(acc, lt0, lg0, zero0, x0 + e, rt, rg, floor_t, floor_g, ln_hi, ln_lo, tab_lds, amb, amb_count);
            one_pass_token(acc, lt1, lg1, zero1, x0 + e + 1, rt, rg, floor_t, floor_g, ln_hi, ln_lo, tab_lds, amb, amb_count);
            tv = L::drop2(tv);
            gv = L::drop2(gv);
            in_a >>= 2;
        }
        const double pt = wave_sum_dpp(acc.pt);
        const double pg = wave_sum_dpp(acc.pg);
        if (lane == 0) {
            seg[2 * (c * NW + wave)] = pt;
            seg[2 * (c * NW + wave) + 1] = pg;
        }
    }
    const double zt = block_sum<NW>(acc.zt, sh.red, tid);
    const double zg = block_sum<NW>(acc.zg, sh.red2, tid);  // its barriers publish seg and the list

    // ---- decision ----
    const double mass = (e_tx + S) / zt;
    const double g_tok = e_gx / zg;
    const bool accepted = ((double)u_acc32 * g_tok < mass);
    if (tid == 0) {
        double ap;
        if (g_tok > 0.0) ap = fmin(1.0, mass / g_tok);
        else ap = mass > 0.0 ? 1.0 : 0.0;
        if (a.out_prob) a.out_prob[row] = (float)ap;
        if (a.out_mass) a.out_mass[row] = (float)mass;
        if (a.out_gtok) a.out_gtok[row] = (float)g_tok;
        if (a.out_asize) a.out_asize[row] = a_size;
        if (a.out_path) a.out_path[row] = 1;
        if (accepted) {
            a.out_accept[row] = 1;
            a.out_resample[row] = -1;
        }
    }
    if (accepted) return;

    // ---- rejected: residual mass per segment (segments in token order), the one that holds the draw ----
    const int n_amb = *amb_count;
    const double inv_zt = 1.0 / zt, inv_zg = 1.0 / zg;
    if (wave == 0) {
        double r = 0.0;
        if (lane < NSEG) {
            r = seg[2 * lane] * inv_zt - seg[2 * lane + 1] * inv_zg;
            r = r > 0.0 ? r : 0.0;
            for (int i = 0; i < n_amb && i < AMB_CAP; ++i) {
                const int v = amb[i].x / EPV;               // vector of the token: chunk v / NT, thread v % NT
                if ((v / NT) * NW + ((v % NT) >> 6) == lane) {
                    const double d = amb[i].et * inv_zt - amb[i].eg * inv_zg;
                    r += d > 0.0 ? d : 0.0;
                }
            }
        }
        const double incl = wave_scan_incl(r);
        const double Z = __shfl(incl, WAVE - 1, WAVE);
        const double cthr = (double)u_res32 * Z;
        const unsigned long long cross = __ballot(lane < NSEG && incl > cthr);
        const unsigned long long has = __ballot(r > 0.0);
        // rounding can leave no crossing: the last segment that holds mass takes the draw
        const int s = cross ? (__ffsll((long long)cross) - 1) : (has ? 63 - __clzll((long long)has) : 0);
        const double before = s ? __shfl(incl, s - 1, WAVE) : 0.0;
        if (lane == 0) {
            sh.bcast[0] = before;
            sh.bcast[1] = cthr;
            sh.bcast[2] = Z;
            sh.ibcast[0] = s;
        }
    }
    __syncthreads();
    // a list that overflowed, or a residual without mass (by rounding): the general path
    // (uniform over the workgroup)
    if (n_amb > AMB_CAP || !(sh.bcast[2] > 0.0)) {
        __syncthreads();
        exact_row<LT, true>(a, row, ex, s_row, false, 0.f, 0.f);
        return;
    }
    const int ent = sh.ibcast[0];
    if (wave == (ent % NW)) {
        const double P = sh.bcast[0], cthr = sh.bcast[1];
        const int vi = (ent / NW) * NT + tid;
        const int x0 = vi * EPV;
        const bool live = FULL || vi < nvec;
        const uint4 ninf = make_uint4(L::NEG_INF_WORD, L::NEG_INF_WORD, L::NEG_INF_WORD, L::NEG_INF_WORD);
        const uint4 gv = live ? gsrc[vi] : ninf;             // this segment of the drafter's row, once more
        const uint4 tv = live ? reinterpret_cast<const uint4*>(s_row)[vi] : ninf;
        const unsigned in_a = live ? (mask[x0 >> 5] >> (x0 & 31)) & ((1u << EPV) - 1u) : 0u;
        double r[EPV];
        double sum = 0.0;
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            r[e] = one_pass_term(L::get(tv, e), L::get(gv, e), ((in_a >> e) & 1u) || (x0 + e == xt), rt, rg, inv_zt,
                                 inv_zg, tab);
            sum += r[e];
        }
        const double incl = wave_scan_incl(sum);
        double excl = __shfl_up(incl, 1, WAVE);
        if (lane == 0) excl = 0.0;
        const unsigned long long cross = __ballot(P + incl > cthr);
        const unsigned long long haspos = __ballot(sum > 0.0);
        // rounding between the segment's mass and its token-by-token evaluation can leave no
        // crossing lane: then the last lane that holds mass takes the draw
        const int owner = cross ? (__ffsll((long long)cross) - 1) : (haspos ? 63 - __clzll((long long)haspos) : 0);
        int found = -1;
        if (lane == owner) {
            double cum = P + excl;
            int lastpos = -1;
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                cum += r[e];
                if (r[e] > 0.0) lastpos = x0 + e;
                if (found < 0 && cum > cthr && r[e] > 0.0) found = x0 + e;
            }
            if (found < 0) found = lastpos;
        }
        found = __shfl(found, owner, WAVE);
        if (found < 0) {
            // no token of the segment holds mass: its mass was rounding noise of the sums (it takes a
            // draw within ~1e-16 of a segment edge).  The first token after it that holds mass is
            // the one the cumulative sum reaches next; failing that, the last one before it.
            const int seg_x0 = ((ent / NW) * NT + (ent % NW) * WAVE) * EPV;   // first token of the segment
            int before = -1, after = INT_MAX;
            for (int v0 = 0; v0 < nvec; v0 += WAVE) {
                const int v = v0 + lane;
                const bool lv = v < nvec;
                const uint4 gq = lv ? gsrc[v] : ninf;
                const uint4 tq = lv ? reinterpret_cast<const uint4*>(s_row)[v] : ninf;
                const unsigned ia = lv ? (mask[(v * EPV) >> 5] >> ((v * EPV) & 31)) & ((1u << EPV) - 1u) : 0u;
                int first = INT_MAX, last = -1;
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    const int x = v * EPV + e;
                    const bool has = one_pass_term(L::get(tq, e), L::get(gq, e), ((ia >> e) & 1u) || x == xt, rt, rg,
                                                   inv_zt, inv_zg, tab) > 0.0;
                    if (has && x >= seg_x0 && x < first) first = x;
                    if (has && x < seg_x0) last = x;
                }
                after = min(after, wave_min(first));
                before = max(before, -wave_min(-last));
            }
            found = after != INT_MAX ? after : before;
        }
        if (lane == 0) {
            a.out_accept[row] = 0;
            a.out_resample[row] = found;
        }
    }
}

// Per-row scalars and table slots, fetched together with the row.
struct RowMeta {
    int xt;        // draft token
    float u_acc;   // acceptance draw
    float lg_tok;  // draft logit of the token
    int nb[4];     // table slots 4*tid .. 4*tid+3 (unspecified where the slot is beyond k)
};

// fp32 path, one workgroup per row.
// FULL: the row fills all NV vector slots of every thread (no bounds checks).
// VT: the token's table row can be read with 16-byte loads (k a multiple of four, table 16-byte
// aligned); the other case is a kernel of its own because a load that only one of two paths
// issues makes the hardware wait counters, which are placed statically, wait for every load.
//
// Exponentials are taken as 2^(l*log2e - c) with one reference c per row, common to all
// terms of that row, so its own rounding cancels in every comparison.  The reference is
// the maximum over the first vector slot of every thread (an eighth of the row at NV = 8)
// rather than the row maximum: any element of the row works, because the sum then holds
// a term equal to one (Z >= 1) and every term is at most Z; rows whose sum exceeds 2^46
// (an element more than 32 above the reference) are left to the exact path.
template <typename LT, int NV, bool FULL, bool VT>
__global__ __launch_bounds__(NT, (NV <= 8 ? 4 : 2)) void verify_fast(VerifyArgs a) {
    using L = Lane<LT>;
    constexpr int EPV = L::EPV;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* s_row = smem + EXP_TABLE_BYTES;           // the fp64 path's table goes in front
    const int row_bytes = (a.V * (int)sizeof(LT) + 15) & ~15;
    FastShared& sh = *reinterpret_cast<FastShared*>(s_row + row_bytes);
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

    // ---- loads, in the order their results are needed to issue further loads ----
    // Vector loads return in order.  The token comes first: the address of its table row depends on
    // it, and that second, dependent load should be in flight together with the streamed rows, not
    // start after the last of them has arrived.
    RowMeta m;
    m.xt = a.tokens[row];
    m.u_acc = a.uniforms[2 * (int64_t)row];
    // stream both rows: NV 16-byte loads per thread and row, coalesced
    uint4 T[NV], G[NV];
    {
        const uint4* tv = reinterpret_cast<const uint4*>(reinterpret_cast<const LT*>(a.target) + (int64_t)lrow * a.stride);
        const uint4* gv = reinterpret_cast<const uint4*>(reinterpret_cast<const LT*>(a.draft) + (int64_t)lrow * a.stride);
#pragma unroll
        for (int c = 0; c < NV; ++c) {
            const int vi = c * NT + tid;
            if (FULL || vi < nvec) {
                T[c] = load_stream16(tv + vi);
                G[c] = load_stream16(gv + vi);
            } else {
                T[c] = make_uint4(L::NEG_INF_WORD, L::NEG_INF_WORD, L::NEG_INF_WORD, L::NEG_INF_WORD);
                G[c] = T[c];
            }
        }
    }
    // the token's table slots 4*tid .. 4*tid+3 and its draft logit
    {
        const int xs0 = ((unsigned)m.xt < (unsigned)V) ? m.xt : 0;
        const int32_t* nrow = a.knn + (int64_t)xs0 * k;
        const int j0 = tid * 4;
        if (VT) {        // k a multiple of four, so a thread's four slots are all inside k or all beyond
            // loaded unconditionally from a clamped slot (no branch around the load, so nothing waits
            // for it here); what threads beyond k read is never looked at (every use checks the slot
            // number against k)
            const int4 q = *reinterpret_cast<const int4*>(nrow + min(j0, k - 4));
            m.nb[0] = q.x; m.nb[1] = q.y; m.nb[2] = q.z; m.nb[3] = q.w;
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) m.nb[q] = (j0 + q < k) ? nrow[j0 + q] : 0;
        }
        m.lg_tok = L::glob(reinterpret_cast<const LT*>(a.draft) + (int64_t)lrow * a.stride, xs0);
    }
    // every load of the row is issued before anything waits for one of them
    __builtin_amdgcn_sched_barrier(0);

    {
        const int xt = m.xt;
        const bool tok_ok = (unsigned)xt < (unsigned)V;
        const int xs = tok_ok ? xt : 0;

        // ---- raw target row to LDS; reference = maximum over vector slot 0 of every thread ----
#pragma unroll
        for (int c = 0; c < NV; ++c) {
            const int vi = c * NT + tid;
            if (FULL || vi < nvec) reinterpret_cast<uint4*>(s_row)[vi] = T[c];
        }
        float rt = neg_inf_f(), rg = neg_inf_f();
#pragma unroll
        for (int e = 0; e < EPV; e += 2) {
            rt = fmaxf(rt, fmaxf(L::get(T[0], e), L::get(T[0], e + 1)));
            rg = fmaxf(rg, fmaxf(L::get(G[0], e), L::get(G[0], e + 1)));
        }
        rt = wave_max(rt);
        rg = wave_max(rg);
        if (lane == 0) { sh.wmax_t[wave] = rt; sh.wmax_g[wave] = rg; }
        __syncthreads();  // the row is in LDS and the wave maxima are published
        rt = sh.wmax_t[0];
        rg = sh.wmax_g[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) {
            rt = fmaxf(rt, sh.wmax_t[w]);
            rg = fmaxf(rg, sh.wmax_g[w]);
        }
        // a sampled part without a finite logit: reference 0 (large rows then overflow and fall through)
        if (rt == neg_inf_f()) rt = 0.f;
        if (rg == neg_inf_f()) rg = 0.f;
        const float ct = rt * LOG2E_F;   // rounded once; common to every term of the row
        const float cg = rg * LOG2E_F;

        // ---- exponentials 2^(l*log2e - c), summed ----
        float st = 0.f, sg = 0.f;
#pragma unroll
        for (int c = 0; c < NV; ++c) {
            float et[EPV], eg[EPV];
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                et[e] = hw_exp2(__builtin_fmaf(L::get(T[c], e), LOG2E_F, -ct));
                eg[e] = hw_exp2(__builtin_fmaf(L::get(G[c], e), LOG2E_F, -cg));
            }
#pragma unroll
            for (int s = EPV / 2; s > 0; s >>= 1)
#pragma unroll
                for (int e = 0; e < s; ++e) {
                    et[e] += et[e + s];
                    eg[e] += eg[e + s];
                }
            st += et[0];
            sg += eg[0];
        }
        st = wave_sum(st);
        sg = wave_sum(sg);

        // ---- neighbour terms of slots 4*tid .. 4*tid+3, scanned within the wavefront ----
        const SlotTerms slots = slot_terms<LT>(m.nb, xt, k, V, a.knn + (int64_t)xs * k, s_row, ct, sh.wtot, sh.wbad);
        if (lane == 0) { sh.wsum_t[wave] = st; sh.wsum_g[wave] = sg; }
        __syncthreads();  // sums and wavefront totals of the neighbour terms are published

        // ---- every wavefront: the bound on its own slots ----
        float Zt = 0.f, Zg = 0.f, woff = 0.f, run_off = 0.f;
        int bad = (tok_ok && row_ok) ? 0 : 1;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            Zt += sh.wsum_t[w];
            Zg += sh.wsum_g[w];
            if (w < wave) woff += sh.wtot[w];
            run_off += sh.wtot[w];
            bad |= sh.wbad[w];
        }
        const float e_tx = hw_exp2(__builtin_fmaf(L::lds(s_row, xs), LOG2E_F, -ct));
        SlotTest test;
        {
            const float R = a.delta * Zt;             // divergence of the prefix, times Zt, < delta * Zt
            test.divergence = a.divergence;
            test.e_tx = e_tx;
            test.lo = R * (1.f - TAU_CUT) - ABS_SLACK;
            test.hi = R * (1.f + TAU_CUT) + ABS_SLACK;
        }
        classify_slots(slots, test, woff, WaveCut{sh.cut_np, sh.cut_df, sh.cut_s});
        __syncthreads();  // the wavefronts' results are published

        // ---- every thread: the cut, the mass, the acceptance test (same inputs, same result) ----
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
        if (first_np == INT_MAX && k > NT * 4) {      // uniform: the walk goes on beyond slot 1024
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
        const float e_gx = hw_exp2(__builtin_fmaf(m.lg_tok, LOG2E_F, -cg));
        const float MA = e_tx + S;                // mass * Zt
        const float lhs = m.u_acc * e_gx * Zt;    // u * g(xt) * Zt * Zg
        const float rhs = MA * Zg;                // mass  * Zt * Zg
        const float slack = acc_slack(k);
        const bool accept = (lhs + slack) < rhs * (1.f - TAU_ACC);
        // a definite rejection settles the row only when no resampled token is asked for
        const bool reject = (a.mode == VERIFY_DECIDE) && (lhs * (1.f - TAU_ACC) > rhs + slack);
        // sums in [1, 2^46]: every term is within 32 of the reference (NaN fails both tests)
        const bool sums_ok = (Zt >= 1.f) && (Zt <= Z_MAX) && (Zg >= 1.f) && (Zg <= Z_MAX);
        const bool settled = !bad && sums_ok && cut_definite && (accept || reject);
        if (__builtin_expect(settled, 1)) {
            if (tid == 0) {
                a.out_accept[row] = accept ? 1 : 0;
                if (a.mode == VERIFY_FULL) a.out_resample[row] = -1;
                const float mass = MA / Zt;
                const float gx = e_gx / Zg;
                if (a.out_prob) a.out_prob[row] = fminf(1.f, mass / gx);
                if (a.out_mass) a.out_mass[row] = mass;
                if (a.out_gtok) a.out_gtok[row] = gx;
                if (a.out_asize) a.out_asize[row] = a_size;
                if (a.out_path) a.out_path[row] = 0;
            }
        } else {
            // not settled in fp32: this workgroup evaluates the row in fp64; the raw target row stays in
            // LDS.  With the resampled token wanted, a usable row with a definite cut is finished in one
            // pass from the registers.
            if (!bad && sums_ok && cut_definite && a.mode == VERIFY_FULL) {
                exact_one_pass<LT, NV, FULL>(a, row, lrow, m.nb, rt, rg, Zt, Zg, a_size, xt, m.lg_tok, m.u_acc,
                                             smem, ex_lds, s_row);
            } else {
                exact_row<LT, true>(a, row, ex_lds, s_row, false, 0.f, 0.f);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// fp64 evaluation of rows the fp32 path did not settle
// ---------------------------------------------------------------------------

// LDS the exact path needs beyond whatever precedes it: reductions, a bitmask
// of A over the vocabulary, one fp64 partial sum per (vector chunk, wavefront).
__host__ __device__ inline size_t exact_table_offset(int V, int threads = NT) {
    const size_t nvec = ((size_t)V + EXV - 1) / EXV;
    const size_t nchunk = (nvec + threads - 1) / threads;
    const size_t off = ((sizeof(ExactShared) + 15) & ~size_t(15)) + (((size_t)V + 31) / 32) * 4 + 8 +
                       nchunk * (threads / WAVE) * sizeof(double);
    return (off + 15) & ~size_t(15);
}
// ... and, last, the table of the exponential.
__host__ __device__ inline size_t exact_lds_bytes(int V, int threads = NT) {
    return exact_table_offset(V, threads) + EXP_TABLE_BYTES;
}

// One residual term: max(0, t_A(x) - g(x)) (or t_A(x) when the residual has no mass).
__device__ __forceinline__ double resid_term(int x, int xt, int V, float lt, float lg, const uint32_t* mask,
                                             double mt, double mg, double inv_zt, double inv_zg,
                                             double mass, int zero_resid, const double* tab) {
    // branch-free: both exponentials are always evaluated, then selected
    const int xm = x < V ? x : V - 1;
    const bool in_a = (x < V) && ((mask[xm >> 5] >> (xm & 31)) & 1u);
    double ta = exp_tab((double)lt - mt, tab) * inv_zt;
    ta = in_a ? 0.0 : ta;
    ta = (x == xt) ? mass : ta;
    const double gv = exp_tab((double)lg - mg, tab) * inv_zg;
    const double r = zero_resid ? ta : ta - gv;
    return r > 0.0 ? r : 0.0;
}

// Evaluates one row in fp64 with the whole workgroup.  ex: LDS region of
// exact_lds_bytes().  lds_row, lds_grow: the raw target / draft row in LDS, or null.  have_max:
// the caller has the row maxima and knows both rows are free of NaN and +inf.
// TNT: threads of the calling workgroup.  Token order of the vector layout: vector vi = chunk*TNT + tid, so (chunk,
// wavefront, lane, element) is ascending token order.  Every pass over the row
// loads the next chunk's vectors before it works on the current one.
template <typename LT, bool VEC, int TNT>
__device__ void exact_row(const VerifyArgs& a, int row, unsigned char* ex, const unsigned char* lds_row,
                          bool have_max, float max_t, float max_g, const unsigned char* lds_grow) {
    constexpr int TNW = TNT / WAVE;
    const bool selected = a.mode == VERIFY_SELECTED;
    const int out = selected ? (int)blockIdx.x : row;   // slot of the outputs this workgroup writes
    using L = Lane<LT>;
    constexpr int EPV = EXV;
    ExactShared& sh = *reinterpret_cast<ExactShared*>(ex);
    uint32_t* mask = reinterpret_cast<uint32_t*>(ex + ((sizeof(ExactShared) + 15) & ~size_t(15)));

    const int tid = threadIdx.x;
    const int lane = tid & (WAVE - 1);
    const int wave = tid >> 6;
    const int V = a.V;
    const int k = a.k;
    const int nwords = (V + 31) >> 5;
    double* tab = reinterpret_cast<double*>(ex + exact_table_offset(V, TNT));
    for (int i = tid; i < 2 * EXP_TABLE_N; i += TNT) tab[i] = EXP_TABLE_HILO[i];   // published by the first barrier below
    double* wtot = reinterpret_cast<double*>(reinterpret_cast<unsigned char*>(mask) + (((size_t)nwords * 4 + 7) & ~size_t(7)));
    const int nvec = (V + EPV - 1) / EPV;
    const int nchunk = (nvec + TNT - 1) / TNT;
    bool row_ok;
    const int lrow = logit_row(a.row_index, a.R, row, &row_ok);
    const LT* trow = reinterpret_cast<const LT*>(a.target) + (int64_t)lrow * a.stride;
    const LT* grow = reinterpret_cast<const LT*>(a.draft) + (int64_t)lrow * a.stride;
    const int xt = a.tokens[row];
    const double delta = (double)a.delta;
    const double u_acc = (double)a.uniforms[2 * (int64_t)row];
    const double u_res = (double)a.uniforms[2 * (int64_t)row + 1];

    // ---- usability and maxima: token and table entries in range, no NaN / +inf ----
    int bad = ((unsigned)xt < (unsigned)V) ? 0 : 1;
    const int32_t* nrow = a.knn + (int64_t)(bad ? 0 : xt) * k;
    if (!row_ok) bad = 1;
    if (!bad)
        for (int j = tid; j < k; j += TNT)
            if ((unsigned)nrow[j] >= (unsigned)V) bad = 1;
    float mtf = neg_inf_f(), mgf = neg_inf_f();
    if (have_max) {
        mtf = max_t;
        mgf = max_g;
    } else {
        float tn[EPV], gn[EPV];
        VecLoad<LT, VEC>::load(trow, lds_row, tid, V, tn);
        VecLoad<LT, VEC>::load(grow, lds_grow, tid, V, gn);
        for (int c = 0; c < nchunk; ++c) {
            float tf[EPV], gf[EPV];
#pragma unroll
            for (int e = 0; e < EPV; ++e) { tf[e] = tn[e]; gf[e] = gn[e]; }
            if (c + 1 < nchunk) {
                VecLoad<LT, VEC>::load(trow, lds_row, (c + 1) * TNT + tid, V, tn);
                VecLoad<LT, VEC>::load(grow, lds_grow, (c + 1) * TNT + tid, V, gn);
            }
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                if (isnan(tf[e]) || isnan(gf[e]) || tf[e] == INFINITY || gf[e] == INFINITY) bad = 1;
                mtf = fmaxf(mtf, tf[e]);
                mgf = fmaxf(mgf, gf[e]);
            }
        }
    }
    const double mt = block_max<TNW>((double)mtf, sh.red, tid);
    const double mg = block_max<TNW>((double)mgf, sh.red2, tid);
    if (mt == -INFINITY || mg == -INFINITY) bad = 1;
    bad = block_or_i<TNW>(bad, sh.ired, tid);
    if (bad) {
        if (tid == 0) {
            if (selected) {
                a.out_resample[out] = -2;
            } else {
                a.out_accept[row] = -1;
                if (a.mode == VERIFY_FULL) a.out_resample[row] = -1;
                if (a.out_prob) a.out_prob[row] = NAN;
                if (a.out_mass) a.out_mass[row] = NAN;
                if (a.out_gtok) a.out_gtok[row] = NAN;
                if (a.out_asize) a.out_asize[row] = -1;
                if (a.out_path) a.out_path[row] = 1;
            }
        }
        return;
    }

    // ---- softmax normalisers ----
    double zt = 0.0, zg = 0.0;
    {
        float tn[EPV], gn[EPV];
        VecLoad<LT, VEC>::load(trow, lds_row, tid, V, tn);
        VecLoad<LT, VEC>::load(grow, lds_grow, tid, V, gn);
        for (int c = 0; c < nchunk; ++c) {
            float tf[EPV], gf[EPV];
#pragma unroll
            for (int e = 0; e < EPV; ++e) { tf[e] = tn[e]; gf[e] = gn[e]; }
            if (c + 1 < nchunk) {
                VecLoad<LT, VEC>::load(trow, lds_row, (c + 1) * TNT + tid, V, tn);
                VecLoad<LT, VEC>::load(grow, lds_grow, (c + 1) * TNT + tid, V, gn);
            }
            double st = 0.0, sg = 0.0;
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                st += exp_tab((double)tf[e] - mt, tab);
                sg += exp_tab((double)gf[e] - mg, tab);
            }
            zt += st;
            zg += sg;
        }
    }
    zt = block_sum<TNW>(zt, sh.red, tid);
    zg = block_sum<TNW>(zg, sh.red2, tid);

    // ---- nearest-first walk over the table row ----
    const double t_tok = exp_tab((double)L::glob(trow, xt) - mt, tab) / zt;
    int a_size;
    double S;
    exact_walk<LT, TNT>(trow, lds_row, nrow, k, xt, mt, zt, a.divergence, t_tok, delta, sh, tid, &a_size, &S, tab);

    const double g_tok = exp_tab((double)L::glob(grow, xt) - mg, tab) / zg;
    const double mass = t_tok + S;
    const bool accepted = (u_acc * g_tok < mass);
    if (tid == 0 && !selected) {
        double ap;
        if (g_tok > 0.0) ap = fmin(1.0, mass / g_tok);
        else ap = mass > 0.0 ? 1.0 : 0.0;
        if (a.out_prob) a.out_prob[row] = (float)ap;
        if (a.out_mass) a.out_mass[row] = (float)mass;
        if (a.out_gtok) a.out_gtok[row] = (float)g_tok;
        if (a.out_asize) a.out_asize[row] = a_size;
        if (a.out_path) a.out_path[row] = 1;
    }
    if (accepted || a.mode == VERIFY_DECIDE) {
        if (tid == 0) {
            if (selected) {
                a.out_resample[out] = -1;
            } else {
                a.out_accept[row] = accepted ? 1 : 0;
                if (a.mode == VERIFY_FULL) a.out_resample[row] = -1;
            }
        }
        return;
    }

    // ---- rejected: distorted target t_A, residual max(0, t_A - g), inverse CDF ----
    for (int w = tid; w < nwords; w += TNT) mask[w] = 0u;
    __syncthreads();
    for (int j = tid; j < a_size; j += TNT) {
        const int n = nrow[j];
        if (n != xt) atomicOr(&mask[n >> 5], 1u << (n & 31));
    }
    __syncthreads();

    const double inv_zt = 1.0 / zt, inv_zg = 1.0 / zg;
    int zero_resid = 0;
    for (int attempt = 0; attempt < 2; ++attempt) {
        // per (chunk, wavefront) partial sums of the residual, in token order
        {
            float tn[EPV], gn[EPV];
            VecLoad<LT, VEC>::load(trow, lds_row, tid, V, tn);
            VecLoad<LT, VEC>::load(grow, lds_grow, tid, V, gn);
            for (int c = 0; c < nchunk; ++c) {
                const int vi = c * TNT + tid;
                float tf[EPV], gf[EPV];
#pragma unroll
                for (int e = 0; e < EPV; ++e) { tf[e] = tn[e]; gf[e] = gn[e]; }
                if (c + 1 < nchunk) {
                    VecLoad<LT, VEC>::load(trow, lds_row, vi + TNT, V, tn);
                    VecLoad<LT, VEC>::load(grow, lds_grow, vi + TNT, V, gn);
                }
                double s = 0.0;
#pragma unroll
                for (int e = 0; e < EPV; ++e)
                    s += resid_term(vi * EPV + e, xt, V, tf[e], gf[e], mask, mt, mg, inv_zt, inv_zg, mass,
                                    zero_resid, tab);
                s = wave_sum(s);
                if (lane == 0) wtot[c * TNW + wave] = s;
            }
        }
        __syncthreads();
        // every wavefront scans the partial sums itself, 64 entries at a time in token order
        const int nent = nchunk * TNW;
        double Z = 0.0;
        for (int base = 0; base < nent; base += WAVE) Z += wave_sum(base + lane < nent ? wtot[base + lane] : 0.0);
        if (!(Z > 0.0) && !zero_resid) {  // residual without mass: sample t_A itself
            zero_resid = 1;
            __syncthreads();
            continue;
        }
        const double cthr = u_res * Z;
        // first (chunk, wavefront) whose running sum exceeds the threshold; P: the sum before it
        double P = 0.0;
        int ent = -1;
        for (int base = 0; base < nent && ent < 0; base += WAVE) {
            const double incl = P + wave_scan_incl(base + lane < nent ? wtot[base + lane] : 0.0);
            const unsigned long long cross = __ballot(base + lane < nent && incl > cthr);
            if (cross) {
                const int l = __ffsll((long long)cross) - 1;
                ent = base + l;
                P = l ? __shfl(incl, l - 1, WAVE) : P;
            } else {
                P = __shfl(incl, WAVE - 1, WAVE);
            }
        }
        if (ent < 0) {   // rounding left no crossing: the last entry takes the draw
            ent = nent - 1;
            P -= wtot[ent];
        }
        if (wave == (ent % TNW)) {
            const int c = ent / TNW;
            const int vi = c * TNT + tid;
            float tf[EPV], gf[EPV];
            VecLoad<LT, VEC>::load(trow, lds_row, vi, V, tf);
            VecLoad<LT, VEC>::load(grow, lds_grow, vi, V, gf);
            double r[EPV];
            double s = 0.0;
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                r[e] = resid_term(vi * EPV + e, xt, V, tf[e], gf[e], mask, mt, mg, inv_zt, inv_zg, mass, zero_resid, tab);
                s += r[e];
            }
            const double incl = wave_scan_incl(s);
            double excl = __shfl_up(incl, 1, WAVE);
            if (lane == 0) excl = 0.0;
            const unsigned long long cross = __ballot(P + incl > cthr);
            const unsigned long long haspos = __ballot(s > 0.0);
            // rounding between the butterfly sum and the scan can leave no crossing lane:
            // then the last lane that holds mass takes the draw
            const int owner = cross ? (__ffsll((long long)cross) - 1)
                                    : (haspos ? 63 - __clzll((long long)haspos) : 0);
            if (lane == owner) {
                double cum = P + excl;
                int found = -1, lastpos = -1;
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    cum += r[e];
                    if (r[e] > 0.0) lastpos = vi * EPV + e;
                    if (found < 0 && cum > cthr && r[e] > 0.0) found = vi * EPV + e;
                }
                if (found < 0) found = lastpos;
                if (!selected) a.out_accept[row] = 0;
                a.out_resample[out] = found;
            }
        }
        break;
    }
}

// Every row through the exact path: for shapes the fast path does not cover.
template <typename LT>
__global__ __launch_bounds__(NT) void verify_exact(VerifyArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    exact_row<LT, false>(a, verification_of_block(blockIdx.x, a.N, a.row_index != nullptr), smem, nullptr, false, 0.f, 0.f);
}

// VERIFY_SELECTED: workgroup i evaluates verification select[i] and writes out_resample[i].
// Few rows per launch, so each gets a workgroup of 512 threads (two wavefronts per SIMD, no register
// spills; 1024 threads measured slower): the fp64 passes of a row are
// latency-bound at one wavefront per SIMD.
constexpr int SEL_NT = 512;
// Evaluates verification v in fp64 with all threads of this workgroup (VERIFY_SELECTED: only
// out_resample[blockIdx.x] is written).  When they fit, both logit rows are first copied into LDS,
// all loads in flight together, so the fp64 passes read LDS.
template <typename LT, bool VEC>
__device__ __forceinline__ void selected_row(const VerifyArgs& a, int v, unsigned char* smem) {
    const unsigned char* lds_t = nullptr;
    const unsigned char* lds_g = nullptr;
    if (VEC && a.stage_rows) {
        const int row_bytes = a.V * (int)sizeof(LT);          // a multiple of 8 (VEC: V % 4 == 0)
        const size_t ex_bytes = (exact_lds_bytes(a.V, SEL_NT) + 15) & ~size_t(15);
        unsigned char* st = smem + ex_bytes;
        unsigned char* sg = st + ((row_bytes + 15) & ~15);
        bool row_ok;
        const int lrow = logit_row(a.row_index, a.R, v, &row_ok);
        const uint2* tsrc = reinterpret_cast<const uint2*>(reinterpret_cast<const LT*>(a.target) + (int64_t)lrow * a.stride);
        const uint2* gsrc = reinterpret_cast<const uint2*>(reinterpret_cast<const LT*>(a.draft) + (int64_t)lrow * a.stride);
        const int n8 = row_bytes >> 3;
        for (int i = threadIdx.x; i < n8; i += SEL_NT) {
            reinterpret_cast<uint2*>(st)[i] = tsrc[i];
            reinterpret_cast<uint2*>(sg)[i] = gsrc[i];
        }
        __syncthreads();
        lds_t = st;
        lds_g = sg;
    }
    exact_row<LT, VEC, SEL_NT>(a, v, smem, lds_t, false, 0.f, 0.f, lds_g);
}

// VERIFY_SELECTED: workgroup i evaluates verification select[i] and writes out_resample[i].
template <typename LT, bool VEC>
__global__ __launch_bounds__(SEL_NT) void resample_selected(VerifyArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int v = a.select[blockIdx.x];
    if (v < 0 || v >= a.N) {   // uniform per workgroup
        if (threadIdx.x == 0) a.out_resample[blockIdx.x] = v < 0 ? v : -2;
        return;
    }
    selected_row<LT, VEC>(a, v, smem);
}

// Second half of a tree step: workgroup b walks tree b over the decisions in a.out_accept (its
// first wavefront), then draws the one residual the walk asks for and writes a.out_resample[b].
template <typename LT, bool VEC>
__global__ __launch_bounds__(SEL_NT) void tree_finish(VerifyArgs a, const int32_t* parent, int M, int32_t* out_len,
                                                      int32_t* out_path) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tree = blockIdx.x;
    int32_t* path = out_path + (int64_t)tree * M;
    int* bcast = reinterpret_cast<int*>(smem);
    if (threadIdx.x < WAVE) {
        int len;
        const int next = walk_tree(a.out_accept + (int64_t)tree * M, nullptr, parent + (int64_t)tree * M, M, tree,
                                   path, &len);
        for (int j = len + threadIdx.x; j < M; j += WAVE) path[j] = -1;
        if (threadIdx.x == 0) {
            out_len[tree] = len;
            bcast[0] = next;
        }
    }
    __syncthreads();
    const int v = bcast[0];
    __syncthreads();              // the exact path reuses this LDS
    if (v < 0) {                  // uniform per workgroup: nothing to resample
        if (threadIdx.x == 0) a.out_resample[tree] = v;
        return;
    }
    selected_row<LT, VEC>(a, v, smem);
}

// ---------------------------------------------------------------------------
// host-side launch
// ---------------------------------------------------------------------------

// Dynamic LDS of verify_fast: raw row, the head of FastShared, then a region that holds either
// the neighbour partial sums or the exact path's data.
template <typename LT>
static size_t fast_lds_bytes(int V) {
    const size_t row_bytes = ((size_t)V * sizeof(LT) + 15) & ~size_t(15);
    size_t tail = exact_lds_bytes(V) > FAST_SHARED_TAIL ? exact_lds_bytes(V) : FAST_SHARED_TAIL;
    const size_t one_pass = one_pass_layout(V).total;
    if (one_pass > tail) tail = one_pass;
    return EXP_TABLE_BYTES + row_bytes + FAST_SHARED_HEAD + tail;
}

// launch == false: only the LDS limits are raised (lantern_prepare), nothing is enqueued.
template <typename LT, int NV>
static hipError_t launch_fast_nv(const VerifyArgs& a, hipStream_t stream, bool launch) {
    const size_t lds = fast_lds_bytes<LT>(a.V);
    const bool full = a.V == NV * NT * Lane<LT>::EPV;
    // three instantiations: whole rows with a vector-readable table, ragged rows with one, and the rest
    const bool vt = ((a.k & 3) == 0) && ((reinterpret_cast<uintptr_t>(a.knn) & 15) == 0);
    if (!launch) {   // every one of them may be needed later
        hipError_t e = allow_lds<&verify_fast<LT, NV, true, true>>(lds);
        if (e == hipSuccess) e = allow_lds<&verify_fast<LT, NV, false, true>>(lds);
        if (e == hipSuccess) e = allow_lds<&verify_fast<LT, NV, false, false>>(lds);
        return e;
    }
    const hipError_t e = (full && vt) ? allow_lds<&verify_fast<LT, NV, true, true>>(lds)
                         : vt         ? allow_lds<&verify_fast<LT, NV, false, true>>(lds)
                                      : allow_lds<&verify_fast<LT, NV, false, false>>(lds);
    if (e != hipSuccess) return e;
    if (full && vt)
        hipLaunchKernelGGL((verify_fast<LT, NV, true, true>), dim3(a.N), dim3(NT), lds, stream, a);
    else if (vt)
        hipLaunchKernelGGL((verify_fast<LT, NV, false, true>), dim3(a.N), dim3(NT), lds, stream, a);
    else
        hipLaunchKernelGGL((verify_fast<LT, NV, false, false>), dim3(a.N), dim3(NT), lds, stream, a);
    return hipGetLastError();
}

template <typename LT>
static hipError_t launch_fast(const VerifyArgs& a, hipStream_t stream, bool launch) {
    const int nvec = a.V / Lane<LT>::EPV;
    const int nv = (nvec + NT - 1) / NT;
    if (nv <= 1) return launch_fast_nv<LT, 1>(a, stream, launch);
    if (nv <= 2) return launch_fast_nv<LT, 2>(a, stream, launch);
    if (nv <= 4) return launch_fast_nv<LT, 4>(a, stream, launch);
    if (nv <= 8) return launch_fast_nv<LT, 8>(a, stream, launch);
    return launch_fast_nv<LT, 16>(a, stream, launch);
}

// Rows the fp32 pass covers: whole 16-byte vectors, at most 16 per thread, k within the scan's depth.
template <typename LT>
static bool fast_shape(int V, int k) {
    constexpr int EPV = Lane<LT>::EPV;
    return (V % EPV) == 0 && (V / EPV + NT - 1) / NT <= 16 && k <= FAST_MAX_K;
}

template <typename LT>
static hipError_t launch_typed(const VerifyArgs& a, hipStream_t stream) {
    const uintptr_t align = reinterpret_cast<uintptr_t>(a.target) | reinterpret_cast<uintptr_t>(a.draft) |
                            (uintptr_t)(a.stride * (int64_t)sizeof(LT));
    if ((align & 15) == 0 && fast_shape<LT>(a.V, a.k)) return launch_fast<LT>(a, stream, true);
    const size_t lds = exact_lds_bytes(a.V);
    const hipError_t e = allow_lds<&verify_exact<LT>>(lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((verify_exact<LT>), dim3(a.N), dim3(NT), lds, stream, a);
    return hipGetLastError();
}

// LDS of the 512-thread kernels; *stage: both logit rows fit beside the exact path's data.
template <typename LT>
static size_t selected_lds_bytes(int V, bool vec, int* stage) {
    const size_t lds = exact_lds_bytes(V, SEL_NT);
    const size_t staged = ((lds + 15) & ~size_t(15)) + 2 * (((size_t)V * sizeof(LT) + 15) & ~size_t(15));
    *stage = (vec && staged <= 150 * 1024) ? 1 : 0;
    return *stage ? staged : lds;
}

template <typename LT>
static hipError_t launch_selected_typed(const VerifyArgs& a_in, const int32_t* parent, int M, int32_t* out_len,
                                        int32_t* out_path, hipStream_t stream) {
    VerifyArgs a = a_in;
    const uintptr_t align = reinterpret_cast<uintptr_t>(a.target) | reinterpret_cast<uintptr_t>(a.draft) |
                            (uintptr_t)(a.stride * (int64_t)sizeof(LT));
    const bool vec = (align & 15) == 0 && (a.V % EXV) == 0;   // rows 16-byte aligned, whole vectors
    const size_t lds = selected_lds_bytes<LT>(a.V, vec, &a.stage_rows);
    if (parent) {   // walk and draw in one launch, one workgroup per tree
        const hipError_t e = vec ? allow_lds<&tree_finish<LT, true>>(lds) : allow_lds<&tree_finish<LT, false>>(lds);
        if (e != hipSuccess) return e;
        if (vec)
            hipLaunchKernelGGL((tree_finish<LT, true>), dim3(a.n_sel), dim3(SEL_NT), lds, stream, a, parent, M, out_len,
                               out_path);
        else
            hipLaunchKernelGGL((tree_finish<LT, false>), dim3(a.n_sel), dim3(SEL_NT), lds, stream, a, parent, M, out_len,
                               out_path);
        return hipGetLastError();
    }
    const hipError_t e = vec ? allow_lds<&resample_selected<LT, true>>(lds) : allow_lds<&resample_selected<LT, false>>(lds);
    if (e != hipSuccess) return e;
    if (vec)
        hipLaunchKernelGGL((resample_selected<LT, true>), dim3(a.n_sel), dim3(SEL_NT), lds, stream, a);
    else
        hipLaunchKernelGGL((resample_selected<LT, false>), dim3(a.n_sel), dim3(SEL_NT), lds, stream, a);
    return hipGetLastError();
}

// Raises, on the current device, the LDS limit of every kernel a verification of this vocabulary
// size and logit type can launch, whatever the alignment of the caller's buffers turns out to be.
template <typename LT>
static hipError_t prepare_typed(int V, int k) {
    // the runtime defers loading a file's kernels to their first use: make that happen now
    hipFuncAttributes attr;
    hipError_t e = hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(&verify_exact<LT>));
    if (e != hipSuccess) return e;
    if (fast_shape<LT>(V, k)) {
        VerifyArgs a{};
        a.V = V;
        a.k = k;
        e = launch_fast<LT>(a, nullptr, false);
    }
    if (e == hipSuccess) e = allow_lds<&verify_exact<LT>>(exact_lds_bytes(V));
    for (int vec = 0; vec < 2 && e == hipSuccess; ++vec) {
        if (vec && (V % EXV) != 0) break;
        int stage;
        const size_t lds = selected_lds_bytes<LT>(V, vec != 0, &stage);
        if (vec) {
            e = allow_lds<&tree_finish<LT, true>>(lds);
            if (e == hipSuccess) e = allow_lds<&resample_selected<LT, true>>(lds);
        } else {
            e = allow_lds<&tree_finish<LT, false>>(lds);
            if (e == hipSuccess) e = allow_lds<&resample_selected<LT, false>>(lds);
        }
    }
    return e;
}

hipError_t prepare_verify(int logits_dtype, int V, int k) {
    return logits_dtype == 0 ? prepare_typed<float>(V, k) : prepare_typed<uint16_t>(V, k);
}

hipError_t launch_resample_selected(const VerifyArgs& a, int logits_dtype, hipStream_t stream) {
    if (logits_dtype == 0) return launch_selected_typed<float>(a, nullptr, 0, nullptr, nullptr, stream);
    return launch_selected_typed<uint16_t>(a, nullptr, 0, nullptr, nullptr, stream);
}

hipError_t launch_tree_finish(const VerifyArgs& a, const int32_t* parent, int M, int32_t* out_len, int32_t* out_path,
                              int logits_dtype, hipStream_t stream) {
    if (logits_dtype == 0) return launch_selected_typed<float>(a, parent, M, out_len, out_path, stream);
    return launch_selected_typed<uint16_t>(a, parent, M, out_len, out_path, stream);
}

hipError_t launch_verify(const VerifyArgs& a, int logits_dtype, hipStream_t stream) {
    if (logits_dtype == 0) return launch_typed<float>(a, stream);
    return launch_typed<uint16_t>(a, stream);
}

}  // namespace lantern
