/*
 * CPU oracle for LANTERN's relaxed-acceptance verification and its codebook
 * nearest-neighbour table.  TEST INFRASTRUCTURE ONLY: it exists so the tests,
 * the smoke check and the bench's CPU-baseline leg have an independent, slow,
 * obviously-correct result to compare the HIP library against.  The product
 * path never calls it, and it shares no code with the HIP sources.
 *
 * Everything is evaluated in fp64, one row at a time, in the order the paper
 * states its steps.  Inputs arrive as fp32 arrays (bf16 and fp32 logits are
 * both exactly representable in fp32) and are widened to fp64 on read.
 *
 * Notation.  The paper writes p for the drafter and q for the target model
 * (Section 2, "Notations").  To keep that from being confused with the
 * opposite convention used elsewhere, this file writes
 *     t(x)  target probability      (the paper's q)
 *     g(x)  drafter probability     (the paper's p)
 *     xt    the draft token         (the paper's x-tilde)
 *
 * Build with -ffp-contract=off: the squared distance of the table build is
 * defined as a sequence of separately rounded fp64 subtract, multiply and add
 * operations, so that an IEEE-754 fp64 implementation elsewhere can reproduce
 * the ordering of near-ties bit for bit.
 *
 * Parity pins (tests marked "not gpu"): hand-derived rows under tests/golden,
 * reduction to standard speculative acceptance at k = 1 and delta = 0, the TVD
 * invariant, brute-force neighbour search, residuals that sum to one, exact
 * enumeration and Monte-Carlo recovery of the target law at k = 1.
 * Parity unpinned: behaviour on real LlamaGen / Anole logits and codebooks.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------- */
/* Codebook neighbour table  B_k  (Section 4.2; Algorithm 2, precompute part) */
/* ------------------------------------------------------------------------- */

typedef struct {
    double dist;
    int32_t idx;
} dist_idx;

static int by_dist_then_idx(const void* pa, const void* pb) {
    const dist_idx* a = (const dist_idx*)pa;
    const dist_idx* b = (const dist_idx*)pb;
    if (a->dist < b->dist) return -1;
    if (a->dist > b->dist) return 1;
    return (a->idx > b->idx) - (a->idx < b->idx);
}

/* Squared l2 distance between codes i and j: differences, squares and the
 * running sum are each rounded to fp64, coordinates taken in index order.
 * Squared distance orders pairs exactly as the l2 distance does. */
static double sq_dist(const float* ci, const float* cj, int d) {
    double acc = 0.0;
    for (int c = 0; c < d; ++c) {
        double diff = (double)ci[c] - (double)cj[c];
        double sq = diff * diff;
        acc = acc + sq;
    }
    return acc;
}

/* Rows [row_begin, row_end) of the table.  Row i holds i itself first, then
 * the k-1 other tokens in increasing distance; equal distances are ordered by
 * the lower token index.  out is [(row_end-row_begin), k].
 * metric 0: squared l2 (the paper's choice, Section 5.1).
 * metric 1: cosine similarity, larger is nearer (ablation of Section 5.3.1);
 *           the key is -cos so that the same ascending order applies.
 * A key that is not a number (the cosine with a code of zero norm, 0/0; a
 * codebook entry that is itself NaN or infinite) stands for a similarity that
 * does not exist: the paper does not treat it, and it is read here as the
 * farthest possible, key +infinity, equal keys by the lower index as always.
 * Returns 0, or -1 on bad arguments. */
int oracle_build_knn_rows(const float* codebook, int V, int d, int k, int metric,
                          int row_begin, int row_end, int32_t* out, int threads) {
    if (!codebook || !out || V < 1 || d < 1 || k < 1 || k > V) return -1;
    if (row_begin < 0 || row_end > V || row_begin > row_end) return -1;
    if (metric != 0 && metric != 1) return -1;
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel num_threads(threads > 0 ? threads : 1)
#endif
    {
        dist_idx* others = (dist_idx*)malloc(sizeof(dist_idx) * (size_t)(V > 1 ? V - 1 : 1));
        if (!others) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        } else {
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 4)
#endif
            for (int i = row_begin; i < row_end; ++i) {
                const float* ci = codebook + (size_t)i * d;
                double ni = 0.0;
                if (metric == 1) {
                    for (int c = 0; c < d; ++c) ni = ni + (double)ci[c] * (double)ci[c];
                    ni = sqrt(ni);
                }
                int m = 0;
                for (int j = 0; j < V; ++j) {
                    if (j == i) continue;
                    const float* cj = codebook + (size_t)j * d;
                    double key;
                    if (metric == 0) {
                        key = sq_dist(ci, cj, d);
                    } else {
                        double dot = 0.0, nj = 0.0;
                        for (int c = 0; c < d; ++c) {
                            dot = dot + (double)ci[c] * (double)cj[c];
                            nj = nj + (double)cj[c] * (double)cj[c];
                        }
                        nj = sqrt(nj);
                        key = -(dot / (ni * nj));
                    }
                    if (key != key) key = HUGE_VAL;
                    others[m].dist = key;
                    others[m].idx = j;
                    ++m;
                }
                qsort(others, (size_t)m, sizeof(dist_idx), by_dist_then_idx);
                int32_t* row = out + (size_t)(i - row_begin) * k;
                row[0] = i;
                for (int s = 1; s < k; ++s) row[s] = others[s - 1].idx;
            }
        }
        free(others);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------- */
/* Row softmax (Section 2: the model's next-token likelihoods)                */
/* ------------------------------------------------------------------------- */

/* Returns 0 when the row is usable: no NaN, no +inf, at least one finite
 * logit.  -inf logits (tokens removed by top-k / top-p filtering upstream)
 * get probability exactly zero. */
static int softmax_row(const float* logits, int V, double* prob) {
    double mx = -INFINITY;
    for (int x = 0; x < V; ++x) {
        double l = (double)logits[x];
        if (isnan(l) || l == INFINITY) return -1;
        if (l > mx) mx = l;
    }
    if (mx == -INFINITY) return -1;
    double z = 0.0;
    for (int x = 0; x < V; ++x) {
        double e = exp((double)logits[x] - mx);
        prob[x] = e;
        z = z + e;
    }
    for (int x = 0; x < V; ++x) prob[x] = prob[x] / z;
    return 0;
}

int oracle_softmax(const float* logits, int V, double* prob) {
    if (!logits || !prob || V < 1) return -1;
    return softmax_row(logits, V, prob);
}

/* ------------------------------------------------------------------------- */
/* One verification on given probability vectors                              */
/* ------------------------------------------------------------------------- */

enum {
    DIAG_ACCEPT_PROB = 0, /* min(1, mass / g(xt))                                   */
    DIAG_MASS = 1,        /* sum of t over A_{k,delta}(xt)                          */
    DIAG_G_TOK = 2,       /* g(xt)                                                  */
    DIAG_T_TOK = 3,       /* t(xt)                                                  */
    DIAG_TVD_WALK = 4,    /* cumulative TVD kept while walking the neighbourhood    */
    DIAG_TVD_DIRECT = 5,  /* 1/2 * sum |t_A - t| evaluated from the definition      */
    DIAG_RESID_Z = 6,     /* normaliser of the residual, 0 when accepted            */
    DIAG_A_SIZE = 7,      /* number of table slots taken into A                     */
    DIAG_MARGIN_ACCEPT = 8, /* |u_acc*g(xt) - mass|                                 */
    DIAG_MARGIN_CUT = 9,    /* min over tested slots of |D_TV + inc - delta|        */
    DIAG_MARGIN_CDF = 10,   /* min over CDF edges of |cum - u_res*Z| (rejected rows)*/
    DIAG_ZERO_RESID = 11,   /* 1 when the residual had no mass and t_A was sampled  */
    DIAG_COUNT = 12
};

int oracle_diag_count(void) { return DIAG_COUNT; }

/* Jensen-Shannon divergence (natural logarithm, Section 5.3.2) between a distorted target ta and
 * the target t, from the definition over the whole vocabulary:
 *     1/2 KL(ta || m) + 1/2 KL(t || m),   m = (ta + t) / 2,   0 ln 0 = 0.
 * Entries where the two agree have m equal to both, so both logarithms are ln 1 = 0 exactly.
 * The divergence is never negative; when the mass moved is around one unit in the last place of
 * t(xt) the two terms at xt cancel down to their rounding errors and the sum can come out below
 * zero: such a value is returned as zero, so that no prefix ever passes a bound of zero. */
static double jsd_full(const double* ta, const double* t, int V) {
    double kl_a = 0.0, kl_t = 0.0;
    for (int x = 0; x < V; ++x) {
        if (ta[x] == t[x]) continue;
        double m = 0.5 * (ta[x] + t[x]);
        if (ta[x] > 0.0) kl_a = kl_a + ta[x] * log(ta[x] / m);
        if (t[x] > 0.0) kl_t = kl_t + t[x] * log(t[x] / m);
    }
    double jsd = 0.5 * kl_a + 0.5 * kl_t;
    return jsd < 0.0 ? 0.0 : jsd;
}

/*
 * t, g: probability vectors of length V.  nbrs: the k table entries of row xt,
 * nearest first.  scratch: V doubles.
 *
 * Steps (Section 4.3; Algorithm 2, inference part; Algorithm 1, verification):
 *  1. Walk the neighbourhood nearest-first keeping the cumulative TVD.  Adding
 *     a neighbour x != xt moves t(x) from x onto xt, which by the definition
 *     of the distorted target raises 1/2*sum|t_A - t| by exactly t(x); adding
 *     xt itself changes nothing.  A neighbour is taken while the TVD after
 *     adding it stays strictly below delta; the first one that does not fit
 *     ends the walk.  xt itself is always taken.
 *  2. mass = t(xt) + cumulative TVD = sum of t over A.
 *  3. Accept iff u_acc < min(1, mass / g(xt)), evaluated as u_acc*g(xt) < mass
 *     (identical for u_acc in [0,1) and g(xt) > 0, and defined at g(xt) = 0).
 *  4. On rejection build the distorted target t_A (mass at xt, zero on the
 *     rest of A, t elsewhere), the residual rho = max(0, t_A - g), and return
 *     the first token, in index order, whose cumulative rho exceeds u_res*Z.
 *     A residual with no mass at all falls back to sampling t_A.
 * optional outputs (may be NULL): rho_out[V] normalised residual, ta_out[V].
 */
static void verify_probs(const double* t, const double* g, int V, int xt,
                         const int32_t* nbrs, int k, int divergence, double delta,
                         double u_acc, double u_res,
                         int32_t* out_accept, int32_t* out_resample,
                         double* diag, double* scratch,
                         double* rho_out, double* ta_out) {
    double d_tv = 0.0;
    int a = 0;
    double margin_cut = INFINITY;
    /* divergence 0: total variation distance (Section 4.3), which for a prefix is the mass it
     * moves onto xt.  divergence 1: Jensen-Shannon (ablation of Section 5.3.2), evaluated on the
     * candidate's distorted target itself, kept in `scratch` while walking. */
    double* cand_ta = scratch;
    if (divergence != 0) memcpy(cand_ta, t, sizeof(double) * (size_t)V);
    for (int j = 0; j < k; ++j) {
        int x = nbrs[j];
        if (x == xt) {
            a = j + 1;
            continue;
        }
        double inc = t[x];
        double cand = d_tv + inc;                       /* mass moved onto xt if x is taken */
        double div;
        if (divergence == 0) {
            div = cand;
        } else {
            cand_ta[x] = 0.0;
            cand_ta[xt] = t[xt] + cand;
            div = jsd_full(cand_ta, t, V);
        }
        double mg = fabs(div - delta);
        if (mg < margin_cut) margin_cut = mg;
        if (div < delta) {
            d_tv = cand;
            a = j + 1;
        } else {
            break;
        }
    }
    double mass = t[xt] + d_tv;
    double gx = g[xt];
    double accept_prob;
    if (gx > 0.0) {
        accept_prob = mass / gx;
        if (accept_prob > 1.0) accept_prob = 1.0;
    } else {
        accept_prob = mass > 0.0 ? 1.0 : 0.0;
    }
    int accepted = (u_acc * gx < mass) ? 1 : 0;

    /* distorted target from its definition, used for the direct TVD and the residual */
    double* ta = scratch;
    memcpy(ta, t, sizeof(double) * (size_t)V);
    for (int j = 0; j < a; ++j)
        if (nbrs[j] != xt) ta[nbrs[j]] = 0.0;
    ta[xt] = mass;
    double tvd_direct = 0.0;
    for (int x = 0; x < V; ++x) tvd_direct = tvd_direct + fabs(ta[x] - t[x]);
    tvd_direct = 0.5 * tvd_direct;
    if (ta_out) memcpy(ta_out, ta, sizeof(double) * (size_t)V);

    double z = 0.0;
    int zero_resid = 0;
    int resample = -1;
    double margin_cdf = INFINITY;
    if (!accepted || rho_out) {
        for (int x = 0; x < V; ++x) {
            double r = ta[x] - g[x];
            if (!(r > 0.0)) r = 0.0;
            z = z + r;
        }
        if (!(z > 0.0)) zero_resid = 1;
        double zz = 0.0;
        if (zero_resid)
            for (int x = 0; x < V; ++x) zz = zz + ta[x];
        else
            zz = z;
        if (rho_out)
            for (int x = 0; x < V; ++x) {
                double r = zero_resid ? ta[x] : ta[x] - g[x];
                if (!(r > 0.0)) r = 0.0;
                rho_out[x] = r / zz;
            }
        if (!accepted) {
            double c = u_res * zz;
            double cum = 0.0;
            for (int x = 0; x < V; ++x) {
                double r = zero_resid ? ta[x] : ta[x] - g[x];
                if (!(r > 0.0)) r = 0.0;
                cum = cum + r;
                double mg = fabs(cum - c);
                if (r > 0.0 && mg < margin_cdf) margin_cdf = mg;
                if (resample < 0 && cum > c) resample = x;
            }
        }
        z = zz;
    }

    *out_accept = accepted;
    *out_resample = accepted ? -1 : resample;
    if (diag) {
        diag[DIAG_ACCEPT_PROB] = accept_prob;
        diag[DIAG_MASS] = mass;
        diag[DIAG_G_TOK] = gx;
        diag[DIAG_T_TOK] = t[xt];
        diag[DIAG_TVD_WALK] = d_tv;
        diag[DIAG_TVD_DIRECT] = tvd_direct;
        diag[DIAG_RESID_Z] = accepted ? 0.0 : z;
        diag[DIAG_A_SIZE] = (double)a;
        diag[DIAG_MARGIN_ACCEPT] = fabs(u_acc * gx - mass);
        diag[DIAG_MARGIN_CUT] = margin_cut;
        diag[DIAG_MARGIN_CDF] = margin_cdf;
        diag[DIAG_ZERO_RESID] = (double)(zero_resid && !accepted);
    }
}

static int row_args_ok(int V, int xt, const int32_t* nbrs, int k) {
    if (xt < 0 || xt >= V) return 0;
    for (int j = 0; j < k; ++j)
        if (nbrs[j] < 0 || nbrs[j] >= V) return 0;
    return 1;
}

/* Single verification on probabilities given directly (lets the tests use
 * dyadic, exactly representable rows).  Returns 0, or -1 on bad arguments. */
int oracle_verify_probs(const double* t, const double* g, int V, int xt,
                        const int32_t* nbrs, int k, double delta,
                        double u_acc, double u_res,
                        int32_t* out_accept, int32_t* out_resample,
                        double* diag, double* rho_out, double* ta_out) {
    if (!t || !g || !nbrs || !out_accept || !out_resample) return -1;
    if (V < 1 || k < 1 || k > V || !(delta >= 0.0)) return -1;
    if (!row_args_ok(V, xt, nbrs, k)) return -1;
    double* scratch = (double*)malloc(sizeof(double) * (size_t)V);
    if (!scratch) return -1;
    verify_probs(t, g, V, xt, nbrs, k, 0, delta, u_acc, u_res, out_accept, out_resample,
                 diag, scratch, rho_out, ta_out);
    free(scratch);
    return 0;
}

/*
 * N independent verifications from logits.  Row i uses target_logits and
 * draft_logits at offset i*row_stride, token draft_tokens[i], table row
 * knn[draft_tokens[i]*k .. +k), uniforms[2i] for acceptance and uniforms[2i+1]
 * for resampling.  out_accept[i] is 1 or 0; out_resample[i] is the resampled
 * token, or -1 when accepted.  A row whose token or table entries fall outside
 * [0,V), or whose logits hold NaN, +inf or nothing finite, gets -1 in both.
 * diag is NULL or [N, oracle_diag_count()].  Returns 0, or -1 on bad arguments.
 */
int oracle_verify_div(const float* target_logits, const float* draft_logits, int N, int V,
                      int64_t row_stride, const int32_t* draft_tokens, const int32_t* knn, int k,
                      int divergence, double delta, const float* uniforms,
                      int32_t* out_accept, int32_t* out_resample, double* diag, int threads);

int oracle_verify(const float* target_logits, const float* draft_logits, int N, int V,
                  int64_t row_stride, const int32_t* draft_tokens, const int32_t* knn, int k,
                  double delta, const float* uniforms,
                  int32_t* out_accept, int32_t* out_resample, double* diag, int threads) {
    return oracle_verify_div(target_logits, draft_logits, N, V, row_stride, draft_tokens, knn, k, 0, delta,
                             uniforms, out_accept, out_resample, diag, threads);
}

/* As oracle_verify with a choice of divergence for the bound on A: 0 total variation
 * distance, 1 Jensen-Shannon divergence (natural logarithm).  With JSD the diagnostic
 * "tvd_walk" still reports the mass moved onto xt. */
int oracle_verify_div(const float* target_logits, const float* draft_logits, int N, int V,
                      int64_t row_stride, const int32_t* draft_tokens, const int32_t* knn, int k,
                      int divergence, double delta, const float* uniforms,
                      int32_t* out_accept, int32_t* out_resample, double* diag, int threads) {
    if (divergence != 0 && divergence != 1) return -1;
    if (N < 0 || V < 1 || k < 1 || k > V || row_stride < V || !(delta >= 0.0)) return -1;
    if (N == 0) return 0;
    if (!target_logits || !draft_logits || !draft_tokens || !knn || !uniforms || !out_accept ||
        !out_resample)
        return -1;
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel num_threads(threads > 0 ? threads : 1)
#endif
    {
        double* buf = (double*)malloc(sizeof(double) * 3 * (size_t)V);
        if (!buf) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        } else {
            double* t = buf;
            double* g = buf + V;
            double* scratch = buf + 2 * (size_t)V;
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
            for (int i = 0; i < N; ++i) {
                double* dg = diag ? diag + (size_t)i * DIAG_COUNT : NULL;
                if (dg)
                    for (int c = 0; c < DIAG_COUNT; ++c) dg[c] = NAN;
                int xt = draft_tokens[i];
                int ok = (xt >= 0 && xt < V) && row_args_ok(V, xt, knn + (size_t)xt * k, k);
                if (ok) ok = softmax_row(target_logits + (size_t)i * row_stride, V, t) == 0;
                if (ok) ok = softmax_row(draft_logits + (size_t)i * row_stride, V, g) == 0;
                if (!ok) {
                    out_accept[i] = -1;
                    out_resample[i] = -1;
                    continue;
                }
                verify_probs(t, g, V, xt, knn + (size_t)xt * k, k, divergence, delta,
                             (double)uniforms[2 * (size_t)i], (double)uniforms[2 * (size_t)i + 1],
                             &out_accept[i], &out_resample[i], dg, scratch, NULL, NULL);
            }
        }
        free(buf);
    }
    return failed ? -1 : 0;
}


/* ------------------------------------------------------------------------- */
/* Greedy decoding variant (Section 4.3, last sentence)                       */
/* ------------------------------------------------------------------------- */

/*
 * Accept xt iff xt = argmax_x t_A(x), where t_A is the distorted target
 * induced by A_{k,delta}(xt): the mass of A at xt, zero on the rest of A, t
 * elsewhere.  The arg-max takes the lowest token index among equal values.
 * out_token[i] is -1 when accepted and that arg-max otherwise (the token
 * greedy decoding of the distorted target emits).  No drafter probabilities
 * and no random draws are involved.
 * diag (optional, [N,3]): mass, the largest t_A outside xt, a_size.
 * Unusable rows get -1 in both outputs, as in oracle_verify.
 */
int oracle_verify_greedy(const float* target_logits, int N, int V, int64_t row_stride,
                         const int32_t* draft_tokens, const int32_t* knn, int k, double delta,
                         int32_t* out_accept, int32_t* out_token, double* diag, int threads) {
    if (N < 0 || V < 1 || k < 1 || k > V || row_stride < V || !(delta >= 0.0)) return -1;
    if (N == 0) return 0;
    if (!target_logits || !draft_tokens || !knn || !out_accept || !out_token) return -1;
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel num_threads(threads > 0 ? threads : 1)
#endif
    {
        double* buf = (double*)malloc(sizeof(double) * 2 * (size_t)V);
        if (!buf) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        } else {
            double* t = buf;
            double* ta = buf + V;
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
            for (int i = 0; i < N; ++i) {
                double* dg = diag ? diag + (size_t)i * 3 : NULL;
                if (dg) dg[0] = dg[1] = dg[2] = NAN;
                int xt = draft_tokens[i];
                int ok = (xt >= 0 && xt < V) && row_args_ok(V, xt, knn + (size_t)xt * k, k);
                if (ok) ok = softmax_row(target_logits + (size_t)i * row_stride, V, t) == 0;
                if (!ok) {
                    out_accept[i] = -1;
                    out_token[i] = -1;
                    continue;
                }
                const int32_t* nbrs = knn + (size_t)xt * k;
                /* the same nearest-first walk as in verify_probs */
                double d_tv = 0.0;
                int a = 0;
                for (int j = 0; j < k; ++j) {
                    int x = nbrs[j];
                    if (x == xt) { a = j + 1; continue; }
                    double cand = d_tv + t[x];
                    if (cand < delta) { d_tv = cand; a = j + 1; } else break;
                }
                double mass = t[xt] + d_tv;
                memcpy(ta, t, sizeof(double) * (size_t)V);
                for (int j = 0; j < a; ++j)
                    if (nbrs[j] != xt) ta[nbrs[j]] = 0.0;
                ta[xt] = mass;
                int best = 0;
                for (int x = 1; x < V; ++x)
                    if (ta[x] > ta[best]) best = x;   /* strict: the lowest index wins ties */
                double other = -1.0;
                for (int x = 0; x < V; ++x)
                    if (x != xt && ta[x] > other) other = ta[x];
                out_accept[i] = (best == xt) ? 1 : 0;
                out_token[i] = (best == xt) ? -1 : best;
                if (dg) { dg[0] = mass; dg[1] = other; dg[2] = (double)a; }
            }
        }
        free(buf);
    }
    return failed ? -1 : 0;
}

/* oracle_verify_probs with a choice of divergence (see oracle_verify_div). */
int oracle_verify_probs_div(const double* t, const double* g, int V, int xt,
                            const int32_t* nbrs, int k, int divergence, double delta,
                            double u_acc, double u_res,
                            int32_t* out_accept, int32_t* out_resample,
                            double* diag, double* rho_out, double* ta_out) {
    if (!t || !g || !nbrs || !out_accept || !out_resample) return -1;
    if (V < 1 || k < 1 || k > V || !(delta >= 0.0)) return -1;
    if (divergence != 0 && divergence != 1) return -1;
    if (!row_args_ok(V, xt, nbrs, k)) return -1;
    double* scratch = (double*)malloc(sizeof(double) * (size_t)V);
    if (!scratch) return -1;
    verify_probs(t, g, V, xt, nbrs, k, divergence, delta, u_acc, u_res, out_accept, out_resample,
                 diag, scratch, rho_out, ta_out);
    free(scratch);
    return 0;
}

int oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------- */
/* Walk of a drafted chain (Algorithm 1, the loop over t = 1..L)              */
/* ------------------------------------------------------------------------- */

/*
 * B chains of L candidates each; chain b owns rows b*L .. b*L+L-1 of accept /
 * resample in drafting order.  The drafts are taken while they are accepted;
 * at the first candidate that is not accepted the loop exits with that row's
 * resampled token.  out_len[b]: number of drafts kept.  out_next[b]: the
 * resampled token that follows them; -1 when all L were accepted (the caller
 * then samples the extra token from the target's next row); -2 when the first
 * row that was not accepted is an unusable one (accept = -1).
 */
int oracle_accept_chains(const int32_t* accept, const int32_t* resample, int B, int L,
                         int32_t* out_len, int32_t* out_next) {
    if (B < 0 || L < 1) return -1;
    if (B == 0) return 0;
    if (!accept || !resample || !out_len || !out_next) return -1;
    for (int b = 0; b < B; ++b) {
        int n = 0;
        int next = -1;
        for (int t = 0; t < L; ++t) {
            int a = accept[(size_t)b * L + t];
            if (a == 1) {
                n = n + 1;
            } else {
                next = (a == 0) ? resample[(size_t)b * L + t] : -2;
                break;
            }
        }
        out_len[b] = n;
        out_next[b] = next;
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Walk of a drafted tree (Algorithm 1 applied along the branches)            */
/* ------------------------------------------------------------------------- */

/*
 * B trees of M candidate nodes each (the paper verifies 60 candidates per
 * step, Appendix on experimental details, and leaves the tree rule to its
 * drafter); tree b owns rows b*M .. b*M+M-1.  parent[i] is the node, within
 * the tree, whose token precedes node i, or -1 when node i directly follows
 * the committed prefix; nodes are listed in drafting order, parent[i] < i.
 * accept / resample hold, per node, the outcome of verifying that node's token
 * against the distributions after its parent's prefix.
 *
 * The rule stated here (it reduces to the chain of Algorithm 1 when every node
 * has one child): standing at a node (at first the committed prefix, -1), its
 * children are tried in index order; the first child whose row says accepted
 * is taken and the walk continues from it.  A child with an unusable row
 * (accept < 0) met before any accepted one ends the walk with next = -2.  When
 * every child was rejected the walk ends with the resampled token of the first
 * child, the candidate Algorithm 1 tries at that position; when the node has
 * no child at all every draft on the branch was accepted and next = -1 (the
 * caller samples the extra token).  A tree with a parent outside [-1, i) is
 * not walked: len 0, next = -3.
 *
 * out_len[b]: number of accepted nodes.  out_path[b*M + j]: the j-th accepted
 * node for j < len, -1 beyond.  out_next[b] as above.
 */
int oracle_accept_trees(const int32_t* accept, const int32_t* resample, const int32_t* parent, int B, int M,
                        int32_t* out_len, int32_t* out_path, int32_t* out_next) {
    if (B < 0 || M < 1) return -1;
    if (B == 0) return 0;
    if (!accept || !resample || !parent || !out_len || !out_path || !out_next) return -1;
    for (int b = 0; b < B; ++b) {
        const int32_t* acc = accept + (size_t)b * M;
        const int32_t* res = resample + (size_t)b * M;
        const int32_t* par = parent + (size_t)b * M;
        int32_t* path = out_path + (size_t)b * M;
        for (int j = 0; j < M; ++j) path[j] = -1;
        int well_formed = 1;
        for (int i = 0; i < M; ++i)
            if (par[i] < -1 || par[i] >= i) well_formed = 0;
        if (!well_formed) {
            out_len[b] = 0;
            out_next[b] = -3;
            continue;
        }
        int cur = -1;
        int len = 0;
        int next = -1;
        for (;;) {
            int first_child = -1;
            int taken = -1;
            int unusable = 0;
            for (int i = cur + 1; i < M; ++i) {
                if (par[i] != cur) continue;
                if (first_child < 0) first_child = i;
                if (acc[i] == 1) { taken = i; break; }
                if (acc[i] < 0) { unusable = 1; break; }
            }
            if (taken >= 0) {
                path[len] = taken;
                len = len + 1;
                cur = taken;
                continue;
            }
            if (unusable) next = -2;
            else if (first_child >= 0) next = res[first_child];
            else next = -1;
            break;
        }
        out_len[b] = len;
        out_next[b] = next;
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Siblings verified one after the other against the residual of the ones     */
/* before (a second rule for draft trees; Section 2, Algorithm 1)             */
/* ------------------------------------------------------------------------- */

/*
 * Algorithm 1 tries one drafted token per position and, when it rejects it,
 * goes on with the residual distribution.  A draft tree offers several tokens
 * for one position.  The rule of oracle_accept_trees tests each of them
 * against the same undistorted target, which does not keep the target law even
 * at k = 1.  The rule here applies Algorithm 1's own step repeatedly: the
 * siblings x_1 .. x_m share the context's target t and drafter g;
 *     t_1 = t
 *     for j = 1 .. m:  verify x_j as Section 4.3 states it, with t_j in place of
 *                      the target (neighbourhood, mass and acceptance all on t_j);
 *                      accepted: x_j is taken;
 *                      rejected: t_{j+1} = the normalised residual of that
 *                                verification, max(0, t_{j,A} - g) / Z
 *     all rejected: the token that follows is drawn from t_{m+1}, i.e. it is the
 *                   resampled token of the last sibling's verification.
 * With tokens drawn independently from g and k = 1 (or delta = 0) this is
 * recursive rejection sampling and the emitted token follows t exactly.
 *
 * One sibling group on explicit probabilities.  xs[m]: the siblings' tokens in
 * the order they are tried; nbrs[j*k .. j*k+k): the table row of xs[j];
 * u_acc[m], u_res[m]: each sibling's own draws.  out_taken: index of the accepted
 * sibling or -1; out_next: the resampled token when all were rejected, else -1;
 * accept_prob[m] (optional): the probability of accepting sibling j given that
 * all before it were rejected (NaN for siblings not reached); final_dist[V]
 * (optional): t_{m+1}, computed even when a sibling was accepted (as if none were).
 * Returns 0, or -1 on bad arguments.
 */
int oracle_sibling_group_probs(const double* t, const double* g, int V, int m, const int32_t* xs,
                               const int32_t* nbrs, int k, int divergence, double delta,
                               const double* u_acc, const double* u_res, int32_t* out_taken,
                               int32_t* out_next, double* accept_prob, double* final_dist) {
    if (!t || !g || !xs || !nbrs || !u_acc || !u_res || !out_taken || !out_next) return -1;
    if (V < 1 || m < 1 || k < 1 || k > V || !(delta >= 0.0)) return -1;
    if (divergence != 0 && divergence != 1) return -1;
    for (int j = 0; j < m; ++j)
        if (!row_args_ok(V, xs[j], nbrs + (size_t)j * k, k)) return -1;
    double* buf = (double*)malloc(sizeof(double) * 3 * (size_t)V);
    if (!buf) return -1;
    double* cur = buf;
    double* rho = buf + V;
    double* scratch = buf + 2 * (size_t)V;
    memcpy(cur, t, sizeof(double) * (size_t)V);
    int taken = -1;
    int next = -1;
    for (int j = 0; j < m; ++j) {
        if (accept_prob) accept_prob[j] = NAN;
    }
    for (int j = 0; j < m; ++j) {
        int32_t acc, res;
        double diag[DIAG_COUNT];
        verify_probs(cur, g, V, xs[j], nbrs + (size_t)j * k, k, divergence, delta, u_acc[j], u_res[j],
                     &acc, &res, diag, scratch, rho, NULL);
        if (accept_prob) accept_prob[j] = diag[DIAG_ACCEPT_PROB];
        if (acc && taken < 0) {
            taken = j;
            if (!final_dist) break;
        }
        if (!acc && taken < 0) next = res;
        memcpy(cur, rho, sizeof(double) * (size_t)V);     /* the next sibling's target */
    }
    if (final_dist) memcpy(final_dist, cur, sizeof(double) * (size_t)V);
    *out_taken = taken;
    *out_next = taken >= 0 ? -1 : next;
    free(buf);
    return 0;
}

/*
 * Walk of B draft trees of M candidates under the rule above, from logits.
 * Candidate i of tree b (at b*M + i) reads logit row row_index[b*M+i] of both
 * matrices, drafts tokens[b*M+i] and owns uniforms[2*(b*M+i) .. +2); parent as
 * in oracle_accept_trees.  Standing at a node, its children are tried in index
 * order as one sibling group on the logit rows of the first child; the accepted
 * child is taken and the walk goes on from it.  out_len, out_path as in
 * oracle_accept_trees; out_next: the resampled token of the last child when
 * every child was rejected; -1 when the last node has no child; -2 when a child
 * that had to be tried is unusable (token, table entry or row index out of
 * range, unusable logits, or a row index other than the first child's); -3 for
 * a malformed parent array.  Returns 0, or -1 on bad arguments.
 */
int oracle_verify_trees_sequential(const float* target_logits, const float* draft_logits, int R, int V,
                                   int64_t row_stride, const int32_t* row_index, const int32_t* parent,
                                   int B, int M, const int32_t* tokens, const int32_t* knn, int k,
                                   int divergence, double delta, const float* uniforms, int32_t* out_len,
                                   int32_t* out_path, int32_t* out_next, int threads) {
    if (divergence != 0 && divergence != 1) return -1;
    if (B < 0 || M < 1 || R < 0 || V < 1 || k < 1 || k > V || row_stride < V || !(delta >= 0.0)) return -1;
    if (B == 0) return 0;
    if (R < 1) return -1;
    if (!target_logits || !draft_logits || !row_index || !parent || !tokens || !knn || !uniforms ||
        !out_len || !out_path || !out_next)
        return -1;
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel num_threads(threads > 0 ? threads : 1)
#endif
    {
        double* buf = (double*)malloc(sizeof(double) * 4 * (size_t)V);
        if (!buf) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        } else {
            double* cur = buf;
            double* g = buf + V;
            double* rho = buf + 2 * (size_t)V;
            double* scratch = buf + 3 * (size_t)V;
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
            for (int b = 0; b < B; ++b) {
                const int32_t* par = parent + (size_t)b * M;
                int32_t* path = out_path + (size_t)b * M;
                for (int j = 0; j < M; ++j) path[j] = -1;
                int well_formed = 1;
                for (int i = 0; i < M; ++i)
                    if (par[i] < -1 || par[i] >= i) well_formed = 0;
                if (!well_formed) {
                    out_len[b] = 0;
                    out_next[b] = -3;
                    continue;
                }
                int node = -1;
                int len = 0;
                int next = -1;
                for (;;) {
                    int taken = -1;
                    int group_row = -1;
                    int have_rows = 0;
                    int stop = 0;
                    next = -1;
                    for (int i = node + 1; i < M && !stop; ++i) {
                        if (par[i] != node) continue;
                        size_t c = (size_t)b * M + i;
                        int r = row_index[c];
                        int xt = tokens[c];
                        if (!have_rows) {             /* first child: the group's context */
                            group_row = r;
                            have_rows = 1;
                            int ok = (r >= 0 && r < R);
                            if (ok) ok = softmax_row(target_logits + (size_t)r * row_stride, V, cur) == 0;
                            if (ok) ok = softmax_row(draft_logits + (size_t)r * row_stride, V, g) == 0;
                            if (!ok) { next = -2; stop = 1; break; }
                        }
                        if (r != group_row || xt < 0 || xt >= V || !row_args_ok(V, xt, knn + (size_t)xt * k, k)) {
                            next = -2;
                            stop = 1;
                            break;
                        }
                        int32_t acc, res;
                        verify_probs(cur, g, V, xt, knn + (size_t)xt * k, k, divergence, delta,
                                     (double)uniforms[2 * c], (double)uniforms[2 * c + 1], &acc, &res, NULL,
                                     scratch, rho, NULL);
                        if (acc) {
                            taken = i;
                            stop = 1;
                        } else {
                            next = res;                                  /* so far the last rejected child */
                            memcpy(cur, rho, sizeof(double) * (size_t)V);  /* the next sibling's target */
                        }
                    }
                    if (taken >= 0) {
                        path[len] = taken;
                        len = len + 1;
                        node = taken;
                        continue;
                    }
                    break;     /* next: -1 no child, -2 unusable, else the last child's resampled token */
                }
                out_len[b] = len;
                out_next[b] = next;
            }
        }
        free(buf);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------- */
/* Random neighbourhoods (Section 5.3.1 and Table 3, the "random selection"   */
/* row of the ablation on latent proximity measures)                          */
/* ------------------------------------------------------------------------- */

/*
 * Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11), written out: ten rounds
 * of two 32x32 -> 64 bit multiplications, the key advanced by the Weyl
 * constants between rounds.
 */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

typedef struct { uint32_t key; int32_t token; } keyed_token;

static int cmp_keyed_token(const void* a, const void* b) {
    const keyed_token* x = (const keyed_token*)a;
    const keyed_token* y = (const keyed_token*)b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    return (x->token > y->token) - (x->token < y->token);
}

/*
 * The paper only says that the k tokens are selected at random.  The reading
 * taken here: B_k(x) holds x itself in slot 0 and then k-1 other tokens, a
 * uniform sample without replacement in uniformly random order, fixed once
 * per token like the nearest-neighbour table.  Every pair (x, y) gets a 32-bit
 * key: word y mod 4 of Philox4x32-10 at counter (y div 4, x, 0, 0) under the
 * key (seed low word, seed high word); row x lists the other tokens by
 * increasing (key, token).  Writes rows r0 .. r1-1 into out[(r1-r0) * k].
 */
int oracle_build_random_rows(int V, int k, uint64_t seed, int r0, int r1, int32_t* out, int threads) {
    if (V < 1 || k < 1 || k > V || r0 < 0 || r1 > V || r0 > r1 || !out) return -1;
    const uint32_t key[2] = {(uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32)};
    int failed = 0;
    (void)threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 16) num_threads(threads > 0 ? threads : 1)
#endif
    for (int x = r0; x < r1; ++x) {
        keyed_token* others = (keyed_token*)malloc(sizeof(keyed_token) * (size_t)V);
        if (!others) {
            failed = 1;
            continue;
        }
        int n = 0;
        for (int y = 0; y < V; ++y) {
            if (y == x) continue;
            uint32_t ctr[4] = {(uint32_t)(y / 4), (uint32_t)x, 0u, 0u};
            uint32_t words[4];
            oracle_philox4x32_10(ctr, key, words);
            others[n].key = words[y % 4];
            others[n].token = y;
            n = n + 1;
        }
        qsort(others, (size_t)n, sizeof(keyed_token), cmp_keyed_token);
        int32_t* row = out + (size_t)(x - r0) * k;
        row[0] = x;
        for (int j = 1; j < k; ++j) row[j] = others[j - 1].token;
        free(others);
    }
    return failed ? -2 : 0;
}
