/*
 * Driver that runs the CPU oracle under AddressSanitizer / UndefinedBehaviorSanitizer.
 * Built by tests/test_oracle_sanitizers.py together with oracle/lantern_oracle.c; reads a
 * stream of commands (int32 opcode, int32 / float64 parameters, raw arrays) from the file named
 * by argv[1] and writes every call's outputs, raw, to the file named by argv[2].  Any sanitizer
 * report aborts the process (-fno-sanitize-recover), which the test sees as a failure.
 */
#include "../oracle/lantern_oracle.c"

#include <stdio.h>

static FILE* fin;
static FILE* fout;

static void* rd(size_t bytes) {
    void* p = malloc(bytes ? bytes : 1);
    if (!p || fread(p, 1, bytes, fin) != bytes) {
        fprintf(stderr, "short read\n");
        exit(3);
    }
    return p;
}
static int32_t rd_i32(void) { int32_t v; if (fread(&v, 4, 1, fin) != 1) exit(3); return v; }
static double rd_f64(void) { double v; if (fread(&v, 8, 1, fin) != 1) exit(3); return v; }
static void wr(const void* p, size_t bytes) { if (fwrite(p, 1, bytes, fout) != bytes) exit(4); }
static void wr_i32(int32_t v) { wr(&v, 4); }

int main(int argc, char** argv) {
    if (argc != 3) return 2;
    fin = fopen(argv[1], "rb");
    fout = fopen(argv[2], "wb");
    if (!fin || !fout) return 2;
    int32_t op;
    while (fread(&op, 4, 1, fin) == 1) {
        if (op == 1) {          /* one verification on explicit probabilities */
            int V = rd_i32(), k = rd_i32(), xt = rd_i32(), divergence = rd_i32();
            double delta = rd_f64(), u_acc = rd_f64(), u_res = rd_f64();
            double* t = rd(sizeof(double) * (size_t)V);
            double* g = rd(sizeof(double) * (size_t)V);
            int32_t* nb = rd(4 * (size_t)k);
            int32_t acc = -7, res = -7;
            double diag[DIAG_COUNT];
            double* rho = malloc(sizeof(double) * (size_t)V);
            double* ta = malloc(sizeof(double) * (size_t)V);
            int rc = oracle_verify_probs_div(t, g, V, xt, nb, k, divergence, delta, u_acc, u_res, &acc, &res, diag,
                                             rho, ta);
            wr_i32(rc); wr_i32(acc); wr_i32(res);
            if (rc == 0) { wr(diag, sizeof diag); wr(rho, sizeof(double) * (size_t)V); wr(ta, sizeof(double) * (size_t)V); }
            free(t); free(g); free(nb); free(rho); free(ta);
        } else if (op == 2) {   /* rows of the neighbour table */
            int V = rd_i32(), d = rd_i32(), k = rd_i32(), metric = rd_i32(), r0 = rd_i32(), r1 = rd_i32(),
                threads = rd_i32();
            float* cb = rd(4 * (size_t)V * d);
            int32_t* out = malloc(4 * (size_t)(r1 - r0) * k + 4);
            int rc = oracle_build_knn_rows(cb, V, d, k, metric, r0, r1, out, threads);
            wr_i32(rc);
            if (rc == 0) wr(out, 4 * (size_t)(r1 - r0) * k);
            free(cb); free(out);
        } else if (op == 3) {   /* N verifications from logits */
            int N = rd_i32(), V = rd_i32(), k = rd_i32(), divergence = rd_i32(), threads = rd_i32();
            double delta = rd_f64();
            float* tl = rd(4 * (size_t)N * V);
            float* dl = rd(4 * (size_t)N * V);
            int32_t* tok = rd(4 * (size_t)N);
            int32_t* knn = rd(4 * (size_t)V * k);
            float* un = rd(4 * 2 * (size_t)N);
            int32_t* acc = malloc(4 * (size_t)N + 4);
            int32_t* res = malloc(4 * (size_t)N + 4);
            double* diag = malloc(sizeof(double) * (size_t)N * DIAG_COUNT + 8);
            int rc = oracle_verify_div(tl, dl, N, V, V, tok, knn, k, divergence, delta, un, acc, res, diag, threads);
            wr_i32(rc);
            if (rc == 0) { wr(acc, 4 * (size_t)N); wr(res, 4 * (size_t)N); wr(diag, sizeof(double) * (size_t)N * DIAG_COUNT); }
            free(tl); free(dl); free(tok); free(knn); free(un); free(acc); free(res); free(diag);
        } else if (op == 4) {   /* greedy variant */
            int N = rd_i32(), V = rd_i32(), k = rd_i32(), threads = rd_i32();
            double delta = rd_f64();
            float* tl = rd(4 * (size_t)N * V);
            int32_t* tok = rd(4 * (size_t)N);
            int32_t* knn = rd(4 * (size_t)V * k);
            int32_t* acc = malloc(4 * (size_t)N + 4);
            int32_t* out = malloc(4 * (size_t)N + 4);
            double* diag = malloc(sizeof(double) * 3 * (size_t)N + 8);
            int rc = oracle_verify_greedy(tl, N, V, V, tok, knn, k, delta, acc, out, diag, threads);
            wr_i32(rc);
            if (rc == 0) { wr(acc, 4 * (size_t)N); wr(out, 4 * (size_t)N); }
            free(tl); free(tok); free(knn); free(acc); free(out); free(diag);
        } else if (op == 5) {   /* chain walk */
            int B = rd_i32(), L = rd_i32();
            int32_t* acc = rd(4 * (size_t)B * L);
            int32_t* res = rd(4 * (size_t)B * L);
            int32_t* len = malloc(4 * (size_t)B + 4);
            int32_t* next = malloc(4 * (size_t)B + 4);
            int rc = oracle_accept_chains(acc, res, B, L, len, next);
            wr_i32(rc);
            if (rc == 0) { wr(len, 4 * (size_t)B); wr(next, 4 * (size_t)B); }
            free(acc); free(res); free(len); free(next);
        } else if (op == 6) {   /* tree walk */
            int B = rd_i32(), M = rd_i32();
            int32_t* acc = rd(4 * (size_t)B * M);
            int32_t* res = rd(4 * (size_t)B * M);
            int32_t* par = rd(4 * (size_t)B * M);
            int32_t* len = malloc(4 * (size_t)B + 4);
            int32_t* path = malloc(4 * (size_t)B * M + 4);
            int32_t* next = malloc(4 * (size_t)B + 4);
            int rc = oracle_accept_trees(acc, res, par, B, M, len, path, next);
            wr_i32(rc);
            if (rc == 0) { wr(len, 4 * (size_t)B); wr(path, 4 * (size_t)B * M); wr(next, 4 * (size_t)B); }
            free(acc); free(res); free(par); free(len); free(path); free(next);
        } else if (op == 7) {   /* rows of the random table */
            int V = rd_i32(), k = rd_i32(), r0 = rd_i32(), r1 = rd_i32(), threads = rd_i32();
            uint64_t seed;
            if (fread(&seed, 8, 1, fin) != 1) exit(3);
            int32_t* out = malloc(4 * (size_t)(r1 - r0) * k + 4);
            int rc = oracle_build_random_rows(V, k, seed, r0, r1, out, threads);
            wr_i32(rc);
            if (rc == 0) wr(out, 4 * (size_t)(r1 - r0) * k);
            free(out);
        } else if (op == 8) {   /* tree walk under the sequential-residual sibling rule, from logits */
            int R = rd_i32(), V = rd_i32(), B = rd_i32(), M = rd_i32(), k = rd_i32(), divergence = rd_i32(),
                threads = rd_i32();
            double delta = rd_f64();
            float* tl = rd(4 * (size_t)R * V);
            float* dl = rd(4 * (size_t)R * V);
            int32_t* ri = rd(4 * (size_t)B * M);
            int32_t* par = rd(4 * (size_t)B * M);
            int32_t* tok = rd(4 * (size_t)B * M);
            int32_t* knn = rd(4 * (size_t)V * k);
            float* un = rd(4 * 2 * (size_t)B * M);
            int32_t* len = malloc(4 * (size_t)B + 4);
            int32_t* path = malloc(4 * (size_t)B * M + 4);
            int32_t* next = malloc(4 * (size_t)B + 4);
            int rc = oracle_verify_trees_sequential(tl, dl, R, V, V, ri, par, B, M, tok, knn, k, divergence, delta, un,
                                                    len, path, next, threads);
            wr_i32(rc);
            if (rc == 0) { wr(len, 4 * (size_t)B); wr(path, 4 * (size_t)B * M); wr(next, 4 * (size_t)B); }
            free(tl); free(dl); free(ri); free(par); free(tok); free(knn); free(un); free(len); free(path); free(next);
        } else {
            fprintf(stderr, "unknown opcode %d\n", op);
            return 5;
        }
    }
    fclose(fin);
    if (fclose(fout) != 0) return 4;
    return 0;
}
