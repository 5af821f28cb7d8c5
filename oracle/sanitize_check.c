/*
 * sanitize_check.c -- drives every entry point of ada_oracle.c on small seeded inputs (ragged sizes, r = 1, r = T,
 * zero rows, forced decisions, both cross readings, greedy variant, causal attention) so that the oracle can be run
 * under AddressSanitizer and UndefinedBehaviorSanitizer:
 *     gcc -O1 -g -fopenmp -fsanitize=address,undefined -fno-sanitize-recover=all ada_oracle.c sanitize_check.c -lm
 * TEST INFRASTRUCTURE ONLY (it checks the checker's memory safety, not the method).  Exit status 0 = every call
 * returned success and the sanitizers found nothing.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int ada_oracle_normalize(const double* X, int T, int d, double* Xhat, double* norms);
int ada_oracle_gram(const double* X, int T, int d, double* G);
int ada_oracle_select_full(const double* X, int T, int d, double tau, int greedy, const int8_t* force, uint8_t* mask,
                           double* gamma, int32_t* r_out, uint64_t* gram_ops);
int ada_oracle_gamma_full_rows(const double* X, int T, int d, const int32_t* rows, int n, double* gamma_out);
int ada_oracle_cascade_step(const double* X, int T, int d, double tau, const int32_t* prev_idx, int r, unsigned flags,
                            const int8_t* force, int32_t* idx, int32_t* adds, int32_t* removes, int32_t* counts,
                            uint64_t* gram_ops, double* gamma, double* gamma_all);
int ada_oracle_assign_nearest(const double* X, int T, int d, const int32_t* idx, int r, int32_t* assign, double* corr);
int ada_oracle_attention_compressed(const double* Q, const double* K, const double* V, int T, int H, int d_h,
                                    const int32_t* idx, int r, const int32_t* assign, unsigned flags, double* out);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static double rnd(void) {                                /* xorshift, uniform in (-1, 1) */
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 4503599627370496.0 - 1.0;
}

#define CHECK(call) do { int rc_ = (call); if (rc_ != 0) { fprintf(stderr, "%s -> %d (T=%d d=%d)\n", #call, rc_, T, d); return 1; } } while (0)

static int one_shape(int T, int d, int K) {
    double* X = malloc(sizeof(double) * T * d);
    double* Xh = malloc(sizeof(double) * T * d);
    double* nr = malloc(sizeof(double) * T);
    double* G = malloc(sizeof(double) * T * T);
    double* gam = malloc(sizeof(double) * T);
    double* gall = malloc(sizeof(double) * T);
    uint8_t* mask = malloc(T);
    int8_t* force = malloc(T);
    int32_t *idx = malloc(4 * T), *adds = malloc(4 * T), *rem = malloc(4 * T), *prev = malloc(4 * T), *rows = malloc(4 * T);
    int32_t* assign = malloc(4 * T);
    double* cen = malloc(sizeof(double) * K * d);
    for (int i = 0; i < K * d; ++i) cen[i] = rnd();
    for (int t = 0; t < T; ++t) {
        const int k = (int)((rnd() + 1.0) * 0.5 * K) % K;
        for (int j = 0; j < d; ++j) X[(size_t)t * d + j] = cen[k * d + j] + 0.001 * rnd();
    }
    if (T > 3) for (int j = 0; j < d; ++j) X[(size_t)3 * d + j] = 0.0;          /* a zero row */
    CHECK(ada_oracle_normalize(X, T, d, Xh, nr));
    CHECK(ada_oracle_gram(X, T, d, G));
    int32_t r = 0, counts[4];
    uint64_t ops = 0;
    for (int greedy = 0; greedy < 2; ++greedy) CHECK(ada_oracle_select_full(X, T, d, 0.1, greedy, NULL, mask, gam, &r, &ops));
    for (int t = 0; t < T; ++t) { force[t] = (int8_t)(t % 3 == 0 ? (t % 2) : -1); rows[t] = T - 1 - t; }
    CHECK(ada_oracle_select_full(X, T, d, 0.1, 0, force, mask, gam, &r, &ops));
    CHECK(ada_oracle_select_full(X, T, d, 0.3, 0, NULL, mask, NULL, &r, NULL));
    CHECK(ada_oracle_gamma_full_rows(X, T, d, rows, T, gam));
    int n = 0;
    for (int t = 0; t < T; ++t) if (mask[t]) prev[n++] = t;
    for (int variant = 0; variant < 4; ++variant) {
        int rr = n;
        if (variant == 1) { rr = 1; prev[0] = 0; }
        if (variant == 2) { rr = T; for (int t = 0; t < T; ++t) prev[t] = t; }
        if (variant == 3) { rr = (T + 1) / 2; for (int t = 0; t < rr; ++t) prev[t] = 2 * t; }
        for (unsigned flags = 0; flags < 2; ++flags) {
            CHECK(ada_oracle_cascade_step(X, T, d, 0.1, prev, rr, flags, NULL, idx, adds, rem, counts, &ops, gam, gall));
            CHECK(ada_oracle_cascade_step(X, T, d, 0.1, prev, rr, flags, force, idx, adds, rem, counts, NULL, NULL, NULL));
        }
        CHECK(ada_oracle_assign_nearest(X, T, d, prev, rr, assign, gam));
        CHECK(ada_oracle_assign_nearest(X, T, d, prev, rr, assign, NULL));
        for (int H = 1; H <= 2; ++H) {
            if (d % H) continue;
            double* out = malloc(sizeof(double) * T * d);
            for (unsigned flags = 0; flags < 2; ++flags)
                CHECK(ada_oracle_attention_compressed(X, Xh, X, T, H, d / H, prev, rr, assign, flags, out));
            free(out);
        }
    }
    free(X); free(Xh); free(nr); free(G); free(gam); free(gall); free(mask); free(force);
    free(idx); free(adds); free(rem); free(prev); free(rows); free(assign); free(cen);
    return 0;
}

int main(void) {
    const int shapes[][3] = {{1, 1, 1}, {2, 3, 1}, {5, 7, 2}, {33, 16, 5}, {64, 10, 9}, {129, 24, 17}};
    for (unsigned i = 0; i < sizeof(shapes) / sizeof(shapes[0]); ++i)
        if (one_shape(shapes[i][0], shapes[i][1], shapes[i][2])) return 1;
    puts("oracle sanitize check ok");
    return 0;
}
