/*
 * ada_oracle.c -- float64 CPU oracle for Gram-threshold representative-token
 * selection and the cascade step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute.  It shares no code, header, table or helper with the
 * HIP path, and nothing in the product path may call it: only the tests, the
 * smoke check and the benchmark's CPU-baseline leg do.
 *
 * Every function is the paper's definition written out:
 *   - row normalisation and Gram matrix ......... Section 2.1
 *   - lower-triangular max correlation, the set R  Definition "Gram threshold" (Section 2.2)
 *   - cascade step ............................... Algorithm 1 (Section 4.1)
 *   - Gram-operation count ....................... eq. (6) and Table 6 (one operation = one Gram entry)
 *   - nearest-representative assignment .......... Section 2.3 (attention on the representative set)
 *   - attention on the representative set ........ eq. (1) (Section 2.3)
 *
 * There is no blocking, fusion or reordering: a Gram entry is one left-to-right
 * dot product of two normalised rows in double precision.  The only concession
 * to speed is an OpenMP "parallel for" over independent tokens, which changes no
 * arithmetic.
 *
 * Readings taken where the paper is silent or at odds with itself (they are the
 * library's readings too, and are listed with their reasons in the design notes):
 *   R1  full selection compares token t against ALL earlier tokens (the
 *       Definition), not only earlier representatives (the Section 2.5 remark);
 *       the latter is available as `greedy` for study.
 *   R2  rep validation maxes over all earlier INHERITED representatives, also
 *       those that are themselves being removed (Algorithm 1, step 4).
 *   R3  the cross step maxes over all valid representatives with no order
 *       restriction (Algorithm 1, step 8); ADA_ORACLE_CROSS_EARLIER_ONLY
 *       restricts it to s < t, the form the proof of the superset proposition needs.
 *   R4  |G| is used everywhere (Definition and Algorithm 1).
 *   R5  a zero row normalises to the zero vector: all its cosines are 0.
 *   R6  gram_ops(full) = T*T; gram_ops(cascade) = r*r + (T-r)*r_valid.
 *   R7  strict "<" against 1 - tau^2 evaluated in double; the empty max is 0.
 *   R8  removed representatives are not reconsidered as additions in the same step
 *       (they are not in the complement of the inherited set).
 *   R15 eq. (1) is a plain softmax over all members of R (no causal mask is printed); ADA_ORACLE_ATTN_CAUSAL
 *       restricts a representative's keys to members of R that are not later than itself in the sequence, as
 *       the decoder-only models of Section 6 would.  Heads lie side by side in a row (head h owns columns
 *       h*d_h .. (h+1)*d_h - 1); every token outside R takes its representative's output row unchanged.
 *   R14 nearest representative: the maximum of |G_ts| runs over the WHOLE set R handed in (earlier and later
 *       tokens alike, as Section 2.3 states it); a member of R is its own representative with correlation 1;
 *       among equal maxima the smallest token id is reported (any of them satisfies the text).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ADA_ORACLE_OK 0
#define ADA_ORACLE_ERR_ARG 1
#define ADA_ORACLE_ERR_INDEX 2
#define ADA_ORACLE_ERR_NOMEM 3

#define ADA_ORACLE_CROSS_EARLIER_ONLY 1u
#define ADA_ORACLE_ATTN_CAUSAL 1u

int ada_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sets the number of OpenMP threads later calls use (n >= 1); returns the previous maximum.  No arithmetic depends
 * on it: every Gram entry is one thread's left-to-right dot product. */
int ada_oracle_set_threads(int n) {
#ifdef _OPENMP
    const int before = omp_get_max_threads();
    if (n >= 1) omp_set_num_threads(n);
    return before;
#else
    (void)n;
    return 1;
#endif
}

/* Section 2.1: Xhat = D^{-1} X with D = diag(||x_t||).  Reading R5 for a zero row. */
int ada_oracle_normalize(const double* X, int T, int d, double* Xhat, double* norms) {
    if (!X || !Xhat || T < 1 || d < 1) return ADA_ORACLE_ERR_ARG;
    for (int t = 0; t < T; ++t) {
        double ss = 0.0;
        for (int k = 0; k < d; ++k) ss += X[(size_t)t * d + k] * X[(size_t)t * d + k];
        double n = sqrt(ss);
        if (norms) norms[t] = n;
        for (int k = 0; k < d; ++k) Xhat[(size_t)t * d + k] = (n > 0.0) ? X[(size_t)t * d + k] / n : 0.0;
    }
    return ADA_ORACLE_OK;
}

/* One Gram entry G_st = <xhat_s, xhat_t> (Section 2.1). */
static double gram_entry(const double* Xhat, int d, int s, int t) {
    const double* a = Xhat + (size_t)s * d;
    const double* b = Xhat + (size_t)t * d;
    double acc = 0.0;
    for (int k = 0; k < d; ++k) acc += a[k] * b[k];
    return acc;
}

/* Section 2.1: the whole T x T Gram matrix, row-major, for small T (tests). */
int ada_oracle_gram(const double* X, int T, int d, double* G) {
    if (!X || !G || T < 1 || d < 1) return ADA_ORACLE_ERR_ARG;
    double* Xhat = (double*)malloc((size_t)T * d * sizeof(double));
    if (!Xhat) return ADA_ORACLE_ERR_NOMEM;
    ada_oracle_normalize(X, T, d, Xhat, NULL);
    for (int s = 0; s < T; ++s)
        for (int t = 0; t < T; ++t) G[(size_t)s * T + t] = gram_entry(Xhat, d, s, t);
    free(Xhat);
    return ADA_ORACLE_OK;
}

static int decide(double gamma, double thr, const int8_t* force, int t) {
    if (force && force[t] >= 0) return force[t] ? 1 : 0;
    return gamma < thr;
}

/*
 * Definition "Gram threshold": gamma_t = max_{s<t} |G_st|, token t is representative
 * iff gamma_t < 1 - tau^2.  The first token has an empty max (gamma_0 = 0) and is
 * always representative.
 *
 * greedy != 0 selects the Section 2.5 variant (compare against earlier
 * REPRESENTATIVES only); it is sequential and is not what the library computes.
 * force (optional, [T]): -1 = decide from gamma; 0 / 1 = take this decision for
 * token t instead (used by parity tests for tokens whose gamma lies within the
 * stated band around the threshold).
 */
int ada_oracle_select_full(const double* X, int T, int d, double tau, int greedy, const int8_t* force,
                           uint8_t* mask, double* gamma, int32_t* r_out, uint64_t* gram_ops) {
    if (!X || !mask || T < 1 || d < 1) return ADA_ORACLE_ERR_ARG;
    if (!(tau > 0.0 && tau < 1.0)) return ADA_ORACLE_ERR_ARG;
    const double thr = 1.0 - tau * tau;
    double* Xhat = (double*)malloc((size_t)T * d * sizeof(double));
    double* g = (double*)malloc((size_t)T * sizeof(double));
    if (!Xhat || !g) { free(Xhat); free(g); return ADA_ORACLE_ERR_NOMEM; }
    ada_oracle_normalize(X, T, d, Xhat, NULL);
    if (!greedy) {
#pragma omp parallel for schedule(dynamic, 8)
        for (int t = 0; t < T; ++t) {
            double m = 0.0;
            for (int s = 0; s < t; ++s) {
                double c = fabs(gram_entry(Xhat, d, s, t));
                if (c > m) m = c;
            }
            g[t] = m;
        }
        for (int t = 0; t < T; ++t) mask[t] = (uint8_t)decide(g[t], thr, force, t);
    } else {
        for (int t = 0; t < T; ++t) {
            double m = 0.0;
            for (int s = 0; s < t; ++s) {
                if (!mask[s]) continue;
                double c = fabs(gram_entry(Xhat, d, s, t));
                if (c > m) m = c;
            }
            g[t] = m;
            mask[t] = (uint8_t)decide(m, thr, force, t);
        }
    }
    int r = 0;
    for (int t = 0; t < T; ++t) r += mask[t];
    if (gamma) memcpy(gamma, g, (size_t)T * sizeof(double));
    if (r_out) *r_out = r;
    if (gram_ops) *gram_ops = (uint64_t)T * (uint64_t)T; /* Table 6: L*T^2 entries for independent selection */
    free(Xhat);
    free(g);
    return ADA_ORACLE_OK;
}

/*
 * gamma_t of the Definition for a chosen list of tokens only, so that full-size
 * inputs can be checked on sampled outputs.  rows[i] in [0,T).
 */
int ada_oracle_gamma_full_rows(const double* X, int T, int d, const int32_t* rows, int n, double* gamma_out) {
    if (!X || !rows || !gamma_out || T < 1 || d < 1 || n < 0) return ADA_ORACLE_ERR_ARG;
    for (int i = 0; i < n; ++i)
        if (rows[i] < 0 || rows[i] >= T) return ADA_ORACLE_ERR_INDEX;
    double* Xhat = (double*)malloc((size_t)T * d * sizeof(double));
    if (!Xhat) return ADA_ORACLE_ERR_NOMEM;
    ada_oracle_normalize(X, T, d, Xhat, NULL);
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n; ++i) {
        int t = rows[i];
        double m = 0.0;
        for (int s = 0; s < t; ++s) {
            double c = fabs(gram_entry(Xhat, d, s, t));
            if (c > m) m = c;
        }
        gamma_out[i] = m;
    }
    free(Xhat);
    return ADA_ORACLE_OK;
}

/*
 * Algorithm 1 (Cascade Token Selection), step by step.
 *
 * prev_idx[r]: the inherited set R^(l) as strictly ascending token ids.
 * flags: ADA_ORACLE_CROSS_EARLIER_ONLY -> reading R3's variant.
 * force (optional, [T]): as in ada_oracle_select_full; for an inherited
 *   representative it overrides the validity decision of step 5, for any other
 *   token the addition decision of step 9.
 * Outputs (caller-allocated): idx[T] ascending R^(l+1); adds[T]; removes[r];
 *   counts[3] = {|R^(l+1)|, |adds|, |removes|}; gram_ops (reading R6);
 *   gamma[T] (optional): gamma^rep for inherited tokens, gamma^cross for the others.
 *   gamma_all[T] (optional): as gamma, but for a non-inherited token the max runs over ALL inherited
 *   representatives instead of the valid ones only (an auxiliary quantity: the cross-Gram row maximum before step 5's
 *   validity is applied; it never enters a decision).
 */
int ada_oracle_cascade_step(const double* X, int T, int d, double tau, const int32_t* prev_idx, int r,
                            unsigned flags, const int8_t* force, int32_t* idx, int32_t* adds,
                            int32_t* removes, int32_t* counts, uint64_t* gram_ops, double* gamma,
                            double* gamma_all) {
    if (!X || !prev_idx || !idx || !adds || !removes || !counts || T < 1 || d < 1) return ADA_ORACLE_ERR_ARG;
    if (!(tau > 0.0 && tau < 1.0)) return ADA_ORACLE_ERR_ARG;
    if (r < 1 || r > T) return ADA_ORACLE_ERR_ARG;
    for (int j = 0; j < r; ++j) {
        if (prev_idx[j] < 0 || prev_idx[j] >= T) return ADA_ORACLE_ERR_INDEX;
        if (j > 0 && prev_idx[j] <= prev_idx[j - 1]) return ADA_ORACLE_ERR_INDEX;
    }
    const double thr = 1.0 - tau * tau;
    const int earlier_only = (flags & ADA_ORACLE_CROSS_EARLIER_ONLY) != 0;

    double* Xhat = (double*)malloc((size_t)T * d * sizeof(double));
    double* g = (double*)calloc((size_t)T, sizeof(double));
    double* g_all = (double*)calloc((size_t)T, sizeof(double));
    uint8_t* inherited = (uint8_t*)calloc((size_t)T, 1);
    uint8_t* valid = (uint8_t*)calloc((size_t)r, 1);
    uint8_t* is_new = (uint8_t*)calloc((size_t)T, 1);
    if (!Xhat || !g || !g_all || !inherited || !valid || !is_new) {
        free(Xhat); free(g); free(g_all); free(inherited); free(valid); free(is_new);
        return ADA_ORACLE_ERR_NOMEM;
    }

    /* step 1: row-normalise */
    ada_oracle_normalize(X, T, d, Xhat, NULL);
    /* step 2: the inherited rows are Xhat[prev_idx[j]]; mark them so the complement is known (step 6) */
    for (int j = 0; j < r; ++j) inherited[prev_idx[j]] = 1;

    /* steps 3-4: gamma^rep_s = max over earlier inherited representatives s' < s of |G_R(s, s')| */
#pragma omp parallel for schedule(dynamic, 8)
    for (int j = 0; j < r; ++j) {
        double m = 0.0;
        for (int i = 0; i < j; ++i) {
            double c = fabs(gram_entry(Xhat, d, prev_idx[i], prev_idx[j]));
            if (c > m) m = c;
        }
        g[prev_idx[j]] = m;
        g_all[prev_idx[j]] = m;
    }
    /* step 5: R_valid */
    int r_valid = 0;
    for (int j = 0; j < r; ++j) {
        valid[j] = (uint8_t)decide(g[prev_idx[j]], thr, force, prev_idx[j]);
        r_valid += valid[j];
    }

    /* steps 6-8: gamma^cross_t = max over s in R_valid of |C(t, s)| for every non-inherited t */
#pragma omp parallel for schedule(dynamic, 8)
    for (int t = 0; t < T; ++t) {
        if (inherited[t]) continue;
        double m = 0.0, m_all = 0.0;
        for (int j = 0; j < r; ++j) {
            if (earlier_only && prev_idx[j] >= t) continue;
            double c = fabs(gram_entry(Xhat, d, t, prev_idx[j]));
            if (c > m_all) m_all = c;               /* auxiliary: before validity */
            if (!valid[j]) continue;
            if (c > m) m = c;
        }
        g[t] = m;
        g_all[t] = m_all;
    }
    /* step 9: R_new */
    for (int t = 0; t < T; ++t)
        if (!inherited[t]) is_new[t] = (uint8_t)decide(g[t], thr, force, t);

    /* step 10: R^(l+1) = R_valid U R_new, ascending; additions and removals for eq. (8) */
    int n_idx = 0, n_add = 0, n_rem = 0, j = 0;
    for (int t = 0; t < T; ++t) {
        if (inherited[t]) {
            if (valid[j]) idx[n_idx++] = t; else removes[n_rem++] = t;
            ++j;
        } else if (is_new[t]) {
            idx[n_idx++] = t;
            adds[n_add++] = t;
        }
    }
    counts[0] = n_idx; counts[1] = n_add; counts[2] = n_rem;
    /* reading R6: entries Algorithm 1 forms -- r x r among the inherited, (T-r) x r_valid across */
    if (gram_ops) *gram_ops = (uint64_t)r * (uint64_t)r + (uint64_t)(T - r) * (uint64_t)r_valid;
    if (gamma) memcpy(gamma, g, (size_t)T * sizeof(double));
    if (gamma_all) memcpy(gamma_all, g_all, (size_t)T * sizeof(double));

    free(Xhat); free(g); free(g_all); free(inherited); free(valid); free(is_new);
    return ADA_ORACLE_OK;
}

/*
 * Section 2.3: a token outside R takes the attention output of its nearest representative, the s* in R that
 * maximises |G_{t s*}| (reading R14).  idx[r]: R as strictly ascending token ids.
 * Outputs: assign[T] = token id of s*(t) (t itself for t in R); corr[T] (optional) = |G_{t s*}| (1 for t in R).
 */
int ada_oracle_assign_nearest(const double* X, int T, int d, const int32_t* idx, int r, int32_t* assign,
                              double* corr) {
    if (!X || !idx || !assign || T < 1 || d < 1) return ADA_ORACLE_ERR_ARG;
    if (r < 1 || r > T) return ADA_ORACLE_ERR_ARG;
    for (int j = 0; j < r; ++j) {
        if (idx[j] < 0 || idx[j] >= T) return ADA_ORACLE_ERR_INDEX;
        if (j > 0 && idx[j] <= idx[j - 1]) return ADA_ORACLE_ERR_INDEX;
    }
    double* Xhat = (double*)malloc((size_t)T * d * sizeof(double));
    uint8_t* in_R = (uint8_t*)calloc((size_t)T, 1);
    if (!Xhat || !in_R) { free(Xhat); free(in_R); return ADA_ORACLE_ERR_NOMEM; }
    ada_oracle_normalize(X, T, d, Xhat, NULL);
    for (int j = 0; j < r; ++j) in_R[idx[j]] = 1;
#pragma omp parallel for schedule(dynamic, 8)
    for (int t = 0; t < T; ++t) {
        if (in_R[t]) {
            assign[t] = t;
            if (corr) corr[t] = 1.0;
            continue;
        }
        double best = -1.0;
        int arg = idx[0];
        for (int j = 0; j < r; ++j) {                 /* ascending token ids: ">" keeps the smallest among equals */
            double c = fabs(gram_entry(Xhat, d, t, idx[j]));
            if (c > best) { best = c; arg = idx[j]; }
        }
        assign[t] = arg;
        if (corr) corr[t] = best;
    }
    free(Xhat); free(in_R);
    return ADA_ORACLE_OK;
}

/*
 * eq. (1) (Section 2.3): per head, O_R = softmax(Q_R K_R^T / sqrt(d_h)) V_R on the r representative rows, then every
 * token t takes the row of its representative assign[t] (reading R15).
 * Q, K, V: T x (H*d_h) row-major.  idx[r]: R ascending.  assign[T]: members of R (as ada_oracle_assign_nearest returns).
 * flags: ADA_ORACLE_ATTN_CAUSAL.  out: T x (H*d_h).
 */
int ada_oracle_attention_compressed(const double* Q, const double* K, const double* V, int T, int H, int d_h,
                                    const int32_t* idx, int r, const int32_t* assign, unsigned flags, double* out) {
    if (!Q || !K || !V || !idx || !assign || !out || T < 1 || H < 1 || d_h < 1) return ADA_ORACLE_ERR_ARG;
    if (r < 1 || r > T) return ADA_ORACLE_ERR_ARG;
    for (int j = 0; j < r; ++j) {
        if (idx[j] < 0 || idx[j] >= T) return ADA_ORACLE_ERR_INDEX;
        if (j > 0 && idx[j] <= idx[j - 1]) return ADA_ORACLE_ERR_INDEX;
    }
    const int causal = (flags & ADA_ORACLE_ATTN_CAUSAL) != 0;
    const size_t D = (size_t)H * (size_t)d_h;
    int32_t* pos = (int32_t*)malloc((size_t)T * sizeof(int32_t));      /* position in R, -1 outside */
    double* O = (double*)malloc((size_t)r * D * sizeof(double));
    if (!pos || !O) { free(pos); free(O); return ADA_ORACLE_ERR_NOMEM; }
    for (int t = 0; t < T; ++t) pos[t] = -1;
    for (int j = 0; j < r; ++j) pos[idx[j]] = j;
    for (int t = 0; t < T; ++t)
        if (assign[t] < 0 || assign[t] >= T || pos[assign[t]] < 0) { free(pos); free(O); return ADA_ORACLE_ERR_INDEX; }
    const double inv_sqrt = 1.0 / sqrt((double)d_h);
#pragma omp parallel for schedule(dynamic, 4) collapse(2)
    for (int h = 0; h < H; ++h) {
        for (int i = 0; i < r; ++i) {
            double* p = (double*)malloc((size_t)r * sizeof(double));
            const double* q = Q + (size_t)idx[i] * D + (size_t)h * d_h;
            const int n = causal ? i + 1 : r;                           /* keys 0 .. n-1 (R is in sequence order) */
            double m = -INFINITY;
            for (int j = 0; j < n; ++j) {
                const double* k = K + (size_t)idx[j] * D + (size_t)h * d_h;
                double s = 0.0;
                for (int c = 0; c < d_h; ++c) s += q[c] * k[c];
                p[j] = s * inv_sqrt;
                if (p[j] > m) m = p[j];
            }
            double z = 0.0;
            for (int j = 0; j < n; ++j) { p[j] = exp(p[j] - m); z += p[j]; }
            double* o = O + (size_t)i * D + (size_t)h * d_h;
            for (int c = 0; c < d_h; ++c) o[c] = 0.0;
            for (int j = 0; j < n; ++j) {
                const double w = p[j] / z;
                const double* v = V + (size_t)idx[j] * D + (size_t)h * d_h;
                for (int c = 0; c < d_h; ++c) o[c] += w * v[c];
            }
            free(p);
        }
    }
    for (int t = 0; t < T; ++t) memcpy(out + (size_t)t * D, O + (size_t)pos[assign[t]] * D, D * sizeof(double));
    free(pos); free(O);
    return ADA_ORACLE_OK;
}
