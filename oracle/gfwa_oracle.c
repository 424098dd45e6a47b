/*
 * GatedFWA CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 implementation of memory-gated sliding-window softmax
 * attention written straight from the definitions in the paper.  It shares no
 * code with the HIP path and must only be used by tests, the smoke check and
 * the cpu_baseline leg of the benchmark.
 *
 * One call handles ONE (batch, head) pair: Q, K, V, dO are [N, d] row-major
 * doubles, alpha / c / L are [N] doubles.  0-indexed positions.
 *
 * Notation (Sec. 3.2 of the paper, with the sign moved: the paper's
 * u_t = -sum alpha, here c_t = +sum alpha, so the paper's bias u_t - u_j equals
 * c_j - c_t):
 *
 *   c_t  = sum_{q<=t} alpha_q                       (inclusive prefix, Sec. 3.2)
 *   S_ti = scale * <q_t, k_i> + (c_i - c_t)         for  t-w < i <= t, i >= 0
 *   P_ti = exp(S_ti) / sum_{j in window(t)} exp(S_tj)   (gated score, Sec. 3.2)
 *   O_t  = sum_i P_ti v_i                           (Eq. 1 and the line after it)
 *   L_t  = log sum_{j in window(t)} exp(S_tj)       (Alg. 2, last step: m + log l)
 *
 * No tiling, no online softmax, no skipping logic: every row materialises its
 * band of logits, takes a max, exponentiates and normalises.
 *
 * Parity pins (tests/test_oracle_*.py): dense N x N brute force; reduction to
 * sliding-window and to causal softmax attention for alpha = 0 (Sec. 3, the
 * two special scores defined after Eq. 1); closed form for Q = 0 with a
 * constant gate; w = 1; row sums; shift invariance of c; finite differences
 * for every gradient; the two independent formulas for d(alpha).
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int gfwa_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sec. 3.2: inclusive prefix sum of the gate, one head. */
void gfwa_oracle_prefix(const double *alpha, double *c, long N) {
    double run = 0.0;
    for (long t = 0; t < N; ++t) {
        run += alpha[t];
        c[t] = run;
    }
}

static inline long window_lo(long t, long w) {
    long lo = t - w + 1; /* keep q-w+1 <= g <= q  (Alg. 2 mask) */
    return lo < 0 ? 0 : lo;
}

/* One row of the band: logits S_t,lo..t into s[0..n), returns n = t-lo+1. */
static long band_logits(const double *Q, const double *K, const double *c, long d, long w,
                        double scale, long t, double *s) {
    long lo = window_lo(t, w);
    for (long i = lo; i <= t; ++i) {
        double dot = 0.0;
        for (long x = 0; x < d; ++x) dot += Q[t * d + x] * K[i * d + x];
        s[i - lo] = scale * dot + (c[i] - c[t]);
    }
    return t - lo + 1;
}

/* Normalise a band row in place: s -> P, returns L = log sum exp. */
static double band_softmax(double *s, long n) {
    double m = s[0];
    for (long j = 1; j < n; ++j)
        if (s[j] > m) m = s[j];
    double l = 0.0;
    for (long j = 0; j < n; ++j) {
        s[j] = exp(s[j] - m);
        l += s[j];
    }
    for (long j = 0; j < n; ++j) s[j] /= l;
    return m + log(l);
}

/*
 * Forward for one head from a given prefix c (Sec. 3.2 score; Alg. 2 outputs).
 * O [N,d], L [N].  P_band, if not NULL, receives the probabilities as a
 * [N, w] array: P_band[t*w + (i - lo(t))], zero-padded on the right.
 */
void gfwa_oracle_forward_c(const double *Q, const double *K, const double *V, const double *c,
                           long N, long d, long w, double scale, double *O, double *L,
                           double *P_band) {
    long wb = w < N ? w : N;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)wb);
#pragma omp for schedule(dynamic, 16)
        for (long t = 0; t < N; ++t) {
            long lo = window_lo(t, w);
            long n = band_logits(Q, K, c, d, w, scale, t, s);
            L[t] = band_softmax(s, n);
            for (long x = 0; x < d; ++x) O[t * d + x] = 0.0;
            for (long j = 0; j < n; ++j)
                for (long x = 0; x < d; ++x) O[t * d + x] += s[j] * V[(lo + j) * d + x];
            if (P_band) {
                for (long j = 0; j < wb; ++j) P_band[t * wb + j] = j < n ? s[j] : 0.0;
            }
        }
        free(s);
    }
}

/* Forward for one head from the gate alpha itself (the full definition). */
void gfwa_oracle_forward(const double *Q, const double *K, const double *V, const double *alpha,
                         long N, long d, long w, double scale, double *O, double *L, double *c_out) {
    double *c = (double *)malloc(sizeof(double) * (size_t)N);
    gfwa_oracle_prefix(alpha, c, N);
    gfwa_oracle_forward_c(Q, K, V, c, N, d, w, scale, O, L, NULL);
    if (c_out) memcpy(c_out, c, sizeof(double) * (size_t)N);
    free(c);
}

/*
 * Backward for one head (App. E.2, Alg. 3, with the scale factor the chain
 * rule requires on dQ and dK).  Given dO, with P and O recomputed here:
 *
 *   D_t   = <dO_t, O_t>
 *   dP_ti = <dO_t, v_i>
 *   dS_ti = P_ti (dP_ti - D_t)
 *   dV_i  = sum_t P_ti dO_t
 *   dQ_t  = scale * sum_i dS_ti k_i
 *   dK_i  = scale * sum_t dS_ti q_t
 *   dc_p  = sum_t dS_tp - sum_i dS_pi      (S depends on c through +c_i - c_t)
 *
 * dc [N] is the gradient w.r.t. the prefix c; gfwa_oracle_dalpha_* turn it
 * into the gradient w.r.t. alpha.  dS_band (optional, [N, min(w,N)]) returns the band of
 * dS for the independent d(alpha) formula.
 */
static void backward_one_head(const double *Q, const double *K, const double *V, const double *c,
                              const double *dO, const double *O_saved, long N, long d, long w,
                              double scale, double *dQ, double *dK, double *dV, double *dc,
                              double *dS_band_out) {
    long wb = w < N ? w : N;
    size_t band = (size_t)N * (size_t)wb;
    double *O = (double *)malloc(sizeof(double) * (size_t)N * (size_t)d);
    double *L = (double *)malloc(sizeof(double) * (size_t)N);
    double *P = (double *)malloc(sizeof(double) * band);
    double *dS = dS_band_out ? dS_band_out : (double *)malloc(sizeof(double) * band);
    double *rowsum = (double *)malloc(sizeof(double) * (size_t)N);

    gfwa_oracle_forward_c(Q, K, V, c, N, d, w, scale, O, L, P);
    const double *Ouse = O_saved ? O_saved : O; /* the output that enters D */

    /* pass over query rows: D, dP, dS, dQ, row sums */
#pragma omp parallel for schedule(dynamic, 16)
    for (long t = 0; t < N; ++t) {
        long lo = window_lo(t, w);
        long n = t - lo + 1;
        double D = 0.0;
        for (long x = 0; x < d; ++x) D += dO[t * d + x] * Ouse[t * d + x];
        double rs = 0.0;
        for (long x = 0; x < d; ++x) dQ[t * d + x] = 0.0;
        for (long j = 0; j < wb; ++j) dS[t * wb + j] = 0.0;
        for (long j = 0; j < n; ++j) {
            long i = lo + j;
            double dP = 0.0;
            for (long x = 0; x < d; ++x) dP += dO[t * d + x] * V[i * d + x];
            double ds = P[t * wb + j] * (dP - D);
            dS[t * wb + j] = ds;
            rs += ds;
            for (long x = 0; x < d; ++x) dQ[t * d + x] += scale * ds * K[i * d + x];
        }
        rowsum[t] = rs;
    }

    /* pass over key columns: dV, dK, column sums.  Key i is seen by rows t = i .. i+w-1. */
#pragma omp parallel for schedule(dynamic, 16)
    for (long i = 0; i < N; ++i) {
        double cs = 0.0;
        for (long x = 0; x < d; ++x) {
            dV[i * d + x] = 0.0;
            dK[i * d + x] = 0.0;
        }
        long thi = i + w - 1;
        if (thi > N - 1) thi = N - 1;
        for (long t = i; t <= thi; ++t) {
            long j = i - window_lo(t, w);
            double p = P[t * wb + j];
            double ds = dS[t * wb + j];
            cs += ds;
            for (long x = 0; x < d; ++x) {
                dV[i * d + x] += p * dO[t * d + x];
                dK[i * d + x] += scale * ds * Q[t * d + x];
            }
        }
        dc[i] = cs - rowsum[i];
    }

    free(O);
    free(L);
    free(P);
    if (!dS_band_out) free(dS);
    free(rowsum);
}

void gfwa_oracle_backward_c(const double *Q, const double *K, const double *V, const double *c,
                            const double *dO, long N, long d, long w, double scale, double *dQ,
                            double *dK, double *dV, double *dc, double *dS_band_out) {
    backward_one_head(Q, K, V, c, dO, NULL, N, d, w, scale, dQ, dK, dV, dc, dS_band_out);
}

/*
 * The same formulas with D_t = <dO_t, O_saved_t> taken on a GIVEN output O_saved [N, d] instead of
 * the output recomputed here.  App. E.2 / Alg. 3 is stated this way: the saved forward output O is
 * an input of the backward and D = rowsum(dO * O) is formed from it.  With O_saved equal to the
 * exact output this is the gradient; with an output that was rounded for storage it is what the
 * algorithm returns on that input, and differs from the gradient by  -P_ti * (D_saved - D)_t  in
 * every dS_ti.  P is still the exact softmax (the logsumexp is recomputed, not taken from outside).
 */
void gfwa_oracle_backward_saved_O(const double *Q, const double *K, const double *V, const double *c,
                                  const double *dO, const double *O_saved, long N, long d, long w,
                                  double scale, double *dQ, double *dK, double *dV, double *dc,
                                  double *dS_band_out) {
    backward_one_head(Q, K, V, c, dO, O_saved, N, d, w, scale, dQ, dK, dV, dc, dS_band_out);
}

/* c_p = sum_{q<=p} alpha_q, so d(alpha_q) = sum_{p>=q} dc_p  (reverse inclusive scan;
 * Sec. 3.3 "gradients into U flow through the same streamed scan"). */
void gfwa_oracle_dalpha_from_dc(const double *dc, double *dalpha, long N) {
    double run = 0.0;
    for (long q = N - 1; q >= 0; --q) {
        run += dc[q];
        dalpha[q] = run;
    }
}

/* Independent formula: alpha_q enters S_ti as -alpha_q exactly when i < q <= t
 * (Fig. 1 caption: the bias is minus the sum of alpha over (i, t]), so
 * d(alpha_q) = - sum over in-window pairs (t, i) with i < q <= t of dS_ti.  O(N w^2): tiny N only. */
void gfwa_oracle_dalpha_direct(const double *dS_band, double *dalpha, long N, long w) {
    long wb = w < N ? w : N;
    for (long q = 0; q < N; ++q) {
        double acc = 0.0;
        for (long t = q; t < N; ++t) {
            long lo = window_lo(t, w);
            for (long i = lo; i < q && i <= t; ++i) acc -= dS_band[t * wb + (i - lo)];
        }
        dalpha[q] = acc;
    }
}

/*
 * Gate activation (Sec. 3.2, the equation that defines alpha from the pre-activation h and the
 * amplitude beta; Alg. 1, the on-chip steps with the overflow-safe softplus; Sec. 3.3 puts the
 * small epsilon into the denominator):
 *
 *   z = beta * h,  nu = max(z, 0),  softplus(z) = nu + log(exp(z - nu) + exp(-nu))
 *   alpha = softplus(z) / (beta + eps)
 *
 * n independent elements.
 */
void gfwa_oracle_gate_activation(const double *h, const double *beta, double eps, double *alpha,
                                 long n) {
    for (long i = 0; i < n; ++i) {
        const double z = beta[i] * h[i];
        const double nu = z > 0.0 ? z : 0.0;
        const double sp = nu + log(exp(z - nu) + exp(-nu));
        alpha[i] = sp / (beta[i] + eps);
    }
}

/*
 * Its derivative (chain rule on the definition above; the paper states no listing for it):
 * with s = softplus(z), sigma = d softplus / dz = 1 / (1 + exp(-z)),
 *
 *   d alpha / d h    = sigma * beta / (beta + eps)
 *   d alpha / d beta = sigma * h / (beta + eps) - s / (beta + eps)^2
 */
void gfwa_oracle_gate_activation_backward(const double *h, const double *beta, double eps,
                                          const double *dalpha, double *dh, double *dbeta, long n) {
    for (long i = 0; i < n; ++i) {
        const double z = beta[i] * h[i];
        const double nu = z > 0.0 ? z : 0.0;
        const double sp = nu + log(exp(z - nu) + exp(-nu));
        const double sig = z >= 0.0 ? 1.0 / (1.0 + exp(-z)) : exp(z) / (1.0 + exp(z));
        const double be = beta[i] + eps;
        dh[i] = dalpha[i] * sig * beta[i] / be;
        dbeta[i] = dalpha[i] * (sig * h[i] / be - sp / (be * be));
    }
}
