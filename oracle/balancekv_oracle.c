/*
 * BalanceKV reference oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, double-precision CPU statement of what the BalanceKV hot path
 * computes (arXiv 2502.07861).  Only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code, header, table
 * or helper with the HIP library and is never used as a fallback for it.
 *
 * Every function takes the algorithm's steps in the paper's order and notation:
 *
 *   bkvo_exact_attention      Eq. 1            softmax(K q / sqrt(d))^T V
 *   bkvo_softmax_balance      Alg. 2           kernel weights + self-balancing walk
 *   bkvo_self_balancing_walk  Alg. 4 (App. A)  the linear walk of ALS21
 *   bkvo_select_half          Alg. 2 output step + the "strictly n/2" rule of
 *                             App. B "Implementation Detail"
 *   bkvo_attend               Alg. 1, output line: weighted softmax estimator
 *   bkvo_uniform              the counter-based generator that supplies the
 *                             "with probability p_j" draws of Alg. 2
 *
 * Pins (tests/test_oracle_*.py): brute-force softmax for Eq. 1 and for the
 * estimator with unit weights; hand-worked walks; Alg. 2 == Alg. 4 run on the
 * explicit (truncated) feature map of App. A; the constant-free discrepancy
 * certificate; the walk's quadratic identity; structure invariants.
 * Parity unpinned: exact kept-index sets on realistic inputs (the paper prints
 * none); they are held only by the necessary conditions above.
 *
 * No blocking, fusion or reordering: loops are written as the definitions read.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------- */
/* Counter-based uniform generator.                                          */
/* u(seed, stream, ctr) in [0,1), a multiple of 2^-24.  Integer arithmetic   */
/* only (two rounds of the SplitMix64 output mixer), so any implementation   */
/* reproduces it bit for bit.                                                 */
/* ------------------------------------------------------------------------- */
static uint64_t mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

uint32_t bkvo_uniform_bits(uint64_t seed, uint64_t stream, uint64_t ctr)
{
    const uint64_t golden = 0x9E3779B97F4A7C15ull;
    uint64_t a = mix64(seed + golden * (stream + 1));
    uint64_t z = mix64(a + golden * (ctr + 1));
    return (uint32_t)(z >> 40);                 /* top 24 bits */
}

double bkvo_uniform(uint64_t seed, uint64_t stream, uint64_t ctr)
{
    return (double)bkvo_uniform_bits(seed, stream, ctr) * (1.0 / 16777216.0);
}

void bkvo_uniform_fill(uint64_t seed, uint64_t stream, uint64_t ctr0, int64_t n, double *out)
{
    for (int64_t j = 0; j < n; ++j) out[j] = bkvo_uniform(seed, stream, ctr0 + (uint64_t)j);
}

/* ------------------------------------------------------------------------- */
/* Eq. 1: Attn(q, K, V) = softmax(K q / sqrt(d))^T V.                         */
/* K [n,d], V [n,s], q [d]  ->  out [s].  The common factor exp(-max) cancels */
/* in the ratio, so subtracting the largest logit leaves Eq. 1 unchanged.     */
/* ------------------------------------------------------------------------- */
void bkvo_exact_attention(const double *q, const double *K, const double *V,
                          int64_t n, int d, int s, double *out)
{
    double *logit = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    double mx = -INFINITY;
    for (int64_t i = 0; i < n; ++i) {
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += K[i * d + c] * q[c];
        logit[i] = dot / sqrt((double)d);
        if (logit[i] > mx) mx = logit[i];
    }
    double Z = 0.0;
    for (int c = 0; c < s; ++c) out[c] = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double e = exp(logit[i] - mx);
        Z += e;
        for (int c = 0; c < s; ++c) out[c] += e * V[i * s + c];
    }
    for (int c = 0; c < s; ++c) out[c] /= Z;
    free(logit);
}

/* ------------------------------------------------------------------------- */
/* Alg. 1, output line: z = sum_l 2^l sum_{C^l} e^{<k,q>/sqrt d} v             */
/*                        / sum_l 2^l sum_{C^l} e^{<k,q>/sqrt d}.              */
/* The levels arrive flattened: token i carries weight w_i = 2^{level(i)}.     */
/* w_i e^{x} = e^{x + ln w_i}; the largest exponent is subtracted top and      */
/* bottom.  lse (optional) = ln of the denominator.  Tokens with w_i = 0 do    */
/* not take part.                                                             */
/* ------------------------------------------------------------------------- */
void bkvo_attend(const double *q, const double *K, const double *V, const double *w,
                 int64_t n, int d, int s, double *out, double *lse)
{
    double *logit = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    double mx = -INFINITY;
    for (int64_t i = 0; i < n; ++i) {
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += K[i * d + c] * q[c];
        logit[i] = (w[i] > 0.0) ? dot / sqrt((double)d) + log(w[i]) : -INFINITY;
        if (logit[i] > mx) mx = logit[i];
    }
    double Z = 0.0;
    for (int c = 0; c < s; ++c) out[c] = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        if (!(w[i] > 0.0)) continue;
        double e = exp(logit[i] - mx);
        Z += e;
        for (int c = 0; c < s; ++c) out[c] += e * V[i * s + c];
    }
    for (int c = 0; c < s; ++c) out[c] /= Z;
    if (lse) *lse = mx + log(Z);
    free(logit);
}

/* ------------------------------------------------------------------------- */
/* Alg. 2, SoftmaxBalance, the sign-assignment loop.                           */
/*                                                                             */
/* Inputs: K [n,d]; V [n,s] or NULL for the scalar value v == 1 (the           */
/* denominator instance of Alg. 1); radii r_key, r_value (<= 0: take the       */
/* largest norm in the input, of the centred keys if `center`); log_c = ln c;  */
/* u [n] the uniform draws; forced [n] or NULL.                                */
/*                                                                             */
/* With R = exp(r_key^2 / (2 sqrt d)) r_value and y_i = e^{<k_i,k_j>/sqrt d}   */
/* <v_i,v_j>, the algorithm only ever uses y^T eta / (c R^2).  Each term of    */
/* that quotient is                                                            */
/*     g_ij = exp((<k_i,k_j> - r_key^2)/sqrt d - ln c) * <v_i,v_j> / r_value^2 */
/* which is what is evaluated here, so that neither R^2 nor c R^2 is ever      */
/* formed (they overflow for realistic key norms).                             */
/*                                                                             */
/* y ranges over the already signed tokens i < j (eta_j is still 0 when y is   */
/* formed, so the i = j entry contributes nothing).                            */
/*                                                                             */
/*   sigma_j = sum_{i<j} eta_i g_ij          (= y^T eta / (c R^2))             */
/*   FAIL if |sigma_j| > 1; the run continues with p clamped to [0,1]          */
/*   p_j = 1/2 - sigma_j / 2                                                   */
/*   eta_j = +1 if u_j < p_j else -1                                           */
/*                                                                             */
/* If `forced` is given, eta_j is taken from it instead (teacher forcing), and */
/* dec[j] still reports what the rule above would have chosen.                 */
/* `center`: keys are shifted by their mean before the inner products          */
/* (App. B.5 item 1); selection only.                                          */
/* `linear_kernel`: g_ij = <k_i,k_j> <v_i,v_j> / (c r_key^2 r_value^2), the    */
/* finite-dimensional walk of Alg. 4, for cross-checks.                        */
/*                                                                             */
/* Outputs (any may be NULL): eta [n] (+1/-1), p [n] (clamped), sig [n],       */
/* dec [n] (+1/-1 by the rule).  Returns the number of FAIL events.            */
/* ------------------------------------------------------------------------- */
int64_t bkvo_softmax_balance(const double *K, const double *V, int64_t n, int d, int s,
                             double r_key, double r_value, double log_c,
                             int center, int linear_kernel,
                             const double *u, const int8_t *forced,
                             int8_t *eta_out, double *p_out, double *sig_out, int8_t *dec_out)
{
    if (n <= 0) return 0;
    double *Kc = (double *)malloc(sizeof(double) * (size_t)n * (size_t)d);
    int8_t *eta = (int8_t *)calloc((size_t)n, 1);
    double sqrt_d = sqrt((double)d);

    /* optional mean shift of the keys */
    memcpy(Kc, K, sizeof(double) * (size_t)n * (size_t)d);
    if (center) {
        for (int c = 0; c < d; ++c) {
            double mu = 0.0;
            for (int64_t i = 0; i < n; ++i) mu += K[i * d + c];
            mu /= (double)n;
            for (int64_t i = 0; i < n; ++i) Kc[i * d + c] = K[i * d + c] - mu;
        }
    }
    /* radii */
    double rk2 = r_key * r_key, rv2 = r_value * r_value;
    if (!(r_key > 0.0)) {
        rk2 = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            double nn = 0.0;
            for (int c = 0; c < d; ++c) nn += Kc[i * d + c] * Kc[i * d + c];
            if (nn > rk2) rk2 = nn;
        }
    }
    if (V && !(r_value > 0.0)) {
        rv2 = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            double nn = 0.0;
            for (int c = 0; c < s; ++c) nn += V[i * s + c] * V[i * s + c];
            if (nn > rv2) rv2 = nn;
        }
    }
    if (!V) rv2 = 1.0;                      /* v == 1: <v_i,v_j> = 1, r_value = 1 */

    int64_t fails = 0;
    for (int64_t j = 0; j < n; ++j) {
        double sigma = 0.0;
        for (int64_t i = 0; i < j; ++i) {
            double kk = 0.0;
            for (int c = 0; c < d; ++c) kk += Kc[i * d + c] * Kc[j * d + c];
            double vv = 1.0;
            if (V) {
                vv = 0.0;
                for (int c = 0; c < s; ++c) vv += V[i * s + c] * V[j * s + c];
            }
            double g;
            if (linear_kernel) g = kk * exp(-log_c) / rk2 * (vv / rv2);
            else               g = exp((kk - rk2) / sqrt_d - log_c) * (vv / rv2);
            sigma += (double)eta[i] * g;
        }
        if (fabs(sigma) > 1.0) ++fails;
        double p = 0.5 - 0.5 * sigma;
        if (p < 0.0) p = 0.0;
        if (p > 1.0) p = 1.0;
        int8_t decision = (u[j] < p) ? 1 : -1;
        eta[j] = forced ? forced[j] : decision;
        if (p_out) p_out[j] = p;
        if (sig_out) sig_out[j] = sigma;
        if (dec_out) dec_out[j] = decision;
    }
    if (eta_out) memcpy(eta_out, eta, (size_t)n);
    free(Kc);
    free(eta);
    return fails;
}

/* The same over n_inst independent blocks laid out [n_inst, n, d]; instances  */
/* are spread over OpenMP threads, each instance runs the serial routine.      */
void bkvo_softmax_balance_batch(const double *K, const double *V, int64_t n_inst, int64_t n,
                                int d, int s, double r_key, double r_value, double log_c,
                                int center, const double *u, const int8_t *forced,
                                int8_t *eta_out, double *p_out, double *sig_out,
                                int8_t *dec_out, int64_t *fails_out, int n_threads)
{
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < n_inst; ++t) {
        int64_t f = bkvo_softmax_balance(
            K + t * n * d, V ? V + t * n * s : NULL, n, d, s, r_key, r_value, log_c, center, 0,
            u + t * n, forced ? forced + t * n : NULL,
            eta_out ? eta_out + t * n : NULL, p_out ? p_out + t * n : NULL,
            sig_out ? sig_out + t * n : NULL, dec_out ? dec_out + t * n : NULL);
        if (fails_out) fails_out[t] = f;
    }
}

int bkvo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------- */
/* Alg. 4, Self-Balancing Walk, on explicit vectors U [n,dim] of norm <= r.    */
/* Keeps the signed sum  wsum = sum_{U+} u - sum_{U-} u  and tests             */
/* <wsum, u_i> against c r^2, as the listing does.                             */
/* ------------------------------------------------------------------------- */
int64_t bkvo_self_balancing_walk(const double *U, int64_t n, int64_t dim, double r, double log_c,
                                 const double *u, int8_t *eps_out, double *p_out)
{
    double *wsum = (double *)calloc((size_t)(dim > 0 ? dim : 1), sizeof(double));
    double cr2 = exp(log_c) * r * r;
    int64_t fails = 0;
    for (int64_t i = 0; i < n; ++i) {
        double dot = 0.0;
        for (int64_t c = 0; c < dim; ++c) dot += wsum[c] * U[i * dim + c];
        if (fabs(dot) > cr2) ++fails;
        double p = 0.5 - dot / (2.0 * cr2);
        if (p < 0.0) p = 0.0;
        if (p > 1.0) p = 1.0;
        int8_t e = (u[i] < p) ? 1 : -1;
        for (int64_t c = 0; c < dim; ++c) wsum[c] += (double)e * U[i * dim + c];
        if (eps_out) eps_out[i] = e;
        if (p_out) p_out[i] = p;
    }
    free(wsum);
    return fails;
}

/* ------------------------------------------------------------------------- */
/* Output step of Alg. 2 and the strict rule.                                  */
/* sigma = '+' if |{eta=+1}| <= |{eta=-1}| else '-'.  Theory mode keeps        */
/* exactly the tokens of sign sigma (at most n/2).  Strict mode ("strictly     */
/* select n/2") tops that set up to exactly n/2 with the other sign's tokens,  */
/* lowest index first.  idx [>= n/2 or n] is written ascending; returns its    */
/* length.                                                                     */
/* ------------------------------------------------------------------------- */
int64_t bkvo_select_half(const int8_t *eta, int64_t n, int strict, int64_t *idx)
{
    int64_t n_plus = 0;
    for (int64_t i = 0; i < n; ++i) n_plus += (eta[i] > 0);
    int8_t sigma = (n_plus <= n - n_plus) ? 1 : -1;
    int64_t n_min = (sigma > 0) ? n_plus : n - n_plus;
    int64_t need = strict ? n / 2 - n_min : 0;       /* majority tokens to add */
    int64_t m = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (eta[i] == sigma) idx[m++] = i;
        else if (need > 0) { idx[m++] = i; --need; }
    }
    return m;
}
