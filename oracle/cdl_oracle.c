/*
 * CPU oracle for the quantized layer step of Coded Deep Learning (CDL).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the method computes, written from the paper's definitions in double
 * precision.  Only the test-suite, the smoke check and the CPU-baseline leg of
 * the benchmark may call it; the GPU library never does, and the two share no
 * code, tables or helpers.
 *
 * Every routine evaluates the definition directly: each element visits every
 * level of the index set, there is no windowing, blocking, recurrence or
 * reordering.  OpenMP is used only to spread independent elements / output
 * rows over the host cores.
 *
 * Notation (Section III-A): theta is one weight or activation, q (here
 * `delta`) the step size, alpha the sharpness, the index set is
 * {lo, ..., lo+n_levels-1}, level i reproduces the value i*delta.
 *
 * Readings where the paper is silent are listed next to the code that takes
 * them; all are repeated in the design notes of the repository.
 *
 * Parity pins: every function below is pinned by a CPU test against a closed
 * form, an invariant, a finite difference or a brute-force / library result;
 * none is "parity unpinned".  The paper's trained-network results (Table I
 * and the figures of Section V) are not reproduced by anything here.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int cdl_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------
 * One element: conditional PMF over the levels (eq. CPMF / eq. PMF, Sec. III-A)
 *
 *   P(i*delta | theta) = exp(-alpha (theta - i delta)^2) / sum_j exp(-alpha (theta - j delta)^2)
 *
 * evaluated as a softmax with the largest score subtracted (the same
 * quotient, safe against underflow of every term).
 * Returns the mode (lowest index on an exact tie of scores: the paper does not
 * say) and the gap between the two largest scores.
 * ---------------------------------------------------------------------- */
static int cpmf_core(double theta, int lo, int n_levels, double delta, double alpha, int top_k,
                     double *P /* n_levels */, double *score_gap /* nullable */)
{
    double s_best = -INFINITY, s_second = -INFINITY;
    int i_best = lo;
    for (int k = 0; k < n_levels; ++k) {
        double d = theta - (double)(lo + k) * delta;
        double s = -alpha * d * d;
        P[k] = s;
        if (s > s_best) { s_second = s_best; s_best = s; i_best = lo + k; }
        else if (s > s_second) { s_second = s; }
    }
    if (top_k > 0 && top_k < n_levels) {
        /*
         * Truncated CPMF (Sec. V-B, the paragraph on quantizing within a mini-batch): only the
         * most probable values keep probability mass, in proportion; all others get 0.
         * Reading: keep the top_k levels of largest probability (= largest score; on equal
         * scores the lower index is kept first), renormalise over them.  The paper uses 5.
         */
        char *keep = (char *)calloc((size_t)n_levels, 1);
        for (int r = 0; r < top_k; ++r) {
            int pick = -1;
            for (int k = 0; k < n_levels; ++k)
                if (!keep[k] && (pick < 0 || P[k] > P[pick])) pick = k;   /* strict >: lower index wins ties */
            keep[pick] = 1;
        }
        for (int k = 0; k < n_levels; ++k) if (!keep[k]) P[k] = -INFINITY;
        free(keep);
    }
    double Z = 0.0;
    for (int k = 0; k < n_levels; ++k) { P[k] = exp(P[k] - s_best); Z += P[k]; }
    for (int k = 0; k < n_levels; ++k) P[k] /= Z;
    if (score_gap) *score_gap = s_best - s_second;
    return i_best;
}

int cdl_oracle_cpmf(double theta, int lo, int n_levels, double delta, double alpha,
                    double *P /* n_levels */, double *score_gap /* nullable */)
{
    return cpmf_core(theta, lo, n_levels, delta, alpha, 0, P, score_gap);
}

int cdl_oracle_cpmf_k(double theta, int lo, int n_levels, double delta, double alpha, int top_k,
                      double *P /* n_levels */, double *score_gap /* nullable */)
{
    return cpmf_core(theta, lo, n_levels, delta, alpha, top_k, P, score_gap);
}

/* Soft deterministic quantizer Q_d(theta) = sum_i P(i delta | theta) * i delta  (eq. softQ, Sec. III-B) */
static double soft_value(const double *P, int lo, int n_levels, double delta)
{
    double e = 0.0;
    for (int k = 0; k < n_levels; ++k) e += P[k] * ((double)(lo + k) * delta);
    return e;
}

typedef struct {
    double mean;      /* E{Q_p}  = Q_d                                    */
    double var;       /* Var{Q_p}                                         */
    double skew_u;    /* Skew_u{Q_p} = E X^3 - E X * E X^2  (Lemma 1)      */
    double cov_x_d2;  /* Cov(X, (theta - X)^2)                             */
} moments_t;

/*
 * Moments of the quantized value X = Q_p(theta) under the CPMF.
 * Var and Skew_u are taken about the mean: Var = E(X-EX)^2 by definition and
 * Skew_u = E(X-EX)^3 + 2 EX Var (expand X = EX + Y with EY = 0 in Lemma 1's
 * definition).  The raw-power form printed in Lemma 1 is the same number but
 * cancels to nothing in double once |i| ~ 100 and the distribution is
 * concentrated; cdl_oracle_lemma1_raw below evaluates it literally so a test
 * can check the two agree where the raw form is still well conditioned.
 */
static moments_t moments(const double *P, double theta, int lo, int n_levels, double delta)
{
    moments_t m;
    m.mean = soft_value(P, lo, n_levels, delta);
    double c2 = 0.0, c3 = 0.0, cov = 0.0;
    for (int k = 0; k < n_levels; ++k) {
        double v = (double)(lo + k) * delta;
        double y = v - m.mean;
        double d = theta - v;
        c2 += P[k] * y * y;
        c3 += P[k] * y * y * y;
        cov += P[k] * y * d * d;
    }
    m.var = c2;
    m.skew_u = c3 + 2.0 * m.mean * c2;
    m.cov_x_d2 = cov;
    return m;
}

/*
 * Partial derivatives of Q_d for one element.
 *   dQd/dtheta = 2 alpha Var                                   (Lemma 1, eq. partialW)
 *   dQd/dq     = (E + 2 alpha theta Var - 2 alpha Skew_u) / q  (Lemma 1, eq. partialQ)
 *   dQd/dalpha = -Cov(X, (theta - X)^2)
 * The paper does not print the last one (Sec. IV-B, after eq. Jgrad_alpha_q, only notes that it
 * has an analytic form).  Differentiating eq. CPMF gives
 * dP_i/dalpha = -P_i (d_i^2 - sum_j P_j d_j^2) with d_i = theta - i q, and
 * summing i q dP_i/dalpha gives the covariance above.
 */
void cdl_oracle_element_k(double theta, int lo, int n_levels, double delta, double alpha, int top_k,
                          int *idx, double *soft, double *score_gap,
                          double *dsoft_dtheta, double *dsoft_ddelta, double *dsoft_dalpha)
{
    double *P = (double *)malloc(sizeof(double) * (size_t)n_levels);
    double gap;
    int mode = cpmf_core(theta, lo, n_levels, delta, alpha, top_k, P, &gap);
    moments_t m = moments(P, theta, lo, n_levels, delta);
    if (idx) *idx = mode;
    if (soft) *soft = m.mean;
    if (score_gap) *score_gap = gap;
    if (dsoft_dtheta) *dsoft_dtheta = 2.0 * alpha * m.var;
    if (dsoft_ddelta) *dsoft_ddelta = (m.mean + 2.0 * alpha * theta * m.var - 2.0 * alpha * m.skew_u) / delta;
    if (dsoft_dalpha) *dsoft_dalpha = -m.cov_x_d2;
    free(P);
}

void cdl_oracle_element(double theta, int lo, int n_levels, double delta, double alpha,
                        int *idx, double *soft, double *score_gap,
                        double *dsoft_dtheta, double *dsoft_ddelta, double *dsoft_dalpha)
{
    cdl_oracle_element_k(theta, lo, n_levels, delta, alpha, 0, idx, soft, score_gap, dsoft_dtheta, dsoft_ddelta, dsoft_dalpha);
}

/* Lemma 1 with Var and Skew_u from raw powers of X exactly as printed. */
void cdl_oracle_lemma1_raw(double theta, int lo, int n_levels, double delta, double alpha,
                           double *dsoft_dtheta, double *dsoft_ddelta)
{
    double *P = (double *)malloc(sizeof(double) * (size_t)n_levels);
    cdl_oracle_cpmf(theta, lo, n_levels, delta, alpha, P, NULL);
    double e1 = 0.0, e2 = 0.0, e3 = 0.0;
    for (int k = 0; k < n_levels; ++k) {
        double v = (double)(lo + k) * delta;
        e1 += P[k] * v; e2 += P[k] * v * v; e3 += P[k] * v * v * v;
    }
    double var = e2 - e1 * e1;
    double skew_u = e3 - e1 * e2;
    *dsoft_dtheta = 2.0 * alpha * var;
    *dsoft_ddelta = (e1 + 2.0 * alpha * theta * var - 2.0 * alpha * skew_u) / delta;
    free(P);
}

/* ------------------------------------------------------------------------
 * Tensor forward: hard index (mode of the CPMF = the value Q_p takes with
 * probability -> 1 as alpha grows, Remark after eq. Qprob) and soft value
 * Q_d (eq. softboth, Sec. IV-B) for every entry.
 * ---------------------------------------------------------------------- */
void cdl_oracle_quantize_fwd_k(const float *theta, int64_t n, int lo, int n_levels,
                               float delta_f, float alpha_f, int top_k,
                               int32_t *idx /* n, nullable */, double *soft /* n, nullable */,
                               double *score_gap /* n, nullable */)
{
    const double delta = (double)delta_f, alpha = (double)alpha_f;
#pragma omp parallel
    {
        double *P = (double *)malloc(sizeof(double) * (size_t)n_levels);
#pragma omp for schedule(static)
        for (int64_t e = 0; e < n; ++e) {
            double gap;
            int mode = cpmf_core((double)theta[e], lo, n_levels, delta, alpha, top_k, P, &gap);
            if (idx) idx[e] = mode;
            if (soft) soft[e] = soft_value(P, lo, n_levels, delta);
            if (score_gap) score_gap[e] = gap;
        }
        free(P);
    }
}

void cdl_oracle_quantize_fwd(const float *theta, int64_t n, int lo, int n_levels,
                             float delta_f, float alpha_f,
                             int32_t *idx /* n, nullable */, double *soft /* n, nullable */,
                             double *score_gap /* n, nullable */)
{
    cdl_oracle_quantize_fwd_k(theta, n, lo, n_levels, delta_f, alpha_f, 0, idx, soft, score_gap);
}

/* ------------------------------------------------------------------------
 * Marginal PMF of the quantized tensor (eq. approx1/n, Sec. IV-C):
 *   marg[k] = (1/n) sum_e P(level k | theta_e)
 * and its Shannon entropy H = -sum_k marg[k] log2 marg[k] in bits (the paper
 * writes "log" and measures the result in bits per weight; terms with
 * marg[k] = 0 contribute 0).  The total for the layer is n*H.
 * One call = one PMF over the whole tensor handed in.
 * ---------------------------------------------------------------------- */
void cdl_oracle_marginal_entropy_k(const float *theta, int64_t n, int lo, int n_levels,
                                   float delta_f, float alpha_f, int top_k,
                                   double *marg /* n_levels */, double *entropy_bits /* 1 */)
{
    const double delta = (double)delta_f, alpha = (double)alpha_f;
    int nthreads = cdl_oracle_num_threads();
    double *partial = (double *)calloc((size_t)nthreads * (size_t)n_levels, sizeof(double));
#pragma omp parallel
    {
#ifdef _OPENMP
        int t = omp_get_thread_num();
#else
        int t = 0;
#endif
        double *mine = partial + (size_t)t * (size_t)n_levels;
        double *P = (double *)malloc(sizeof(double) * (size_t)n_levels);
#pragma omp for schedule(static)
        for (int64_t e = 0; e < n; ++e) {
            cpmf_core((double)theta[e], lo, n_levels, delta, alpha, top_k, P, NULL);
            for (int k = 0; k < n_levels; ++k) mine[k] += P[k];
        }
        free(P);
    }
    double H = 0.0;
    for (int k = 0; k < n_levels; ++k) {
        double s = 0.0;
        for (int t = 0; t < nthreads; ++t) s += partial[(size_t)t * (size_t)n_levels + k];
        marg[k] = (n > 0) ? s / (double)n : 0.0;
        if (marg[k] > 0.0) H -= marg[k] * log2(marg[k]);
    }
    *entropy_bits = H;
    free(partial);
}

void cdl_oracle_marginal_entropy(const float *theta, int64_t n, int lo, int n_levels,
                                 float delta_f, float alpha_f,
                                 double *marg /* n_levels */, double *entropy_bits /* 1 */)
{
    cdl_oracle_marginal_entropy_k(theta, n, lo, n_levels, delta_f, alpha_f, 0, marg, entropy_bits);
}

/* ------------------------------------------------------------------------
 * Tensor backward (Sec. IV-B): with g[e] = dL/dQ_p(theta_e) from the layer,
 *   dtheta[e] = g[e] * dQd/dtheta                    (eq. partialX3 / partialW3)
 *   d_delta   = sum_e g[e] * dQd/dq                  (eq. Jgradqw / Jgradqx)
 *   d_alpha   = sum_e g[e] * dQd/dalpha              (eq. Jgradq_alpha_w / Jgrad_alpha_q)
 * ---------------------------------------------------------------------- */
void cdl_oracle_quantize_bwd_k(const float *theta, const float *g, int64_t n, int lo, int n_levels,
                               float delta_f, float alpha_f, int top_k,
                               double *dtheta /* n, nullable */,
                               double *d_delta, double *d_alpha)
{
    const double delta = (double)delta_f, alpha = (double)alpha_f;
    double sd = 0.0, sa = 0.0;
#pragma omp parallel reduction(+ : sd, sa)
    {
        double *P = (double *)malloc(sizeof(double) * (size_t)n_levels);
#pragma omp for schedule(static)
        for (int64_t e = 0; e < n; ++e) {
            double th = (double)theta[e], ge = (double)g[e];
            cpmf_core(th, lo, n_levels, delta, alpha, top_k, P, NULL);
            moments_t m = moments(P, th, lo, n_levels, delta);
            double d_th = 2.0 * alpha * m.var;
            double d_q = (m.mean + 2.0 * alpha * th * m.var - 2.0 * alpha * m.skew_u) / delta;
            double d_al = -m.cov_x_d2;
            if (dtheta) dtheta[e] = ge * d_th;
            sd += ge * d_q;
            sa += ge * d_al;
        }
        free(P);
    }
    *d_delta = sd;
    *d_alpha = sa;
}

void cdl_oracle_quantize_bwd(const float *theta, const float *g, int64_t n, int lo, int n_levels,
                             float delta_f, float alpha_f,
                             double *dtheta /* n, nullable */,
                             double *d_delta, double *d_alpha)
{
    cdl_oracle_quantize_bwd_k(theta, g, n, lo, n_levels, delta_f, alpha_f, 0, dtheta, d_delta, d_alpha);
}

/*
 * The three quantities Lemma 1 is written in, for every entry of a tensor: E{Q_p}, Var{Q_p} and
 * Skew_u{Q_p} under the (possibly truncated) CPMF of that entry.
 */
void cdl_oracle_moments_k(const float *theta, int64_t n, int lo, int n_levels,
                          float delta_f, float alpha_f, int top_k,
                          double *mean /* n */, double *var /* n */, double *skew_u /* n */)
{
    const double delta = (double)delta_f, alpha = (double)alpha_f;
#pragma omp parallel
    {
        double *P = (double *)malloc(sizeof(double) * (size_t)n_levels);
#pragma omp for schedule(static)
        for (int64_t e = 0; e < n; ++e) {
            double th = (double)theta[e];
            cpmf_core(th, lo, n_levels, delta, alpha, top_k, P, NULL);
            moments_t m = moments(P, th, lo, n_levels, delta);
            mean[e] = m.mean;
            var[e] = m.var;
            skew_u[e] = m.skew_u;
        }
        free(P);
    }
}

/* ------------------------------------------------------------------------
 * The probabilistic quantizer itself (eq. Qprob, Sec. III-A): theta is mapped to level i with
 * probability P(i q | theta).  The draw is made by inversion with one uniform number u in [0,1)
 * per entry, supplied by the caller: levels are taken in increasing order and the draw is the
 * first level whose cumulative probability exceeds u (the paper does not say how the draw is
 * made; any method with the right distribution is the same quantizer, inversion is the one that
 * can be compared entry by entry).  `margin` is the distance from u to the nearest end of the
 * chosen level's cumulative interval: a different rounding of the cumulative sums can only
 * change draws whose margin is of that size.
 * ---------------------------------------------------------------------- */
void cdl_oracle_quantize_draw(const float *theta, const float *u, int64_t n, int lo, int n_levels,
                              float delta_f, float alpha_f, int top_k,
                              int32_t *idx /* n */, double *margin /* n, nullable */)
{
    const double delta = (double)delta_f, alpha = (double)alpha_f;
#pragma omp parallel
    {
        double *P = (double *)malloc(sizeof(double) * (size_t)n_levels);
#pragma omp for schedule(static)
        for (int64_t e = 0; e < n; ++e) {
            cpmf_core((double)theta[e], lo, n_levels, delta, alpha, top_k, P, NULL);
            const double ue = (double)u[e];
            double cdf = 0.0, below = 0.0;
            int pick = -1, last_pos = 0;
            for (int k = 0; k < n_levels; ++k) {
                if (P[k] > 0.0) last_pos = k;
                if (pick < 0) {
                    below = cdf;
                    cdf += P[k];
                    if (cdf > ue) pick = k;
                }
            }
            if (pick < 0) { pick = last_pos; }   /* u beyond the rounded total: the last level that can occur */
            idx[e] = lo + pick;
            if (margin) {
                double a = ue - below, b = cdf - ue;
                margin[e] = a < b ? a : b;
            }
        }
        free(P);
    }
}

/* ------------------------------------------------------------------------
 * Gradient of the entropy term of the objective (eq. obj / eq. opt4, Sec. IV-D; Algorithm 1, the
 * step that computes the partials of H(w) and H(x)).  The paper prints no formula for these
 * partials (it only notes that they have an analytic form); this is the derivation used.
 *
 * H = -sum_k m_k log2 m_k with the marginal PMF m_k = (1/n) sum_e P_k(theta_e)  (eq. approx1/n).
 * For any parameter x:  dH/dx = -sum_k (log2 m_k + 1/ln 2) dm_k/dx = -sum_k log2(m_k) dm_k/dx,
 * because sum_k m_k = 1.  dm_k/dx = (1/n) sum_e dP_k(theta_e)/dx, and with d_k = theta - k q the
 * derivatives of the CPMF are (eq. partialw2 and eq. partialq2 of Appendix B; the third follows
 * in the same way from eq. CPMF):
 *   dP_k/dtheta = -2 alpha P_k d_k + 2 alpha P_k sum_j P_j d_j
 *   dP_k/dq     =  2 alpha P_k k d_k - 2 alpha P_k sum_j P_j j d_j
 *   dP_k/dalpha = -P_k d_k^2 + P_k sum_j P_j d_j^2
 * Outputs (each multiplied by `scale`, e.g. lambda * n for the total-bits term lambda * n * H):
 *   dtheta[e] = dH/dtheta_e,   d_delta = dH/dq,   d_alpha = dH/dalpha,
 * and, on request, the contribution of every entry to the last two (term_delta, term_alpha).
 * The marginal PMF is an input (the one the forward pass produced); levels with m_k = 0
 * contribute nothing (their P_k vanish wherever they are evaluated to working precision).
 * ---------------------------------------------------------------------- */
void cdl_oracle_entropy_bwd(const float *theta, int64_t n, int lo, int n_levels,
                            float delta_f, float alpha_f, int top_k,
                            const double *marg /* n_levels */, double scale,
                            double *dtheta /* n, nullable */, double *d_delta, double *d_alpha,
                            double *term_delta /* n, nullable */, double *term_alpha /* n, nullable */)
{
    const double delta = (double)delta_f, alpha = (double)alpha_f;
    double *ell = (double *)malloc(sizeof(double) * (size_t)n_levels);
    for (int k = 0; k < n_levels; ++k) ell[k] = marg[k] > 0.0 ? log2(marg[k]) : 0.0;
    const double inv_n = n > 0 ? 1.0 / (double)n : 0.0;
    double sd = 0.0, sa = 0.0;
#pragma omp parallel reduction(+ : sd, sa)
    {
        double *P = (double *)malloc(sizeof(double) * (size_t)n_levels);
#pragma omp for schedule(static)
        for (int64_t e = 0; e < n; ++e) {
            const double th = (double)theta[e];
            cpmf_core(th, lo, n_levels, delta, alpha, top_k, P, NULL);
            double e_d = 0.0, e_jd = 0.0, e_d2 = 0.0;
            for (int k = 0; k < n_levels; ++k) {
                const double j = (double)(lo + k), d = th - j * delta;
                e_d += P[k] * d; e_jd += P[k] * j * d; e_d2 += P[k] * d * d;
            }
            double g_th = 0.0, g_q = 0.0, g_al = 0.0;
            for (int k = 0; k < n_levels; ++k) {
                const double j = (double)(lo + k), d = th - j * delta;
                const double dP_th = -2.0 * alpha * P[k] * d + 2.0 * alpha * P[k] * e_d;
                const double dP_q = 2.0 * alpha * P[k] * j * d - 2.0 * alpha * P[k] * e_jd;
                const double dP_al = -P[k] * d * d + P[k] * e_d2;
                g_th -= ell[k] * dP_th;
                g_q -= ell[k] * dP_q;
                g_al -= ell[k] * dP_al;
            }
            g_th *= inv_n * scale; g_q *= inv_n * scale; g_al *= inv_n * scale;
            if (dtheta) dtheta[e] = g_th;
            sd += g_q;
            sa += g_al;
            if (term_delta) term_delta[e] = g_q;
            if (term_alpha) term_alpha[e] = g_al;
        }
        free(P);
    }
    free(ell);
    *d_delta = sd;
    *d_alpha = sa;
}

/* ------------------------------------------------------------------------
 * Layer compute over quantized operands (Sec. IV-A: forward and backward
 * passes run on the quantized weights and activations; Algorithm 1, the
 * forward and backward steps).  Operands are level indices; the quantized
 * values are a_idx*delta_a and b_idx*delta_b, so
 *   acc[m,n] = sum_k a_idx[m,k] * b_idx[n,k]          (exact integers)
 *   y[m,n]   = delta_a * delta_b * acc[m,n]
 * Both index matrices are row-major with the contraction index contiguous.
 * The indices are the level indices themselves, whatever the level set (the
 * paper's unsigned b-bit set {0, ..., 2^b - 1} of eq. repo_alphabet reaches 255
 * for the 8-bit first and last layers of Sec. V-B), hence 16-bit here; how a
 * library stores them is its own business.
 * ---------------------------------------------------------------------- */
void cdl_oracle_qgemm_fwd(const int16_t *a_idx, const int16_t *b_idx, int M, int N, int K,
                          float delta_a, float delta_b,
                          int32_t *acc /* M*N, nullable */, double *y /* M*N, nullable */)
{
    const double scale = (double)delta_a * (double)delta_b;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            int64_t s = 0;
            for (int k = 0; k < K; ++k)
                s += (int64_t)a_idx[(size_t)m * K + k] * (int64_t)b_idx[(size_t)n * K + k];
            if (acc) acc[(size_t)m * N + n] = (int32_t)s;
            if (y) y[(size_t)m * N + n] = scale * (double)s;
        }
    }
}

/*
 * The same layer compute for a convolutional layer (Sec. II: fully-connected and convolutional layers are
 * treated alike; Sec. IV-A: the forward pass runs on the quantized weights and activations; the ResNets of
 * Sec. V are stacks of such layers), written out as the definition of a 2-D cross-correlation with zero
 * padding - no im2col matrix is formed:
 *   acc[b,p,q,n] = sum_{r,s,c} x_idx[b, p*stride + r - pad, q*stride + s - pad, c] * w_idx[n,r,s,c]
 * over the taps whose input pixel lies inside the image (pixels outside count as level index 0, i.e. the
 * quantized value 0), y = delta_x * delta_w * acc.  Layouts: x [B][H][W][C], w [N][R][S][C], outputs
 * [B][P][Q][N] with P = (H + 2 pad - R) / stride + 1, Q = (W + 2 pad - S) / stride + 1.
 */
void cdl_oracle_qconv_fwd(const int16_t *x_idx, const int16_t *w_idx, int B, int H, int W, int C,
                          int N, int R, int S, int stride, int pad, float delta_x, float delta_w,
                          int32_t *acc /* B*P*Q*N, nullable */, double *y /* B*P*Q*N, nullable */)
{
    const int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    const double scale = (double)delta_x * (double)delta_w;
#pragma omp parallel for schedule(static) collapse(2)
    for (int b = 0; b < B; ++b) {
        for (int p = 0; p < P; ++p) {
            for (int q = 0; q < Q; ++q) {
                for (int n = 0; n < N; ++n) {
                    int64_t sum = 0;
                    for (int r = 0; r < R; ++r) {
                        const int h = p * stride + r - pad;
                        if (h < 0 || h >= H) continue;
                        for (int s = 0; s < S; ++s) {
                            const int w = q * stride + s - pad;
                            if (w < 0 || w >= W) continue;
                            const int16_t *xp = x_idx + (((size_t)b * H + h) * W + w) * C;
                            const int16_t *wp = w_idx + (((size_t)n * R + r) * S + s) * C;
                            for (int c = 0; c < C; ++c) sum += (int64_t)xp[c] * (int64_t)wp[c];
                        }
                    }
                    const size_t o = (((size_t)b * P + p) * Q + q) * N + n;
                    if (acc) acc[o] = (int32_t)sum;
                    if (y) y[o] = scale * (double)sum;
                }
            }
        }
    }
}

/*
 * Backward of the convolution above with respect to its two quantized operands (Algorithm 1, backward step, for
 * a convolutional layer): with g = dL/dy, fp32 [B][P][Q][N], xhat = delta_x * x_idx and what = delta_w * w_idx,
 *   d_x_hat[b,h,w,c] = sum over (p,q,r,s,n) with p*stride + r - pad = h and q*stride + s - pad = w of
 *                      g[b,p,q,n] * what[n,r,s,c]
 *   d_w_hat[n,r,s,c] = sum over (b,p,q) whose tap (r,s) lies inside the image of
 *                      g[b,p,q,n] * xhat[b, p*stride + r - pad, q*stride + s - pad, c]
 * i.e. every product x*w that enters y[b,p,q,n] hands g[b,p,q,n] times the other factor to each of its factors.
 */
void cdl_oracle_qconv_bwd(const float *g, const int16_t *x_idx, const int16_t *w_idx, int B, int H, int W, int C,
                          int N, int R, int S, int stride, int pad, float delta_x, float delta_w,
                          double *d_x_hat /* B*H*W*C, nullable */, double *d_w_hat /* N*R*S*C, nullable */)
{
    const int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
    if (d_x_hat) {
#pragma omp parallel for schedule(static) collapse(2)
        for (int b = 0; b < B; ++b)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    for (int c = 0; c < C; ++c) {
                        double sum = 0.0;
                        for (int p = 0; p < P; ++p) {
                            const int r = h - p * stride + pad;
                            if (r < 0 || r >= R) continue;
                            for (int q = 0; q < Q; ++q) {
                                const int s = w - q * stride + pad;
                                if (s < 0 || s >= S) continue;
                                const float *gp = g + (((size_t)b * P + p) * Q + q) * N;
                                for (int n = 0; n < N; ++n)
                                    sum += (double)gp[n] * (double)w_idx[(((size_t)n * R + r) * S + s) * C + c];
                            }
                        }
                        d_x_hat[(((size_t)b * H + h) * W + w) * C + c] = (double)delta_w * sum;
                    }
    }
    if (d_w_hat) {
#pragma omp parallel for schedule(static) collapse(2)
        for (int n = 0; n < N; ++n)
            for (int r = 0; r < R; ++r)
                for (int s = 0; s < S; ++s)
                    for (int c = 0; c < C; ++c) {
                        double sum = 0.0;
                        for (int b = 0; b < B; ++b)
                            for (int p = 0; p < P; ++p) {
                                const int h = p * stride + r - pad;
                                if (h < 0 || h >= H) continue;
                                for (int q = 0; q < Q; ++q) {
                                    const int w = q * stride + s - pad;
                                    if (w < 0 || w >= W) continue;
                                    sum += (double)g[(((size_t)b * P + p) * Q + q) * N + n] *
                                           (double)x_idx[(((size_t)b * H + h) * W + w) * C + c];
                                }
                            }
                        d_w_hat[(((size_t)n * R + r) * S + s) * C + c] = (double)delta_x * sum;
                    }
    }
}

/*
 * Backward of the same product with respect to the two quantized operands.
 * With Yhat = Ahat . Bhat^T, Ahat = delta_a*a_idx, Bhat = delta_b*b_idx and
 * g = dL/dYhat (kept in fp32: the paper quantizes weights and activations,
 * never the gradient signal):
 *   d_a_hat[m,k] = sum_n g[m,n] * Bhat[n,k] = delta_b * sum_n g[m,n] b_idx[n,k]
 *   d_b_hat[n,k] = sum_m g[m,n] * Ahat[m,k] = delta_a * sum_m g[m,n] a_idx[m,k]
 * These are dL/dQ_p(x) and dL/dQ_p(w) of Sec. IV-B, the factors that the
 * quantizer backward multiplies by dQd/dtheta.
 */
void cdl_oracle_qgemm_bwd(const float *g, const int16_t *a_idx, const int16_t *b_idx,
                          int M, int N, int K, float delta_a, float delta_b,
                          double *d_a_hat /* M*K, nullable */, double *d_b_hat /* N*K, nullable */)
{
    if (d_a_hat) {
#pragma omp parallel for schedule(static)
        for (int m = 0; m < M; ++m)
            for (int k = 0; k < K; ++k) {
                double s = 0.0;
                for (int n = 0; n < N; ++n)
                    s += (double)g[(size_t)m * N + n] * (double)b_idx[(size_t)n * K + k];
                d_a_hat[(size_t)m * K + k] = (double)delta_b * s;
            }
    }
    if (d_b_hat) {
#pragma omp parallel for schedule(static)
        for (int n = 0; n < N; ++n)
            for (int k = 0; k < K; ++k) {
                double s = 0.0;
                for (int m = 0; m < M; ++m)
                    s += (double)g[(size_t)m * N + n] * (double)a_idx[(size_t)m * K + k];
                d_b_hat[(size_t)n * K + k] = (double)delta_a * s;
            }
    }
}

/* ------------------------------------------------------------------------
 * Bits per entry of a quantized tensor under Huffman coding of its level indices (Sec. V-A,
 * eq. Nofbits: the paper reports the average Huffman code length per weight / activation of a layer).  counts[k] = number of entries equal to level lo+k.
 * A Huffman code is built by repeatedly merging the two least frequent nodes; the total code
 * length in bits is the sum of the weights of all merged nodes, and it is the same for every
 * Huffman tree of the same counts (ties may be broken either way), so only the total is returned
 * besides the counts.  Reading for the degenerate case the paper does not mention: a tensor in
 * which a single level occurs costs one bit per entry; an empty tensor costs 0.
 * ---------------------------------------------------------------------- */
void cdl_oracle_huffman_bits(const int16_t *idx, int64_t n, int lo, int n_levels,
                             int64_t *counts /* n_levels */, double *total_bits, double *bits_per_entry)
{
    for (int k = 0; k < n_levels; ++k) counts[k] = 0;
    for (int64_t e = 0; e < n; ++e) {
        int k = (int)idx[e] - lo;
        if (k >= 0 && k < n_levels) counts[k] += 1;
    }
    int64_t *w = (int64_t *)malloc(sizeof(int64_t) * (size_t)n_levels);
    int m = 0;
    for (int k = 0; k < n_levels; ++k) if (counts[k] > 0) w[m++] = counts[k];
    double total = 0.0;
    if (m == 1) total = (double)w[0];
    while (m > 1) {
        /* the two smallest weights */
        int a = 0, b = 1;
        if (w[b] < w[a]) { a = 1; b = 0; }
        for (int i = 2; i < m; ++i) {
            if (w[i] < w[a]) { b = a; a = i; }
            else if (w[i] < w[b]) { b = i; }
        }
        int64_t merged = w[a] + w[b];
        total += (double)merged;
        /* replace a by the merged node, remove b */
        w[a] = merged;
        w[b] = w[m - 1];
        --m;
    }
    free(w);
    *total_bits = total;
    *bits_per_entry = n > 0 ? total / (double)n : 0.0;
}
