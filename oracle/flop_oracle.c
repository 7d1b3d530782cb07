/*
 * fp64 CPU oracle for the FLOP gated factorized linear layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the HIP path and the
 * product never calls it: only the test-suite, the smoke check and the
 * benchmark's CPU-baseline leg may load it.
 *
 * Everything is evaluated in double precision, row-major, contiguous
 * (leading dimension == number of columns), with straightforward loops.
 * OpenMP only spreads independent output rows over threads; no blocking,
 * fusion or reordering beyond the definitions below.
 *
 * Notation (Section 4.1, "Structured Pruning using Factorization", batched
 * row form of W = P G Q):
 *   x[n,d]  tokens          Q[r,d]  rows q_k        P[dout,r]  columns p_k
 *   alpha[r], u[r], z[r]    one gate per rank-1 component, shared by the batch
 *   h = x Q^T   g = h .* z   y = g P^T
 *
 * Parity pins (tests marked "not gpu"): closed-form sampler points (train and
 * deterministic mode, value and slope), noise at the ends of its range, Monte-Carlo
 * agreement of the sampler with Eq.(3), all-gates-open == dense product via a
 * library matmul, closing a gate == deleting the component, finite differences
 * for every gradient, brute-force compaction, one-hot embedding equivalence.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* logistic function, written so that neither branch overflows */
static double logistic(double t)
{
    if (t >= 0.0) return 1.0 / (1.0 + exp(-t));
    double e = exp(t);
    return e / (1.0 + e);
}

/*
 * Hard-Concrete inverse CDF (Section 3, the unnumbered display defining
 * s, s-bar and z), with the temperature beta of the cited Louizos et al. form;
 * beta = 1 is the paper's expression.
 *   mode 0 (training):      s = sigmoid((log u - log(1-u) + alpha) / beta)
 *   mode 1 (deterministic): s = sigmoid(alpha)            (u is not read)
 *   sbar = s (r - l) + l ;  z = min(1, max(0, sbar))
 * dzda (may be NULL) receives dz/dalpha: the clamp passes gradient where
 * 0 <= sbar <= 1, and d sbar / d alpha = (r - l) s (1 - s) / beta
 * (no 1/beta in deterministic mode).
 */
void oracle_gate_sample(const double *alpha, const double *u, int64_t r,
                        double beta, double l, double rr, int mode,
                        double *z, double *dzda)
{
    for (int64_t k = 0; k < r; ++k) {
        double t, inv_temp;
        if (mode == 0) {
            t = (log(u[k]) - log1p(-u[k]) + alpha[k]) / beta;
            inv_temp = 1.0 / beta;
        } else {
            t = alpha[k];
            inv_temp = 1.0;
        }
        double s = logistic(t);
        double one_minus_s = logistic(-t);
        double sbar = s * (rr - l) + l;
        double zk = sbar;
        if (zk < 0.0) zk = 0.0;
        if (zk > 1.0) zk = 1.0;
        z[k] = zk;
        if (dzda) {
            int inside = (sbar >= 0.0 && sbar <= 1.0);
            dzda[k] = inside ? (rr - l) * s * one_minus_s * inv_temp : 0.0;
        }
    }
}

/*
 * Expected L0 norm, Eq.(3), with the temperature written out:
 *   p_k = P[z_k > 0] = sigmoid(alpha_k - beta * log(-l / r))
 *   out = sum_k w_k p_k          (w == NULL means w_k = 1)
 * The weights are the parameter-block sizes of Section 4.3 (s(alpha)).
 * grad (may be NULL) receives d out / d alpha_k = w_k p_k (1 - p_k).
 */
void oracle_expected_l0(const double *alpha, const double *w, int64_t R,
                        double beta, double l, double rr,
                        double *out, double *grad)
{
    double shift = beta * log(-l / rr);
    double sum = 0.0;
    for (int64_t k = 0; k < R; ++k) {
        double p = logistic(alpha[k] - shift);
        double q = logistic(-(alpha[k] - shift));
        double wk = w ? w[k] : 1.0;
        sum += wk * p;
        if (grad) grad[k] = wk * p * q;
    }
    *out = sum;
}

/*
 * Forward of the gated factorized layer (Section 4.1, W = P G Q applied to
 * each token):  h = x Q^T,  g = h .* z,  y = g P^T.
 * h and g are returned too (either may be NULL).
 */
void oracle_fwd(int64_t n, int64_t d, int64_t r, int64_t dout,
                const double *x, const double *Q, const double *P,
                const double *z, double *h, double *g, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double *grow = (double *)malloc((size_t)r * sizeof(double));
        for (int64_t k = 0; k < r; ++k) {
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (int64_t j = 0; j < d; ++j) acc += x[i * d + j] * Q[k * d + j];
            if (h) h[i * r + k] = acc;
            grow[k] = acc * z[k];
            if (g) g[i * r + k] = grow[k];
        }
        for (int64_t m = 0; m < dout; ++m) {
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (int64_t k = 0; k < r; ++k) acc += grow[k] * P[m * r + k];
            y[i * dout + m] = acc;
        }
        free(grow);
    }
}

/*
 * Second, independent evaluation of the same map through the sum of rank-1
 * components (Section 4.1):  W = sum_k z_k p_k q_k  (dout x d),  y = x W^T.
 * W (dout*d) is returned as well.
 */
void oracle_fwd_rank1(int64_t n, int64_t d, int64_t r, int64_t dout,
                      const double *x, const double *Q, const double *P,
                      const double *z, double *W, double *y)
{
    memset(W, 0, (size_t)(dout * d) * sizeof(double));
    for (int64_t k = 0; k < r; ++k)
        for (int64_t m = 0; m < dout; ++m) {
            double c = z[k] * P[m * r + k];
            for (int64_t j = 0; j < d; ++j) W[m * d + j] += c * Q[k * d + j];
        }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int64_t m = 0; m < dout; ++m) {
            double acc = 0.0;
            for (int64_t j = 0; j < d; ++j) acc += x[i * d + j] * W[m * d + j];
            y[i * dout + m] = acc;
        }
}

/*
 * Backward of the layer by the chain rule through y = ((x Q^T) .* z) P^T and
 * z = G(u; alpha) (Section 3: gradient updates reach both theta and alpha).
 * Given dy[n,dout]:
 *   dg = dy P                 dP = dy^T g
 *   dz_k = sum_i dg_ik h_ik   dh = dg .* z
 *   dx = dh Q                 dQ = dh^T x
 *   dalpha_k = dz_k * dzda_k
 * u is data and receives no gradient.  Any output pointer may be NULL.
 */
void oracle_bwd(int64_t n, int64_t d, int64_t r, int64_t dout,
                const double *dy, const double *x, const double *Q,
                const double *P, const double *z, const double *dzda,
                double *dx, double *dQ, double *dP, double *dz, double *dalpha)
{
    size_t nr = (size_t)n * (size_t)r;
    double *h = (double *)malloc(nr * sizeof(double));
    double *g = (double *)malloc(nr * sizeof(double));
    double *dg = (double *)calloc(nr, sizeof(double));
    double *dh = (double *)malloc(nr * sizeof(double));
    double *dzv = (double *)calloc((size_t)r, sizeof(double));

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t k = 0; k < r; ++k) {
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (int64_t j = 0; j < d; ++j) acc += x[i * d + j] * Q[k * d + j];
            h[i * r + k] = acc;
            g[i * r + k] = acc * z[k];
        }
        /* dg_i = dy_i P */
        for (int64_t m = 0; m < dout; ++m) {
            double a = dy[i * dout + m];
            for (int64_t k = 0; k < r; ++k) dg[i * r + k] += a * P[m * r + k];
        }
        for (int64_t k = 0; k < r; ++k) dh[i * r + k] = dg[i * r + k] * z[k];
        /* dx_i = dh_i Q */
        if (dx) {
            for (int64_t j = 0; j < d; ++j) dx[i * d + j] = 0.0;
            for (int64_t k = 0; k < r; ++k) {
                double a = dh[i * r + k];
                for (int64_t j = 0; j < d; ++j) dx[i * d + j] += a * Q[k * d + j];
            }
        }
    }

    /* dz_k = sum_i dg_ik h_ik (sequential over tokens, fixed order) */
    for (int64_t i = 0; i < n; ++i)
        for (int64_t k = 0; k < r; ++k) dzv[k] += dg[i * r + k] * h[i * r + k];

    if (dP) {
#pragma omp parallel for schedule(static)
        for (int64_t m = 0; m < dout; ++m) {
            for (int64_t k = 0; k < r; ++k) dP[m * r + k] = 0.0;
            for (int64_t i = 0; i < n; ++i) {
                double a = dy[i * dout + m];
                for (int64_t k = 0; k < r; ++k) dP[m * r + k] += a * g[i * r + k];
            }
        }
    }
    if (dQ) {
#pragma omp parallel for schedule(static)
        for (int64_t k = 0; k < r; ++k) {
            for (int64_t j = 0; j < d; ++j) dQ[k * d + j] = 0.0;
            for (int64_t i = 0; i < n; ++i) {
                double a = dh[i * r + k];
                for (int64_t j = 0; j < d; ++j) dQ[k * d + j] += a * x[i * d + j];
            }
        }
    }
    for (int64_t k = 0; k < r; ++k) {
        if (dz) dz[k] = dzv[k];
        if (dalpha) dalpha[k] = dzv[k] * dzda[k];
    }
    free(h); free(g); free(dg); free(dh); free(dzv);
}

/*
 * Compaction for inference (Sections 4.1 and 4.4): component k is kept iff
 * z_k > 0; survivors keep their original (ascending) order.
 *   idx[0..r'-1]  kept indices          zc = z[idx]
 *   Pc[dout, r']  = P[:, idx]           Qc[r', d] = Q[idx, :]
 * With absorb != 0 the gate value is folded into Q:  Qc[t,:] = z[idx[t]] * Q[idx[t],:].
 * Outputs are sized for the worst case by the caller (r' <= r) but written
 * densely with leading dimensions r' (Pc) and d (Qc).  Returns r'.
 */
int64_t oracle_compact(int64_t d, int64_t r, int64_t dout,
                       const double *z, const double *Q, const double *P,
                       int absorb, int64_t *idx, double *Qc, double *Pc, double *zc)
{
    int64_t rp = 0;
    for (int64_t k = 0; k < r; ++k)
        if (z[k] > 0.0) idx[rp++] = k;
    for (int64_t t = 0; t < rp; ++t) {
        int64_t k = idx[t];
        if (zc) zc[t] = z[k];
        if (Qc)
            for (int64_t j = 0; j < d; ++j)
                Qc[t * d + j] = absorb ? z[k] * Q[k * d + j] : Q[k * d + j];
    }
    if (Pc)
        for (int64_t m = 0; m < dout; ++m)
            for (int64_t t = 0; t < rp; ++t) Pc[m * rp + t] = P[m * r + idx[t]];
    return rp;
}

/*
 * One cluster of the gated adaptive embedding (Section 4.2): the cluster owns
 * vocabulary ids [lo, hi), an embedding table E[hi-lo, dc], a projection
 * O[dc, d] and gates z[dc]; the embedding of word id t is (E[t-lo,:] .* z) O,
 * i.e. row t-lo of E G O.  Tokens whose id lies outside [lo, hi) are left
 * untouched in y, so calling this once per cluster fills every row.
 */
void oracle_embed_fwd(int64_t nt, const int64_t *ids, int64_t lo, int64_t hi,
                      int64_t dc, int64_t d, const double *E, const double *O,
                      const double *z, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nt; ++i) {
        if (ids[i] < lo || ids[i] >= hi) continue;
        const double *e = E + (ids[i] - lo) * dc;
        for (int64_t m = 0; m < d; ++m) y[i * d + m] = 0.0;
        for (int64_t a = 0; a < dc; ++a) {
            double ga = e[a] * z[a];
            for (int64_t m = 0; m < d; ++m) y[i * d + m] += ga * O[a * d + m];
        }
    }
}

/*
 * Backward of one embedding cluster.  For every token i of the cluster
 * (row = ids[i]-lo, e = E[row,:], g = e .* z):
 *   dg_i = dy_i O^T          dO += g_i^T dy_i
 *   dE[row,:] += dg_i .* z   (tokens repeating a word accumulate)
 *   dz += dg_i .* e          dalpha = dz .* dzda
 * dE[hi-lo, dc], dO[dc, d], dz[dc], dalpha[dc] are overwritten.
 */
void oracle_embed_bwd(int64_t nt, const int64_t *ids, int64_t lo, int64_t hi,
                      int64_t dc, int64_t d, const double *dy, const double *E,
                      const double *O, const double *z, const double *dzda,
                      double *dE, double *dO, double *dz, double *dalpha)
{
    memset(dE, 0, (size_t)((hi - lo) * dc) * sizeof(double));
    memset(dO, 0, (size_t)(dc * d) * sizeof(double));
    double *dzv = (double *)calloc((size_t)dc, sizeof(double));
    double *dg = (double *)calloc((size_t)(nt * dc) + 1, sizeof(double));

    /* dg_i = dy_i O^T, one token per iteration */
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nt; ++i) {
        if (ids[i] < lo || ids[i] >= hi) continue;
        for (int64_t a = 0; a < dc; ++a) {
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (int64_t m = 0; m < d; ++m) acc += dy[i * d + m] * O[a * d + m];
            dg[i * dc + a] = acc;
        }
    }
    /* dO[a,:] = sum_i g_ia dy_i, tokens in order; rows a are independent */
#pragma omp parallel for schedule(static)
    for (int64_t a = 0; a < dc; ++a)
        for (int64_t i = 0; i < nt; ++i) {
            if (ids[i] < lo || ids[i] >= hi) continue;
            double ga = E[(ids[i] - lo) * dc + a] * z[a];
            for (int64_t m = 0; m < d; ++m) dO[a * d + m] += ga * dy[i * d + m];
        }
    /* scatter-add into dE and the gate gradient, tokens in order */
    for (int64_t i = 0; i < nt; ++i) {
        if (ids[i] < lo || ids[i] >= hi) continue;
        int64_t row = ids[i] - lo;
        for (int64_t a = 0; a < dc; ++a) {
            dE[row * dc + a] += dg[i * dc + a] * z[a];
            dzv[a] += dg[i * dc + a] * E[row * dc + a];
        }
    }
    for (int64_t a = 0; a < dc; ++a) {
        if (dz) dz[a] = dzv[a];
        if (dalpha) dalpha[a] = dzv[a] * dzda[a];
    }
    free(dzv); free(dg);
}

/*
 * Deterministic inference mask (Section 4.4, second paragraph): every gate gets
 * its Eq.(3) value p_k = sigmoid(alpha_k - beta * log(-l / r)); the `keep`
 * largest stay, the others are set to zero.  p is increasing in alpha, so the
 * gates are ranked by alpha itself (ranking the rounded p could only add ties);
 * equal alphas: the lower index wins.  Selection by repeated search for the
 * best remaining gate, O(R * keep), on purpose.
 * z[k] = p_k for the kept gates, 0 otherwise.  Returns the number kept
 * (= min(keep, R), keep < 0 counts as 0).
 */
int64_t oracle_topk_mask(const double *alpha, int64_t R, int64_t keep,
                         double beta, double l, double rr, double *z)
{
    double shift = beta * log(-l / rr);
    char *taken = (char *)calloc((size_t)(R > 0 ? R : 1), 1);
    int64_t kept = 0;
    for (int64_t k = 0; k < R; ++k) z[k] = 0.0;
    for (int64_t t = 0; t < keep && t < R; ++t) {
        int64_t best = -1;
        for (int64_t k = 0; k < R; ++k) {
            if (taken[k]) continue;
            if (best < 0 || alpha[k] > alpha[best]) best = k;   /* strict: ties keep the lower index */
        }
        taken[best] = 1;
        z[best] = logistic(alpha[best] - shift);
        ++kept;
    }
    free(taken);
    return kept;
}

/*
 * Augmented-Lagrangian size penalty (Section 4.3):
 *   g(lambda, alpha) = lambda1 (s - t) + lambda2 (s - t)^2,    s = scale * sum_k w_k p_k  (Eq.(3), block sizes w)
 * with the gradients of the adversarial game: descent on alpha, ascent on lambda,
 *   dg/dalpha_k = (lambda1 + 2 lambda2 (s - t)) * scale * w_k p_k (1 - p_k)
 *   dg/dlambda1 = s - t            dg/dlambda2 = (s - t)^2
 * scale turns the expected parameter count into the unit of t (1 for counts,
 * 1 / total for a fraction).  out = {g, dg/dlambda1, dg/dlambda2}; dalpha (may
 * be NULL) is overwritten.
 */
void oracle_lagrangian(const double *alpha, const double *w, int64_t R,
                       double beta, double l, double rr,
                       double scale, double t, double lambda1, double lambda2,
                       double *out, double *dalpha)
{
    double shift = beta * log(-l / rr);
    double s = 0.0;
    for (int64_t k = 0; k < R; ++k) s += (w ? w[k] : 1.0) * logistic(alpha[k] - shift);
    s *= scale;
    double viol = s - t;
    out[0] = lambda1 * viol + lambda2 * viol * viol;
    out[1] = viol;
    out[2] = viol * viol;
    if (dalpha)
        for (int64_t k = 0; k < R; ++k) {
            double p = logistic(alpha[k] - shift), q = logistic(-(alpha[k] - shift));
            dalpha[k] = (lambda1 + 2.0 * lambda2 * viol) * scale * (w ? w[k] : 1.0) * p * q;
        }
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
