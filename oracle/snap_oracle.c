/*
 * CPU oracle for the GPU-resident local solver of Snap ML (arXiv 1803.06333, Section 3.1):
 * stochastic coordinate descent (SCD) for generalized linear models, eq. (1),
 *
 *        min_alpha  f(A alpha) + sum_i g_i(alpha_i),        shared vector v := A alpha.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, sequential fp64
 * implementation written from the paper; it shares no code with the HIP library and must only be
 * used by tests, the smoke check and the benchmark's CPU-baseline leg.
 *
 * The GPU solver of the paper is asynchronous; its synchronous limit -- one coordinate at a time,
 * every update seeing the fully updated v -- is what is written out here.  Data are fp32 (as the
 * GPU path stores them); the model, v and every sum are fp64.
 *
 * Notation: X is n x d (examples x features), y the labels, lambda > 0, and
 *
 *        P(w) = (1/n) sum_i loss(y_i, x_i.w) + (lambda/2) ||w||^2 .
 *
 *  primal form: coordinates are features, alpha = w, A = X, v = X w (length n);
 *               f(v) = (1/n) sum_i loss(y_i, v_i),  g_j(w_j) = (lambda/2) w_j^2.
 *  dual form: coordinates are examples, alpha in [0,1]^n, A = X^T diag(y),
 *               v = X^T (y o alpha) (length d), w = v/(lambda n); f(v) = ||v||^2/(2 lambda n^2);
 *               hinge:    g_i(a) = -a/n + indicator[0,1](a);
 *               logistic: g_i(a) = (a ln a + (1-a) ln(1-a))/n on (0,1).
 *
 * An optional l1 term (eq. (1) admits lasso and elastic-net regularisers) turns the primal
 * regulariser into g_j(w) = (lambda/2) w^2 + lambda1 |w|.
 *
 * The paper leaves the objective scaling, the update formulas, the random-key generator and the
 * duality gap unstated; the readings taken are written next to each function.
 *
 * Pinned (tests/test_oracle_*.py): ridge against the normal equations, logistic against brute
 * force and an independent quasi-Newton solve, hinge against brute-force primal minimisation and
 * the box/monotonicity invariants, the gap against its closed forms and P - P*, the sparse
 * products against dense matmul, the logistic dual against the primal logistic solution (strong
 * duality, alpha* = sigmoid(-y x.w*)) and brute force.  Parity unpinned: nothing in this file.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { LOSS_RIDGE = 0, LOSS_LOGISTIC = 1, LOSS_HINGE = 2 };

/* ------------------------------------------------------------------------------------------- */
/* Permutation of the coordinates (Section 3.2, "Streaming Permutation Generation"): one 32-bit  */
/* pseudo-random key per coordinate from an xorshift generator, then a sort of the keys carrying */
/* the indices.  Reading taken: the key is a pure function of (seed, chunk, coordinate) -- a      */
/* 64-bit integer mix seeds a 32-bit xorshift state (forced non-zero), four rounds of the        */
/* (13,17,5) xorshift follow -- so that any number of threads produce the same keys; ties between */
/* equal keys are broken by the smaller coordinate index.                                        */
/* ------------------------------------------------------------------------------------------- */
static uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

uint32_t oracle_key(uint64_t seed, uint32_t chunk, uint32_t c)
{
    uint64_t z = mix64(seed ^ mix64((uint64_t)chunk + 0x632BE59BD9B4E019ull));
    z = mix64(z + (uint64_t)c * 0x9E3779B97F4A7C15ull);
    uint32_t x = (uint32_t)(z ^ (z >> 32));
    if (x == 0u) x = 0x6C078965u;
    for (int r = 0; r < 4; ++r) {
        x ^= x << 13;
        x ^= x >> 17;
        x ^= x << 5;
    }
    return x;
}

static int cmp_u64(const void *a, const void *b)
{
    uint64_t x = *(const uint64_t *)a, y = *(const uint64_t *)b;
    return (x > y) - (x < y);
}

/* keys_out may be NULL.  perm_out[k] = the coordinate visited k-th. */
int oracle_perm(uint64_t seed, uint32_t chunk, uint32_t m, uint32_t *keys_out, uint32_t *perm_out)
{
    uint64_t *comp = (uint64_t *)malloc((size_t)(m ? m : 1) * sizeof(uint64_t));
    if (!comp) return -1;
    for (uint32_t c = 0; c < m; ++c) {
        uint32_t k = oracle_key(seed, chunk, c);
        if (keys_out) keys_out[c] = k;
        comp[c] = ((uint64_t)k << 32) | c;      /* unique composites: equal keys order by index */
    }
    qsort(comp, m, sizeof(uint64_t), cmp_u64);
    for (uint32_t k = 0; k < m; ++k) perm_out[k] = (uint32_t)(comp[k] & 0xFFFFFFFFu);
    free(comp);
    return 0;
}

/* ------------------------------------------------------------------------------------------- */
/* Scalar pieces of the losses                                                                   */
/* ------------------------------------------------------------------------------------------- */
static double sigmoid(double t)            /* 1/(1+exp(-t)), overflow safe */
{
    if (t >= 0) return 1.0 / (1.0 + exp(-t));
    double e = exp(t);
    return e / (1.0 + e);
}

static double log1pexp(double t)           /* log(1+exp(t)), overflow safe */
{
    return t > 0 ? t + log1p(exp(-t)) : log1p(exp(t));
}

static double loss_value(int loss, double y, double z)
{
    switch (loss) {
    case LOSS_RIDGE: return 0.5 * (z - y) * (z - y);
    case LOSS_LOGISTIC: return log1pexp(-y * z);
    default: { double m = 1.0 - y * z; return m > 0 ? m : 0.0; }
    }
}

/* d loss / d z  (ridge, logistic) */
static double loss_d1(int loss, double y, double z)
{
    if (loss == LOSS_RIDGE) return z - y;
    return -y * sigmoid(-y * z);
}

/* d^2 loss / d z^2 (ridge, logistic) */
static double loss_d2(int loss, double y, double z)
{
    if (loss == LOSS_RIDGE) return 1.0;
    double p = sigmoid(-y * z);
    return p * (1.0 - p);
}

/* ------------------------------------------------------------------------------------------- */
/* One primal coordinate update (Section 3.1).  Ridge: the exact minimiser of P along w_j        */
/* (closed form).  Logistic: one Newton step on the coordinate problem from the current w_j,     */
/* with the exact first and second derivative, both inner products of the column with a function */
/* of v:                                                                                         */
/*     g = (1/n) sum_i a_ij loss'(y_i, v_i) + lambda w_j                                         */
/*     h = (1/n) sum_i a_ij^2 loss''(y_i, v_i) + lambda          ( >= lambda > 0 )               */
/*     delta = -g/h ;  w_j += delta ;  v_i += delta a_ij on the column's support.                */
/* With an l1 term the same quadratic model of the loss along w_j,                               */
/*     gf delta + (hf/2) delta^2,  gf = (1/n) sum a loss',  hf = (1/n) sum a^2 loss'',            */
/* plus (lambda/2)(w+delta)^2 + lambda1 |w+delta| is minimised exactly by soft-thresholding:      */
/*     w_new = S(hf w - gf, lambda1) / (hf + lambda),   S(t, k) = sign(t) max(|t| - k, 0)         */
/* (lambda1 = 0 gives the step above; for ridge loss it is the exact coordinate minimiser).       */
/* ------------------------------------------------------------------------------------------- */
static double soft_threshold(double t, double k)
{
    if (t > k) return t - k;
    if (t < -k) return t + k;
    return 0.0;
}

static double primal_step(double gsum, double hsum, double n, double lambda, double lambda1, double wj)
{
    double gf = gsum / n, hf = hsum / n;
    if (lambda1 == 0.0) return -(gf + lambda * wj) / (hf + lambda);
    return soft_threshold(hf * wj - gf, lambda1) / (hf + lambda) - wj;
}

static void primal_update_sparse(int loss, int64_t n, const int64_t *colptr, const int32_t *row,
                                 const float *val, const float *y, double lambda, double lambda1,
                                 int64_t j, double *w, double *v)
{
    double g = 0.0, h = 0.0;
    for (int64_t k = colptr[j]; k < colptr[j + 1]; ++k) {
        double a = val[k];
        int64_t i = row[k];
        g += a * loss_d1(loss, y[i], v[i]);
        h += a * a * loss_d2(loss, y[i], v[i]);
    }
    double delta = primal_step(g, h, (double)n, lambda, lambda1, w[j]);
    w[j] += delta;
    for (int64_t k = colptr[j]; k < colptr[j + 1]; ++k) v[row[k]] += delta * (double)val[k];
}

/* Coordinates c0 + perm[0..mc) are visited in that order (c0 = first coordinate of the chunk). */
void oracle_epoch_primal_sparse(int loss, int64_t n, const int64_t *colptr, const int32_t *row,
                                const float *val, const float *y, double lambda, double lambda1,
                                const uint32_t *perm, int64_t c0, int64_t mc, double *w, double *v)
{
    for (int64_t k = 0; k < mc; ++k)
        primal_update_sparse(loss, n, colptr, row, val, y, lambda, lambda1, c0 + perm[k], w, v);
}

/* Dense column-major matrix: element (i, j) at A[j*n + i]. */
void oracle_epoch_primal_dense(int loss, int64_t n, const float *A, const float *y, double lambda,
                               double lambda1, const uint32_t *perm, int64_t c0, int64_t mc, double *w,
                               double *v)
{
    for (int64_t k = 0; k < mc; ++k) {
        int64_t j = c0 + perm[k];
        const float *a = A + (size_t)j * (size_t)n;
        double g = 0.0, h = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            g += (double)a[i] * loss_d1(loss, y[i], v[i]);
            h += (double)a[i] * (double)a[i] * loss_d2(loss, y[i], v[i]);
        }
        double delta = primal_step(g, h, (double)n, lambda, lambda1, w[j]);
        w[j] += delta;
        for (int64_t i = 0; i < n; ++i) v[i] += delta * (double)a[i];
    }
}

/* ------------------------------------------------------------------------------------------- */
/* One dual coordinate update for the hinge loss (closed form with box clipping).  The dual       */
/*     D(alpha) = (1/n) sum_i alpha_i - (lambda/2) ||w(alpha)||^2,   w = v/(lambda n)             */
/* is quadratic in alpha_i: dD/dalpha_i = (1 - m)/n with m = y_i x_i.w, and -d2D = q/n with        */
/* q = ||x_i||^2/(lambda n); its maximiser over [0,1] is clip(alpha_i + (1-m)/q, 0, 1).           */
/* An empty row (q = 0) has dD/dalpha_i = 1/n > 0, so alpha_i = 1; v does not change.             */
/* ------------------------------------------------------------------------------------------- */
void oracle_epoch_dual_hinge(int64_t n, const int64_t *rowptr, const int32_t *col, const float *val,
                             const float *y, double lambda, const uint32_t *perm, int64_t c0,
                             int64_t mc, double *alpha, double *v)
{
    const double ln = lambda * (double)n;
    for (int64_t k = 0; k < mc; ++k) {
        int64_t i = c0 + perm[k];
        double dot = 0.0, nrm = 0.0;
        for (int64_t t = rowptr[i]; t < rowptr[i + 1]; ++t) {
            dot += (double)val[t] * v[col[t]];
            nrm += (double)val[t] * (double)val[t];
        }
        double anew;
        if (nrm == 0.0) {
            anew = 1.0;
        } else {
            double m = (double)y[i] * dot / ln;
            double q = nrm / ln;
            anew = alpha[i] + (1.0 - m) / q;
            if (anew < 0.0) anew = 0.0;
            if (anew > 1.0) anew = 1.0;
        }
        double delta = anew - alpha[i];
        alpha[i] = anew;
        if (delta != 0.0)
            for (int64_t t = rowptr[i]; t < rowptr[i + 1]; ++t)
                v[col[t]] += delta * (double)y[i] * (double)val[t];
    }
}

/* ------------------------------------------------------------------------------------------- */
/* Sparse / dense products (the definitions, row by row)                                         */
/* compressed(ptr, idx, val) with m major slices: out = M x (one dot per slice) when trans = 0,  */
/* out = M^T x (scatter of x[slice] * slice) when trans = 1.  A CSR of X is X itself; a CSC of X  */
/* is the CSR of X^T.                                                                            */
/* ------------------------------------------------------------------------------------------- */
void oracle_compressed_matvec(int64_t m, int64_t len_out, const int64_t *ptr, const int32_t *idx,
                              const float *val, const double *x, int trans, double *out)
{
    if (!trans) {
#pragma omp parallel for schedule(dynamic, 256)
        for (int64_t s = 0; s < m; ++s) {
            double acc = 0.0;
            for (int64_t k = ptr[s]; k < ptr[s + 1]; ++k) acc += (double)val[k] * x[idx[k]];
            out[s] = acc;
        }
    } else {
        for (int64_t r = 0; r < len_out; ++r) out[r] = 0.0;
        for (int64_t s = 0; s < m; ++s)
            for (int64_t k = ptr[s]; k < ptr[s + 1]; ++k) out[idx[k]] += (double)val[k] * x[s];
    }
}

/* column-major n x d: out = A x (length n) when trans = 0, out = A^T u (length d) when trans = 1 */
void oracle_dense_matvec(int64_t n, int64_t d, const float *A, const double *x, int trans, double *out)
{
    if (!trans) {
        for (int64_t i = 0; i < n; ++i) out[i] = 0.0;
        for (int64_t j = 0; j < d; ++j) {
            const float *a = A + (size_t)j * (size_t)n;
            for (int64_t i = 0; i < n; ++i) out[i] += (double)a[i] * x[j];
        }
    } else {
#pragma omp parallel for
        for (int64_t j = 0; j < d; ++j) {
            const float *a = A + (size_t)j * (size_t)n;
            double acc = 0.0;
            for (int64_t i = 0; i < n; ++i) acc += (double)a[i] * x[i];
            out[j] = acc;
        }
    }
}

/* ------------------------------------------------------------------------------------------- */
/* One dual coordinate update for the logistic loss (Section 3.1: no closed form, a single       */
/* Newton step from the previous value).  With the conjugate of the logistic loss the dual is    */
/*     D(alpha) = -(1/n) sum_i [alpha_i ln alpha_i + (1-alpha_i) ln(1-alpha_i)]                   */
/*                - (lambda/2) ||w(alpha)||^2,     alpha in (0,1)^n,  w = v/(lambda n),           */
/* and along alpha_i, with m = y_i x_i.w and q = ||x_i||^2/(lambda n),                            */
/*     -n dD/dalpha_i = ln(alpha_i/(1-alpha_i)) + m,     -n d2D/dalpha_i^2 = 1/(alpha_i(1-alpha_i)) + q. */
/* Readings taken where the paper is silent: the start is alpha_i = 1/2 (the entropy is not       */
/* defined at Algorithm 1's alpha = 0; 1/2 is the dual optimum of w = 0), and the Newton iterate   */
/* is clipped to [2^-20, 1 - 2^-20], both exactly representable in fp32.                          */
/* ------------------------------------------------------------------------------------------- */
#define ORACLE_ALPHA_EPS (1.0 / 1048576.0)

void oracle_epoch_dual_logistic(int64_t n, const int64_t *rowptr, const int32_t *col, const float *val,
                                const float *y, double lambda, const uint32_t *perm, int64_t c0,
                                int64_t mc, double *alpha, double *v)
{
    const double ln = lambda * (double)n;
    for (int64_t k = 0; k < mc; ++k) {
        int64_t i = c0 + perm[k];
        double dot = 0.0, nrm = 0.0;
        for (int64_t t = rowptr[i]; t < rowptr[i + 1]; ++t) {
            dot += (double)val[t] * v[col[t]];
            nrm += (double)val[t] * (double)val[t];
        }
        double a = alpha[i];
        double m = (double)y[i] * dot / ln;
        double q = nrm / ln;
        double g = log(a) - log1p(-a) + m;
        double h = 1.0 / (a * (1.0 - a)) + q;
        double anew = a - g / h;
        if (anew < ORACLE_ALPHA_EPS) anew = ORACLE_ALPHA_EPS;
        if (anew > 1.0 - ORACLE_ALPHA_EPS) anew = 1.0 - ORACLE_ALPHA_EPS;
        double delta = anew - a;
        alpha[i] = anew;
        if (delta != 0.0)
            for (int64_t t = rowptr[i]; t < rowptr[i + 1]; ++t)
                v[col[t]] += delta * (double)y[i] * (double)val[t];
    }
}

/* ------------------------------------------------------------------------------------------- */
/* Objectives.  Reading taken for the scaling that eq. (1) leaves open:                          */
/*     P(w) = (1/n) sum_i loss(y_i, z_i) + (lambda/2) ||w||^2,   z = X w.                         */
/* ------------------------------------------------------------------------------------------- */
double oracle_primal_objective(int loss, int64_t n, int64_t d, const double *z, const float *y,
                               const double *w, double lambda, double lambda1)
{
    double s = 0.0, r = 0.0, a = 0.0;
#pragma omp parallel for reduction(+ : s)
    for (int64_t i = 0; i < n; ++i) s += loss_value(loss, y[i], z[i]);
    for (int64_t j = 0; j < d; ++j) {
        r += w[j] * w[j];
        a += fabs(w[j]);
    }
    return s / (double)n + 0.5 * lambda * r + lambda1 * a;
}

/* Hinge dual value D(alpha) from alpha and v = X^T (y o alpha). */
double oracle_hinge_dual_objective(int64_t n, int64_t d, const double *alpha, const double *v, double lambda)
{
    double sa = 0.0, vv = 0.0;
    for (int64_t i = 0; i < n; ++i) sa += alpha[i];
    for (int64_t j = 0; j < d; ++j) vv += v[j] * v[j];
    double ln = lambda * (double)n;
    return sa / (double)n - 0.5 * lambda * vv / (ln * ln);
}

/* Logistic dual value D(alpha) from alpha and v = X^T (y o alpha)  (0 ln 0 := 0). */
double oracle_logistic_dual_objective(int64_t n, int64_t d, const double *alpha, const double *v, double lambda)
{
    double ent = 0.0, vv = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double a = alpha[i], b = 1.0 - alpha[i];
        ent += (a > 0.0 ? a * log(a) : 0.0) + (b > 0.0 ? b * log(b) : 0.0);
    }
    for (int64_t j = 0; j < d; ++j) vv += v[j] * v[j];
    double ln = lambda * (double)n;
    return -ent / (double)n - 0.5 * lambda * vv / (ln * ln);
}

/* ------------------------------------------------------------------------------------------- */
/* Duality gap (the paper does not define one; reading taken: the Fenchel-Rockafellar gap of     */
/* eq. (1) with the dual candidate u = grad f(v)).                                               */
/*                                                                                               */
/* Primal form, smooth loss, two ways that must agree:                                            */
/*  (a) "Fenchel" form  G = P(w) - D(u),  D(u) = -f*(u) - sum_j g_j*(-a_j.u)                      */
/*        ridge:    u = (v - y)/n,        f*(u) = u.y + (n/2)||u||^2                              */
/*        logistic: u_i = -y_i p_i/n, p_i = sigmoid(-y_i v_i),                                    */
/*                  f*(u) = (1/n) sum_i [p_i ln p_i + (1-p_i) ln(1-p_i)]     (0 ln 0 := 0)         */
/*        g_j*(t) = t^2/(2 lambda);  with an l1 term  g_j*(t) = max(|t| - lambda1, 0)^2/(2 lambda) */
/*  (b) gradient form   G = ||X^T u + lambda w||^2 / (2 lambda) = ||grad P(w)||^2/(2 lambda).     */
/* ------------------------------------------------------------------------------------------- */
static double xlogx(double p) { return p > 0.0 ? p * log(p) : 0.0; }

/* z_in = X^T u must be supplied (length d), u = grad f(v); computed by the caller with the
 * matvec above so that this function stays a direct transcription of the formulas. */
void oracle_primal_dual_candidate(int loss, int64_t n, const double *v, const float *y, double *u)
{
    for (int64_t i = 0; i < n; ++i) u[i] = loss_d1(loss, y[i], v[i]) / (double)n;
}

double oracle_primal_gap_fenchel(int loss, int64_t n, int64_t d, const double *v, const float *y,
                                 const double *w, const double *u, const double *xtu, double lambda,
                                 double lambda1)
{
    double P = oracle_primal_objective(loss, n, d, v, y, w, lambda, lambda1);
    double fstar = 0.0;
    if (loss == LOSS_RIDGE) {
        for (int64_t i = 0; i < n; ++i) fstar += u[i] * (double)y[i] + 0.5 * (double)n * u[i] * u[i];
    } else {
        for (int64_t i = 0; i < n; ++i) {
            double p = sigmoid(-(double)y[i] * v[i]);
            fstar += xlogx(p) + xlogx(1.0 - p);
        }
        fstar /= (double)n;
    }
    double gstar = 0.0;
    for (int64_t j = 0; j < d; ++j) {
        double t = fabs(xtu[j]) - lambda1;
        if (t > 0.0) gstar += t * t;
    }
    gstar /= 2.0 * lambda;
    double D = -fstar - gstar;
    return P - D;
}

double oracle_primal_gap_gradient(int64_t d, const double *w, const double *xtu, double lambda)
{
    double s = 0.0;
    for (int64_t j = 0; j < d; ++j) {
        double t = xtu[j] + lambda * w[j];
        s += t * t;
    }
    return s / (2.0 * lambda);
}

/* Hinge, dual form: w = v/(lambda n), margins m_i = y_i x_i.w (supplied as xw = X w),
 *   P = (1/n) sum max(0, 1 - m_i) + (lambda/2)||w||^2,  D = (1/n) sum alpha_i - (lambda/2)||w||^2,
 *   G = P - D. */
void oracle_hinge_primal_dual(int64_t n, int64_t d, const double *alpha, const double *v,
                              const double *xw, const float *y, double lambda, double *P, double *D)
{
    double ln = lambda * (double)n, ww = 0.0, hs = 0.0, sa = 0.0;
    for (int64_t j = 0; j < d; ++j) ww += (v[j] / ln) * (v[j] / ln);
    for (int64_t i = 0; i < n; ++i) {
        double m = 1.0 - (double)y[i] * xw[i];
        hs += m > 0 ? m : 0.0;
        sa += alpha[i];
    }
    *P = hs / (double)n + 0.5 * lambda * ww;
    *D = sa / (double)n - 0.5 * lambda * ww;
}

/* Logistic, dual form: w = v/(lambda n), xw = X w supplied;
 *   P = (1/n) sum log(1 + exp(-y_i x_i.w)) + (lambda/2)||w||^2,  D as above,  G = P - D. */
void oracle_logistic_primal_dual(int64_t n, int64_t d, const double *alpha, const double *v,
                                 const double *xw, const float *y, double lambda, double *P, double *D)
{
    double ln = lambda * (double)n, ww = 0.0, ls = 0.0;
    for (int64_t j = 0; j < d; ++j) ww += (v[j] / ln) * (v[j] / ln);
    for (int64_t i = 0; i < n; ++i) ls += log1pexp(-(double)y[i] * xw[i]);
    *P = ls / (double)n + 0.5 * lambda * ww;
    *D = oracle_logistic_dual_objective(n, d, alpha, v, lambda);
}
