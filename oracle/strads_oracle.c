/*
 * CPU oracle for one scheduling round of SAP-scheduled Lasso coordinate descent.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the slow, plain statement of what the
 * round computes, written from the paper (Section 2.1: Algorithm 1, eq. (1),
 * eq. (2), Steps 1-4; Section 4 items 1-2; Theorem 1).  Only the tests, the
 * smoke check and the benchmark's CPU-baseline leg may call it.  It shares no
 * source, header, table or helper with the HIP library.
 *
 * Precision: inputs and state are fp32 arrays; every sum of products is
 * accumulated in fp64 and rounded to fp32 once, when it is stored.  The
 * sampling key is the one place where fp32 arithmetic is *specified* bit by
 * bit (so that index decisions can be compared exactly); see
 * oracle_log2_spec() and oracle_priority_key().
 *
 * Loops are written in the order of the definition; OpenMP is used only
 * across independent outputs (columns, Gram entries, rows).  No blocking, no
 * fusion, no BLAS.
 *
 * Pins (tests/test_oracle_*.py): Philox known-answer vectors from the
 * Random123 publication; log2 against libm in fp64; sampling law against
 * successive-sampling probabilities (chi-square); Gram against an fp64 matmul;
 * greedy filter against brute-force subset enumeration; soft-threshold closed
 * form; orthonormal-design exact solution; KKT at convergence and agreement
 * with an independent library Lasso solver; monotone descent for sequential
 * updates; residual invariant r = y - X beta.  The round with update-aware
 * dependencies (oracle_round_dynamic, tests/test_oracle_dynamic.py): equality
 * with the plain round where the two must coincide (no conflicts; every
 * candidate moves), brute-force enumeration, hand-built three-column designs,
 * and the same fixed point.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* --------------------------------------------------------------------------
 * Counter-based random numbers: Philox-4x32 with 10 rounds
 * (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3",
 * SC'11).  The paper under study only says "draw from p(j)"; the generator is
 * this build's choice and is keyed by (seed, round t, coordinate j) so that a
 * draw does not depend on how the work is split.
 * ------------------------------------------------------------------------ */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;   /* Weyl increments of the key schedule */
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Uniform in (0,1) for (seed, t, j): the top 23 bits m of the first Philox
 * word give u = (2m+1) * 2^-24, every value exactly representable in fp32,
 * never 0 and never 1. */
float oracle_uniform(uint64_t seed, uint64_t t, uint64_t j)
{
    uint32_t ctr[4] = { (uint32_t)j, (uint32_t)(j >> 32), (uint32_t)t, (uint32_t)(t >> 32) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    uint32_t m = out[0] >> 9;
    return (float)(2u * m + 1u) * 0x1.0p-24f;
}

/* --------------------------------------------------------------------------
 * The specified base-2 logarithm for positive normal fp32 x.
 *   x = 2^e * m, m in [1,2); if m > sqrt(2): m /= 2, e += 1
 *   f = m - 1  (exact);  log2(x) ~= e + f * Q(f), Q of degree 8, Horner with
 *   fused multiply-adds in the order written here.
 * Every operation is a correctly rounded IEEE fp32 operation, so any
 * conforming implementation returns the same bits.
 * ------------------------------------------------------------------------ */
static const float L2Q[9] = {
     0x1.715476p+0f, -0x1.715474p-1f,  0x1.ec73dep-2f, -0x1.715994p-2f,  0x1.26d01cp-2f,
    -0x1.e9d1e6p-3f,  0x1.ba8738p-3f, -0x1.a59aeap-3f,  0x1.f841dcp-4f
};

float oracle_log2_spec(float x)
{
    uint32_t bits;
    memcpy(&bits, &x, 4);
    int32_t e = (int32_t)(bits >> 23) - 127;
    uint32_t man = bits & 0x007FFFFFu;
    uint32_t mbits;
    if (man > 0x003504F3u) { mbits = man | 0x3F000000u; e += 1; }   /* m in (sqrt2/2, 1) */
    else                   { mbits = man | 0x3F800000u; }          /* m in [1, sqrt2]   */
    float m;
    memcpy(&m, &mbits, 4);
    float f = m - 1.0f;
    float q = L2Q[8];
    for (int i = 7; i >= 0; --i) q = fmaf(q, f, L2Q[i]);
    return fmaf(f, q, (float)e);
}

/* Step 1 of SAP for Lasso with Theorem 1's weight: p(j) proportional to
 * w_j = (delta beta_j)^2 + eta.  Drawing P' distinct coordinates with
 * probability proportional to w (successive sampling without replacement) is
 * done with the Gumbel-top-k identity: perturb log w_j by independent Gumbel
 * noise -log(-log u_j) and take the P' largest.  Base 2 is used throughout,
 * which scales and shifts every key alike and leaves the order unchanged. */
float oracle_priority_key(float dbeta, float eta, uint64_t seed, uint64_t t, uint64_t j)
{
    float w = fmaf(dbeta, dbeta, eta);
    float u = oracle_uniform(seed, t, j);
    float e = -oracle_log2_spec(u);            /* > 0 : an exponential variate in base-2 units */
    return oracle_log2_spec(w) - oracle_log2_spec(e);
}

/* The weight of coordinate j under the three priorities the paper names:
 *   0  (delta beta_j)^2 + eta    Theorem 1 (the one this build's rounds use by default)
 *   1  |delta beta_j| + eta      Algorithm 1 and Step 1 as printed
 *   2  1                         no priority: the uniform draw of the comparison
 *                                schedulers of Section 5.1 (static correlation, Shotgun) */
float oracle_priority_weight(float dbeta, float eta, int32_t priority)
{
    if (priority == 1) return fabsf(dbeta) + eta;
    if (priority == 2) return 1.0f;
    return fmaf(dbeta, dbeta, eta);
}

float oracle_priority_key_mode(float dbeta, float eta, uint64_t seed, uint64_t t, uint64_t j, int32_t priority)
{
    float w = oracle_priority_weight(dbeta, eta, priority);
    float u = oracle_uniform(seed, t, j);
    float e = -oracle_log2_spec(u);
    return oracle_log2_spec(w) - oracle_log2_spec(e);
}

void oracle_priority_keys_mode(int64_t J, const float *dbeta, float eta, uint64_t seed, uint64_t t,
                               int32_t priority, float *keys)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < J; ++j)
        keys[j] = oracle_priority_key_mode(dbeta[j], eta, seed, t, (uint64_t)j, priority);
}

void oracle_priority_keys(int64_t J, const float *dbeta, float eta, uint64_t seed, uint64_t t, float *keys)
{
    oracle_priority_keys_mode(J, dbeta, eta, seed, t, 0, keys);
}

typedef struct { float key; int32_t j; } keyed_t;

static int keyed_desc(const void *pa, const void *pb)
{
    const keyed_t *a = (const keyed_t *)pa, *b = (const keyed_t *)pb;
    if (a->key > b->key) return -1;
    if (a->key < b->key) return 1;
    return (a->j > b->j) - (a->j < b->j);      /* equal keys: smaller index first */
}

/* The candidate set U: the min(P', J) coordinates with the largest keys, in
 * descending key order (= draw order of successive sampling). */
int32_t oracle_draw(int64_t J, const float *keys, int32_t l_prime, int32_t *cand)
{
    if (J <= 0 || l_prime <= 0) return 0;
    keyed_t *a = (keyed_t *)malloc((size_t)J * sizeof(keyed_t));
    if (!a) return -1;
    for (int64_t j = 0; j < J; ++j) { a[j].key = keys[j]; a[j].j = (int32_t)j; }
    qsort(a, (size_t)J, sizeof(keyed_t), keyed_desc);
    int32_t L = (int64_t)l_prime < J ? l_prime : (int32_t)J;
    for (int32_t i = 0; i < L; ++i) cand[i] = a[i].j;
    free(a);
    return L;
}

/* --------------------------------------------------------------------------
 * Step 2: dependencies d(x_a, x_b) = |x_a^T x_b| among the candidates.
 * X is dense column-major (column j at X + j*N).  G is L x L row-major, full
 * (both triangles and the diagonal), each entry an fp64 sum rounded to fp32.
 * ------------------------------------------------------------------------ */
void oracle_gram_dense(int64_t N, const float *X, const int32_t *cand, int32_t L, float *G)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t a = 0; a < L; ++a) {
        const float *xa = X + (int64_t)cand[a] * N;
        for (int32_t b = a; b < L; ++b) {
            const float *xb = X + (int64_t)cand[b] * N;
            double s = 0.0;
            for (int64_t i = 0; i < N; ++i) s += (double)xa[i] * (double)xb[i];
            G[(int64_t)a * L + b] = (float)s;
            G[(int64_t)b * L + a] = (float)s;
        }
    }
}

/* The same dependencies for chosen rows of G only (row rows[t] against every candidate; out is
 * n_rows x L, row-major), and for chosen pairs (out[t] = x_{cand[pa[t]]}^T x_{cand[pb[t]]}): the same
 * definition, for candidate sets whose whole Gram would take the CPU minutes. */
void oracle_gram_rows_dense(int64_t N, const float *X, const int32_t *cand, int32_t L,
                            const int32_t *rows, int32_t n_rows, float *out)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int32_t t = 0; t < n_rows; ++t) {
        for (int32_t b = 0; b < L; ++b) {
            const float *xa = X + (int64_t)cand[rows[t]] * N;
            const float *xb = X + (int64_t)cand[b] * N;
            double s = 0.0;
            for (int64_t i = 0; i < N; ++i) s += (double)xa[i] * (double)xb[i];
            out[(int64_t)t * L + b] = (float)s;
        }
    }
}

void oracle_gram_pairs_dense(int64_t N, const float *X, const int32_t *cand, const int32_t *pa,
                             const int32_t *pb, int64_t n_pairs, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n_pairs; ++t) {
        const float *xa = X + (int64_t)cand[pa[t]] * N;
        const float *xb = X + (int64_t)cand[pb[t]] * N;
        double s = 0.0;
        for (int64_t i = 0; i < N; ++i) s += (double)xa[i] * (double)xb[i];
        out[t] = (float)s;
    }
}

/* CSC design: column j holds rows row_idx[col_ptr[j] .. col_ptr[j+1]) in
 * increasing order with the matching values. */
void oracle_gram_csc(const float *val, const int32_t *row_idx, const int64_t *col_ptr,
                     const int32_t *cand, int32_t L, float *G)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t a = 0; a < L; ++a) {
        int64_t a0 = col_ptr[cand[a]], a1 = col_ptr[cand[a] + 1];
        for (int32_t b = a; b < L; ++b) {
            int64_t b0 = col_ptr[cand[b]], b1 = col_ptr[cand[b] + 1];
            double s = 0.0;
            int64_t p = a0, q = b0;
            while (p < a1 && q < b1) {
                if (row_idx[p] < row_idx[q]) ++p;
                else if (row_idx[p] > row_idx[q]) ++q;
                else { s += (double)val[p] * (double)val[q]; ++p; ++q; }
            }
            G[(int64_t)a * L + b] = (float)s;
            G[(int64_t)b * L + a] = (float)s;
        }
    }
}

/* The set B_1 of Algorithm 1: walk the candidates in draw order and keep one
 * iff its dependency with every coordinate kept so far is strictly below rho.
 * Stops once p_max are kept (p_max <= 0: no cap).  kept_pos receives positions
 * into the candidate list, in increasing order.  Returns |B_1|. */
int32_t oracle_filter(int32_t L, const float *G, float rho, int32_t p_max, int32_t *kept_pos)
{
    int32_t k = 0;
    for (int32_t a = 0; a < L; ++a) {
        if (p_max > 0 && k >= p_max) break;
        int ok = 1;
        for (int32_t i = 0; i < k && ok; ++i)
            if (!(fabsf(G[(int64_t)a * L + kept_pos[i]]) < rho)) ok = 0;
        if (ok) kept_pos[k++] = a;
    }
    return k;
}

/* --------------------------------------------------------------------------
 * eq. (2): with unit-norm columns and r = y - X beta held at its value from
 * the start of the round,  x_j^T y - sum_{k != j} x_j^T x_k beta_k = x_j^T r + beta_j.
 * ------------------------------------------------------------------------ */
void oracle_dots_dense(int64_t N, const float *X, const int32_t *cols, int32_t k, const float *r, double *z)
{
#pragma omp parallel for schedule(static)
    for (int32_t c = 0; c < k; ++c) {
        const float *x = X + (int64_t)cols[c] * N;
        double s = 0.0;
        for (int64_t i = 0; i < N; ++i) s += (double)x[i] * (double)r[i];
        z[c] = s;
    }
}

void oracle_dots_csc(const float *val, const int32_t *row_idx, const int64_t *col_ptr,
                     const int32_t *cols, int32_t k, const float *r, double *z)
{
#pragma omp parallel for schedule(static)
    for (int32_t c = 0; c < k; ++c) {
        double s = 0.0;
        for (int64_t p = col_ptr[cols[c]]; p < col_ptr[cols[c] + 1]; ++p)
            s += (double)val[p] * (double)r[row_idx[p]];
        z[c] = s;
    }
}

/* Soft-thresholding operator S(a, lambda) = sign(a) * max(|a| - lambda, 0). */
double oracle_soft_threshold(double a, double lambda)
{
    double m = fabs(a) - lambda;
    if (!(m > 0.0)) return 0.0;
    return a < 0.0 ? -m : m;
}

/* Apply eq. (2) to every kept coordinate (all from the same stale r), record
 * the change (Step 4: delta beta_j feeds the next draw).  inv_kappa = 1 is eq. (2) as printed
 * (squared loss, unit-norm columns); for the logistic loss see oracle_logistic_weights. */
void oracle_update(int32_t k, const int32_t *cols, const double *z, float lambda, double inv_kappa,
                   float *beta, float *dbeta, double *delta)
{
    for (int32_t c = 0; c < k; ++c) {
        int32_t j = cols[c];
        double old = (double)beta[j];
        float nb = (float)oracle_soft_threshold(z[c] * inv_kappa + old, (double)lambda * inv_kappa);
        double d = (double)nb - old;
        delta[c] = d;
        dbeta[j] = (float)fabs(d);
        beta[j] = nb;
    }
}

/* r <- r - sum_{j in B} x_j * delta_j  */
void oracle_residual_dense(int64_t N, const float *X, const int32_t *cols, int32_t k,
                           const double *delta, float *r)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        double s = 0.0;
        for (int32_t c = 0; c < k; ++c) s += (double)X[(int64_t)cols[c] * N + i] * delta[c];
        r[i] = (float)((double)r[i] - s);
    }
}

void oracle_residual_csc(int64_t N, const float *val, const int32_t *row_idx, const int64_t *col_ptr,
                         const int32_t *cols, int32_t k, const double *delta, float *r)
{
    double *acc = (double *)calloc((size_t)N, sizeof(double));
    if (!acc) return;
    for (int32_t c = 0; c < k; ++c)
        for (int64_t p = col_ptr[cols[c]]; p < col_ptr[cols[c] + 1]; ++p)
            acc[row_idx[p]] += (double)val[p] * delta[c];
    for (int64_t i = 0; i < N; ++i) r[i] = (float)((double)r[i] - acc[i]);
    free(acc);
}

/* eq. (1) with squared loss: F = 1/2 ||r||^2 + lambda * sum |beta_j|. */
double oracle_objective(int64_t N, const float *r, int64_t J, const float *beta, float lambda)
{
    double s = 0.0, l1 = 0.0;
    for (int64_t i = 0; i < N; ++i) s += (double)r[i] * (double)r[i];
    for (int64_t j = 0; j < J; ++j) l1 += fabs((double)beta[j]);
    return 0.5 * s + (double)lambda * l1;
}

/* --------------------------------------------------------------------------
 * Logistic loss.  Section 2.1 lets L in eq. (1) be the squared or the logistic loss and says the
 * latter is handled in the same way as in the parallel coordinate descent work it cites;
 * no formula is given.  Taken here: labels y_i in {-1, +1},
 *      L(beta) = sum_i log(1 + exp(-y_i m_i)),   m = X beta,
 * whose derivative along coordinate j is -x_j^T w with w_i = y_i / (1 + exp(y_i m_i)), and whose
 * second derivative along a unit-norm column is at most 1/4.  A coordinate update minimises the
 * quadratic upper bound with that curvature, kappa = 1/4:
 *      beta_j <- S(beta_j + (x_j^T w) / kappa, lambda / kappa),
 * which never increases the objective when applied one coordinate at a time.  Everything else of
 * Algorithm 1 is unchanged; w takes the place of the residual in eq. (2) and in the optimality test,
 * and the state vector kept between rounds is v = -X beta (so that the same residual update
 * v <- v - sum x_j delta_j maintains it): w_i = y_i / (1 + exp(-y_i v_i)).
 * ------------------------------------------------------------------------ */
void oracle_logistic_weights(int64_t N, const float *y, const float *v, float *w)
{
    for (int64_t i = 0; i < N; ++i)
        w[i] = (float)((double)y[i] / (1.0 + exp(-(double)y[i] * (double)v[i])));
}

/* eq. (1) with the logistic loss: sum_i log(1 + exp(y_i v_i)) + lambda sum |beta_j|, v = -X beta. */
double oracle_objective_logistic(int64_t N, const float *y, const float *v, int64_t J, const float *beta,
                                 float lambda)
{
    double s = 0.0, l1 = 0.0;
    for (int64_t i = 0; i < N; ++i) {
        const double t = (double)y[i] * (double)v[i];
        s += t > 0.0 ? t + log1p(exp(-t)) : log1p(exp(t));
    }
    for (int64_t j = 0; j < J; ++j) l1 += fabs((double)beta[j]);
    return s + (double)lambda * l1;
}

/* Optimality (KKT) violation of eq. (1) at beta, g = X^T r:
 *   beta_j == 0 : max(|g_j| - lambda, 0);   beta_j != 0 : |g_j - lambda*sign(beta_j)|.
 * Returns the maximum over j; g_out (may be NULL) receives g. */
static double kkt_violation(double g, float beta, float lambda)
{
    if (beta == 0.0f) { double v = fabs(g) - (double)lambda; return v > 0.0 ? v : 0.0; }
    return fabs(g - (beta > 0.0f ? (double)lambda : -(double)lambda));
}

double oracle_kkt_dense(int64_t N, int64_t J, const float *X, const float *r, const float *beta,
                        float lambda, double *g_out)
{
    double worst = 0.0;
#pragma omp parallel for schedule(static) reduction(max : worst)
    for (int64_t j = 0; j < J; ++j) {
        const float *x = X + j * N;
        double s = 0.0;
        for (int64_t i = 0; i < N; ++i) s += (double)x[i] * (double)r[i];
        if (g_out) g_out[j] = s;
        double v = kkt_violation(s, beta[j], lambda);
        if (v > worst) worst = v;
    }
    return worst;
}

double oracle_kkt_csc(int64_t J, const float *val, const int32_t *row_idx, const int64_t *col_ptr,
                      const float *r, const float *beta, float lambda, double *g_out)
{
    double worst = 0.0;
#pragma omp parallel for schedule(static) reduction(max : worst)
    for (int64_t j = 0; j < J; ++j) {
        double s = 0.0;
        for (int64_t p = col_ptr[j]; p < col_ptr[j + 1]; ++p) s += (double)val[p] * (double)r[row_idx[p]];
        if (g_out) g_out[j] = s;
        double v = kkt_violation(s, beta[j], lambda);
        if (v > worst) worst = v;
    }
    return worst;
}

/* --------------------------------------------------------------------------
 * One whole round of Algorithm 1 (dense or CSC), in the paper's order:
 * draw U -> dependencies -> choose B_1 -> update in parallel -> bookkeeping.
 * State (beta, dbeta, r) is updated in place.  The per-stage results are
 * returned through the out pointers (any of G, z, delta may be NULL).
 * forced_cand / forced_kept_pos (may be NULL) replace the oracle's own index
 * decisions; the parity harness uses them to keep comparing floating-point
 * work after an admissible near-tie sent the two sides different ways.
 * Returns |B_1|, or a negative number on allocation failure.
 * ------------------------------------------------------------------------ */
typedef struct {
    int64_t N, J;
    const float *X;            /* dense: J columns of N ; CSC: values */
    const int32_t *row_idx;    /* CSC only (NULL selects dense) */
    const int64_t *col_ptr;    /* CSC only */
    float lambda, rho, eta;
    int32_t l_prime, p_max;
    uint64_t seed;
    int32_t priority;          /* see oracle_priority_weight */
    int32_t deps;              /* 0: Algorithm 1's dependency check; 2: none (every candidate is
                                  dispatched, up to p_max: the Shotgun scheduler of Section 5.1).
                                  1 is oracle_round_dynamic's rule and is not read here. */
    int32_t n_shards;          /* S scheduler shards taking turns (Section 3); <= 1: one scheduler */
    int32_t loss;              /* 0: squared loss (the state vector is r = y - X beta);
                                  1: logistic loss (state vector v = -X beta, see oracle_logistic_weights) */
    const float *y;            /* logistic loss only: the N labels */
} oracle_problem_t;

/* The vector that eq. (2)'s dot products are taken with: the residual itself, or the logistic
 * weights computed from the state vector (the caller frees *owned if it is not NULL). */
static const float *dots_vector(const oracle_problem_t *p, const float *r, float **owned)
{
    *owned = NULL;
    if (p->loss != 1) return r;
    *owned = (float *)malloc((size_t)(p->N > 0 ? p->N : 1) * sizeof(float));
    if (!*owned) return NULL;
    oracle_logistic_weights(p->N, p->y, r, *owned);
    return *owned;
}

/* Step 1 for round t.  With S > 1 scheduler shards (Section 3, "Implementation Overview"): every
 * coordinate belongs to exactly one shard for good, shard s = t mod S has the turn in round t, and it
 * draws its P' candidates from its own coordinates only, with p_s(j) the same priority restricted
 * to them.  The paper assigns coordinates to shards at random; here coordinate j belongs to shard
 * j mod S.  The random number of coordinate j is keyed by j itself, whatever the sharding.
 * Returns the number of candidates (min(P', size of the shard)) or -1. */
static int32_t draw_for_round(const oracle_problem_t *p, uint64_t t, const float *dbeta, int32_t *cand)
{
    const int64_t S = p->n_shards > 1 ? p->n_shards : 1;
    const int64_t s = (int64_t)(t % (uint64_t)S);
    const int64_t Js = p->J > s ? (p->J - s + S - 1) / S : 0;
    float *keys = (float *)malloc((size_t)(Js > 0 ? Js : 1) * sizeof(float));
    if (!keys) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < Js; ++i) {
        const int64_t j = i * S + s;
        keys[i] = oracle_priority_key_mode(dbeta[j], p->eta, p->seed, t, (uint64_t)j, p->priority);
    }
    int32_t L = oracle_draw(Js, keys, p->l_prime, cand);     /* positions within the shard */
    free(keys);
    for (int32_t a = 0; a < L; ++a) cand[a] = (int32_t)((int64_t)cand[a] * S + s);
    return L;
}

int32_t oracle_round(const oracle_problem_t *p, uint64_t t, float *beta, float *dbeta, float *r,
                     const int32_t *forced_cand, int32_t forced_n_cand,
                     const int32_t *forced_kept_pos, int32_t forced_n_kept,
                     int32_t *cand, int32_t *n_cand_out, int32_t *kept_pos, int32_t *kept_cols,
                     float *G_out, double *z_out, double *delta_out)
{
    int32_t L;
    if (forced_cand) {
        L = forced_n_cand;
        memcpy(cand, forced_cand, (size_t)L * sizeof(int32_t));
    } else {
        L = draw_for_round(p, t, dbeta, cand);
        if (L < 0) return -1;
    }
    *n_cand_out = L;

    int32_t k;
    if (p->deps == 2 && !forced_kept_pos) {
        /* no dependency check: the first p_max candidates (all of them without a cap) */
        k = (p->p_max > 0 && p->p_max < L) ? p->p_max : L;
        for (int32_t a = 0; a < k; ++a) kept_pos[a] = a;
        if (G_out) memset(G_out, 0, (size_t)L * (size_t)L * sizeof(float));
    } else if (forced_kept_pos && !G_out) {
        k = forced_n_kept;
        memcpy(kept_pos, forced_kept_pos, (size_t)k * sizeof(int32_t));
    } else {
        float *G = G_out ? G_out : (float *)malloc((size_t)(L > 0 ? L : 1) * (size_t)(L > 0 ? L : 1) * sizeof(float));
        if (!G) return -1;
        if (p->row_idx) oracle_gram_csc(p->X, p->row_idx, p->col_ptr, cand, L, G);
        else            oracle_gram_dense(p->N, p->X, cand, L, G);
        if (forced_kept_pos) {
            k = forced_n_kept;
            memcpy(kept_pos, forced_kept_pos, (size_t)k * sizeof(int32_t));
        } else {
            k = oracle_filter(L, G, p->rho, p->p_max, kept_pos);
        }
        if (!G_out) free(G);
    }
    for (int32_t c = 0; c < k; ++c) kept_cols[c] = cand[kept_pos[c]];

    double *z = z_out ? z_out : (double *)malloc((size_t)(k > 0 ? k : 1) * sizeof(double));
    double *d = delta_out ? delta_out : (double *)malloc((size_t)(k > 0 ? k : 1) * sizeof(double));
    if (!z || !d) return -1;
    float *w_owned;
    const float *dv = dots_vector(p, r, &w_owned);
    if (!dv) return -1;
    if (p->row_idx) oracle_dots_csc(p->X, p->row_idx, p->col_ptr, kept_cols, k, dv, z);
    else            oracle_dots_dense(p->N, p->X, kept_cols, k, dv, z);
    free(w_owned);
    oracle_update(k, kept_cols, z, p->lambda, p->loss == 1 ? 4.0 : 1.0, beta, dbeta, d);
    if (p->row_idx) oracle_residual_csc(p->N, p->X, p->row_idx, p->col_ptr, kept_cols, k, d, r);
    else            oracle_residual_dense(p->N, p->X, kept_cols, k, d, r);
    if (!z_out) free(z);
    if (!delta_out) free(d);
    return k;
}

/* --------------------------------------------------------------------------
 * Round with update-aware ("dynamic") dependencies.
 *
 * Section 1 ("Dynamic Block Structures") observes that a coefficient which
 * stays where it is during a round neither disturbs nor is disturbed by the
 * parallel update of a correlated one, however large the correlation; Step 4
 * of Section 2 has the scheduler remove such dependencies.  In eq. (2) the
 * interference of k with j's update is x_j^T x_k * (change of beta_k), which
 * vanishes exactly when beta_k does not change.  So the dependency used by
 * Step 2 becomes
 *      d_t(a, b) = |x_a^T x_b|   if both a and b would move this round,
 *                = 0             otherwise,
 * where "a would move" means its update from the residual of the start of the
 * round, S(x_a^T r + beta_a, lambda) - beta_a, is not zero.  Everything else
 * is Algorithm 1 unchanged: draw U, choose B_1 greedily in draw order under
 * d_t < rho (and the cap p_max), update B_1 from the same r, bookkeeping.  A
 * kept coordinate that does not move gets delta beta = 0, as in Algorithm 1.
 *
 * Outputs per candidate (L entries each; any may be NULL): z_cand = x^T r,
 * delta_cand = tentative change, mover = 1/0.  G_out (L x L, may be NULL)
 * receives d_t's signed values (x_a^T x_b for mover pairs, 0 elsewhere).
 * forced_cand / forced_mover / forced_kept_pos replace the oracle's own index
 * decisions (see oracle_round); a candidate forced to "does not move" is
 * committed with change 0.
 * Returns |B_1| or a negative number on allocation failure.
 * ------------------------------------------------------------------------ */
int32_t oracle_round_dynamic(const oracle_problem_t *p, uint64_t t, float *beta, float *dbeta, float *r,
                             const int32_t *forced_cand, int32_t forced_n_cand,
                             const uint8_t *forced_mover,
                             const int32_t *forced_kept_pos, int32_t forced_n_kept,
                             int32_t *cand, int32_t *n_cand_out, uint8_t *mover_out,
                             double *z_cand_out, double *delta_cand_out,
                             int32_t *kept_pos, int32_t *kept_cols, float *G_out,
                             double *z_out, double *delta_out)
{
    int32_t L;
    if (forced_cand) {
        L = forced_n_cand;
        memcpy(cand, forced_cand, (size_t)L * sizeof(int32_t));
    } else {
        L = draw_for_round(p, t, dbeta, cand);
        if (L < 0) return -1;
    }
    *n_cand_out = L;
    const size_t Ls = (size_t)(L > 0 ? L : 1);

    /* every candidate's update from the residual as it stands */
    double *zc = (double *)malloc(Ls * sizeof(double));
    double *dc = (double *)malloc(Ls * sizeof(double));
    float *nb = (float *)malloc(Ls * sizeof(float));
    uint8_t *mv = (uint8_t *)malloc(Ls);
    float *G = G_out ? G_out : (float *)malloc(Ls * Ls * sizeof(float));
    if (!zc || !dc || !nb || !mv || !G) return -1;
    float *w_owned;
    const float *dv = dots_vector(p, r, &w_owned);
    if (!dv) return -1;
    if (p->row_idx) oracle_dots_csc(p->X, p->row_idx, p->col_ptr, cand, L, dv, zc);
    else            oracle_dots_dense(p->N, p->X, cand, L, dv, zc);
    free(w_owned);
    const double ik = p->loss == 1 ? 4.0 : 1.0;
    for (int32_t a = 0; a < L; ++a) {
        const double old = (double)beta[cand[a]];
        nb[a] = (float)oracle_soft_threshold(zc[a] * ik + old, (double)p->lambda * ik);
        dc[a] = (double)nb[a] - old;
        mv[a] = forced_mover ? (uint8_t)(forced_mover[a] != 0) : (uint8_t)(dc[a] != 0.0);
        if (!mv[a]) { dc[a] = 0.0; nb[a] = beta[cand[a]]; }
    }

    /* dependencies among the candidates, kept only between two movers */
    if (p->row_idx) oracle_gram_csc(p->X, p->row_idx, p->col_ptr, cand, L, G);
    else            oracle_gram_dense(p->N, p->X, cand, L, G);
    for (int32_t a = 0; a < L; ++a)
        for (int32_t b = 0; b < L; ++b)
            if (!(mv[a] && mv[b])) G[(int64_t)a * L + b] = 0.0f;

    int32_t k;
    if (forced_kept_pos) {
        k = forced_n_kept;
        memcpy(kept_pos, forced_kept_pos, (size_t)k * sizeof(int32_t));
    } else {
        k = oracle_filter(L, G, p->rho, p->p_max, kept_pos);
    }

    /* commit B_1 (all from the same r), then the residual */
    double *dk = delta_out ? delta_out : (double *)malloc((size_t)(k > 0 ? k : 1) * sizeof(double));
    if (!dk) return -1;
    for (int32_t c = 0; c < k; ++c) {
        const int32_t a = kept_pos[c], j = cand[a];
        kept_cols[c] = j;
        if (z_out) z_out[c] = zc[a];
        dk[c] = dc[a];
        dbeta[j] = (float)fabs(dc[a]);
        beta[j] = nb[a];
    }
    if (p->row_idx) oracle_residual_csc(p->N, p->X, p->row_idx, p->col_ptr, kept_cols, k, dk, r);
    else            oracle_residual_dense(p->N, p->X, kept_cols, k, dk, r);

    if (mover_out) memcpy(mover_out, mv, (size_t)L);
    if (z_cand_out) memcpy(z_cand_out, zc, (size_t)L * sizeof(double));
    if (delta_cand_out) memcpy(delta_cand_out, dc, (size_t)L * sizeof(double));
    if (!delta_out) free(dk);
    if (!G_out) free(G);
    free(zc); free(dc); free(nb); free(mv);
    return k;
}
