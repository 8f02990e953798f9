/*
 * CPU oracle for the decentralized momentum updates -- TEST INFRASTRUCTURE.
 *
 * Plain, slow, fp64 loops that evaluate the paper's definitions one statement
 * at a time.  Nothing here is shared with the GPU library: no header, no
 * helper, no table.  Only tests, the smoke check and the benchmark's
 * "cpu_baseline" leg may call it; the product path never does.
 *
 * Build with -ffp-contract=off so that every line below is evaluated as
 * written (one rounding per operation, no fused multiply-add).
 *
 * Conventions: stacked arrays are row-major n x d (row i = node i, notation
 * of the appendix "Preliminary"); a weight matrix W is a neighbour list in
 * CSR form (row i lists the j with w_ij > 0, self included -- Sec.
 * "Decentralized Momentum SGD", eq. (2) and the definition of N_i);
 * a time-varying W is `period` such lists, iteration k using phase k mod period.
 *
 * Pins (tests marked "not gpu"): library momentum SGD for W = I, the DSGD
 * compact form for beta = 0, the momentum-free second-order recursions of the
 * appendix "Reformulation of DmSGD and DecentLaM", the alternative forms of
 * the corrected gradient, node-average and zero-sum invariants, exact rational
 * brute force on tiny cases, the fixed-point equations of the appendix
 * "Limiting Bias of Decentralized Algorithms", automatic differentiation and
 * finite differences for the least-squares gradient, hand-written neighbour
 * tables for the topologies.  The two sibling methods AWC-DmSGD and DA-DmSGD
 * are this file's reading of one-sentence descriptions ("parity weakly
 * pinned"): their pins (W = I, beta = 0, node average, dense-matrix brute force,
 * directly solved fixed points) fix the arithmetic of the reading, not the
 * reading itself.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_RING = 0, ORACLE_EXP_STATIC = 1, ORACLE_EXP_ONEPEER = 2, ORACLE_EXP_SYM = 3,
       ORACLE_MESH = 4, ORACLE_BIPARTITE_MATCH = 5 };

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of hop exponents of the exponential graphs: hops 2^0 .. 2^floor(log2(n-1))
 * (appendix "Network topologies", exponential-graph item). */
static int hop_count(int n)
{
    int tau = 0;
    while (n > 1 && (1 << tau) <= n - 1) tau++;
    return tau; /* 0 when n == 1 */
}

/* Append j to row (kept in first-occurrence order, no duplicates). */
static int push_unique(int32_t* row, int len, int32_t j)
{
    for (int t = 0; t < len; ++t)
        if (row[t] == j) return len;
    row[len] = j;
    return len + 1;
}

static int wrap(int j, int n) { return ((j % n) + n) % n; }

/* splitmix64, the published 64-bit mixing generator; drives the random matching. */
static uint64_t splitmix64(uint64_t* state)
{
    uint64_t z = (*state += 0x9E3779B97F4A7C15ULL);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* Partner of every node in the bipartite random match of phase p ("all nodes are evenly divided
 * into two groups randomly per iteration; communication only within each pair"; same seed on all
 * nodes).  Recipe (an interface both sides must share, like a file format): Fisher-Yates shuffle
 * of 0..n-1 from the top with index splitmix64() % (t+1), generator seeded with
 * seed ^ (0xD1B54A32D192ED03 * (p+1)); shuffled position q pairs with position q + n/2; an odd
 * node out stays alone (partner = itself). */
static void match_partners(int n, uint64_t seed, int p, int32_t* partner)
{
    int32_t* perm = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
    for (int i = 0; i < n; ++i) perm[i] = i;
    uint64_t state = seed ^ (0xD1B54A32D192ED03ULL * ((uint64_t)p + 1));
    for (int t = n - 1; t > 0; --t) {
        int q = (int)(splitmix64(&state) % (uint64_t)(t + 1));
        int32_t tmp = perm[t]; perm[t] = perm[q]; perm[q] = tmp;
    }
    for (int i = 0; i < n; ++i) partner[i] = i;
    for (int q = 0; q < n / 2; ++q) {
        partner[perm[q]] = perm[q + n / 2];
        partner[perm[q + n / 2]] = perm[q];
    }
    free(perm);
}

/* Neighbour set of node i in phase p, self first.
 *   ring:                 i, i-1, i+1 (mod n)                          -- "Ring" item
 *   static exponential:   i, i+2^0, i+2^1, ... (mod n)                 -- exponential-graph item, directed reading
 *   one-peer exponential: i, i+2^p (mod n)                             -- one neighbour per iteration (Introduction)
 *   symmetric exponential: i, i+2^0, i-2^0, i+2^1, i-2^1, ... (mod n)  -- "Symmetric Exponential Graph" item
 *   mesh:                 R x C grid (R the largest divisor of n with R*R <= n, node i at row i/C,
 *                         column i%C), neighbours up, down, left, right, no wrap-around -- "Mesh" item;
 *                         the paper's drawing of it is lost, this is the reading taken
 *   bipartite match:      i and its partner of this phase                -- "Bipartite Random Match" item
 * Reading: node i *receives from* the listed nodes. */
static int neighbours(int kind, int n, int p, int i, const int32_t* partner, int32_t* row)
{
    int len = 0;
    len = push_unique(row, len, i);
    if (kind == ORACLE_RING) {
        len = push_unique(row, len, wrap(i - 1, n));
        len = push_unique(row, len, wrap(i + 1, n));
    } else if (kind == ORACLE_EXP_STATIC) {
        int tau = hop_count(n);
        for (int t = 0; t < tau; ++t) len = push_unique(row, len, wrap(i + (1 << t), n));
    } else if (kind == ORACLE_EXP_ONEPEER) {
        if (n > 1) len = push_unique(row, len, wrap(i + (1 << p), n));
    } else if (kind == ORACLE_EXP_SYM) {
        int tau = hop_count(n);
        for (int t = 0; t < tau; ++t) {
            len = push_unique(row, len, wrap(i + (1 << t), n));
            len = push_unique(row, len, wrap(i - (1 << t), n));
        }
    } else if (kind == ORACLE_MESH) {
        int R = 1;
        for (int r = 1; r * r <= n; ++r)
            if (n % r == 0) R = r;
        int C = n / R, a = i / C, b = i % C;
        if (a > 0) len = push_unique(row, len, i - C);
        if (a + 1 < R) len = push_unique(row, len, i + C);
        if (b > 0) len = push_unique(row, len, i - 1);
        if (b + 1 < C) len = push_unique(row, len, i + 1);
    } else if (kind == ORACLE_BIPARTITE_MATCH) {
        len = push_unique(row, len, partner[i]);
    }
    return len;
}

/* Sizes first (row_ptr == NULL), then fill.  row_ptr holds period*(n+1) absolute offsets into
 * col_idx / w (phase-major).
 * Weights: Metropolis-Hastings rule (the paper cites it for all its topologies without printing
 * it; reading taken: w_ij = 1/(1 + max(deg_i, deg_j)) for j != i, w_ii = 1 - sum_j w_ij, deg =
 * neighbours other than the node itself).  Where every neighbour of i has i's degree the rule
 * gives 1/|N_i| for all entries and is evaluated as (float)1/(float)|N_i|.  The two directed
 * exponential graphs are not undirected graphs, so the rule does not apply; they carry the
 * uniform 1/|N_i|. */
int oracle_topology(int kind, int n, uint64_t seed, int phases, int32_t* period_out, int64_t* nnz_out,
                    int32_t* row_ptr, int32_t* col_idx, float* w)
{
    if (n < 1 || kind < 0 || kind > 5) return -1;
    int period = 1;
    if (kind == ORACLE_EXP_ONEPEER && n > 1) period = hop_count(n);
    if (kind == ORACLE_BIPARTITE_MATCH) {
        if (phases < 1) return -1;
        period = phases;
    }
    int undirected = (kind != ORACLE_EXP_STATIC && kind != ORACLE_EXP_ONEPEER);
    int32_t* tmp = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n + 2));
    int32_t* other = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n + 2));
    int32_t* partner = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
    int32_t* deg = (int32_t*)malloc(sizeof(int32_t) * (size_t)n);
    if (!tmp || !other || !partner || !deg) { free(tmp); free(other); free(partner); free(deg); return -2; }
    int64_t nnz = 0;
    for (int p = 0; p < period; ++p) {
        if (kind == ORACLE_BIPARTITE_MATCH) match_partners(n, seed, p, partner);
        for (int i = 0; i < n; ++i) deg[i] = neighbours(kind, n, p, i, partner, tmp) - 1;
        for (int i = 0; i < n; ++i) {
            int len = neighbours(kind, n, p, i, partner, tmp);
            if (row_ptr) {
                row_ptr[p * (n + 1) + i] = (int32_t)nnz;
                int same_degree = 1;
                for (int t = 1; t < len; ++t) same_degree = same_degree && (deg[tmp[t]] == deg[i]);
                double rest = 0.0;
                for (int t = 0; t < len; ++t) {
                    col_idx[nnz + t] = tmp[t];
                    if (!undirected || same_degree) {
                        w[nnz + t] = 1.0f / (float)len;
                    } else if (t > 0) {
                        int big = deg[i] > deg[tmp[t]] ? deg[i] : deg[tmp[t]];
                        w[nnz + t] = 1.0f / (float)(1 + big);
                        rest = rest + (double)w[nnz + t];
                    }
                }
                if (undirected && !same_degree) w[nnz] = (float)(1.0 - rest);
            }
            nnz += len;
        }
        if (row_ptr) row_ptr[p * (n + 1) + n] = (int32_t)nnz;
    }
    free(tmp); free(other); free(partner); free(deg);
    *period_out = period;
    *nnz_out = nnz;
    return 0;
}

/* Partial averaging, eq. (3): out_i = sum_{j in N_i} w_ij in_j, terms added in
 * list order.  `in` and `out` must not overlap. */
static void partial_average(int n, int64_t d, const int32_t* row_ptr, const int32_t* col_idx,
                            const float* w, const double* in, double* out)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < n; ++i) {
        for (int64_t c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int32_t e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
                double wij = (double)w[e];
                acc = acc + wij * in[(int64_t)col_idx[e] * d + c];
            }
            out[(int64_t)i * d + c] = acc;
        }
    }
}

/* DSGD, eqs. (4)-(5): x^{k+1/2} = x - gamma g ; x^{k+1} = W x^{k+1/2}. */
int oracle_dsgd_step(int n, int64_t d, int period, const int32_t* row_ptr, const int32_t* col_idx,
                     const float* w, double gamma, int64_t k,
                     const double* x, const double* g, double* x_out)
{
    const int32_t* rp = row_ptr + (k % period) * (n + 1);
    double* half = (double*)malloc(sizeof(double) * (size_t)n * (size_t)(d > 0 ? d : 1));
    if (!half) return -2;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < n; ++i)
        for (int64_t c = 0; c < d; ++c) {
            int64_t q = (int64_t)i * d + c;
            half[q] = x[q] - gamma * g[q];
        }
    partial_average(n, d, rp, col_idx, w, half, x_out);
    free(half);
    return 0;
}

/* DmSGD, Algorithm 1:
 *   m^{k+1} = beta m^k + g^k            (momentum update)
 *   x^{k+1/2} = x^k - gamma m^{k+1}     (local model update)
 *   x^{k+1} = sum_j w_ij x_j^{k+1/2}    (partial average)          */
int oracle_dmsgd_step(int n, int64_t d, int period, const int32_t* row_ptr, const int32_t* col_idx,
                      const float* w, double gamma, double beta, int64_t k,
                      const double* x, const double* m, const double* g,
                      double* x_out, double* m_out)
{
    const int32_t* rp = row_ptr + (k % period) * (n + 1);
    double* half = (double*)malloc(sizeof(double) * (size_t)n * (size_t)(d > 0 ? d : 1));
    if (!half) return -2;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < n; ++i)
        for (int64_t c = 0; c < d; ++c) {
            int64_t q = (int64_t)i * d + c;
            double m_new = beta * m[q] + g[q];
            m_out[q] = m_new;
            half[q] = x[q] - gamma * m_new;
        }
    partial_average(n, d, rp, col_idx, w, half, x_out);
    free(half);
    return 0;
}

/* AWC-DmSGD (Sec. "Experiments", list of compared algorithms: the
 * adaptation-with-combination form of DSGD, whose recursion x <- W x - gamma grad
 * is printed in the discussion that follows the DSGD-as-SGD proposition,
 * accelerated with momentum).  PARITY WEAKLY PINNED: the paper prints no recursion
 * for the momentum version; reading taken: the gradient in that recursion is
 * replaced by the momentum buffer of Algorithm 1,
 *   m^{k+1} = beta m^k + g^k
 *   x^{k+1} = sum_j w_ij x_j^k - gamma m_i^{k+1}                           */
int oracle_awc_dmsgd_step(int n, int64_t d, int period, const int32_t* row_ptr, const int32_t* col_idx,
                          const float* w, double gamma, double beta, int64_t k,
                          const double* x, const double* m, const double* g,
                          double* x_out, double* m_out)
{
    const int32_t* rp = row_ptr + (k % period) * (n + 1);
    partial_average(n, d, rp, col_idx, w, x, x_out);
#pragma omp parallel for schedule(static)
    for (int i = 0; i < n; ++i)
        for (int64_t c = 0; c < d; ++c) {
            int64_t q = (int64_t)i * d + c;
            double m_new = beta * m[q] + g[q];
            m_out[q] = m_new;
            x_out[q] = x_out[q] - gamma * m_new;
        }
    return 0;
}

/* DA-DmSGD (Sec. "Related work" and "Experiments": DmSGD with an additional
 * partial averaging over the momentum, two partial averages per iteration).
 * PARITY WEAKLY PINNED: no recursion is printed; reading taken: Algorithm 1
 * with its momentum buffer averaged as well,
 *   mh_i    = beta m_i^k + g_i^k
 *   x^{k+1} = sum_j w_ij (x_j^k - gamma mh_j)
 *   m^{k+1} = sum_j w_ij mh_j                                              */
int oracle_da_dmsgd_step(int n, int64_t d, int period, const int32_t* row_ptr, const int32_t* col_idx,
                         const float* w, double gamma, double beta, int64_t k,
                         const double* x, const double* m, const double* g,
                         double* x_out, double* m_out)
{
    const int32_t* rp = row_ptr + (k % period) * (n + 1);
    size_t cnt = (size_t)n * (size_t)(d > 0 ? d : 1);
    double* mh = (double*)malloc(sizeof(double) * cnt);
    double* half = (double*)malloc(sizeof(double) * cnt);
    if (!mh || !half) { free(mh); free(half); return -2; }
#pragma omp parallel for schedule(static)
    for (int i = 0; i < n; ++i)
        for (int64_t c = 0; c < d; ++c) {
            int64_t q = (int64_t)i * d + c;
            mh[q] = beta * m[q] + g[q];
            half[q] = x[q] - gamma * mh[q];
        }
    partial_average(n, d, rp, col_idx, w, half, x_out);
    partial_average(n, d, rp, col_idx, w, mh, m_out);
    free(mh);
    free(half);
    return 0;
}

/* DecentLaM, Algorithm 2 with the corrected gradient of the equation that
 * follows the "Efficient implementation" paragraph:
 *   gt_i  = (1/gamma) x_i - (1/gamma) sum_j w_ij (x_j - gamma g_j)
 *   m^{k+1} = beta m^k + gt            (momentum update)
 *   x^{k+1} = x^k - gamma m^{k+1}      (local model update)
 * Reading: the two 1/gamma terms are evaluated as one division of the
 * difference, (x_i - z_i) / gamma. */
int oracle_decentlam_step(int n, int64_t d, int period, const int32_t* row_ptr,
                          const int32_t* col_idx, const float* w, double gamma, double beta,
                          int64_t k, const double* x, const double* m, const double* g,
                          double* x_out, double* m_out)
{
    const int32_t* rp = row_ptr + (k % period) * (n + 1);
    size_t cnt = (size_t)n * (size_t)(d > 0 ? d : 1);
    double* local = (double*)malloc(sizeof(double) * cnt);
    double* z = (double*)malloc(sizeof(double) * cnt);
    if (!local || !z) { free(local); free(z); return -2; }
#pragma omp parallel for schedule(static)
    for (int i = 0; i < n; ++i)
        for (int64_t c = 0; c < d; ++c) {
            int64_t q = (int64_t)i * d + c;
            local[q] = x[q] - gamma * g[q];
        }
    partial_average(n, d, rp, col_idx, w, local, z);
#pragma omp parallel for schedule(static)
    for (int i = 0; i < n; ++i)
        for (int64_t c = 0; c < d; ++c) {
            int64_t q = (int64_t)i * d + c;
            double gt = (x[q] - z[q]) / gamma;
            double m_new = beta * m[q] + gt;
            m_out[q] = m_new;
            x_out[q] = x[q] - gamma * m_new;
        }
    free(local);
    free(z);
    return 0;
}

/* DecentLaM without the momentum array, appendix "Reformulation of DecentLaM":
 *   x^{k+1} = W (x^k - gamma g^k) + beta (x^k - x^{k-1})
 * Reading for a learning rate that changes between iterations (the appendix derives the constant
 * case): eliminating m^k = (x^{k-1} - x^k)/gamma_{k-1} from Algorithm 2 gives the factor
 * beta * gamma_k / gamma_{k-1} in front of the difference.  m^0 = 0 corresponds to x^{-1} = x^0. */
int oracle_decentlam_xprev_step(int n, int64_t d, int period, const int32_t* row_ptr,
                                const int32_t* col_idx, const float* w, double gamma, double gamma_prev,
                                double beta, int64_t k, const double* x, const double* x_prev,
                                const double* g, double* x_out)
{
    const int32_t* rp = row_ptr + (k % period) * (n + 1);
    size_t cnt = (size_t)n * (size_t)(d > 0 ? d : 1);
    double* local = (double*)malloc(sizeof(double) * cnt);
    double* z = (double*)malloc(sizeof(double) * cnt);
    if (!local || !z) { free(local); free(z); return -2; }
    for (int i = 0; i < n; ++i)
        for (int64_t c = 0; c < d; ++c) {
            int64_t q = (int64_t)i * d + c;
            local[q] = x[q] - gamma * g[q];
        }
    partial_average(n, d, rp, col_idx, w, local, z);
    double factor = beta * gamma / gamma_prev;
    for (int i = 0; i < n; ++i)
        for (int64_t c = 0; c < d; ++c) {
            int64_t q = (int64_t)i * d + c;
            x_out[q] = z[q] + factor * (x[q] - x_prev[q]);
        }
    free(local);
    free(z);
    return 0;
}

/* Least-squares gradient of f_i(x) = (scale/2) ||A_i x - y_i||^2 (appendix
 * "Experimental setting for linear regression": grad f_i = A_i^T (A_i x - b_i),
 * scale = 1 there):
 *   res_i = A_i x_i - y_i ; g_i = scale A_i^T res_i ; loss_i = (scale/2) ||res_i||^2
 * A is n x b x d, y is n x b (fp32 data), x is n x d. */
int oracle_lsq_grad(int n, int b, int64_t d, const float* A, const float* y, const double* x,
                    double scale, double* g_out, double* loss_out)
{
    double* res = (double*)malloc(sizeof(double) * (size_t)n * (size_t)b);
    if (!res) return -2;
#pragma omp parallel for schedule(static) collapse(2)
    for (int i = 0; i < n; ++i)
        for (int r = 0; r < b; ++r) {
            const float* a = A + ((int64_t)i * b + r) * d;
            double acc = 0.0;
            for (int64_t c = 0; c < d; ++c) acc = acc + (double)a[c] * x[(int64_t)i * d + c];
            res[(int64_t)i * b + r] = acc - (double)y[(int64_t)i * b + r];
        }
#pragma omp parallel for schedule(static)
    for (int i = 0; i < n; ++i) {
        double* gi = g_out + (int64_t)i * d;
        for (int64_t c = 0; c < d; ++c) gi[c] = 0.0;
        for (int r = 0; r < b; ++r) {
            const float* a = A + ((int64_t)i * b + r) * d;
            double rr = res[(int64_t)i * b + r];
            for (int64_t c = 0; c < d; ++c) gi[c] = gi[c] + (double)a[c] * rr;
        }
        double sq = 0.0;
        for (int r = 0; r < b; ++r) sq = sq + res[(int64_t)i * b + r] * res[(int64_t)i * b + r];
        for (int64_t c = 0; c < d; ++c) gi[c] = scale * gi[c];
        if (loss_out) loss_out[i] = 0.5 * scale * sq;
    }
    free(res);
    return 0;
}

/* Diagnostics on the stacked state (notation of the appendix "Preliminary"; the relative error
 * is the y-axis of the linear-regression experiment):
 *   out[0] = sum_i ||x_i - xbar||^2  with xbar = (1/n) sum_i x_i     (consensus distance)
 *   out[1] = ||xbar||^2
 *   out[2] = sum_i ||x_i - ref||^2   (0 if ref == NULL)
 *   out[3] = ||ref||^2               (0 if ref == NULL)
 *   out[4] = ||m||_F^2               (0 if m == NULL)
 * Two passes per column: mean first, deviations second. */
int oracle_stats(int n, int64_t d, const double* x, const double* m, const double* ref, double* out)
{
    double cons = 0.0, xbar2 = 0.0, err = 0.0, ref2 = 0.0, m2 = 0.0;
    for (int64_t c = 0; c < d; ++c) {
        double mean = 0.0;
        for (int i = 0; i < n; ++i) mean = mean + x[(int64_t)i * d + c];
        mean = mean / (double)n;
        for (int i = 0; i < n; ++i) {
            double dev = x[(int64_t)i * d + c] - mean;
            cons = cons + dev * dev;
            if (ref) {
                double e = x[(int64_t)i * d + c] - ref[c];
                err = err + e * e;
            }
            if (m) m2 = m2 + m[(int64_t)i * d + c] * m[(int64_t)i * d + c];
        }
        xbar2 = xbar2 + mean * mean;
        if (ref) ref2 = ref2 + ref[c] * ref[c];
    }
    out[0] = cons; out[1] = xbar2; out[2] = err; out[3] = ref2; out[4] = m2;
    return 0;
}

/* Stochastic version of the least-squares gradient: the sample xi_i of Algorithms 1 and 2 is a
 * list of bs row indices rows[i*bs + t] into node i's local data (repeats allowed):
 *   res_t = a_t . x_i - y_i[r_t] ;  g_i = scale sum_t a_t res_t ;  loss_i = (scale/2) sum_t res_t^2
 * with a_t the r_t-th row of A_i. */
int oracle_lsq_grad_rows(int n, int b, int64_t d, const float* A, const float* y, const double* x,
                         const int32_t* rows, int bs, double scale, double* g_out, double* loss_out)
{
    for (int i = 0; i < n; ++i) {
        double* gi = g_out + (int64_t)i * d;
        for (int64_t c = 0; c < d; ++c) gi[c] = 0.0;
        double sq = 0.0;
        for (int t = 0; t < bs; ++t) {
            int r = rows[(int64_t)i * bs + t];
            if (r < 0 || r >= b) return -1;
            const float* a = A + ((int64_t)i * b + r) * d;
            double res = 0.0;
            for (int64_t c = 0; c < d; ++c) res = res + (double)a[c] * x[(int64_t)i * d + c];
            res = res - (double)y[(int64_t)i * b + r];
            for (int64_t c = 0; c < d; ++c) gi[c] = gi[c] + (double)a[c] * res;
            sq = sq + res * res;
        }
        for (int64_t c = 0; c < d; ++c) gi[c] = scale * gi[c];
        if (loss_out) loss_out[i] = 0.5 * scale * sq;
    }
    return 0;
}
