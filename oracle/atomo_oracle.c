/*
 * ATOMO oracle: a plain, slow, double-precision CPU statement of what the
 * gradient encoder/decoder of "ATOMO: Communication-efficient Learning via
 * Atomic Sparsification" (arXiv 1806.04090) computes.
 *
 * THIS IS TEST INFRASTRUCTURE.  Only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code, header, table
 * or helper with the HIP library and neither side includes the other.
 *
 * Every function takes its predecessor's output as an explicit argument so
 * that intermediate results of another implementation can be spliced into
 * the chain:  svd -> probabilities -> bernoulli mask -> weights -> decode.
 *
 * Parity pins: every function below is pinned by tests that do not call it
 * to produce the expected value (closed forms, brute force, known answers).
 * The one thing that cannot be pinned value-by-value is the identity of a
 * singular vector inside a cluster of (nearly) equal singular values, which
 * is not unique; those are pinned through residuals only.
 *
 * Build:  gcc -O2 -fPIC -shared -o libatomo_oracle.so atomo_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as   */
/* easy as 1, 2, 3", SC'11).  The paper only fixes the distribution of the   */
/* Bernoulli draws (Section 3, text after eq. (vhat)); the generator, and    */
/* how a 32-bit word becomes a uniform, is this build's reading.             */
/* ------------------------------------------------------------------------ */

void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t prod1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(prod0 >> 32), lo0 = (uint32_t)prod0;
        uint32_t hi1 = (uint32_t)(prod1 >> 32), lo1 = (uint32_t)prod1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;           /* the key schedule advances after every round */
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * The uniform attached to atom i of stream `stream` under `seed`:
 * counter = (i/4 as 64 bits, stream as 64 bits), key = seed as 64 bits, atom i
 * takes output word i mod 4; u = (word >> 8) * 2^-24, exact in single
 * precision, u in [0,1).
 */
void oracle_uniforms(uint64_t seed, uint64_t stream, int64_t first, int64_t count, float* u)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    for (int64_t t = 0; t < count; ++t) {
        uint64_t i = (uint64_t)(first + t);
        uint64_t blk = i >> 2;
        uint32_t ctr[4] = { (uint32_t)blk, (uint32_t)(blk >> 32),
                            (uint32_t)stream, (uint32_t)(stream >> 32) };
        uint32_t out[4];
        oracle_philox4x32_10(ctr, key, out);
        u[t] = (float)(out[i & 3] >> 8) * 0x1.0p-24f;
    }
}

/*
 * t_i ~ Bernoulli(p_i), independent (Section 3, text after eq. (vhat)).
 * The decision u < p is taken in single precision on the single-precision p
 * handed in, so that any implementation given the same p takes the same one.
 */
void oracle_bernoulli_mask(const float* p, int64_t n, uint64_t seed, uint64_t stream, uint8_t* mask)
{
    for (int64_t i = 0; i < n; ++i) {
        float u;
        oracle_uniforms(seed, stream, i, 1, &u);
        mask[i] = (u < p[i]) ? 1 : 0;
    }
}

/* ------------------------------------------------------------------------ */
/* Algorithm 1 (ATOMO probabilities), Section 3.                             */
/* ------------------------------------------------------------------------ */

typedef struct { double mag; int64_t pos; } mag_pos;

static int by_mag_desc(const void* a, const void* b)
{
    const mag_pos* x = (const mag_pos*)a;
    const mag_pos* y = (const mag_pos*)b;
    if (x->mag > y->mag) return -1;
    if (x->mag < y->mag) return 1;
    return (x->pos > y->pos) - (x->pos < y->pos);
}

/*
 * p = argmin sum lambda_i^2/p_i  s.t. 0 < p_i <= 1, sum p_i = s   (eq. (opt_prob1)).
 * Algorithm 1 reaches this minimiser exactly, and the KKT appendix writes it in
 * closed form (eq. (p_i)): with |lambda| sorted descending and
 *     T_k = sum_{j > k} |lambda_j|           (what the atoms after the first k add up to),
 * n_s is the smallest k for which the largest remaining atom fits under the
 * remaining budget,  |lambda_{k+1}| (s - k) <= T_k,  and then
 *     p_i = 1                               for the n_s largest atoms,
 *     p_i = |lambda_i| (s - n_s) / T_{n_s}  for the others.
 * The oracle is that definition written out: sort, tail sums, search for n_s,
 * one pass that fills p (scattered back to the caller's order).  Readings:
 *  - the sums in Algorithm 1's test and update run over |lambda_j| (the tail
 *    sum), as eq. (p_i) confirms, and the budget in the test is what remains
 *    after the atoms already set to 1;
 *  - lambda_i = 0 gets p_i = 0 (KKT appendix, consequence 2): once T_k = 0 only
 *    zeros remain and the search stops there instead of dividing by zero.  With
 *    s >= #nonzeros every nonzero atom gets p = 1 (KKT appendix, consequence 1).
 * Returns n_s.
 */
int64_t oracle_probabilities(const double* lambda, int64_t n, double s, double* p)
{
    if (n <= 0) return 0;
    mag_pos* a = (mag_pos*)malloc((size_t)n * sizeof(mag_pos));
    double* T = (double*)malloc((size_t)(n + 1) * sizeof(double));
    for (int64_t i = 0; i < n; ++i) { a[i].mag = fabs(lambda[i]); a[i].pos = i; }
    qsort(a, (size_t)n, sizeof(mag_pos), by_mag_desc);
    T[n] = 0.0;
    for (int64_t k = n - 1; k >= 0; --k) T[k] = T[k + 1] + a[k].mag;      /* T[k] = sum of a[k..n) */

    /* n_s: first k with T_k = 0 (nothing but zeros left) or |lambda_{k+1}| (s - k) <= T_k; k = n ends it */
    int64_t n_s = 0;
    while (n_s < n && T[n_s] > 0.0 && a[n_s].mag * (s - (double)n_s) > T[n_s]) ++n_s;

    const double budget = s - (double)n_s;
    const double rest = n_s < n ? T[n_s] : 0.0;
    for (int64_t i = 0; i < n; ++i) {
        if (i < n_s) p[a[i].pos] = 1.0;
        else p[a[i].pos] = rest > 0.0 ? a[i].mag * budget / rest : 0.0;
    }
    free(a); free(T);
    return n_s;
}

/* ------------------------------------------------------------------------ */
/* Singular value decomposition (Section 5, Notation): X = sum sigma_i u_i v_i^T */
/* ------------------------------------------------------------------------ */

/*
 * Thin SVD of the m x n row-major matrix G by unblocked cyclic one-sided
 * (Hestenes) Jacobi in double.  r = min(m, n).  On return sigma[0..r) is
 * descending, U is m x r and V is n x r, both column-major with orthonormal
 * columns, and G = sum_i sigma_i u_i v_i^T.  Columns that belong to a zero
 * singular value are an arbitrary orthonormal completion.  Returns the number
 * of sweeps taken (negative if the sweep limit was hit).
 */
int oracle_svd(int32_t m, int32_t n, const double* G, double* sigma, double* U, double* V)
{
    const int tall = (m >= n);
    const int32_t M = tall ? m : n;        /* length of the vectors that get orthogonalised */
    const int32_t r = tall ? n : m;        /* how many of them */
    /* W: M x r column-major, columns = columns of G (tall) or rows of G (wide). */
    double* W = (double*)malloc((size_t)M * r * sizeof(double));
    double* Z = (double*)calloc((size_t)r * r, sizeof(double));     /* accumulated rotations, column-major */
    for (int32_t j = 0; j < r; ++j) {
        for (int32_t i = 0; i < M; ++i)
            W[(size_t)j * M + i] = tall ? G[(size_t)i * n + j] : G[(size_t)j * n + i];
        Z[(size_t)j * r + j] = 1.0;
    }
    /* stop once every pair's cosine is at the rounding level of an M-term dot product */
    const double tol = 4.0 * 2.3e-16 * sqrt((double)M);
    const int max_sweeps = 60;
    /* vectors at or below this length are rounding residue of a rank-deficient input: they are left
       alone during the sweeps and reported as sigma = 0 */
    double frob2 = 0.0;
    for (size_t e = 0; e < (size_t)M * r; ++e) frob2 += W[e] * W[e];
    const double zero_below = (double)M * (double)r * 2.3e-16 * sqrt(frob2);
    int sweeps = 0, rotated = 1;
    while (rotated && sweeps < max_sweeps) {
        rotated = 0;
        ++sweeps;
        for (int32_t p = 0; p < r - 1; ++p) {
            for (int32_t q = p + 1; q < r; ++q) {
                double* wp = W + (size_t)p * M;
                double* wq = W + (size_t)q * M;
                double alpha = 0.0, beta = 0.0, gamma = 0.0;
                for (int32_t i = 0; i < M; ++i) {
                    alpha += wp[i] * wp[i];
                    beta  += wq[i] * wq[i];
                    gamma += wp[i] * wq[i];
                }
                if (gamma == 0.0 || fabs(gamma) <= tol * sqrt(alpha * beta)) continue;
                if (sqrt(alpha) <= zero_below || sqrt(beta) <= zero_below) continue;
                rotated = 1;
                double zeta = (beta - alpha) / (2.0 * gamma);
                double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                double c = 1.0 / sqrt(1.0 + t * t);
                double sn = c * t;
                for (int32_t i = 0; i < M; ++i) {
                    double x = wp[i], y = wq[i];
                    wp[i] = c * x - sn * y;
                    wq[i] = sn * x + c * y;
                }
                double* zp = Z + (size_t)p * r;
                double* zq = Z + (size_t)q * r;
                for (int32_t i = 0; i < r; ++i) {
                    double x = zp[i], y = zq[i];
                    zp[i] = c * x - sn * y;
                    zq[i] = sn * x + c * y;
                }
            }
        }
    }
    /* column norms are the singular values; order them descending */
    mag_pos* order = (mag_pos*)malloc((size_t)r * sizeof(mag_pos));
    for (int32_t j = 0; j < r; ++j) {
        double nrm2 = 0.0;
        const double* wj = W + (size_t)j * M;
        for (int32_t i = 0; i < M; ++i) nrm2 += wj[i] * wj[i];
        order[j].mag = sqrt(nrm2);
        order[j].pos = j;
    }
    qsort(order, (size_t)r, sizeof(mag_pos), by_mag_desc);

    double* longv  = tall ? U : V;     /* M x r: normalised columns of W */
    double* shortv = tall ? V : U;     /* r x r: columns of Z */
    for (int32_t k = 0; k < r; ++k) {
        int32_t j = (int32_t)order[k].pos;
        double sg = order[k].mag;
        memcpy(shortv + (size_t)k * r, Z + (size_t)j * r, (size_t)r * sizeof(double));
        if (sg > zero_below && sg > 0.0) {
            sigma[k] = sg;
            for (int32_t i = 0; i < M; ++i) longv[(size_t)k * M + i] = W[(size_t)j * M + i] / sg;
        } else {
            sigma[k] = 0.0;
            for (int32_t i = 0; i < M; ++i) longv[(size_t)k * M + i] = 0.0;
        }
    }
    /* orthonormal completion of the long vectors that belong to sigma = 0 */
    int32_t next_axis = 0;
    for (int32_t k = 0; k < r; ++k) {
        if (sigma[k] != 0.0) continue;
        double* col = longv + (size_t)k * M;
        while (next_axis < M) {
            for (int32_t i = 0; i < M; ++i) col[i] = 0.0;
            col[next_axis++] = 1.0;
            for (int pass = 0; pass < 2; ++pass) {
                for (int32_t q = 0; q < r; ++q) {
                    if (q == k || (sigma[q] == 0.0 && q > k)) continue;
                    const double* other = longv + (size_t)q * M;
                    double d = 0.0;
                    for (int32_t i = 0; i < M; ++i) d += other[i] * col[i];
                    for (int32_t i = 0; i < M; ++i) col[i] -= d * other[i];
                }
            }
            double nrm2 = 0.0;
            for (int32_t i = 0; i < M; ++i) nrm2 += col[i] * col[i];
            if (nrm2 > 0.25) {
                double inv = 1.0 / sqrt(nrm2);
                for (int32_t i = 0; i < M; ++i) col[i] *= inv;
                break;
            }
        }
    }
    free(order); free(W); free(Z);
    return rotated ? -sweeps : sweeps;
}

/* ------------------------------------------------------------------------ */
/* Rescale (eq. (vhat)): a kept atom carries lambda_i / p_i.                  */
/* ------------------------------------------------------------------------ */

/*
 * Kept atoms in ascending atom index.  idx/w must hold n entries at most.
 * Returns the number kept.  An atom with p_i = 0 is never kept (its mask bit
 * cannot be set because u >= 0), which is the 0/0 := 0 reading of eq. (vhat).
 */
int64_t oracle_pack_weights(const double* lambda, const double* p, const uint8_t* mask, int64_t n,
                            int64_t* idx, double* w)
{
    int64_t k = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (!mask[i]) continue;
        idx[k] = i;
        w[k] = lambda[i] / p[i];
        ++k;
    }
    return k;
}

/* ------------------------------------------------------------------------ */
/* Decode (eq. (vhat)):  g_hat = sum over kept atoms of (lambda_i/p_i) a_i.   */
/* ------------------------------------------------------------------------ */

/*
 * out (m x n row-major) += scale * sum_k w[k] * Ucols[:,k] * Vcols[:,k]^T.
 * Ucols is m x k, Vcols is n x k, column-major (one kept atom per column).
 * Accumulating lets the caller sum several messages (the parameter-server
 * average of Section 2 uses scale = 1/P).
 */
void oracle_decode_svd_accumulate(int32_t m, int32_t n, int64_t k, const double* w,
                                  const double* Ucols, const double* Vcols, double scale, double* out)
{
    for (int64_t a = 0; a < k; ++a) {
        const double* u = Ucols + (size_t)a * m;
        const double* v = Vcols + (size_t)a * n;
        for (int32_t i = 0; i < m; ++i) {
            double ui = scale * w[a] * u[i];
            double* row = out + (size_t)i * n;
            for (int32_t j = 0; j < n; ++j) row[j] += ui * v[j];
        }
    }
}

/* Entry-wise atoms a_i = e_i:  out[idx[k]] += scale * val[k]. */
void oracle_decode_entrywise_accumulate(int64_t k, const int64_t* idx, const double* val, double scale, double* out)
{
    for (int64_t a = 0; a < k; ++a) out[idx[a]] += scale * val[a];
}

/* ------------------------------------------------------------------------ */
/* l_q quantisation (Section 4): 1-bit QSGD (q = 2), TernGrad (q = inf).      */
/* ------------------------------------------------------------------------ */

/*
 * ||g||_q for q in (0, inf]; q_is_inf != 0 selects the maximum norm.
 * Plain left-to-right sums in double.
 */
double oracle_lq_norm(const double* g, int64_t n, double q, int q_is_inf)
{
    double acc = 0.0;
    if (q_is_inf) {
        for (int64_t i = 0; i < n; ++i) { double a = fabs(g[i]); if (a > acc) acc = a; }
        return acc;
    }
    if (q == 2.0) {
        for (int64_t i = 0; i < n; ++i) acc += g[i] * g[i];
        return sqrt(acc);
    }
    if (q == 1.0) {
        for (int64_t i = 0; i < n; ++i) acc += fabs(g[i]);
        return acc;
    }
    for (int64_t i = 0; i < n; ++i) if (g[i] != 0.0) acc += pow(fabs(g[i]), q);
    return pow(acc, 1.0 / q);
}

/*
 * The probabilities of l_q quantisation, p_i = |g_i| / ||g||_q (text before
 * Theorem (lqgrad)); an all-zero g gives p = 0.  Returns the norm.
 */
double oracle_lq_probabilities(const double* g, int64_t n, double q, int q_is_inf, double* p)
{
    double norm = oracle_lq_norm(g, n, q, q_is_inf);
    for (int64_t i = 0; i < n; ++i) p[i] = norm > 0.0 ? fabs(g[i]) / norm : 0.0;
    return norm;
}

/* L_q(g)_i = ||g||_q sign(g_i) zeta_i:  out[idx[k]] += scale * sign[k] * norm. */
void oracle_decode_lq_accumulate(int64_t k, const int64_t* idx, const int8_t* sign, double norm, double scale, double* out)
{
    for (int64_t a = 0; a < k; ++a) out[idx[a]] += scale * (double)sign[a] * norm;
}

