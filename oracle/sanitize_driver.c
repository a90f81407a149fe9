/*
 * Host sanitizer driver for the oracle (TEST INFRASTRUCTURE, like the oracle itself).
 *
 * Calls every function of atomo_oracle.c on small inputs that reach its edge cases (empty and
 * single-element inputs, all-zero and rank-deficient matrices, tall / wide / square shapes, budgets
 * below one and above the number of atoms) so that a build with
 *     gcc -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all -static-libasan \
 *         sanitize_driver.c atomo_oracle.c -lm
 * reports any out-of-bounds access, use of freed memory, leak or undefined arithmetic.  It checks
 * only what the sanitizers cannot (that results are finite and a few invariants); values are pinned
 * by the test-suite.  Exit status 0 = clean.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
void oracle_uniforms(uint64_t seed, uint64_t stream, int64_t first, int64_t count, float* u);
void oracle_bernoulli_mask(const float* p, int64_t n, uint64_t seed, uint64_t stream, uint8_t* mask);
int64_t oracle_probabilities(const double* lambda, int64_t n, double s, double* p);
int oracle_svd(int32_t m, int32_t n, const double* G, double* sigma, double* U, double* V);
int64_t oracle_pack_weights(const double* lambda, const double* p, const uint8_t* mask, int64_t n, int64_t* idx, double* w);
void oracle_decode_svd_accumulate(int32_t m, int32_t n, int64_t k, const double* w, const double* Ucols,
                                  const double* Vcols, double scale, double* out);
void oracle_decode_entrywise_accumulate(int64_t k, const int64_t* idx, const double* val, double scale, double* out);
double oracle_lq_norm(const double* g, int64_t n, double q, int q_is_inf);
double oracle_lq_probabilities(const double* g, int64_t n, double q, int q_is_inf, double* p);
void oracle_decode_lq_accumulate(int64_t k, const int64_t* idx, const int8_t* sign, double norm, double scale, double* out);

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

/* small deterministic generator for the inputs (not the method's Philox) */
static uint64_t lcg_state = 0x9E3779B97F4A7C15ull;
static double next_unit(void)
{
    lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(lcg_state >> 11) / 9007199254740992.0 - 0.5;
}

static void chain_on_matrix(int32_t m, int32_t n, int rank_limit, double s)
{
    const int32_t r = m < n ? m : n;
    double* G = (double*)calloc((size_t)m * n, sizeof(double));
    /* rank_limit > 0: a sum of that many outer products; 0: dense random; < 0: all zeros */
    if (rank_limit == 0) {
        for (size_t e = 0; e < (size_t)m * n; ++e) G[e] = next_unit();
    } else if (rank_limit > 0) {
        for (int k = 0; k < rank_limit; ++k) {
            double* a = (double*)malloc((size_t)m * sizeof(double));
            double* b = (double*)malloc((size_t)n * sizeof(double));
            for (int i = 0; i < m; ++i) a[i] = next_unit();
            for (int j = 0; j < n; ++j) b[j] = next_unit();
            for (int i = 0; i < m; ++i)
                for (int j = 0; j < n; ++j) G[(size_t)i * n + j] += a[i] * b[j];
            free(a); free(b);
        }
    }
    double* sigma = (double*)malloc((size_t)r * sizeof(double));
    double* U = (double*)malloc((size_t)m * r * sizeof(double));
    double* V = (double*)malloc((size_t)n * r * sizeof(double));
    const int sweeps = oracle_svd(m, n, G, sigma, U, V);
    CHECK(sweeps > 0);
    for (int i = 0; i < r; ++i) CHECK(isfinite(sigma[i]) && sigma[i] >= 0.0 && (i == 0 || sigma[i] <= sigma[i - 1]));

    double* p = (double*)malloc((size_t)r * sizeof(double));
    const int64_t ns = oracle_probabilities(sigma, r, s, p);
    CHECK(ns >= 0 && ns <= r);
    float* p32 = (float*)malloc((size_t)r * sizeof(float));
    for (int i = 0; i < r; ++i) { CHECK(p[i] >= 0.0 && p[i] <= 1.0); p32[i] = (float)p[i]; }
    uint8_t* mask = (uint8_t*)malloc((size_t)r);
    oracle_bernoulli_mask(p32, r, 7, 3, mask);
    int64_t* idx = (int64_t*)malloc((size_t)r * sizeof(int64_t));
    double* w = (double*)malloc((size_t)r * sizeof(double));
    const int64_t kept = oracle_pack_weights(sigma, p, mask, r, idx, w);
    CHECK(kept >= 0 && kept <= r);
    /* kept columns, column-major m x kept and n x kept */
    double* Uk = (double*)malloc((size_t)(kept ? kept : 1) * m * sizeof(double));
    double* Vk = (double*)malloc((size_t)(kept ? kept : 1) * n * sizeof(double));
    for (int64_t a = 0; a < kept; ++a) {
        for (int i = 0; i < m; ++i) Uk[(size_t)a * m + i] = U[(size_t)idx[a] * m + i];
        for (int j = 0; j < n; ++j) Vk[(size_t)a * n + j] = V[(size_t)idx[a] * n + j];
    }
    double* out = (double*)calloc((size_t)m * n, sizeof(double));
    oracle_decode_svd_accumulate(m, n, kept, w, Uk, Vk, 0.5, out);
    for (size_t e = 0; e < (size_t)m * n; ++e) CHECK(isfinite(out[e]));
    free(G); free(sigma); free(U); free(V); free(p); free(p32); free(mask); free(idx); free(w); free(Uk); free(Vk); free(out);
}

static void chain_on_vector(int64_t n, double s, int zeros)
{
    double* g = (double*)malloc((size_t)(n ? n : 1) * sizeof(double));
    for (int64_t i = 0; i < n; ++i) g[i] = zeros ? 0.0 : next_unit() * ((i % 17 == 0) ? 100.0 : 1.0);
    double* p = (double*)malloc((size_t)(n ? n : 1) * sizeof(double));
    oracle_probabilities(g, n, s, p);
    float* p32 = (float*)malloc((size_t)(n ? n : 1) * sizeof(float));
    double total = 0.0;
    for (int64_t i = 0; i < n; ++i) { CHECK(p[i] >= 0.0 && p[i] <= 1.0); total += p[i]; p32[i] = (float)p[i]; }
    CHECK(total <= s * (1.0 + 1e-12) + 1e-300);
    uint8_t* mask = (uint8_t*)malloc((size_t)(n ? n : 1));
    oracle_bernoulli_mask(p32, n, 1, 2, mask);
    int64_t* idx = (int64_t*)malloc((size_t)(n ? n : 1) * sizeof(int64_t));
    double* val = (double*)malloc((size_t)(n ? n : 1) * sizeof(double));
    const int64_t kept = oracle_pack_weights(g, p, mask, n, idx, val);
    double* out = (double*)calloc((size_t)(n ? n : 1), sizeof(double));
    oracle_decode_entrywise_accumulate(kept, idx, val, 1.0, out);
    for (int64_t i = 0; i < n; ++i) CHECK(isfinite(out[i]));

    /* l_q quantisation of the same vector: q = 2, q = inf, q = 1, q = 1.5 */
    const double qs[4] = {2.0, 0.0, 1.0, 1.5};
    for (int t = 0; t < 4; ++t) {
        const int is_inf = (t == 1);
        const double norm = oracle_lq_probabilities(g, n, qs[t], is_inf, p);
        CHECK(isfinite(norm) && norm >= 0.0);
        CHECK(oracle_lq_norm(g, n, qs[t], is_inf) == norm);
        for (int64_t i = 0; i < n; ++i) { CHECK(p[i] >= 0.0 && p[i] <= 1.0 + 1e-15); p32[i] = (float)p[i]; }
        oracle_bernoulli_mask(p32, n, 5, (uint64_t)t, mask);
        int8_t* sign = (int8_t*)malloc((size_t)(n ? n : 1));
        int64_t k = 0;
        for (int64_t i = 0; i < n; ++i)
            if (mask[i]) { idx[k] = i; sign[k] = g[i] < 0.0 ? -1 : 1; ++k; }
        for (int64_t i = 0; i < n; ++i) out[i] = 0.0;
        oracle_decode_lq_accumulate(k, idx, sign, norm, 0.25, out);
        free(sign);
    }
    free(g); free(p); free(p32); free(mask); free(idx); free(val); free(out);
}

int main(void)
{
    /* Philox: block function and the uniform mapping across a block boundary and a 32-bit counter carry */
    uint32_t ctr[4] = {0xFFFFFFFFu, 0, 1, 2}, key[2] = {3, 4}, out4[4];
    oracle_philox4x32_10(ctr, key, out4);
    float u[9];
    oracle_uniforms(0xFFFFFFFFFFFFFFFFull, 0x100000000ull, ((int64_t)1 << 34) - 3, 9, u);
    for (int i = 0; i < 9; ++i) CHECK(u[i] >= 0.0f && u[i] < 1.0f);
    oracle_uniforms(0, 0, 0, 0, u);

    /* Algorithm 1: empty, one element, zeros, budget below one / between / at / above the number of atoms */
    double p1[8];
    CHECK(oracle_probabilities(p1, 0, 2.0, p1) == 0);
    const double one[1] = {-3.0};
    oracle_probabilities(one, 1, 0.25, p1); CHECK(p1[0] == 0.25);
    oracle_probabilities(one, 1, 5.0, p1); CHECK(p1[0] == 1.0);
    const double lam[6] = {4.0, 0.0, -1.0, 1.0, 0.0, 1e-300};
    const double budgets[5] = {0.5, 2.0, 3.0, 4.0, 9.0};
    for (int b = 0; b < 5; ++b) {
        oracle_probabilities(lam, 6, budgets[b], p1);
        CHECK(p1[1] == 0.0 && p1[4] == 0.0);
        for (int i = 0; i < 6; ++i) CHECK(p1[i] >= 0.0 && p1[i] <= 1.0);
    }

    chain_on_matrix(1, 1, 0, 1.0);
    chain_on_matrix(1, 7, 0, 1.0);
    chain_on_matrix(7, 1, 0, 0.5);
    chain_on_matrix(6, 6, 0, 2.0);
    chain_on_matrix(5, 12, 0, 3.0);
    chain_on_matrix(12, 5, 0, 8.0);          /* budget above the number of atoms */
    chain_on_matrix(9, 14, 2, 3.0);          /* rank 2: orthonormal completion of the zero singular values */
    chain_on_matrix(14, 9, 1, 1.0);
    chain_on_matrix(4, 6, -1, 2.0);          /* all zeros */

    chain_on_vector(0, 1.0, 0);
    chain_on_vector(1, 1.0, 0);
    chain_on_vector(5, 2.5, 1);
    chain_on_vector(1000, 10.0, 0);
    chain_on_vector(1000, 2000.0, 0);

    if (failures) { fprintf(stderr, "%d checks failed\n", failures); return 1; }
    printf("oracle sanitizer driver: clean\n");
    return 0;
}
