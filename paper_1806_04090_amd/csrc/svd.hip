// Spectral-ATOMO encoder (Section 5 of arXiv 1806.04090): batched blocked one-sided Jacobi SVD on
// fp32 MFMA, followed by Algorithm 1 on the singular values, Philox Bernoulli sampling and packing
// of the kept singular triplets.
//
// Layout.  For a matrix G (rows x cols) let r = min(rows, cols) and M = max(rows, cols).  The r
// vectors of length M that get orthogonalised (the rows of G, or of G^T when rows > cols) are the
// rows of a workspace matrix W = [A | T]: A (r x M) starts as those vectors, T (r x r) starts as the
// identity.  Every rotation is applied to whole rows of W, so at all times  A = T * A0  with T
// orthogonal, and on convergence row i of A is sigma_i times one singular vector and row i of T is
// the matching singular vector of the other side.  Rows are padded to blocks of 32 (plus one extra
// zero block if the number of blocks is odd); columns of A and T are padded to multiples of 64 with
// zeros, so the kernels need no edge handling.
//
// One Jacobi "step" visits, for every matrix at once, one round of a round-robin tournament over
// its row blocks: for each pair of blocks (64 rows)
//     svd_gram   : partial 64x64 Gram matrices of the pair over column chunks      (MFMA)
//     svd_eig    : sums the partials, diagonalises the Gram matrix by two-sided Jacobi in LDS,
//                  re-orthogonalises the accumulated rotation (one Newton-Schulz step, MFMA) and
//                  orders its columns by decreasing eigenvalue
//     svd_update : rows <- Q^T rows over all of W                                   (MFMA)
// A sweep is R = (#blocks - 1) rounds.  Matrices with fewer blocks simply run through their sweeps
// faster; a matrix stops when, in one sweep, no pair of rows had |cos| above the threshold.
#include <cfloat>
#include <cmath>
#include <vector>

#include "atomo_internal.h"
#include "block_algorithm1.h"

namespace atomo {

namespace {

constexpr int BS = 32;          // rows per block
constexpr int PR = 64;          // rows per pair
constexpr int KCG = 512;        // columns per svd_gram work item
constexpr int KCU = 256;        // columns per svd_update work item (4 waves x 64)
constexpr int QSZ = PR * PR;
constexpr int MAX_R = ALG1_MAX;

typedef float floatx16 __attribute__((ext_vector_type(16)));

enum { ST_DONE_AT = 0, ST_SWEEPS = 1, ST_OFFMAX = 2, ST_ARRIVE = 3, ST_SCALE = 4, ST_SCALE_NEXT = 5, ST_WORDS = 8 };

// Rows whose squared norm is below ZERO_REL * (largest squared row norm of the matrix) are rounding
// residue of the fp32 updates (about 32 ulp of the dominant rows): their directions carry no
// information, so they neither count in the convergence test nor get rotated among themselves.
constexpr float ZERO_REL = 3.64e-12f;       // (32 * 2^-24)^2

struct SvdMat {
    float* W;                // rows_alloc x ldw
    int ldw, r, M, Mp, rows_alloc;
    int nb2, R, npairs, nchg, nchu;
    float* gram;             // [npairs][nchg][64*64]
    float* Q;                // [npairs][64*64]
    int* state;              // [ST_WORDS]
    float* sig_raw;          // [rows_alloc]
    const float* G;
    long long ldg;
    int rows, cols, transposed;
    int* count;
    int* idx;
    float* w;
    float* U;
    float* V;
    int capacity;
    float* sigma_out;        // may be null
    float* p_out;            // may be null
    unsigned long long stream_id;
    int* src_row;            // [capacity]
    float* src_inv;          // [capacity]
};

struct Work { int mat, a, b, c; };

__device__ inline void pair_blocks(int nb2, int round, int k, int& bi, int& bj)
{
    const int n1 = nb2 - 1;
    int a, b;
    if (k == 0) { a = n1; b = round; }
    else { a = (round + k) % n1; b = (round - k + n1) % n1; }
    bi = a < b ? a : b;
    bj = a < b ? b : a;
}

// True if work for `step` of this matrix should be skipped (finished earlier, or past the sweep limit).
__device__ inline bool skip_step(const SvdMat& m, int step, int max_sweeps)
{
    const int done_at = m.state[ST_DONE_AT];
    if (done_at != 0 && step >= done_at) return true;
    return step / m.R >= max_sweeps;
}

// ------------------------------------------------------------------------------------------------
// prepare: W = [A | T], padded
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void svd_prepare(const SvdMat* mats, const Work* work)
{
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    const int row0 = wk.a * BS;
    const int c = wk.b * 256 + threadIdx.x;
    if (wk.a == 0 && wk.b == 0 && threadIdx.x < ST_WORDS) m.state[threadIdx.x] = 0;
    if (c >= m.ldw) return;
    for (int i = row0; i < row0 + BS; ++i) {
        float v = 0.0f;
        if (i < m.r) {
            if (c < m.M) v = m.transposed ? m.G[(long long)c * m.ldg + i] : m.G[(long long)i * m.ldg + c];
            else if (c - m.Mp == i) v = 1.0f;
        }
        m.W[(size_t)i * m.ldw + c] = v;
    }
}

// ------------------------------------------------------------------------------------------------
// gram: partial Gram matrix of one 64-row pair over one column chunk
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void svd_gram(const SvdMat* mats, const Work* work, int step, int max_sweeps)
{
    __shared__ float tile[PR][68];
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    if (skip_step(m, step, max_sweeps)) return;
    int bi, bj;
    pair_blocks(m.nb2, step % m.R, wk.a, bi, bj);
    const int c_begin = wk.b * KCG;
    const int c_end = min(m.Mp, c_begin + KCG);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int qi = wave >> 1, qj = wave & 1;
    const int h = lane >> 5, l32 = lane & 31;
    // loader mapping: 16 threads per row (float4 each), 16 rows per pass, 4 passes
    const int lrow = tid >> 4, lc4 = (tid & 15) * 4;

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    for (int c0 = c_begin; c0 < c_end; c0 += 64) {
        float4 ld[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int lr = lrow + 16 * p;                       // 0..63
            const int grow = (lr < BS ? bi * BS + lr : bj * BS + lr - BS);
            ld[p] = *(const float4*)(m.W + (size_t)grow * m.ldw + c0 + lc4);
        }
        __syncthreads();                                         // previous tile fully consumed
#pragma unroll
        for (int p = 0; p < 4; ++p) *(float4*)&tile[lrow + 16 * p][lc4] = ld[p];
        __syncthreads();
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const float4 a = *(const float4*)&tile[qi * BS + l32][h * 32 + 4 * s];
            const float4 b = *(const float4*)&tile[qj * BS + l32][h * 32 + 4 * s];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
        }
    }
    float* out = m.gram + ((size_t)wk.a * m.nchg + wk.b) * QSZ;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int i = qi * BS + 8 * (v >> 2) + 4 * h + (v & 3);
        out[i * PR + qj * BS + l32] = acc[v];
    }
}

// ------------------------------------------------------------------------------------------------
// eig: 64x64 symmetric eigen-decomposition by parallel-ordered two-sided Jacobi in LDS
// ------------------------------------------------------------------------------------------------
constexpr int LDA = 65;

__global__ __launch_bounds__(256) void svd_eig(const SvdMat* mats, const Work* work, int step, int max_sweeps,
                                               float stop_cosine, int* flags)
{
    __shared__ float A[PR * LDA];
    __shared__ float Qm[PR * LDA];
    __shared__ float rc[32], rs[32];
    __shared__ int rp[32], rq[32];
    __shared__ float ev[PR];
    __shared__ int dest[PR];
    __shared__ float red[8];
    __shared__ int rotated;

    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    if (skip_step(m, step, max_sweeps)) return;
    const int round = step % m.R;
    int bi, bj;
    pair_blocks(m.nb2, round, wk.a, bi, bj);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // 1. sum the partial Gram matrices in a fixed order
    {
        const float* g = m.gram + (size_t)wk.a * m.nchg * QSZ;
        for (int e = tid; e < QSZ; e += 256) {
            float sum = 0.0f;
            for (int c = 0; c < m.nchg; ++c) sum += g[(size_t)c * QSZ + e];
            const int i = e >> 6, j = e & 63;
            A[i * LDA + j] = sum;
            Qm[i * LDA + j] = (i == j) ? 1.0f : 0.0f;
        }
    }
    __syncthreads();
    // symmetrise (the two off-diagonal quadrants were accumulated in different orders)
    for (int e = tid; e < QSZ; e += 256) {
        const int i = e >> 6, j = e & 63;
        if (i < j) {
            const float v = 0.5f * (A[i * LDA + j] + A[j * LDA + i]);
            A[i * LDA + j] = v;
            A[j * LDA + i] = v;
        }
    }
    __syncthreads();

    // 2. largest |cos| between two rows of the pair, before rotating (rows at the rounding floor
    //    are measured against the floor instead of their own length), and the largest squared norm
    const float z2 = ZERO_REL * __int_as_float(m.state[ST_SCALE]);
    {
        float mx = 0.0f, dmax = 0.0f;
        for (int e = tid; e < QSZ; e += 256) {
            const int i = e >> 6, j = e & 63;
            if (i < j) {
                const float dii = A[i * LDA + i], djj = A[j * LDA + j];
                if (dii > 0.0f && djj > 0.0f) mx = fmaxf(mx, fabsf(A[i * LDA + j]) / fmaxf(sqrtf(dii * djj), z2));
            } else if (i == j) {
                dmax = fmaxf(dmax, A[i * LDA + i]);
            }
        }
        for (int o = 32; o > 0; o >>= 1) {
            mx = fmaxf(mx, __shfl_down(mx, o));
            dmax = fmaxf(dmax, __shfl_down(dmax, o));
        }
        if (lane == 0) { red[wave] = mx; red[4 + wave] = dmax; }
        __syncthreads();
        if (tid == 0) {
            mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
            dmax = fmaxf(fmaxf(red[4], red[5]), fmaxf(red[6], red[7]));
            atomicMax((unsigned int*)&m.state[ST_OFFMAX], __float_as_uint(mx));
            atomicMax((unsigned int*)&m.state[ST_SCALE_NEXT], __float_as_uint(dmax));
        }
    }

    // 3. Jacobi sweeps, round-robin over 64 indices: 63 steps of 32 disjoint rotations
    for (int isw = 0; isw < 3; ++isw) {
        if (tid == 0) rotated = 0;
        for (int t = 0; t < 63; ++t) {
            if (tid < 32) {
                int a, b;
                if (tid == 0) { a = 63; b = t; }
                else { a = (t + tid) % 63; b = (t - tid + 63) % 63; }
                const int p = a < b ? a : b, q = a < b ? b : a;
                const float app = A[p * LDA + p], aqq = A[q * LDA + q], apq = A[p * LDA + q];
                float c = 1.0f, s = 0.0f;
                if (apq != 0.0f && fabsf(apq) > 1e-7f * fmaxf(sqrtf(fabsf(app * aqq)), z2)) {
                    const float zeta = (aqq - app) / (2.0f * apq);
                    const float tt = copysignf(1.0f, zeta) / (fabsf(zeta) + sqrtf(1.0f + zeta * zeta));
                    c = 1.0f / sqrtf(1.0f + tt * tt);
                    s = c * tt;
                    rotated = 1;
                }
                rc[tid] = c; rs[tid] = s; rp[tid] = p; rq[tid] = q;
            }
            __syncthreads();
            // A <- J^T A J on 2x2 blocks (row pair a, column pair b)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int blk = tid + 256 * e;
                const int a = blk >> 5, b = blk & 31;
                const float ca = rc[a], sa = rs[a], cb = rc[b], sb = rs[b];
                const int pa = rp[a], qa = rq[a], pb = rp[b], qb = rq[b];
                const float x00 = A[pa * LDA + pb], x01 = A[pa * LDA + qb];
                const float x10 = A[qa * LDA + pb], x11 = A[qa * LDA + qb];
                const float y00 = ca * x00 - sa * x10, y01 = ca * x01 - sa * x11;
                const float y10 = sa * x00 + ca * x10, y11 = sa * x01 + ca * x11;
                A[pa * LDA + pb] = cb * y00 - sb * y01;
                A[pa * LDA + qb] = sb * y00 + cb * y01;
                A[qa * LDA + pb] = cb * y10 - sb * y11;
                A[qa * LDA + qb] = sb * y10 + cb * y11;
            }
            // Q <- Q J
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int item = tid + 256 * e;
                const int i = item >> 5, b = item & 31;
                const float cb = rc[b], sb = rs[b];
                const int pb = rp[b], qb = rq[b];
                const float x = Qm[i * LDA + pb], y = Qm[i * LDA + qb];
                Qm[i * LDA + pb] = cb * x - sb * y;
                Qm[i * LDA + qb] = sb * x + cb * y;
            }
            __syncthreads();
        }
        if (rotated == 0) break;
        __syncthreads();
    }

    // 4. eigenvalues, and where each eigenvector goes: decreasing eigenvalue over the live rows of
    //    the pair, padding rows stay padding rows
    const int nI = max(0, min(BS, m.r - bi * BS)), nJ = max(0, min(BS, m.r - bj * BS));
    if (tid < PR) {
        const bool live = tid < BS ? tid < nI : tid - BS < nJ;
        ev[tid] = live ? A[tid * LDA + tid] : -FLT_MAX;
    }
    __syncthreads();
    if (tid < PR) {
        const float mine = ev[tid];
        int rank = 0;
        for (int j = 0; j < PR; ++j) {
            const float o = ev[j];
            rank += (o > mine) || (o == mine && j < tid);
        }
        int slot;
        if (rank < nI) slot = rank;
        else if (rank < nI + nJ) slot = BS + rank - nI;
        else {
            const int pad = rank - nI - nJ;                      // padding rows, in order
            slot = pad < BS - nI ? nI + pad : BS + nJ + pad - (BS - nI);
        }
        dest[tid] = slot;
    }
    __syncthreads();

    // 5. one Newton-Schulz step  Q <- Q (1.5 I - 0.5 Q^T Q): removes the drift of thousands of fp32 rotations
    const int qi = wave >> 1, qj = wave & 1, h = lane >> 5, l32 = lane & 31;
    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    for (int k = 0; k < PR; k += 2) {
        const float a = Qm[(k + h) * LDA + qi * BS + l32];       // (Q^T)[i][k]
        const float b = Qm[(k + h) * LDA + qj * BS + l32];       // Q[k][j]
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int i = qi * BS + 8 * (v >> 2) + 4 * h + (v & 3), j = qj * BS + l32;
        A[i * LDA + j] = (i == j ? 1.5f : 0.0f) - 0.5f * acc[v];  // F = 1.5 I - 0.5 Q^T Q
    }
    __syncthreads();
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    for (int k = 0; k < PR; k += 2) {
        const float a = Qm[(qi * BS + l32) * LDA + k + h];       // Q[i][k]
        const float b = A[(k + h) * LDA + qj * BS + l32];        // F[k][j]
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
    }
    // 6. write Q with its columns permuted to their destination rows
    float* qout = m.Q + (size_t)wk.a * QSZ;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int i = qi * BS + 8 * (v >> 2) + 4 * h + (v & 3), j = qj * BS + l32;
        qout[i * PR + dest[j]] = acc[v];
    }

    // 7. end of a sweep: the last pair to arrive decides whether the matrix is finished
    if (round == m.R - 1 && tid == 0) {
        __threadfence();
        const int arrived = atomicAdd(&m.state[ST_ARRIVE], 1);
        if (arrived == m.npairs - 1) {
            __threadfence();
            const float worst = __uint_as_float(atomicAdd((unsigned int*)&m.state[ST_OFFMAX], 0u));
            const int sweeps = m.state[ST_SWEEPS] + 1;
            m.state[ST_SWEEPS] = sweeps;
            atomicMax(&flags[FLAG_MAX_SWEEPS], sweeps);
            if (worst < stop_cosine) m.state[ST_DONE_AT] = step + 1;
            else if (sweeps >= max_sweeps) atomicMax(&flags[FLAG_NOCONV], 1);
            m.state[ST_OFFMAX] = 0;
            m.state[ST_ARRIVE] = 0;
            const unsigned int grown = atomicAdd((unsigned int*)&m.state[ST_SCALE_NEXT], 0u);
            if (grown > (unsigned int)m.state[ST_SCALE]) m.state[ST_SCALE] = (int)grown;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// update: rows of the pair <- Q^T rows, over one 256-column chunk of W (in place)
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void svd_update(const SvdMat* mats, const Work* work, int step, int max_sweeps)
{
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    if (skip_step(m, step, max_sweeps)) return;
    int bi, bj;
    pair_blocks(m.nb2, step % m.R, wk.a, bi, bj);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, l32 = lane & 31;
    const int c0 = wk.b * KCU + wave * 64;
    if (c0 >= m.ldw) return;
    const float* q = m.Q + (size_t)wk.a * QSZ;

    floatx16 acc[2][2];                                          // [column parity][row block]
#pragma unroll
    for (int e = 0; e < 2; ++e)
#pragma unroll
        for (int ib = 0; ib < 2; ++ib)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[e][ib][v] = 0.0f;

    float* rowI = m.W + (size_t)bi * BS * m.ldw + c0 + 2 * l32;
    float* rowJ = m.W + (size_t)bj * BS * m.ldw + c0 + 2 * l32;
#pragma unroll 4
    for (int s = 0; s < 32; ++s) {
        const int k = 2 * s + h;                                 // local row of the pair, 0..63
        const float* src = (k < BS ? rowI + (size_t)k * m.ldw : rowJ + (size_t)(k - BS) * m.ldw);
        const float2 x = *(const float2*)src;
        const float q0 = q[k * PR + l32];                        // (Q^T)[i][k], i in block 0
        const float q1 = q[k * PR + BS + l32];                   //              i in block 1
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(q0, x.x, acc[0][0], 0, 0, 0);
        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(q0, x.y, acc[1][0], 0, 0, 0);
        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(q1, x.x, acc[0][1], 0, 0, 0);
        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(q1, x.y, acc[1][1], 0, 0, 0);
    }
#pragma unroll
    for (int ib = 0; ib < 2; ++ib) {
        float* base = (ib == 0 ? rowI : rowJ);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = 8 * (v >> 2) + 4 * h + (v & 3);
            *(float2*)(base + (size_t)i * m.ldw) = make_float2(acc[0][ib][v], acc[1][ib][v]);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// finalise: singular values, Algorithm 1, Bernoulli draws, message
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void svd_norms(const SvdMat* mats, const Work* work, int init)
{
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = wk.a * 4 + wave;
    if (row >= m.rows_alloc) return;
    const float* a = m.W + (size_t)row * m.ldw;
    float sum = 0.0f;
    for (int c = lane * 4; c < m.Mp; c += 256) {
        const float4 x = *(const float4*)(a + c);
        sum += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
    }
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_down(sum, o);
    if (lane == 0) {
        if (init) {                                                  // before the first sweep: scale of the matrix
            atomicMax((unsigned int*)&m.state[ST_SCALE], __float_as_uint(sum));
            atomicMax((unsigned int*)&m.state[ST_SCALE_NEXT], __float_as_uint(sum));
        } else {
            m.sig_raw[row] = row < m.r ? sqrtf(sum) : 0.0f;
        }
    }
}

// One workgroup per matrix.  Sorts sigma (descending), runs Algorithm 1 on it, draws the Bernoulli
// mask (eq. (vhat): t_i ~ Bernoulli(p_i)) and writes the message header with weights sigma_i / p_i.
__global__ __launch_bounds__(256) void svd_select(const SvdMat* mats, double s, unsigned long long seed, int* flags)
{
    __shared__ float key[ALG1_MAX];
    __shared__ int src[ALG1_MAX];
    __shared__ Alg1Scratch sc;
    __shared__ int ipart[256];

    const SvdMat m = mats[blockIdx.x];
    const int tid = threadIdx.x;
    const int r = m.r;
    int P = 1;
    while (P < r) P <<= 1;
    for (int i = tid; i < P; i += 256) {
        key[i] = i < r ? m.sig_raw[i] : -1.0f;
        src[i] = i;
    }
    __syncthreads();
    block_sort_desc(key, src, P);
    const int ns = block_algorithm1(key, r, s, sc);
    const double tail_ns = sc.tail_ns;

    const int per = (r + 255) / 256;
    const int lo = min(r, tid * per), hi = min(r, lo + per);
    // pass 1: probabilities and how many atoms this slice keeps; pass 2: ordered compaction
    int kept_local = 0;
    for (int i = lo; i < hi; ++i) {
        const float p = alg1_probability(key[i], i, ns, s, tail_ns);
        const u32x4 rnd = philox4x32_10((unsigned long long)(i >> 2), m.stream_id, seed);
        const uint32_t word = (i & 3) == 0 ? rnd.x : (i & 3) == 1 ? rnd.y : (i & 3) == 2 ? rnd.z : rnd.w;
        if (m.sigma_out) m.sigma_out[i] = key[i];
        if (m.p_out) m.p_out[i] = p;
        kept_local += u01(word) < p;
    }
    ipart[tid] = kept_local;
    __syncthreads();
    int pos = 0;
    for (int t = 0; t < tid; ++t) pos += ipart[t];
    if (tid == 255) {
        const int total = pos + kept_local;
        *m.count = total;
        if (total > m.capacity) atomicMax(&flags[FLAG_CAPACITY], 1);
    }
    for (int i = lo; i < hi; ++i) {
        const float p = alg1_probability(key[i], i, ns, s, tail_ns);
        const u32x4 rnd = philox4x32_10((unsigned long long)(i >> 2), m.stream_id, seed);
        const uint32_t word = (i & 3) == 0 ? rnd.x : (i & 3) == 1 ? rnd.y : (i & 3) == 2 ? rnd.z : rnd.w;
        if (u01(word) < p) {
            if (pos < m.capacity) {
                m.idx[pos] = i;
                m.w[pos] = key[i] / p;
                m.src_row[pos] = src[i];
                m.src_inv[pos] = 1.0f / key[i];
            }
            ++pos;
        }
    }
}

// Copies the kept singular vectors into the message: grid = (matrix, slot).
__global__ __launch_bounds__(256) void svd_pack(const SvdMat* mats, const Work* work)
{
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    const int slot = wk.a;
    const int kept = min(*m.count, m.capacity);
    if (slot >= kept) return;
    const int row = m.src_row[slot];
    const float inv = m.src_inv[slot];
    const float* a = m.W + (size_t)row * m.ldw;
    float* long_out = m.transposed ? m.U + (size_t)slot * m.rows : m.V + (size_t)slot * m.cols;
    float* short_out = m.transposed ? m.V + (size_t)slot * m.cols : m.U + (size_t)slot * m.rows;
    for (int c = threadIdx.x; c < m.M; c += 256) long_out[c] = a[c] * inv;
    for (int c = threadIdx.x; c < m.r; c += 256) short_out[c] = a[m.Mp + c];
}

struct Plan {
    std::vector<SvdMat> mats;
    std::vector<Work> prep, gram, eig, upd, norms, pack;
    int max_R = 1;
    size_t bytes = 0;
    SvdMat* d_mats = nullptr;    // device copies of `mats` and of the concatenated work lists
    Work* d_work = nullptr;
};

// Lays the workspace out (base == nullptr: sizes only).
void build_plan(const atomo_mat* mats, int n_mats, const atomo_svd_msg* msgs, float* sigma_out, float* p_out,
                uint64_t stream_base, void* base, Plan& plan)
{
    Carver carve(base);
    plan.mats.resize(n_mats);
    plan.d_mats = carve.take<SvdMat>(n_mats);
    size_t atom_off = 0;
    for (int j = 0; j < n_mats; ++j) {
        SvdMat& m = plan.mats[j];
        const atomo_mat& a = mats[j];
        m.rows = a.rows; m.cols = a.cols;
        m.transposed = a.rows > a.cols;
        m.r = m.transposed ? a.cols : a.rows;
        m.M = m.transposed ? a.rows : a.cols;
        m.Mp = (int)align_up(m.M, 64);
        m.ldw = m.Mp + (int)align_up(m.r, 64);
        const int nb = (m.r + BS - 1) / BS;
        m.nb2 = nb + (nb & 1);
        m.rows_alloc = m.nb2 * BS;
        m.R = m.nb2 - 1;
        m.npairs = m.nb2 / 2;
        m.nchg = (m.Mp + KCG - 1) / KCG;
        m.nchu = (m.ldw + KCU - 1) / KCU;
        m.W = carve.take<float>((size_t)m.rows_alloc * m.ldw);
        m.gram = carve.take<float>((size_t)m.npairs * m.nchg * QSZ);
        m.Q = carve.take<float>((size_t)m.npairs * QSZ);
        m.state = carve.take<int>(ST_WORDS);
        m.sig_raw = carve.take<float>(m.rows_alloc);
        m.G = a.data; m.ldg = a.ld;
        if (msgs) {
            const atomo_svd_msg& g = msgs[j];
            m.count = g.count; m.idx = g.idx; m.w = g.w; m.U = g.U; m.V = g.V;
            m.capacity = g.capacity < m.r ? g.capacity : m.r;
        } else {
            m.count = nullptr; m.idx = nullptr; m.w = nullptr; m.U = nullptr; m.V = nullptr; m.capacity = 1;
        }
        m.src_row = carve.take<int>(m.capacity);
        m.src_inv = carve.take<float>(m.capacity);
        m.sigma_out = sigma_out ? sigma_out + atom_off : nullptr;
        m.p_out = p_out ? p_out + atom_off : nullptr;
        atom_off += m.r;
        m.stream_id = stream_base + (uint64_t)j;
        if (m.R > plan.max_R) plan.max_R = m.R;
        for (int b = 0; b < m.nb2; ++b)
            for (int c = 0; c < (m.ldw + 255) / 256; ++c) plan.prep.push_back(Work{j, b, c, 0});
        for (int k = 0; k < m.npairs; ++k) {
            for (int c = 0; c < m.nchg; ++c) plan.gram.push_back(Work{j, k, c, 0});
            plan.eig.push_back(Work{j, k, 0, 0});
            for (int c = 0; c < m.nchu; ++c) plan.upd.push_back(Work{j, k, c, 0});
        }
        for (int g = 0; g < m.rows_alloc / 4; ++g) plan.norms.push_back(Work{j, g, 0, 0});
        for (int k = 0; k < m.capacity; ++k) plan.pack.push_back(Work{j, k, 0, 0});
    }
    const size_t n_work = plan.prep.size() + plan.gram.size() + plan.eig.size() + plan.upd.size() +
                          plan.norms.size() + plan.pack.size();
    plan.d_work = carve.take<Work>(n_work);
    plan.bytes = carve.off;
}

}  // namespace

int svd_workspace_bytes(const atomo_mat* mats, int n_mats, size_t* bytes)
{
    for (int j = 0; j < n_mats; ++j) {
        if (mats[j].rows <= 0 || mats[j].cols <= 0) return ATOMO_EINVAL;
        if ((mats[j].rows < mats[j].cols ? mats[j].rows : mats[j].cols) > MAX_R) return ATOMO_EINVAL;
    }
    Plan plan;
    build_plan(mats, n_mats, nullptr, nullptr, nullptr, 0, nullptr, plan);
    *bytes = plan.bytes;
    return ATOMO_OK;
}

int encode_svd(atomo_ctx* ctx, const atomo_mat* mats, int n_mats, double s, uint64_t seed, uint64_t stream_base,
               const atomo_svd_options* opt, const atomo_svd_msg* msgs, float* sigma_out, float* p_out,
               hipStream_t stream)
{
    const int max_sweeps = opt ? opt->max_sweeps : 12;
    const float stop_cosine = opt ? opt->stop_cosine : 1e-4f;

    Plan sizing;
    build_plan(mats, n_mats, msgs, sigma_out, p_out, stream_base, nullptr, sizing);
    int rc = ensure_workspace(ctx, sizing.bytes);
    if (rc != ATOMO_OK) return rc;

    Plan plan;
    build_plan(mats, n_mats, msgs, sigma_out, p_out, stream_base, ctx->ws, plan);

    SvdMat* d_mats = plan.d_mats;
    Work* d_work = plan.d_work;
    const size_t n_work = plan.prep.size() + plan.gram.size() + plan.eig.size() + plan.upd.size() +
                          plan.norms.size() + plan.pack.size();
    std::vector<Work> all;
    all.reserve(n_work);
    const size_t o_prep = 0;
    all.insert(all.end(), plan.prep.begin(), plan.prep.end());
    const size_t o_gram = all.size();
    all.insert(all.end(), plan.gram.begin(), plan.gram.end());
    const size_t o_eig = all.size();
    all.insert(all.end(), plan.eig.begin(), plan.eig.end());
    const size_t o_upd = all.size();
    all.insert(all.end(), plan.upd.begin(), plan.upd.end());
    const size_t o_norms = all.size();
    all.insert(all.end(), plan.norms.begin(), plan.norms.end());
    const size_t o_pack = all.size();
    all.insert(all.end(), plan.pack.begin(), plan.pack.end());

    rc = upload(ctx, d_mats, plan.mats.data(), plan.mats.size() * sizeof(SvdMat), stream);
    if (rc != ATOMO_OK) return rc;
    rc = upload(ctx, d_work, all.data(), all.size() * sizeof(Work), stream);
    if (rc != ATOMO_OK) return rc;

    svd_prepare<<<(unsigned)plan.prep.size(), 256, 0, stream>>>(d_mats, d_work + o_prep);
    svd_norms<<<(unsigned)plan.norms.size(), 256, 0, stream>>>(d_mats, d_work + o_norms, 1);
    const int n_steps = max_sweeps * plan.max_R;
    for (int step = 0; step < n_steps; ++step) {
        svd_gram<<<(unsigned)plan.gram.size(), 256, 0, stream>>>(d_mats, d_work + o_gram, step, max_sweeps);
        svd_eig<<<(unsigned)plan.eig.size(), 256, 0, stream>>>(d_mats, d_work + o_eig, step, max_sweeps, stop_cosine,
                                                               ctx->d_flags);
        svd_update<<<(unsigned)plan.upd.size(), 256, 0, stream>>>(d_mats, d_work + o_upd, step, max_sweeps);
    }
    svd_norms<<<(unsigned)plan.norms.size(), 256, 0, stream>>>(d_mats, d_work + o_norms, 0);
    svd_select<<<(unsigned)n_mats, 256, 0, stream>>>(d_mats, s, (unsigned long long)seed, ctx->d_flags);
    svd_pack<<<(unsigned)plan.pack.size(), 256, 0, stream>>>(d_mats, d_work + o_pack);
    ATOMO_HIP(ctx, hipGetLastError());
    return ATOMO_OK;
}

}  // namespace atomo
