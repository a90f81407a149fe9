// Spectral-ATOMO encoder (Section 5 of arXiv 1806.04090): batched blocked one-sided Jacobi SVD on
// fp32 MFMA, followed by Algorithm 1 on the singular values, Philox Bernoulli sampling and packing
// of the kept singular triplets.
//
// Layout.  For a matrix G (rows x cols) let r = min(rows, cols) and M = max(rows, cols).  The r
// vectors of length M that get orthogonalised (the rows of G, or of G^T when rows > cols) are the
// rows of a workspace matrix W = [A | T]: A (r x M) starts as those vectors (times a power of two
// that brings the largest entry into [1, 2)), T (r x r) starts as the identity.  Every rotation is
// applied to whole rows of W, so at all times  A = T * A0  with T orthogonal, and on convergence row
// i of A is sigma_i times one singular vector and row i of T is the matching singular vector of the
// other side.  Rows are padded to blocks of 32 (plus one extra zero block if the number of blocks is
// odd); columns of A and T are padded to multiples of 64 with zeros: no edge handling in the kernels.
//
// One Jacobi "tick" visits, for every matrix of the call at once, one round of a round-robin
// tournament over its row blocks.  A sweep is R = (#blocks - 1) rounds.
//
// Small matrices (fewer than 16 row blocks) iterate in data space, in two groups (eight blocks and more; fewer) on two
// forked streams of the context; per tick and group, two launches:
//     svd_eig     : per block pair (64 rows), sums the partial Gram matrices of the pair and diagonalises the
//                   sum (see svd_eig.hip)
//     svd_rowgram : per 64-column chunk of W, rows <- Q^T rows for every pair, then the partial Gram matrices
//                   of the pairs of the next tick from the rows it still holds in LDS              (MFMA)
// and stop after the first sweep in which no pair of rows had |cos| above the threshold.
//
// Large matrices iterate in Gram space: the rotations of a pair depend on the rows only through
// their Gram matrix, so the r x r matrix C = A A^T is formed once (svd_fullgram, MFMA), the sweeps
// rotate C two-sidedly and accumulate the rotations in Tgs, and only when a sweep finds C diagonal to
// the threshold are the accumulated rotations applied to the data as one contraction W <- Tgs * W
// (svd_apply, MFMA).  fp32 rounding makes C drift from the true Gram matrix of the rotated rows, so
// after every application C is formed afresh from the data (svd_fullgram again); the matrix is
// finished when that fresh C is diagonal to the threshold, otherwise the sweeps continue
// from it.  The O(M r^2) work thus happens in two or three large contractions instead of in every
// round.  A Gram-space tick is one launch of svd_eig: the pair problems of the tick, and as extra
// workgroups the two-sided update C <- D^T C D, Tgs <- D^T Tgs of the previous tick (twosided_tile in
// svd_common.h; D = the block rotations of that round).  C alternates between two buffers by tick
// parity and every pair problem brings its own 64x64 block up to date (svd_eig.hip, step 1).
// Which blocks form the pairs of a Gram-space tick is read from a table that a further workgroup of the
// launch before has written: the heaviest off-diagonal blocks first (GS_WINDOW in svd_common.h), or the
// rounds of the fixed tournament.
// A call with many Gram-space matrices (SPLIT_TWO_SIDED) runs the update as a kernel of its own in front of
// the pair problems instead (svd_twosided_strip): C is then updated in place and is never behind.
#include <cfloat>
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "svd_common.h"

namespace atomo {

namespace {

using namespace svd;

__device__ inline bool refreshing(const SvdMat& m)
{
    return m.gs && m.state[ST_DONE_AT] == 0 && m.state[ST_MODE] == MODE_NEED_REFRESH;
}

// data-space matrix whose last sweep asked for the check of its whole Gram matrix (DS_VERIFY)
__device__ inline bool verifying(const SvdMat& m)
{
    return !m.gs && m.state[ST_DONE_AT] == 0 && m.state[ST_VERIFY] == 1;
}

// ------------------------------------------------------------------------------------------------
// reset / absmax / prepare
// ------------------------------------------------------------------------------------------------
// Gram-space matrices: the pairing of the first ticks is that of the fixed tournament (no block weights exist yet).
__device__ inline void first_pairs(const SvdMat& m)
{
    for (int e = threadIdx.x; e < 3 * m.npairs; e += 256) {
        const int t = e / m.npairs, k = e - t * m.npairs;
        int bi, bj;
        pair_blocks(m.nb2, t % m.R, k, bi, bj);
        m.sched[(size_t)e * 2] = bi;
        m.sched[(size_t)e * 2 + 1] = bj;
        m.where[(size_t)t * m.nb2 + bi] = 2 * k;
        m.where[(size_t)t * m.nb2 + bj] = 2 * k + 1;
        // where the two blocks sat in the round before (tick 0 has none: its pair problems read C as it is)
        const int before = (t + m.R - 1) % m.R;
        const int ki = pair_of_block(m.nb2, before, bi), kj = pair_of_block(m.nb2, before, bj);
        int xi0, xi1, xj0, xj1;
        pair_blocks(m.nb2, before, ki, xi0, xi1);
        pair_blocks(m.nb2, before, kj, xj0, xj1);
        write_pair_desc(m, t, k, bi, bj, 2 * ki + (bi == xi1), xi0, xi1, 2 * kj + (bj == xj1), xj0, xj1);
    }
}

// The state words of every matrix (workgroups below `reset_wgs`) and, in the same launch, the first pairings of the
// Gram-space matrices (one workgroup each behind them; they touch no state word).
__global__ __launch_bounds__(256) void svd_reset(const SvdMat* mats, int n_mats, int reset_wgs, const Work* gs_list)
{
    if ((int)blockIdx.x >= reset_wgs) {
        first_pairs(mats[gs_list[blockIdx.x - reset_wgs].mat]);
        return;
    }
    const int t = blockIdx.x * 256 + threadIdx.x;
    const int j = t / ST_WORDS, w = t % ST_WORDS;
    if (j < n_mats) mats[j].state[w] = (w == ST_FIRST) ? 1 : (w == ST_DMIN) ? 0x7f800000 : 0;
}

__global__ __launch_bounds__(256) void svd_absmax(const SvdMat* mats, const Work* work)
{
    __shared__ float red[4];
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    const int row0 = wk.a * BS;
    const int c = wk.b * 256 + threadIdx.x;
    float mx = 0.0f;
    if (c < m.M) {
        // all loads of the column piece in flight at once: one at a time, the pass is a chain of memory latencies
        float v[BS];
        const long long by_row = m.transposed ? 1 : m.ldg, by_col = m.transposed ? m.ldg : 1;
        const float* g = m.G + c * by_col;
#pragma unroll
        for (int k = 0; k < BS; ++k) v[k] = g[min(row0 + k, m.r - 1) * by_row];    // (a row read twice changes no maximum)
#pragma unroll
        for (int k = 0; k < BS; ++k) mx = fmaxf(mx, fabsf(v[k]));
    }
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_down(mx, o));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        if (mx > 0.0f && mx <= FLT_MAX) atomicMax((unsigned int*)&m.state[ST_ABSMAX], __float_as_uint(mx));
    }
}

__global__ __launch_bounds__(256) void svd_prepare(const SvdMat* mats, const Work* work)
{
    __shared__ float part[4][BS];
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    const int row0 = wk.a * BS;
    const int c = wk.b * 256 + threadIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int e = scale_exponent(m);
    if (wk.a == 0 && wk.b == 0 && threadIdx.x == 0) m.state[ST_EXP] = e;
    const float factor = ldexpf(1.0f, -e);
    // the scaled copy, and on the way the squared norm of every row's piece of 256 columns (summed over the lanes in
    // a fixed order): svd_scale adds the pieces up, so the copy is not read again for the scale of the matrix
    for (int i = row0; i < row0 + BS; ++i) {
        float v = 0.0f, sq = 0.0f;
        if (i < m.r && c < m.ldw) {
            if (c < m.M) {
                v = factor * (m.transposed ? m.G[(long long)c * m.ldg + i] : m.G[(long long)i * m.ldg + c]);
                sq = v * v;
            } else if (c - m.Mp == i) {
                v = 1.0f;
            }
        }
        if (c < m.ldw) m.W0[(size_t)i * m.ldw + c] = v;
        for (int o = 32; o > 0; o >>= 1) sq += __shfl_down(sq, o);
        if (lane == 0) part[wave][i - row0] = sq;
    }
    __syncthreads();
    if (threadIdx.x < BS)
        m.rowsq[(size_t)(row0 + threadIdx.x) * ((m.ldw + 255) / 256) + wk.b] =
            ((part[0][threadIdx.x] + part[1][threadIdx.x]) + part[2][threadIdx.x]) + part[3][threadIdx.x];
}

// The scale of every matrix before the first sweep: its largest squared row norm, from the pieces that svd_prepare
// left.  One workgroup per matrix.
__global__ __launch_bounds__(256) void svd_scale(const SvdMat* mats)
{
    __shared__ float red[4];
    const SvdMat m = mats[blockIdx.x];
    if (m.thin) return;
    const int pieces = (m.ldw + 255) / 256;
    float mx = 0.0f;
    for (int row = threadIdx.x; row < m.rows_alloc; row += 256) {
        float sum = 0.0f;
        for (int p = 0; p < pieces; ++p) sum += m.rowsq[(size_t)row * pieces + p];
        mx = fmaxf(mx, sum);
    }
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_down(mx, o));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        m.state[ST_SCALE] = __float_as_int(mx);
        m.state[ST_SCALE_NEXT] = __float_as_int(mx);
    }
}

// ------------------------------------------------------------------------------------------------
// fullgram: partial sums, over one column chunk, of tile (ti, tj), ti <= tj, of the Gram matrix of all rows
// (Gram-space matrices at a refresh, data-space matrices at the check of DS_VERIFY)
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void svd_fullgram(const SvdMat* mats, const Work* work)
{
    __shared__ float tile[2 * PR][68];
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    if (!refreshing(m) && !verifying(m)) return;
    const int cur = m.state[ST_CUR] & 1;
    const float* const w0 = m.W0;
    const float* const w1 = m.W1;
    // what svd_apply has just written; a data-space matrix has the one buffer
    const float* W = (m.gs && (m.state[ST_FIRST] ? cur : cur ^ 1) != 0) ? w1 : w0;
    const int ti = wk.a, tj = wk.b, nt = m.nb2 / 2, chunk = wk.c;
    const int rowA0 = ti * PR, rowB0 = tj * PR;
    const int out_index = ti * nt - ti * (ti - 1) / 2 + (tj - ti);
    const bool same = ti == tj;
    const int c_begin = chunk * KCG;
    const int c_end = min(m.Mp, c_begin + KCG);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int qi = wave >> 1, qj = wave & 1;
    const int h = lane >> 5, l32 = lane & 31;
    // loader mapping: 16 threads per row (float4 each), 16 rows per pass
    const int lrow = tid >> 4, lc4 = (tid & 15) * 4;
    const int boff = same ? 0 : PR;                              // where the B rows sit in the tile

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    // (native vector type: an array of the float4 class ended up in scratch memory here)
    floatx4 ld[8];
    auto fetch = [&](int c0) {
#pragma unroll
        for (int p = 0; p < 4; ++p)
            ld[p] = *(const floatx4*)(W + (size_t)(rowA0 + lrow + 16 * p) * m.ldw + c0 + lc4);
        if (!same) {
#pragma unroll
            for (int p = 0; p < 4; ++p)
                ld[4 + p] = *(const floatx4*)(W + (size_t)(rowB0 + lrow + 16 * p) * m.ldw + c0 + lc4);
        }
    };
    if (c_begin < c_end) fetch(c_begin);
    for (int c0 = c_begin; c0 < c_end; c0 += 64) {
        __syncthreads();                                         // previous tile fully consumed
#pragma unroll
        for (int p = 0; p < 4; ++p) *(floatx4*)&tile[lrow + 16 * p][lc4] = ld[p];
        if (!same) {
#pragma unroll
            for (int p = 0; p < 4; ++p) *(floatx4*)&tile[PR + lrow + 16 * p][lc4] = ld[4 + p];
        }
        __syncthreads();
        if (c0 + 64 < c_end) fetch(c0 + 64);                     // the next tile's loads overlap this tile's products
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const float4 a = *(const float4*)&tile[qi * BS + l32][h * 32 + 4 * s];
            const float4 b = *(const float4*)&tile[boff + qj * BS + l32][h * 32 + 4 * s];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
        }
    }
    float* out = m.gramf + ((size_t)out_index * m.nchg + chunk) * QSZ;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int i = qi * BS + 8 * (v >> 2) + 4 * h + (v & 3);
        out[i * PR + qj * BS + l32] = acc[v];
    }
}

// Sums the partial tiles of the full Gram matrix into C (both triangles), resets Tgs to I, and takes the largest
// |cos| between two rows of the tile from the sums it has just formed (the diagonal entries that the cosines need
// belong to the two diagonal tiles: every workgroup sums those 2 x 64 entries itself, in the order in which their
// own workgroups do).  The last tile of a matrix to finish decides whether the matrix is done or sweeps on.
__global__ __launch_bounds__(256) void svd_fullgram_reduce(const SvdMat* mats, const Work* work, int tick, int max_sweeps,
                                                           float stop_cosine, float fresh_stop, int* flags)
{
    __shared__ float t[PR][PR + 1];
    __shared__ float diag[2][PR];
    __shared__ float red[12];
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    if (!refreshing(m)) return;
    const int ti = wk.a, tj = wk.b, nt = m.nb2 / 2;
    auto tile_of = [&](int a, int b) { return a * nt - a * (a - 1) / 2 + (b - a); };
    const float* g = m.gramf + (size_t)tile_of(ti, tj) * m.nchg * QSZ;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // sixteen independent sums per thread, chunk after chunk in a fixed order: sixteen loads in flight
    float sums[QSZ / 256];
#pragma unroll
    for (int p = 0; p < QSZ / 256; ++p) sums[p] = 0.0f;
    float dsum = 0.0f;
    const int dt = tid < PR ? ti : tj, de = (tid & (PR - 1)) * (PR + 1);
    const float* gd = m.gramf + (size_t)tile_of(dt, dt) * m.nchg * QSZ + de;
    for (int c = 0; c < m.nchg; ++c) {
#pragma unroll
        for (int p = 0; p < QSZ / 256; ++p) sums[p] += g[(size_t)c * QSZ + tid + 256 * p];
        if (tid < 2 * PR) dsum += gd[(size_t)c * QSZ];
    }
#pragma unroll
    for (int p = 0; p < QSZ / 256; ++p) {
        const int e = tid + 256 * p;
        t[e >> 6][e & 63] = sums[p];
    }
    if (tid < 2 * PR) diag[tid >> 6][tid & (PR - 1)] = dsum;
    __syncthreads();
    const int Rp = m.rows_alloc;
    float* C = c_of_parity(m, tick);                             // the C that this tick's svd_eig reads
    const bool first = m.state[ST_FIRST] != 0;
    const float z2 = ZERO_REL * __int_as_float(m.state[ST_SCALE]);
    float mx = 0.0f, dmax = 0.0f, dmin = __int_as_float(0x7f800000);
    for (int e = tid; e < QSZ; e += 256) {
        const int i = e >> 6, j = e & 63;
        const float v = ti == tj ? 0.5f * (t[i][j] + t[j][i]) : t[i][j];
        C[(size_t)(ti * PR + i) * m.ldc + tj * PR + j] = v;
        if (ti == tj && i == j) {
            m.cref[ti * PR + i] = v;                             // the row's squared norm, measured on the data
            if (first) m.cref0[ti * PR + i] = v;
        }
        m.CT[(size_t)(ti * PR + i) * m.ldc + Rp + tj * PR + j] = (ti == tj && i == j) ? 1.0f : 0.0f;
        if (ti != tj) {                                          // mirrored tile: row index runs over j
            C[(size_t)(tj * PR + i) * m.ldc + ti * PR + j] = t[j][i];
            m.CT[(size_t)(tj * PR + i) * m.ldc + Rp + ti * PR + j] = 0.0f;
        }
        // the check, on the upper triangle of the whole matrix
        const int gi = ti * PR + i, gj = tj * PR + j;
        if (gi < gj) {
            const float dii = diag[0][i], djj = diag[1][j];
            if (dii > 0.0f && djj > 0.0f) mx = fmaxf(mx, fabsf(v) / fmaxf(sqrtf(dii * djj), z2));
        } else if (gi == gj) {
            dmax = fmaxf(dmax, v);
            if (v > z2) dmin = fminf(dmin, v);
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        mx = fmaxf(mx, __shfl_down(mx, o));
        dmax = fmaxf(dmax, __shfl_down(dmax, o));
        dmin = fminf(dmin, __shfl_down(dmin, o));
    }
    if (lane == 0) { red[wave] = mx; red[4 + wave] = dmax; red[8 + wave] = dmin; }
    __syncthreads();
    if (tid != 0) return;
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    dmax = fmaxf(fmaxf(red[4], red[5]), fmaxf(red[6], red[7]));
    dmin = fminf(fminf(red[8], red[9]), fminf(red[10], red[11]));
    atomicMax((unsigned int*)&m.state[ST_FRESH], __float_as_uint(mx));
    atomicMax((unsigned int*)&m.state[ST_SCALE_NEXT], __float_as_uint(dmax));
    atomicMin((unsigned int*)&m.state[ST_DMIN], __float_as_uint(dmin));
    __threadfence();
    const int arrived = atomicAdd(&m.state[ST_ARRIVE2], 1);
    if (arrived != m.ntiles - 1) return;
    __threadfence();
    const float fresh = __uint_as_float(atomicAdd((unsigned int*)&m.state[ST_FRESH], 0u));
    const int sweeps = m.state[ST_SWEEPS];
    if (!m.state[ST_FIRST]) m.state[ST_CUR] = (m.state[ST_CUR] & 1) ^ 1;     // svd_apply wrote the other buffer
    m.state[ST_FIRST] = 0;
    m.state[ST_REFRESHES] += 1;
    if (fresh < fresh_stop || sweeps >= max_sweeps) {
        m.state[ST_MODE] = MODE_DONE;
        m.state[ST_DONE_AT] = tick + 1;
        if (!(fresh < stop_cosine)) atomicMax(&flags[FLAG_NOCONV], 1);
    } else {
        m.state[ST_MODE] = MODE_SWEEPS;
        m.state[ST_FRESH_AT] = tick + 1;
    }
    m.state[ST_FRESH] = 0;
    m.state[ST_ARRIVE2] = 0;
    m.state[ST_OFFMAX] = 0;
    const unsigned int grown = atomicAdd((unsigned int*)&m.state[ST_SCALE_NEXT], 0u);
    if (grown > (unsigned int)m.state[ST_SCALE]) m.state[ST_SCALE] = (int)grown;
    // how far apart the rows are, for the resolution of the sweeps that follow (GS_NOISE)
    const float lo = __uint_as_float(atomicAdd((unsigned int*)&m.state[ST_DMIN], 0u));
    const float hi = __uint_as_float(grown);
    const float noise = (lo > 0.0f && lo <= hi) ? fminf(GS_NOISE * sqrtf(hi / lo), GS_NOISE_CAP) : 0.0f;
    m.state[ST_NOISE] = __float_as_int(noise);
    m.state[ST_DMIN] = 0x7f800000;
}

// Data-space matrices (DS_VERIFY): largest |cos| between any two rows from the partial tiles that svd_fullgram has
// just formed; the last tile to finish decides whether the matrix is done.  One workgroup per 64x64 tile.
__global__ __launch_bounds__(256) void svd_ds_verify(const SvdMat* mats, const Work* work, int tick, int max_sweeps,
                                                     float stop_cosine, int* flags)
{
    __shared__ float dI[PR], dJ[PR], red[4];
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    if (!verifying(m)) return;
    const int ti = wk.a, tj = wk.b, nt = m.nb2 / 2;
    auto tile_of = [&](int a, int b) { return a * nt - a * (a - 1) / 2 + (b - a); };
    const float* gt = m.gramf + (size_t)tile_of(ti, tj) * m.nchg * QSZ;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < 2 * PR) {                                          // squared norms of the tile's rows and columns
        const int k = tid & (PR - 1), t = tid < PR ? ti : tj;
        const float* gd = m.gramf + (size_t)tile_of(t, t) * m.nchg * QSZ + k * PR + k;
        float sum = 0.0f;
        for (int c = 0; c < m.nchg; ++c) sum += gd[(size_t)c * QSZ];
        (tid < PR ? dI : dJ)[k] = sum;
    }
    __syncthreads();
    const float z2 = ZERO_REL * __int_as_float(m.state[ST_SCALE]);
    float mx = 0.0f;
    for (int e = tid; e < QSZ; e += 256) {
        const int i = e >> 6, j = e & 63;
        if (ti == tj && i >= j) continue;
        float sum = 0.0f;
        for (int c = 0; c < m.nchg; ++c) sum += gt[(size_t)c * QSZ + e];
        const float dii = dI[i], djj = dJ[j];
        if (dii > 0.0f && djj > 0.0f) mx = fmaxf(mx, fabsf(sum) / fmaxf(sqrtf(dii * djj), z2));
    }
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_down(mx, o));
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    if (tid != 0) return;
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    atomicMax((unsigned int*)&m.state[ST_FRESH], __float_as_uint(mx));
    __threadfence();
    const int arrived = atomicAdd(&m.state[ST_ARRIVE2], 1);
    if (arrived != m.ntiles - 1) return;
    __threadfence();
    const float fresh = __uint_as_float(atomicAdd((unsigned int*)&m.state[ST_FRESH], 0u));
    m.state[ST_REFRESHES] += 1;
    if (fresh < stop_cosine) m.state[ST_DONE_AT] = tick;         // this tick's launches already skip the matrix
    else if (m.state[ST_SWEEPS] >= max_sweeps) atomicMax(&flags[FLAG_NOCONV], 1);
    m.state[ST_VERIFY] = 0;
    m.state[ST_FRESH] = 0;
    m.state[ST_ARRIVE2] = 0;
}

// ------------------------------------------------------------------------------------------------
// rowgram: data-space matrices, the row update of a tick and the pair Gram matrices of the next in one pass
// over W.  A work item owns a run of 64-column chunks of W = [A | T] of one matrix, with all its rows.  Per chunk:
//   - all rows of the chunk into LDS;
//   - a wave takes a pair of the tick and replaces its 64 rows by Q^T rows, in LDS (only that wave touches
//     those rows); pairs that the pair problem left alone keep their rows;
//   - the rotated rows go back to memory;
//   - (chunks of A) a wave takes a pair of the next tick and forms the quadrants aa, ab and bb of its 64x64
//     Gram matrix over the chunk's columns from LDS; ba mirrors ab and is not written.  A work item with
//     several chunks adds them up in its own partial matrix, in chunk order.
// tick = -1: no update, the Gram matrices of tick 0.
// ------------------------------------------------------------------------------------------------
constexpr int XLD = 68;                 // row stride of the chunk in LDS (16-byte reads down a column of rows: no bank conflicts)
constexpr int ROWGRAM_MAX_PARTIALS = 48;    // partial Gram matrices per pair that svd_eig adds up, at most
constexpr size_t ROWGRAM_LDS_MAX = (size_t)GS_MIN_BLOCKS * BS * XLD * sizeof(float);   // data-space matrices have fewer blocks

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void svd_rowgram(const SvdMat* mats, const Work* work, int tick, int max_sweeps)
{
    extern __shared__ float xs[];                                // [rows_alloc][XLD]
    __shared__ int moved[GS_MIN_BLOCKS];                        // per row block: its pair was rotated in this tick
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    const bool rotate = tick >= 0 && !skip_step(m, tick, max_sweeps);
    const bool gram = wk.c >= 0 && !skip_step(m, tick + 1, max_sweeps);
    if (!rotate && !gram) return;
    // (the wave index as a scalar: addresses that depend on it are then scalar too)
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, l32 = lane & 31;
    const int lrow = tid >> 4, lc4 = (tid & 15) * 4;             // loader mapping: 16 threads per row, 16 rows per pass
    const int round = rotate ? tick % m.R : 0, next_round = (tick + 1) % m.R;
    if (tid < m.nb2) moved[tid] = rotate && !m.idle[pair_of_block(m.nb2, round, tid)];

    // (pointers read from the descriptor are generic to the compiler, and every generic load waits for the LDS
    // traffic in flight; these are known to be global memory)
    typedef __attribute__((address_space(1))) float gfloat;
    typedef __attribute__((address_space(1))) floatx4 gfloatx4;
    const gfloat* const Qg = (const gfloat*)m.Q;

    float q0[32], q1[32];
    auto load_q = [&](int k) {
        // scalar base (forced: the compiler otherwise forms a 64-bit lane address for each of the 64 loads), one
        // 32-bit lane offset
        const unsigned long long qa = (unsigned long long)(Qg + (size_t)k * QSZ);
        const gfloat* q = (const gfloat*)(((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(qa >> 32)) << 32) |
                                          (unsigned)__builtin_amdgcn_readfirstlane((int)qa));
        const unsigned at = h * PR + l32;
#pragma unroll
        for (int s = 0; s < 32; ++s) {
            q0[s] = (q + 2 * s * PR)[at];                        // (Q^T)[i][k], i in block 0
            q1[s] = (q + 2 * s * PR + BS)[at];                   //              i in block 1
        }
    };

    for (int sc = 0; sc < wk.b; ++sc) {
        const int c0 = (wk.a + sc) * 64;
        gfloat* const wcol = (gfloat*)m.W0 + (size_t)lrow * m.ldw + c0 + lc4;
        float* const xrow = xs + lrow * XLD + lc4;
        int k = wave;
        // (a loaded value is a per-lane value to the compiler: as a scalar it makes the branch and the addresses scalar)
        bool active = rotate && k < m.npairs && !__builtin_amdgcn_readfirstlane(m.idle[k]);
        if (active) load_q(k);                                   // in flight while the chunk is staged
        if (sc > 0) __syncthreads();                             // the previous chunk's products have read LDS
        // all rows of the chunk into LDS, 128 rows (8 passes of 16) at a time; rows_alloc is a multiple of 64
        int p0 = 0;
        for (; p0 + 128 <= m.rows_alloc; p0 += 128) {
            floatx4 ld[8];
#pragma unroll
            for (int p = 0; p < 8; ++p) ld[p] = *(const gfloatx4*)(wcol + (size_t)(p0 + 16 * p) * m.ldw);
#pragma unroll
            for (int p = 0; p < 8; ++p) *(floatx4*)(xrow + (p0 + 16 * p) * XLD) = ld[p];
        }
        if (p0 < m.rows_alloc) {
            floatx4 ld[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) ld[p] = *(const gfloatx4*)(wcol + (size_t)(p0 + 16 * p) * m.ldw);
#pragma unroll
            for (int p = 0; p < 4; ++p) *(floatx4*)(xrow + (p0 + 16 * p) * XLD) = ld[p];
        }
        __syncthreads();

        if (rotate) {
            while (true) {
                if (active) {
                    int bi, bj;
                    pair_blocks(m.nb2, round, k, bi, bj);
                    float* const xi = xs + bi * BS * XLD + l32;
                    float* const xj = xs + bj * BS * XLD + l32;
                    floatx16 acc[2][2];                          // [column half][row block]
#pragma unroll
                    for (int e = 0; e < 2; ++e)
#pragma unroll
                        for (int ib = 0; ib < 2; ++ib)
#pragma unroll
                            for (int v = 0; v < 16; ++v) acc[e][ib][v] = 0.0f;
#pragma unroll
                    for (int s = 0; s < 32; ++s) {
                        const float* xr = s < 16 ? xi + (2 * s + h) * XLD : xj + (2 * s + h - BS) * XLD;
                        const float xa = xr[0], xb = xr[32];
                        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(q0[s], xa, acc[0][0], 0, 0, 0);
                        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(q0[s], xb, acc[1][0], 0, 0, 0);
                        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(q1[s], xa, acc[0][1], 0, 0, 0);
                        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(q1[s], xb, acc[1][1], 0, 0, 0);
                    }
#pragma unroll
                    for (int ib = 0; ib < 2; ++ib) {
                        float* const xo = ib == 0 ? xi : xj;
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int i = 8 * (v >> 2) + 4 * h + (v & 3);
                            xo[i * XLD] = acc[0][ib][v];
                            xo[i * XLD + 32] = acc[1][ib][v];
                        }
                    }
                }
                k += 4;
                if (k >= m.npairs) break;
                active = !__builtin_amdgcn_readfirstlane(m.idle[k]);
                if (active) load_q(k);
            }
            __syncthreads();
            for (int row = 0; row < m.rows_alloc; row += 16)
                if (moved[(row + lrow) >> 5]) *(gfloatx4*)(wcol + (size_t)row * m.ldw) = *(const floatx4*)(xrow + row * XLD);
        }

        if (gram) {
            for (int k = wave; k < m.npairs; k += 4) {
                int bi, bj;
                pair_blocks(m.nb2, next_round, k, bi, bj);
                const float* const pi = xs + (bi * BS + l32) * XLD + h * 32;
                const float* const pj = xs + (bj * BS + l32) * XLD + h * 32;
                floatx16 aa, ab, bb;
#pragma unroll
                for (int v = 0; v < 16; ++v) aa[v] = ab[v] = bb[v] = 0.0f;
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const float4 a = *(const float4*)(pi + 4 * s);
                    const float4 b = *(const float4*)(pj + 4 * s);
                    aa = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, a.x, aa, 0, 0, 0);
                    ab = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, ab, 0, 0, 0);
                    bb = __builtin_amdgcn_mfma_f32_32x32x2f32(b.x, b.x, bb, 0, 0, 0);
                    aa = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, a.y, aa, 0, 0, 0);
                    ab = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, ab, 0, 0, 0);
                    bb = __builtin_amdgcn_mfma_f32_32x32x2f32(b.y, b.y, bb, 0, 0, 0);
                    aa = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, a.z, aa, 0, 0, 0);
                    ab = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, ab, 0, 0, 0);
                    bb = __builtin_amdgcn_mfma_f32_32x32x2f32(b.z, b.z, bb, 0, 0, 0);
                    aa = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, a.w, aa, 0, 0, 0);
                    ab = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, ab, 0, 0, 0);
                    bb = __builtin_amdgcn_mfma_f32_32x32x2f32(b.w, b.w, bb, 0, 0, 0);
                }
                gfloat* const out = (gfloat*)m.gram + ((size_t)k * m.nchp + wk.c) * QSZ + l32;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int i = 8 * (v >> 2) + 4 * h + (v & 3);
                    gfloat* const o = out + i * PR;
                    if (sc == 0) {
                        o[0] = aa[v];
                        o[BS] = ab[v];
                        o[BS * PR + BS] = bb[v];
                    } else {                                     // (written by this same lane for the chunk before)
                        o[0] += aa[v];
                        o[BS] += ab[v];
                        o[BS * PR + BS] += bb[v];
                    }
                }
            }
        }
    }
}

// Gram-space matrices: one tile of the two-sided update per workgroup (see twosided_tile).
__global__ __launch_bounds__(256) void svd_twosided(const SvdMat* mats, const Work* work, int n_items, int tick)
{
    __shared__ float xs[PR * TLD];
    twosided_tile(mats, work, (int)blockIdx.x, n_items, tick, xs, (int)threadIdx.x);
}

// The two-sided update of a call with many Gram-space matrices (C updated in place, see SPLIT_TWO_SIDED): a
// workgroup takes up to STRIP consecutive 64x64 tiles of the 64 rows of pair a - tiles (a, b) of C for kind 1,
// column chunks of Tgs for kind 2 -, so the chain of dependent look-ups (work item, descriptor, pairing) and the
// operand Qa^T are paid once per strip, and the loads of the next tile are in flight during the products of the
// current one.  Same arithmetic, tile by tile, as twosided_tile.
constexpr int STRIP = 4;                // (2 and 8 measure within 3 % of it)

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3))) void svd_twosided_strip(const SvdMat* mats, const Work* work, int tick)
{
    __shared__ float xs[PR * TLD];                               // the tile
    __shared__ float ys[PR * TLD];                               // Qa^T * tile
    __shared__ float rs[PR];                                     // 1 / |row| of the pair's rows for the block weights
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    if (m.state[(tick & 1) ? ST_QTICK_ODD : ST_QTICK] != tick + 1) return;    // svd_eig did not rotate in this tick
    const int kind = wk.c, first = wk.b;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int qi = wave >> 1, qj = wave & 1, h = lane >> 5, l32 = lane & 31;
    const int n_all = kind == 1 ? m.npairs : m.rows_alloc / PR;
    const int count = min(STRIP, n_all - first);
    int ai, aj;
    tick_pair(m, tick, wk.a, ai, aj);
    __shared__ int cbs[2 * STRIP];                               // kind 1: the two column blocks of every tile
    if (tid < STRIP) {
        int b0 = 0, b1 = 0;
        if (kind == 1 && tid < count) tick_pair(m, tick, first + tid, b0, b1);
        cbs[2 * tid] = b0;
        cbs[2 * tid + 1] = b1;
    }
    __syncthreads();
    float* const CT = m.CT;
    // (the rotations from their transposed copies, 16 bytes of a row per load, consecutive lanes consecutive rows;
    // instruction (u, x) of a product contracts the indices 8 u + x, lanes 0..31, and 8 u + 4 + x, lanes 32..63)
    const float* qa = m.QT + ((size_t)(tick & 1) * m.npairs + wk.a) * QSZ;
    const float* dd = m.dd + (size_t)(tick & 1) * m.rows_alloc;
    auto row_of = [&](int i) { return i < BS ? ai * BS + i : aj * BS + i - BS; };
    auto col_of = [&](int t, int j) {
        return kind == 1 ? (j < BS ? cbs[2 * t] * BS + j : cbs[2 * t + 1] * BS + j - BS) : m.rows_alloc + (first + t) * PR + j;
    };
    floatx4 qa_regs[PR / 8], qb_regs[PR / 8], tile_regs[QSZ / 1024];
    // thread tid loads four entries of row tid / 16 + 16 p of the tile: rows of block ai for p < 2, of block aj from
    // there on (32-bit element offsets: a C | Tgs buffer has at most 2048 x 4096 elements)
    const int ldc = m.ldc;
    const int lrow = tid >> 4, lc4 = (tid & 15) * 4;
    const int load_lo = (ai * BS + lrow) * ldc, load_hi = (aj * BS + lrow) * ldc;
    auto fetch_tile = [&](int t) {
        const int col = col_of(t, lc4);
#pragma unroll
        for (int p = 0; p < QSZ / 1024; ++p)
            tile_regs[p] = *(const floatx4*)(CT + (p < 2 ? load_lo + 16 * p * ldc : load_hi + 16 * (p - 2) * ldc) + col);
    };
    auto fetch_qb = [&](int t) {
        const float* qb = m.QT + ((size_t)(tick & 1) * m.npairs + first + t) * QSZ;
#pragma unroll
        for (int u = 0; u < PR / 8; ++u) qb_regs[u] = *(const floatx4*)(qb + ((2 * u + h) * PR + qj * BS + l32) * 4);    // Qb[8 u + 4 h ..][j]
    };
    fetch_tile(0);
#pragma unroll
    for (int u = 0; u < PR / 8; ++u) qa_regs[u] = *(const floatx4*)(qa + ((2 * u + h) * PR + qi * BS + l32) * 4);       // (Qa^T)[i][8 u + 4 h ..]
    if (kind == 1) {
        fetch_qb(0);
        if (tid < PR) {
            const float x = dd[row_of(tid)];
            rs[tid] = x > 0.0f ? __builtin_amdgcn_rsqf(x) : 0.0f;
        }
    }
#pragma unroll 1
    for (int t = 0; t < count; ++t) {
#pragma unroll
        for (int p = 0; p < QSZ / 1024; ++p)
#pragma unroll
            for (int x = 0; x < 4; ++x) xs[(lrow + 16 * p) * TLD + lc4 + x] = tile_regs[p][x];
        __syncthreads();                                         // the tile is staged (and ys of the tile before is spent)
        if (t + 1 < count) fetch_tile(t + 1);
        floatx16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
        for (int u = 0; u < PR / 8; ++u)
#pragma unroll
            for (int x = 0; x < 4; ++x)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(qa_regs[u][x], xs[(8 * u + 4 * h + x) * TLD + qj * BS + l32], acc, 0, 0, 0);
        if (kind == 1) {
#pragma unroll
            for (int v = 0; v < 16; ++v) ys[(qi * BS + 8 * (v >> 2) + 4 * h + (v & 3)) * TLD + qj * BS + l32] = acc[v];
        }
        __syncthreads();                                         // xs is spent, ys complete
        if (kind == 1) {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
            for (int u = 0; u < PR / 8; ++u)
#pragma unroll
                for (int x = 0; x < 4; ++x)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ys[(qi * BS + l32) * TLD + 8 * u + 4 * h + x], qb_regs[u][x], acc, 0, 0, 0);
            if (t + 1 < count) fetch_qb(t + 1);
        }
        // result rows 8 (v / 4) + 4 h + (v mod 4) of block (qi ? aj : ai), column qj * 32 + l32 of the tile
        const int store0 = ((qi ? aj : ai) * BS + 4 * h) * ldc + col_of(t, qj * BS + l32);
#pragma unroll
        for (int v = 0; v < 16; ++v) CT[store0 + (8 * (v >> 2) + (v & 3)) * ldc] = acc[v];
        if (kind == 1) {
            // the weight of this block of the new C (see twosided_tile)
            const int brow = qi ? aj : ai, bcol = cbs[2 * t + qj];
            const float xc = dd[bcol * BS + l32];
            const float rcol = xc > 0.0f ? __builtin_amdgcn_rsqf(xc) : 0.0f;
            float sum = 0.0f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int li = 8 * (v >> 2) + 4 * h + (v & 3);
                const float w = acc[v] * rs[qi * BS + li] * rcol;
                if (brow != bcol || li != l32) sum = fmaf(w, w, sum);
            }
            for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
            if (lane == 0) {
                m.bw[((size_t)((tick + 1) & 1) * m.nb2 + brow) * m.nb2 + bcol] = sum;
                if (wk.a == 0 && first + t == 0 && wave == 0) m.state[ST_WSTAMP + ((tick + 1) & 1)] = tick + 2;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// apply: W[other] <- Tgs * W[cur] for a Gram-space matrix.  128 x 128 output tile per workgroup (a wave: 64 x 64, four
// 32 x 32 accumulators); both operands go through LDS in steps of 32 of the contraction index, double-buffered: the
// next step's tiles are on their way from memory while the current ones are multiplied.
// ------------------------------------------------------------------------------------------------
constexpr int AP_TILE = 128;            // output rows and columns per workgroup
constexpr int AP_K = 16;                // contraction indices per step
constexpr int AP_LDA = AP_TILE + 1;     // Tgs tile, stored [k][row]: odd stride, the 16-k segments of a row land in different banks
constexpr int AP_LDB = AP_TILE + 4;     // W tile, stored [k][column]: 16-byte stores

__global__ __launch_bounds__(256) void svd_apply(const SvdMat* mats, const Work* work)
{
    __shared__ float at[2][AP_K * AP_LDA];
    __shared__ float bt[2][AP_K * AP_LDB];
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    if (!refreshing(m) || m.state[ST_FIRST]) return;
    const int cur = m.state[ST_CUR] & 1;
    float* const w0 = m.W0;
    float* const w1 = m.W1;
    const float* src = cur ? w1 : w0;
    float* dst = cur ? w0 : w1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, l32 = lane & 31;
    const int Rp = m.rows_alloc;
    const int row0 = wk.a * AP_TILE, c0 = wk.b * AP_TILE;
    const float* T = m.CT + Rp;                                  // Tgs: columns Rp.. of [C | Tgs]
    const int wr = (wave >> 1) * 64, wc = (wave & 1) * 64;       // the wave's corner of the tile

    // staging: thread -> (row, AP_K / 2 contraction indices) of the Tgs tile and (contraction index, a run of columns) of
    // the W tile, AP_Q 16-byte pieces each
    constexpr int AP_Q = AP_K / 8;
    const int a_row = tid >> 1, a_k = (tid & 1) * (AP_K / 2);
    const int b_k = tid / (256 / AP_K), b_c = (tid % (256 / AP_K)) * (4 * AP_Q);
    const bool a_live = row0 + a_row < Rp, b_live = c0 + b_c < m.ldw;       // (rows come in multiples of 64, columns of 16)
    const float* a_src = T + (size_t)(row0 + a_row) * m.ldc + a_k;
    const float* b_src = src + (size_t)b_k * m.ldw + c0 + b_c;
    floatx4 ra[AP_Q], rb[AP_Q];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int q = 0; q < AP_Q; ++q) {
            ra[q] = a_live ? *(const floatx4*)(a_src + k0 + 4 * q) : floatx4{0.0f, 0.0f, 0.0f, 0.0f};
            rb[q] = b_live ? *(const floatx4*)(b_src + (size_t)k0 * m.ldw + 4 * q) : floatx4{0.0f, 0.0f, 0.0f, 0.0f};
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int q = 0; q < AP_Q; ++q) {
#pragma unroll
            for (int x = 0; x < 4; ++x) at[buf][(a_k + 4 * q + x) * AP_LDA + a_row] = ra[q][x];
            *(floatx4*)&bt[buf][b_k * AP_LDB + b_c + 4 * q] = rb[q];
        }
    };

    floatx16 acc[2][2];                                          // [row block][column block]
#pragma unroll
    for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ib][jb][v] = 0.0f;

    fetch(0);
    stage(0);
    __syncthreads();
    int buf = 0;
    for (int k0 = 0; k0 < Rp; k0 += AP_K) {
        const bool more = k0 + AP_K < Rp;
        if (more) fetch(k0 + AP_K);
        const float* ap = at[buf] + h * AP_LDA + wr + l32;
        const float* bp = bt[buf] + h * AP_LDB + wc + l32;
#pragma unroll
        for (int s = 0; s < AP_K / 2; ++s) {
            const float a0 = ap[2 * s * AP_LDA], a1 = ap[2 * s * AP_LDA + BS];
            const float b0 = bp[2 * s * AP_LDB], b1 = bp[2 * s * AP_LDB + BS];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
        if (more) stage(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }
#pragma unroll
    for (int ib = 0; ib < 2; ++ib)
#pragma unroll
        for (int jb = 0; jb < 2; ++jb) {
            const int col = c0 + wc + jb * BS + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + wr + ib * BS + 8 * (v >> 2) + 4 * h + (v & 3);
                if (row < Rp && col < m.ldw) dst[(size_t)row * m.ldw + col] = acc[ib][jb][v];
            }
        }
}

// ------------------------------------------------------------------------------------------------
// finalise: singular values, Algorithm 1, Bernoulli draws, message
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void svd_norms(const SvdMat* mats, const Work* work)
{
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = wk.a * 4 + wave;
    if (row >= m.rows_alloc) return;
    // a Gram-space matrix ends on a refresh, whose Gram matrix has the squared norms of the final rows on its
    // diagonal (cref): svd_select takes its singular values from there
    if (m.gs) return;
    const float* a = current_w(m) + (size_t)row * m.ldw;
    float sum = 0.0f;
    // eight loads in flight per lane, added in the order of the columns
    for (int c0 = lane * 4; c0 < m.Mp; c0 += 8 * 256) {
        float4 x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int c = c0 + 256 * u;
            x[u] = c < m.Mp ? *(const float4*)(a + c) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (c0 + 256 * u < m.Mp) sum += x[u].x * x[u].x + x[u].y * x[u].y + x[u].z * x[u].z + x[u].w * x[u].w;
    }
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_down(sum, o);
    // singular values, input scaling undone
    if (lane == 0) m.sig_raw[row] = row < m.r ? ldexpf(sqrtf(sum), m.state[ST_EXP]) : 0.0f;
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
        key[i] = i < r ? (m.gs ? ldexpf(sqrtf(m.cref[i]), m.state[ST_EXP]) : m.sig_raw[i]) : -1.0f;
        src[i] = i;
    }
    __syncthreads();
    block_sort_desc(key, src, P);
    // Rows at the rounding floor of the fp32 iteration (ZERO_REL) were left as they were: what they hold is residue
    // of the updates, not atoms of the matrix.  Their singular value is reported as 0 (which is within that floor
    // of the truth), so p = 0 and they are never sampled.
    {
        const float floor = sqrtf(ZERO_REL) * key[0];
        __syncthreads();
        for (int i = tid; i < r; i += 256)
            if (key[i] <= floor) key[i] = 0.0f;
        __syncthreads();
    }
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
    const int owners = (r + per - 1) / per;                        // threads whose slice is not empty
    int pos = 0;
    for (int t = 0; t < min(tid, owners); ++t) pos += ipart[t];
    if (tid == 0) {
        m.report[0] = m.state[ST_SWEEPS];
        m.report[1] = m.state[ST_REFRESHES];
    }
    if (tid == 255) {
        const int total = pos + kept_local;
        *m.count = total;
        if (total > m.capacity) atomicMax(&flags[FLAG_CAPACITY], 1);
    }
    const float unscale = ldexpf(1.0f, -m.state[ST_EXP]);       // sigma in the units of the scaled rows of W
    for (int i = lo; i < hi; ++i) {
        const float p = alg1_probability(key[i], i, ns, s, tail_ns);
        const u32x4 rnd = philox4x32_10((unsigned long long)(i >> 2), m.stream_id, seed);
        const uint32_t word = (i & 3) == 0 ? rnd.x : (i & 3) == 1 ? rnd.y : (i & 3) == 2 ? rnd.z : rnd.w;
        if (u01(word) < p) {
            if (pos < m.capacity) {
                const float weight = key[i] / p;
                const float fold = m.w ? 1.0f : weight;         // folded message: the weight goes into U
                m.idx[pos] = i;
                if (m.w) m.w[pos] = weight;
                m.src_row[pos] = src[i];
                m.src_inv[pos] = (m.transposed ? fold : 1.0f) / (key[i] * unscale);   // U is the long side iff rows > cols
                m.src_fold[pos] = m.transposed ? 1.0f : fold;
            }
            ++pos;
        }
    }
}

// Most sweeps any Gram-space matrix and any data-space matrix of the call took, and the fewest sweeps after which a
// Gram-space matrix asked for a refresh (0: none did), into pinned host memory that the next calls read without
// waiting (atomo_svd_options.adaptive).  One workgroup.
__device__ inline void sweep_hint(const SvdMat* mats, int n_mats, int* out)
{
    __shared__ int red[3][256];
    const int never = 1 << 30;
    int gs = 0, ds = 0, ask = never;
    for (int j = threadIdx.x; j < n_mats; j += 256) {
        const SvdMat& m = mats[j];
        if (m.thin) continue;
        const int sw = m.report[0];
        if (m.gs) gs = max(gs, sw); else ds = max(ds, sw);
        if (m.gs) ask = min(ask, m.state[ST_FIRST_ASK] > 0 ? m.state[ST_FIRST_ASK] : never);
    }
    red[0][threadIdx.x] = gs;
    red[1][threadIdx.x] = ds;
    red[2][threadIdx.x] = ask;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) {
            red[0][threadIdx.x] = max(red[0][threadIdx.x], red[0][threadIdx.x + off]);
            red[1][threadIdx.x] = max(red[1][threadIdx.x], red[1][threadIdx.x + off]);
            red[2][threadIdx.x] = min(red[2][threadIdx.x], red[2][threadIdx.x + off]);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        out[0] = red[0][0];
        out[1] = red[1][0];
        out[3] = red[2][0] == never ? 0 : red[2][0];
        out[2] = 1;
    }
}

// Copies the kept singular vectors into the message: one workgroup per (matrix, slot); with `hint_out`, one more
// behind them that writes the sweep counts for the next calls.
__global__ __launch_bounds__(256) void svd_pack(const SvdMat* mats, const Work* work, int n_pack, int n_mats, int* hint_out)
{
    if ((int)blockIdx.x >= n_pack) {
        sweep_hint(mats, n_mats, hint_out);
        return;
    }
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    const int slot = wk.a;
    const int kept = min(*m.count, m.capacity);
    if (slot >= kept) return;
    const int row = m.src_row[slot];
    const float inv = m.src_inv[slot];
    const float* a = current_w(m) + (size_t)row * m.ldw;
    float* long_out = m.transposed ? m.U + (size_t)slot * m.rows : m.V + (size_t)slot * m.cols;
    float* short_out = m.transposed ? m.V + (size_t)slot * m.cols : m.U + (size_t)slot * m.rows;
    for (int c0 = threadIdx.x; c0 < m.M; c0 += 8 * 256) {         // eight loads in flight per thread
        float x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = c0 + 256 * u < m.M ? a[c0 + 256 * u] : 0.0f;
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (c0 + 256 * u < m.M) long_out[c0 + 256 * u] = x[u] * inv;
    }
    const float fold = m.src_fold[slot];
    for (int c = threadIdx.x; c < m.r; c += 256) short_out[c] = a[m.Mp + c] * fold;
}

struct Plan {
    std::vector<SvdMat> mats;
    std::vector<Work> prep, fullgram, tiles, apply, eig_gs, twosided, strips, pack;
    // the data-space matrices in two groups that iterate side by side: [0] those of DS_VERIFY_MIN_R ticks per sweep
    // and more, [1] the smaller ones (few pairs, many rounds that rotate all index pairs, done after few ticks)
    std::vector<Work> rowgram[2], eig_ds[2];
    std::vector<Work> norms[2];                    // four rows of a data-space matrix per item: the final row norms
    std::vector<Work> ds_full, ds_tiles;           // data-space matrices that check their whole Gram matrix (DS_VERIFY)
    std::vector<int> ds_periods;                   // their distinct R
    std::vector<Work> thin_chunks, thin_list;      // thin matrices: (matrix, chunk of positions); (matrix)
    std::vector<Work> thin_direct, thin_copied;    // the chunks again, split by whether G is used in place
    std::vector<Work> gs_list;                     // the Gram-space matrices
    std::vector<int> gs_periods;     // distinct R of the Gram-space matrices
    int max_R = 1;
    int max_R_ds[2] = {1, 1};        // largest R in each group of data-space matrices
    size_t rowgram_lds[2] = {0, 0};  // LDS bytes of a svd_rowgram workgroup: all rows of the group's tallest matrix
    bool own_update = false;         // the two-sided update runs as launches of its own (see SPLIT_TWO_SIDED)
    size_t bytes = 0;
    SvdMat* d_mats = nullptr;        // device copies of `mats` and of the concatenated work lists
    Work* d_work = nullptr;
    size_t n_work() const
    {
        return prep.size() + rowgram[0].size() + rowgram[1].size() + fullgram.size() + tiles.size() + apply.size() +
               eig_gs.size() + eig_ds[0].size() + eig_ds[1].size() +
               twosided.size() + strips.size() + ds_full.size() + ds_tiles.size() + norms[0].size() + norms[1].size() + pack.size() + 2 * thin_chunks.size() + thin_list.size() +
               gs_list.size();
    }
};

// With more update tiles per tick than this (a 512-row matrix has 128: 33 or more such matrices) the two-sided update
// is the bulk of a tick and runs as a kernel of its own, in front of the pair problems of the next tick instead of
// beside them.  C is then up to date whenever a pair problem reads it, so it is updated in place (one buffer instead
// of two alternating ones, which a batch of that size no longer finds in the last-level cache) and the pair problems
// read their block as it is instead of bringing it up to date themselves.
constexpr size_t SPLIT_TWO_SIDED = 4096;

// Lays the workspace out (base == nullptr: sizes only).
void build_plan(const atomo_mat* mats, int n_mats, const atomo_svd_msg* msgs, float* sigma_out, float* p_out,
                uint64_t stream_base, const uint64_t* stream_ids, void* base, Plan& plan)
{
    Carver carve(base);
    plan.mats.resize(n_mats);
    plan.d_mats = carve.take<SvdMat>(n_mats);
    size_t atom_off = 0;
    size_t update_tiles = 0;
    for (int j = 0; j < n_mats; ++j) {
        const int r = mats[j].rows < mats[j].cols ? mats[j].rows : mats[j].cols;
        const int nb = (r + BS - 1) / BS, nb2 = nb + (nb & 1);
        if (r > THIN_R && nb2 >= GS_MIN_BLOCKS) update_tiles += (size_t)(nb2 / 2) * (nb2 / 2 + nb2 * BS / PR);
    }
    plan.own_update = update_tiles > SPLIT_TWO_SIDED;
    const bool gs_chain = update_tiles > 0 && !plan.own_update;    // Gram-space matrices, one launch per tick
    for (int j = 0; j < n_mats; ++j) {
        SvdMat& m = plan.mats[j];
        const atomo_mat& a = mats[j];
        m.rows = a.rows; m.cols = a.cols;
        m.transposed = a.rows > a.cols;
        m.r = m.transposed ? a.cols : a.rows;
        m.M = m.transposed ? a.rows : a.cols;
        m.thin = m.r <= THIN_R;
        m.stream_id = stream_ids ? stream_ids[j] : stream_base + (uint64_t)j;
        m.G = a.data; m.ldg = a.ld;
        if (msgs) {
            const atomo_svd_msg& g = msgs[j];
            m.count = g.count; m.idx = g.idx; m.w = g.w; m.U = g.U; m.V = g.V;
            m.capacity = g.capacity < m.r ? g.capacity : m.r;
        } else {
            m.count = nullptr; m.idx = nullptr; m.w = nullptr; m.U = nullptr; m.V = nullptr; m.capacity = 1;
        }
        m.sigma_out = sigma_out ? sigma_out + atom_off : nullptr;
        m.p_out = p_out ? p_out + atom_off : nullptr;
        atom_off += m.r;
        if (m.thin) {
            // chunks of 1024 positions, larger only to keep a matrix under 128 chunks
            const int64_t per = ((int64_t)m.M + 128 * 1024 - 1) / (128 * 1024);
            m.tchunk = m.M <= 1024 ? (int)align_up(m.M, 256) : (int)(1024 * per);
            m.nchg = (m.M + m.tchunk - 1) / m.tchunk;
            m.Mp = m.M; m.ldw = 0; m.nb2 = 0; m.rows_alloc = THIN_R; m.R = 1; m.npairs = 0; m.nchu = 0; m.gs = 0;
            m.ntiles = 0; m.ldc = 0;
            m.W0 = nullptr; m.W1 = nullptr; m.CT = nullptr; m.CT2 = nullptr; m.cref = nullptr; m.cref0 = nullptr; m.rowsq = nullptr;
            m.sched = nullptr; m.where = nullptr; m.bw = nullptr; m.dd = nullptr; m.idle = nullptr;
            m.gram = carve.take<float>((size_t)m.nchg * THIN_R * THIN_R);
            m.Q = carve.take<float>(2 * THIN_R * THIN_R);
            m.B = carve.take<float>((size_t)m.M * m.r);
            m.state = carve.take<int>(ST_WORDS);
            m.sig_raw = carve.take<float>(THIN_R);
            m.src_row = carve.take<int>(m.capacity);
            m.src_inv = carve.take<float>(m.capacity);
            m.src_fold = carve.take<float>(m.capacity);
            const bool direct = m.transposed && m.ldg == m.r;
            m.X = direct ? m.G : m.B;
            for (int c = 0; c < m.nchg; ++c) {
                plan.thin_chunks.push_back(Work{j, c, 0, 0});
                (direct ? plan.thin_direct : plan.thin_copied).push_back(Work{j, c, 0, 0});
            }
            plan.thin_list.push_back(Work{j, 0, 0, 0});
            continue;
        }
        m.tchunk = 0; m.B = nullptr; m.X = nullptr;
        m.Mp = (int)align_up(m.M, 64);
        m.ldw = m.Mp + (int)align_up(m.r, 64);
        const int nb = (m.r + BS - 1) / BS;
        m.nb2 = nb + (nb & 1);
        m.rows_alloc = m.nb2 * BS;
        m.R = m.nb2 - 1;
        m.npairs = m.nb2 / 2;
        m.nchg = (m.Mp + KCG - 1) / KCG;
        m.nchu = (m.ldw + KCU - 1) / KCU;
        m.gs = m.nb2 >= GS_MIN_BLOCKS;
        // data space: work items of svd_rowgram over A, of `run` 64-column chunks each, at most ROWGRAM_MAX_PARTIALS
        const int chunks_a = m.Mp / 64;
        int run = (chunks_a + ROWGRAM_MAX_PARTIALS - 1) / ROWGRAM_MAX_PARTIALS;
        // Beside Gram-space matrices, whose chain of launches sets the time of the call and whose every launch wants 160
        // free compute units at once, the small data-space matrices (done in a third of that time) take four chunks per
        // work item: a quarter of the workgroups, each four times as long (3.03 -> 2.97 ms for the ResNet-18 set; six
        // chunks 2.96, nine 3.25: their chain is then the longest).
        if (gs_chain && m.nb2 - 1 < DS_VERIFY_MIN_R) run = std::max(run, 4);
        m.nchp = m.gs ? 0 : (chunks_a + run - 1) / run;
        const int nt = m.nb2 / 2;
        m.ntiles = nt * (nt + 1) / 2;
        m.ldc = 2 * m.rows_alloc;
        m.W0 = carve.take<float>((size_t)m.rows_alloc * m.ldw);
        m.W1 = m.gs ? carve.take<float>((size_t)m.rows_alloc * m.ldw) : nullptr;
        m.CT = m.gs ? carve.take<float>((size_t)m.rows_alloc * m.ldc) : nullptr;
        // (the same buffer twice: C is updated in place, and svd_eig reads its block of C as it is)
        m.CT2 = !m.gs ? nullptr : plan.own_update ? m.CT : carve.take<float>((size_t)m.rows_alloc * m.ldc);
        const bool ds_verify = !m.gs && m.R >= DS_VERIFY_MIN_R;
        m.gram = m.gs ? nullptr : carve.take<float>((size_t)m.npairs * m.nchp * QSZ);
        m.gramf = m.gs || ds_verify ? carve.take<float>((size_t)m.ntiles * m.nchg * QSZ) : nullptr;
        m.Q = m.gs ? nullptr : carve.take<float>((size_t)m.npairs * QSZ);
        m.QT = m.gs ? carve.take<float>((size_t)2 * m.npairs * QSZ) : nullptr;
        m.DB = m.gs && !plan.own_update ? carve.take<float>((size_t)m.npairs * QSZ) : nullptr;
        m.idle = m.gs ? nullptr : carve.take<int>(m.npairs);
        m.state = carve.take<int>(ST_WORDS);
        const size_t state_off = carve.last;
        m.sig_raw = carve.take<float>(m.rows_alloc);
        m.rowsq = carve.take<float>((size_t)m.rows_alloc * ((m.ldw + 255) / 256));
        m.cref = m.gs ? carve.take<float>(m.rows_alloc) : nullptr;
        m.cref0 = m.gs ? carve.take<float>(m.rows_alloc) : nullptr;
        m.sched = m.gs ? carve.take<int>((size_t)3 * m.npairs * 2) : nullptr;
        m.pdesc = m.gs ? carve.take<int>((size_t)m.npairs * 3 * PD_WORDS) : nullptr;
        const size_t pdesc_off = carve.last;
        m.where = m.gs ? carve.take<int>((size_t)3 * m.nb2) : nullptr;
        m.bw = m.gs ? carve.take<float>((size_t)2 * m.nb2 * m.nb2) : nullptr;
        m.dd = m.gs ? carve.take<float>((size_t)2 * m.rows_alloc) : nullptr;
        m.src_row = carve.take<int>(m.capacity);
        m.src_inv = carve.take<float>(m.capacity);
        m.src_fold = carve.take<float>(m.capacity);
        if (m.R > plan.max_R) plan.max_R = m.R;
        const int grp = m.R >= DS_VERIFY_MIN_R ? 0 : 1;           // (data-space matrices)
        if (!m.gs && m.R > plan.max_R_ds[grp]) plan.max_R_ds[grp] = m.R;
        for (int b = 0; b < m.nb2; ++b)
            for (int c = 0; c < (m.ldw + 255) / 256; ++c) plan.prep.push_back(Work{j, b, c, 0});
        for (int k = 0; k < m.npairs; ++k) {
            // (offsets from the matrices' descriptors, which are the first thing in the workspace)
            if (m.gs)
                plan.eig_gs.push_back(Work{j, k, (int)(unsigned)(state_off / HOT_UNIT),
                                           (int)(unsigned)((pdesc_off + (size_t)k * 3 * PD_WORDS * sizeof(int)) / HOT_UNIT)});
            else
                plan.eig_ds[grp].push_back(Work{j, k, 0, 0});
            if (m.gs) {
                // (tiles of C, two products each, and tiles of Tgs, one product, two and two: svd_eig's update
                // workgroups take four consecutive tiles each, and the slowest of them sets when the launch ends)
                static_assert(PR == 2 * BS, "a pair's strip of C has as many tiles as its strip of Tgs");
                for (int q = 0; q < m.npairs; q += 2) {
                    for (int e = q; e < std::min(q + 2, m.npairs); ++e) plan.twosided.push_back(Work{j, k, e, 1});
                    for (int e = q; e < std::min(q + 2, m.rows_alloc / PR); ++e) plan.twosided.push_back(Work{j, k, e, 2});
                }
                if (plan.own_update) {
                    for (int k2 = 0; k2 < m.npairs; k2 += STRIP) plan.strips.push_back(Work{j, k, k2, 1});
                    for (int c = 0; c < m.rows_alloc / PR; c += STRIP) plan.strips.push_back(Work{j, k, c, 2});
                }
            }
        }
        if (!m.gs) {
            for (int c = 0; c < m.nchp; ++c) plan.rowgram[grp].push_back(Work{j, c * run, std::min(run, chunks_a - c * run), c});
            for (int c = chunks_a; c < m.ldw / 64; ++c) plan.rowgram[grp].push_back(Work{j, c, 1, -1});   // the chunks of T
            plan.rowgram_lds[grp] = std::max(plan.rowgram_lds[grp], (size_t)m.rows_alloc * XLD * sizeof(float));
        }
        if (m.gs) {
            plan.gs_list.push_back(Work{j, 0, 0, 0});
            bool seen = false;
            for (int p : plan.gs_periods) seen = seen || p == m.R;
            if (!seen) plan.gs_periods.push_back(m.R);
            for (int ti = 0; ti < nt; ++ti)
                for (int tj = ti; tj < nt; ++tj) {
                    plan.tiles.push_back(Work{j, ti, tj, 0});
                    for (int c = 0; c < m.nchg; ++c) plan.fullgram.push_back(Work{j, ti, tj, c});
                }
            for (int t = 0; t < (m.rows_alloc + AP_TILE - 1) / AP_TILE; ++t)
                for (int c = 0; c < (m.ldw + AP_TILE - 1) / AP_TILE; ++c) plan.apply.push_back(Work{j, t, c, 0});
        }
        if (ds_verify) {
            bool seen = false;
            for (int p : plan.ds_periods) seen = seen || p == m.R;
            if (!seen) plan.ds_periods.push_back(m.R);
            for (int ti = 0; ti < nt; ++ti)
                for (int tj = ti; tj < nt; ++tj) {
                    plan.ds_tiles.push_back(Work{j, ti, tj, 0});
                    for (int c = 0; c < m.nchg; ++c) plan.ds_full.push_back(Work{j, ti, tj, c});
                }
        }
        if (!m.gs)                                               // (Gram-space matrices: svd_select reads cref)
            for (int g = 0; g < m.rows_alloc / 4; ++g) plan.norms[grp].push_back(Work{j, g, 0, 0});
        for (int k = 0; k < m.capacity; ++k) plan.pack.push_back(Work{j, k, 0, 0});
    }
    deal_to_dies(plan.strips);                                   // a matrix's strips, which share its rotations, on one die
    // the work items of the tallest matrices first: they set the duration of the launch
    for (auto& list : plan.rowgram)
        std::stable_sort(list.begin(), list.end(), [&](const Work& a, const Work& b) {
            return plan.mats[a.mat].rows_alloc * (a.c >= 0 ? 2 : 1) > plan.mats[b.mat].rows_alloc * (b.c >= 0 ? 2 : 1);
        });
    plan.d_work = carve.take<Work>(plan.n_work());
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
    build_plan(mats, n_mats, nullptr, nullptr, nullptr, 0, nullptr, nullptr, plan);
    *bytes = plan.bytes;
    return ATOMO_OK;
}

int encode_svd(atomo_ctx* ctx, const atomo_mat* mats, int n_mats, double s, uint64_t seed, uint64_t stream_base,
               const atomo_svd_options* opt, const atomo_svd_msg* msgs, float* sigma_out, float* p_out,
               hipStream_t stream)
{
    const int max_sweeps = opt && opt->max_sweeps > 0 ? opt->max_sweeps : 16;
    const float stop_cosine = opt && opt->stop_cosine > 0.0f ? opt->stop_cosine : 1e-4f;
    // (defaults: one round per pair problem in Gram space, where a tick is one launch and the chain of ticks sets the
    // time of a call; on the data a second round where the first left more than a tenth of the largest cosine: those
    // matrices then need 5 - 6 sweeps instead of 8 - 10, at a third more per tick)
    const int max_inner = opt && opt->max_inner_sweeps > 0 ? opt->max_inner_sweeps : 1;
    const float inner_reduction = opt && opt->inner_reduction > 0.0f ? opt->inner_reduction : 0.01f;
    const int max_inner_ds = opt && opt->max_inner_sweeps > 0 ? opt->max_inner_sweeps : 2;
    const float inner_reduction_ds = opt && opt->inner_reduction > 0.0f ? opt->inner_reduction : 0.1f;
    const float fresh_stop = stop_cosine;
    const int full_period = opt && opt->full_period > 0 ? opt->full_period : 12;
    const int cyclic = opt && opt->block_order == 1 ? 1 : 0;
    const int adaptive = opt ? opt->adaptive : 0;

    // Sweep limits of this call.  With `adaptive`, what the most recent finished call with the same shapes needed plus
    // the margin; a call that used up a reduced limit tells nothing about what was needed and is followed by a full one.
    int limit_gs = max_sweeps, limit_ds = max_sweeps;
    // ... and the first sweep boundary at which the Gram-space matrices can get a refresh: the margin before the first
    // one that a matrix of that call asked for (0: every boundary).  The refresh launches of an idle boundary cost what
    // five empty launches cost, on the chain of launches that sets the time of the call.
    int ask_from = 0;
    SweepHint* hint = nullptr;
    if (adaptive > 0) {
        uint64_t sig = 1469598103934665603ull ^ (uint64_t)n_mats;
        for (int j = 0; j < n_mats; ++j) {
            sig = (sig ^ (uint64_t)(uint32_t)mats[j].rows) * 1099511628211ull;
            sig = (sig ^ (uint64_t)(uint32_t)mats[j].cols) * 1099511628211ull;
        }
        // The slot this call will use: with four calls in flight its last user is the oldest of them; wait for that one
        // first, so that a host that runs four calls ahead of the device still finds a finished call to learn from.
        hint = &ctx->hints[ctx->hint_next];
        ctx->hint_next = (ctx->hint_next + 1) % (int)(sizeof(ctx->hints) / sizeof(ctx->hints[0]));
        if (hint->pending) {
            ATOMO_HIP(ctx, hipEventSynchronize(hint->done));
            hint->pending = false;
        }
        const SweepHint* best = nullptr;
        for (SweepHint& h : ctx->hints) {
            if (h.seq == 0) continue;
            if (h.pending) {
                const hipError_t q = hipEventQuery(h.done);
                if (q == hipSuccess) h.pending = false;
                else (void)hipGetLastError();                    // "not ready" is an answer, not an error to keep
            }
            if (!h.pending && h.sig == sig && h.host[2] == 1 && (!best || h.seq > best->seq)) best = &h;
        }
        if (best) {
            const int g = best->host[0], d = best->host[1];
            if (!(g >= best->limit_gs && best->limit_gs < max_sweeps)) {
                limit_gs = std::min(max_sweeps, std::max(1, g + adaptive));
                ask_from = std::max(0, best->host[3] - adaptive);
            }
            if (!(d >= best->limit_ds && best->limit_ds < max_sweeps)) limit_ds = std::min(max_sweeps, std::max(1, d + adaptive));
        }
        if (!hint->host) {
            ATOMO_HIP(ctx, hipHostMalloc((void**)&hint->host, 4 * sizeof(int32_t), hipHostMallocDefault));
            ATOMO_HIP(ctx, hipHostGetDevicePointer((void**)&hint->dev, hint->host, 0));
            ATOMO_HIP(ctx, hipEventCreateWithFlags(&hint->done, hipEventDisableTiming));
        }
        hint->host[0] = hint->host[1] = hint->host[2] = hint->host[3] = 0;
        hint->sig = sig;
        hint->seq = ++ctx->hint_seq;
        hint->limit_gs = limit_gs;
        hint->limit_ds = limit_ds;
    }

    if ((size_t)n_mats > ctx->report_cap) {                      // (hipFree waits for the device)
        if (ctx->d_report) ATOMO_HIP(ctx, hipFree(ctx->d_report));
        ctx->d_report = nullptr;
        ctx->report_cap = 0;
        const size_t want = align_up((size_t)n_mats, 256);
        if (hipMalloc((void**)&ctx->d_report, want * 2 * sizeof(int32_t)) != hipSuccess) return ATOMO_ENOMEM;
        ctx->report_cap = want;
    }
    Plan sizing;
    const uint64_t* stream_ids = opt ? opt->stream_ids : nullptr;
    build_plan(mats, n_mats, msgs, sigma_out, p_out, stream_base, stream_ids, nullptr, sizing);
    if (sizing.bytes >= (HOT_UNIT << 32)) return ATOMO_EINVAL;   // (the work items address the workspace in 32 bits of 16-byte units)
    const bool tables_intact = ctx->svd_tables_intact;
    const void* const ws_before = ctx->ws;
    int rc = ensure_workspace(ctx, sizing.bytes);
    if (rc != ATOMO_OK) return rc;

    Plan plan;
    build_plan(mats, n_mats, msgs, sigma_out, p_out, stream_base, stream_ids, ctx->ws, plan);
    SvdMat* d_mats = plan.d_mats;
    for (int j = 0; j < n_mats; ++j) plan.mats[j].report = ctx->d_report + 2 * j;
    ctx->report_n = (size_t)n_mats;

    std::vector<Work> all;
    all.reserve(plan.n_work());
    auto place = [&](const std::vector<Work>& list) {
        const Work* at = plan.d_work + all.size();
        all.insert(all.end(), list.begin(), list.end());
        return at;
    };
    const Work* w_prep = place(plan.prep);
    const Work* w_rowgram[2] = {place(plan.rowgram[0]), place(plan.rowgram[1])};
    const Work* w_fullgram = place(plan.fullgram);
    const Work* w_tiles = place(plan.tiles);
    const Work* w_apply = place(plan.apply);
    const Work* w_eig_gs = place(plan.eig_gs);
    const Work* w_eig_ds[2] = {place(plan.eig_ds[0]), place(plan.eig_ds[1])};
    const Work* w_twosided = place(plan.twosided);
    const Work* w_strips = place(plan.strips);
    const Work* w_ds_full = place(plan.ds_full);
    const Work* w_ds_tiles = place(plan.ds_tiles);
    const Work* w_norms[2] = {place(plan.norms[0]), place(plan.norms[1])};
    const Work* w_pack = place(plan.pack);
    const Work* w_thin_chunks = place(plan.thin_chunks);
    const Work* w_thin_list = place(plan.thin_list);
    const Work* w_thin_direct = place(plan.thin_direct);
    const Work* w_thin_copied = place(plan.thin_copied);
    const Work* w_gs_list = place(plan.gs_list);

    // the tables go up unless the workspace still holds these very bytes (see atomo_ctx::svd_tables)
    {
        const size_t mats_bytes = plan.mats.size() * sizeof(SvdMat), work_bytes = all.size() * sizeof(Work);
        const bool same = tables_intact && ws_before == ctx->ws && ctx->svd_tables_stream == stream &&
                          ctx->svd_tables.size() == mats_bytes + work_bytes &&
                          memcmp(ctx->svd_tables.data(), plan.mats.data(), mats_bytes) == 0 &&
                          memcmp(ctx->svd_tables.data() + mats_bytes, all.data(), work_bytes) == 0;
        if (!same) {
            rc = upload(ctx, d_mats, plan.mats.data(), mats_bytes, stream);
            if (rc != ATOMO_OK) return rc;
            rc = upload(ctx, plan.d_work, all.data(), work_bytes, stream);
            if (rc != ATOMO_OK) return rc;
            ctx->svd_tables.resize(mats_bytes + work_bytes);
            memcpy(ctx->svd_tables.data(), plan.mats.data(), mats_bytes);
            memcpy(ctx->svd_tables.data() + mats_bytes, all.data(), work_bytes);
            ctx->svd_tables_stream = stream;
        }
    }

    auto grid = [](const std::vector<Work>& list) { return (unsigned)list.size(); };
    {
        ProfScope ps(ctx, ATOMO_K_SVD_PREPARE, stream);
        const int reset_wgs = (n_mats * ST_WORDS + 255) / 256;
        svd_reset<<<(unsigned)reset_wgs + grid(plan.gs_list), 256, 0, stream>>>(d_mats, n_mats, reset_wgs, w_gs_list);
        if (!plan.prep.empty()) {
            svd_absmax<<<grid(plan.prep), 256, 0, stream>>>(d_mats, w_prep);
            svd_prepare<<<grid(plan.prep), 256, 0, stream>>>(d_mats, w_prep);
            svd_scale<<<(unsigned)n_mats, 256, 0, stream>>>(d_mats);
        }
    }
    // The data-space matrices iterate on streams of their own from here to the end, the large ones on one, the small
    // ones on another (one fork, one join each): a tick lasts as long as its slowest pair problem, and the small
    // matrices have far more rounds that rotate all index pairs (every third, or every single one) than the large.
    // The Gram-space matrices iterate on the caller's stream, one launch per tick: svd_eig of tick t, which
    // carries the two-sided update of tick t-1 as extra workgroups.  That works because C alternates between
    // two buffers: the update of tick t-1 reads the C of parity t-1 and writes parity t, while svd_eig of tick
    // t forms its own 64x64 block from the C of parity t-1 and the rotations of tick t-1, which are
    // double-buffered by tick parity as well.
    // Thin matrices go in front of the small ones when there are Gram-space matrices to overlap with.
    const bool have_ds[2] = {!plan.rowgram[0].empty(), !plan.rowgram[1].empty()};
    const bool have_gs = !plan.twosided.empty(), have_thin = !plan.thin_list.empty();
    const bool use_side[2] = {have_ds[0], have_ds[1] || (have_thin && have_gs)};
    const int n_two = (int)plan.twosided.size();
    if (use_side[0] || use_side[1]) {
        rc = ensure_side_streams(ctx);
        if (rc != ATOMO_OK) return rc;
        ATOMO_HIP(ctx, hipEventRecord(ctx->ev_fork, stream));
        if (use_side[0]) ATOMO_HIP(ctx, hipStreamWaitEvent(ctx->side, ctx->ev_fork, 0));
        if (use_side[1]) ATOMO_HIP(ctx, hipStreamWaitEvent(ctx->side2, ctx->ev_fork, 0));
    }
    if (have_thin) {
        hipStream_t s_thin = have_gs ? ctx->side2 : stream;
        // a pass over the data does the work of many sweeps of the blocked iteration: one rotating pass per eight
        // sweeps of the limit, and the pass that confirms (no input tried, however graded or rank-deficient, has
        // needed more than two rotating passes)
        const int passes = std::max(2, std::min(THIN_PASSES, 1 + (max_sweeps + 7) / 8));
        ProfScope ps(ctx, ATOMO_K_SVD_THIN, s_thin);
        launch_thin_absmax(d_mats, w_thin_direct, (int)plan.thin_direct.size(), w_thin_copied, (int)plan.thin_copied.size(),
                           s_thin);
        for (int pass = 0; pass < passes; ++pass)
            launch_thin_pass(d_mats, w_thin_chunks, (int)plan.thin_chunks.size(), w_thin_list, (int)plan.thin_list.size(),
                             pass, passes - 1, stop_cosine, ctx->d_flags, s_thin);
    }
    if (have_ds[0] || have_ds[1]) {
        hipStream_t s_ds[2] = {ctx->side, ctx->side2};
        const int ds_ticks[2] = {have_ds[0] ? limit_ds * plan.max_R_ds[0] : 0, have_ds[1] ? limit_ds * plan.max_R_ds[1] : 0};
        // at a sweep boundary: the whole-Gram-matrix check of the matrices whose sweep asked for it (DS_VERIFY; they
        // are all in the first group)
        auto verify = [&](int tick) {
            bool boundary = false;
            for (int period : plan.ds_periods) boundary = boundary || (tick % period == 0 && tick <= limit_ds * period);
            if (!boundary) return;
            ProfScope ps(ctx, ATOMO_K_SVD_REFRESH, s_ds[0]);
            svd_fullgram<<<grid(plan.ds_full), 256, 0, s_ds[0]>>>(d_mats, w_ds_full);
            svd_ds_verify<<<grid(plan.ds_tiles), 256, 0, s_ds[0]>>>(d_mats, w_ds_tiles, tick, limit_ds, stop_cosine, ctx->d_flags);
        };
        // more LDS than a launch gets by default: raised once per context
        if (std::max(plan.rowgram_lds[0], plan.rowgram_lds[1]) > ctx->rowgram_lds) {
            ATOMO_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(svd_rowgram),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)ROWGRAM_LDS_MAX));
            ctx->rowgram_lds = ROWGRAM_LDS_MAX;
        }
        // (the two groups' launches are enqueued alternately, so that both streams have work from the start)
        for (int tick = -1; tick < std::max(ds_ticks[0], ds_ticks[1]); ++tick)
            for (int g = 0; g < 2; ++g) {
                if (!have_ds[g] || tick >= ds_ticks[g]) continue;
                if (tick >= 0) {
                    ProfScope ps(ctx, ATOMO_K_SVD_EIG, s_ds[g]);
                    launch_svd_eig(d_mats, w_eig_ds[g], (int)plan.eig_ds[g].size(), nullptr, 0, nullptr, 0, 0, tick, limit_ds, 0,
                                   stop_cosine, max_inner_ds, inner_reduction_ds, full_period, 0, ctx->d_flags, s_ds[g]);
                }
                {
                    // tick -1: the Gram matrices of the first tick's pairs
                    ProfScope ps(ctx, tick < 0 ? ATOMO_K_SVD_GRAM : ATOMO_K_SVD_UPDATE, s_ds[g]);
                    svd_rowgram<<<grid(plan.rowgram[g]), 256, plan.rowgram_lds[g], s_ds[g]>>>(d_mats, w_rowgram[g], tick, limit_ds);
                }
                if (g == 0 && tick >= 0) verify(tick + 1);
            }
    }
    // the singular values of the data-space matrices, at the end of their own chains
    for (int g = 0; g < 2; ++g)
        if (!plan.norms[g].empty()) {
            hipStream_t s_g = g == 0 ? ctx->side : ctx->side2;
            ProfScope ps(ctx, ATOMO_K_SVD_FINALIZE, s_g);
            svd_norms<<<grid(plan.norms[g]), 256, 0, s_g>>>(d_mats, w_norms[g]);
        }
    if (use_side[0]) ATOMO_HIP(ctx, hipEventRecord(ctx->ev_join, ctx->side));
    if (use_side[1]) ATOMO_HIP(ctx, hipEventRecord(ctx->ev_join2, ctx->side2));
    if (have_gs) {
        const int n_ticks = limit_gs * plan.max_R + 1;
        // Few matrices: the two-sided update of the previous tick rides in the launch of the pair problems (one launch
        // per tick on the chain of dependent ticks), C alternates between two buffers and is one tick behind.
        // Many matrices (SPLIT_TWO_SIDED): the update is the bulk of a tick, and as extra 1024-thread workgroups of
        // svd_eig (128 registers per lane, one or two workgroups per compute unit) it runs at a fraction of the rate of
        // its own kernel of 256-thread workgroups, which is launched in front of the pair problems.  (On a stream of
        // its own beside the pair problems of the next tick it slowed those down by more than it gained.)
        const bool own_launch = plan.own_update;
        for (int tick = 0; tick < n_ticks; ++tick) {
            // the previous tick's update for every matrix, and the pair problems of the matrices that sweep on
            if (tick > 0) {
                if (own_launch) {
                    ProfScope ps(ctx, ATOMO_K_SVD_UPDATE, stream);
                    svd_twosided_strip<<<grid(plan.strips), 256, 0, stream>>>(d_mats, w_strips, tick - 1);
                }
                {
                    ProfScope ps(ctx, ATOMO_K_SVD_EIG, stream);
                    launch_svd_eig(d_mats, w_eig_gs, (int)plan.eig_gs.size(), w_twosided, own_launch ? 0 : n_two, w_gs_list,
                                   (int)plan.gs_list.size(), cyclic, tick, limit_gs, ask_from, stop_cosine, max_inner,
                                   inner_reduction, full_period, 0, ctx->d_flags, stream);
                }
            }
            bool boundary = false;
            for (int period : plan.gs_periods)
                boundary = boundary || (tick % period == 0 && tick <= limit_gs * period && (tick == 0 || tick >= ask_from * period));
            if (boundary) {
                // a sweep boundary of some matrix: those that asked for it get a fresh Gram matrix (their Tgs is
                // complete now), and their pair problems of this tick run in a launch of their own
                {
                    ProfScope ps(ctx, ATOMO_K_SVD_REFRESH, stream);
                    if (tick > 0) svd_apply<<<grid(plan.apply), 256, 0, stream>>>(d_mats, w_apply);   // (tick 0: nothing to apply yet)
                    svd_fullgram<<<grid(plan.fullgram), 256, 0, stream>>>(d_mats, w_fullgram);
                    svd_fullgram_reduce<<<grid(plan.tiles), 256, 0, stream>>>(d_mats, w_tiles, tick, limit_gs, stop_cosine,
                                                                              fresh_stop, ctx->d_flags);
                }
                {
                    ProfScope ps(ctx, ATOMO_K_SVD_EIG, stream);
                    launch_svd_eig(d_mats, w_eig_gs, (int)plan.eig_gs.size(), nullptr, 0, nullptr, 0, 0, tick, limit_gs,
                                   ask_from, stop_cosine, max_inner, inner_reduction, full_period, 1, ctx->d_flags, stream);
                }
            }
        }
        {
            ProfScope ps(ctx, ATOMO_K_SVD_UPDATE, stream);
            if (own_launch) svd_twosided_strip<<<grid(plan.strips), 256, 0, stream>>>(d_mats, w_strips, n_ticks - 1);
            else svd_twosided<<<(unsigned)n_two, 256, 0, stream>>>(d_mats, w_twosided, n_two, n_ticks - 1);
        }
    }
    if (use_side[0]) ATOMO_HIP(ctx, hipStreamWaitEvent(stream, ctx->ev_join, 0));
    if (use_side[1]) ATOMO_HIP(ctx, hipStreamWaitEvent(stream, ctx->ev_join2, 0));
    {
        ProfScope ps(ctx, ATOMO_K_SVD_FINALIZE, stream);
        svd_select<<<(unsigned)n_mats, 256, 0, stream>>>(d_mats, s, (unsigned long long)seed, ctx->d_flags);
        const unsigned pack_wgs = grid(plan.pack) + (hint ? 1u : 0u);     // the hint rides behind the pack items
        if (pack_wgs > 0)
            svd_pack<<<pack_wgs, 256, 0, stream>>>(d_mats, w_pack, (int)plan.pack.size(), n_mats, hint ? hint->dev : nullptr);
        if (have_thin) launch_thin_pack(d_mats, w_thin_chunks, (int)plan.thin_chunks.size(), stream);
    }
    if (hint) {
        ATOMO_HIP(ctx, hipEventRecord(hint->done, stream));
        hint->pending = true;
    }
    ATOMO_HIP(ctx, hipGetLastError());
    ctx->svd_tables_intact = true;                               // until anything asks for the workspace again
    return ATOMO_OK;
}

int svd_sweeps(atomo_ctx* ctx, hipStream_t stream, int32_t* sweeps, int32_t* refreshes, int n_mats)
{
    if ((size_t)n_mats != ctx->report_n) return ATOMO_EINVAL;
    ATOMO_HIP(ctx, hipStreamSynchronize(stream));
    std::vector<int32_t> host(2 * (size_t)n_mats);
    ATOMO_HIP(ctx, hipMemcpy(host.data(), ctx->d_report, host.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
    for (int j = 0; j < n_mats; ++j) {
        sweeps[j] = host[2 * j];
        if (refreshes) refreshes[j] = host[2 * j + 1];
    }
    return ATOMO_OK;
}

}  // namespace atomo
