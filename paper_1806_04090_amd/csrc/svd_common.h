// Definitions shared by the translation units of the Jacobi SVD (device descriptors, schedule).
#pragma once

#include "atomo_internal.h"
#include "block_algorithm1.h"

namespace atomo {
namespace svd {

constexpr int BS = 32;          // rows per block
constexpr int PR = 64;          // rows per pair
constexpr int KCG = 512;        // columns per Gram work item
constexpr int KCU = 256;        // columns per row-update / apply work item (4 waves x 64)
constexpr int QSZ = PR * PR;
constexpr int MAX_R = ALG1_MAX;
constexpr int GS_MIN_BLOCKS = 16; // matrices with at least this many row blocks iterate in Gram space
constexpr int THIN_R = 32;        // matrices with at most this many vectors on the shorter side take the thin path (svd_thin.hip)
constexpr int THIN_PASSES = 8;    // at most this many passes over the data for a thin matrix

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Per-matrix state words (device, int32).
enum {
    ST_DONE_AT = 0,     // tick from which the matrix is finished (0 = still running)
    ST_SWEEPS = 1,      // Jacobi sweeps completed
    ST_OFFMAX = 2,      // largest |cos| seen in the current sweep (float bits)
    ST_ARRIVE = 3,      // workgroups of svd_eig that finished the last round of the sweep
    ST_SCALE = 4,       // largest squared row norm (float bits), fixed during a sweep
    ST_SCALE_NEXT = 5,  // candidate for the next sweep
    ST_MODE = 6,        // Gram-space matrices: MODE_*
    ST_CUR = 7,         // Gram-space matrices: which of the two W buffers holds A
    ST_FIRST = 8,       // Gram-space matrices: 1 until the first refresh has run (nothing to apply yet)
    ST_FRESH = 9,       // largest |cos| of the freshly computed Gram matrix (float bits)
    ST_ARRIVE2 = 10,    // workgroups of svd_fullgram_reduce that finished
    ST_EXP = 11,        // input was multiplied by 2^-ST_EXP before the iteration
    ST_ABSMAX = 12,     // largest |entry| of the input (float bits)
    ST_REFRESHES = 14,  // Gram-space matrices: fresh Gram matrices formed so far
    ST_QTICK = 13,      // Gram-space matrices: 1 + the last even tick in which svd_eig produced rotations
    ST_QTICK_ODD = 15,  //                      the same for odd ticks (rotations are double-buffered by tick parity)
    ST_FRESH_AT = 16,   // Gram-space matrices: 1 + the tick whose refresh wrote C from the data (svd_eig reads it as is)
    ST_SAT_OUT = 17,    // Gram-space matrices: 1 if a row sat out of some pair problem in the current sweep (GS_RELIABLE)
    ST_DMIN = 18,       // Gram-space matrices: smallest squared row norm above the floor seen by the running refresh (float bits)
    ST_NOISE = 19,      // Gram-space matrices: cosines below this are not resolved by the Gram arithmetic (float bits), see GS_NOISE
    ST_WSTAMP = 20,     // Gram-space matrices: word 20 + (t & 1) holds t + 1 once the block weights of the C after t ticks are written
    ST_CYCLIC_FROM = 22, // Gram-space matrices: ticks from this one on are paired by the fixed tournament (0 = not set)
    ST_VERIFY = 23,     // data-space matrices: 1 = the sweep that just ended was close enough for the whole-Gram-matrix check (DS_VERIFY)
    ST_FIRST_ASK = 24,  // Gram-space matrices: the sweep count at which the matrix first asked for a refresh (0 = not yet)
    ST_WORDS = 28
};

enum { MODE_NEED_REFRESH = 0, MODE_SWEEPS = 1, MODE_DONE = 2 };

// Rows whose squared norm is below ZERO_REL * (largest squared row norm of the matrix) are rounding
// residue of the fp32 updates (about 32 ulp of the dominant rows): their directions carry no
// information, so they neither count in the convergence test nor get rotated among themselves.
constexpr float ZERO_REL = 3.64e-12f;       // (32 * 2^-24)^2

// Gram space.  A diagonal entry of C that has shrunk far below what it was when C was last formed from the
// data is the difference of nearly equal numbers: what is left is rounding noise of the size of the old
// value times the unit roundoff times the number of updates.  Every row therefore carries a reference value
// (its squared norm at the last refresh, pushed through the rotations like the diagonal itself, without the
// off-diagonal terms), and a row whose diagonal entry is below GS_RELIABLE x reference sits out: it is not
// rotated and does not count in the convergence test until the next refresh measures it on the data again.
constexpr float GS_RELIABLE = 1.0e-5f;
// A sweep in which some row sat out ends with a refresh: the rows that wait are measured again at once (a
// refresh costs about a tenth of a sweep), so a row can shrink by GS_RELIABLE per sweep, not per several sweeps.
// Gradients of low rank (a fully connected layer sees at most batch-size atoms) converge in two thirds of the sweeps.

// Order of the block pairs in Gram space.  The C of a Gram-space matrix is all there, so the pairing of a tick need not
// follow the fixed tournament: the pairs are chosen greedily by the weight of their off-diagonal block, heaviest first, as in the dynamic ordering of Becka, Oksa and Vajtersic for the parallel
// block-Jacobi method.  The weights known when tick t + 1 is planned (during tick t) are those of the C after
// t - 1 ticks; the pairs of ticks t - 1 and t, whose rotations they do not contain yet, count as zero.
// The largest cosine that decides whether a sweep (still nb - 1 ticks) has resolved the matrix is taken over the
// pairs of its last GS_WINDOW ticks only: they are the heaviest ones of that moment.
// The weight of a block is the sum of its squared entries in the scaling of the first refresh, c_ij^2 / (ref_i ref_j)
// with reference squared norms that follow the rows through the rotations like those of GS_RELIABLE but are never
// measured again.  With a fixed scaling this is the classical dynamic ordering on D^-1/2 C D^-1/2, and rows that
// shrink towards the floor (a rank-deficient gradient) lose their weight as they shrink; squared cosines of the
// current norms would keep them at the top of every tick, at the expense of the pairs of rows that carry the matrix.
constexpr int GS_WINDOW = 5;
// The fixed tournament, which visits every pair whatever the weights say, takes over again from this sweep on, and
// already after the first sweep in which a row sat out (GS_RELIABLE): rows that collapse - a gradient of low rank,
// duplicated rows, a steeply graded spectrum - have to be brought down by the rows that carry the matrix, and
// weights cannot rank those rotations against the ones among the large rows.
constexpr int GS_DYNAMIC_SWEEPS = 10;

// Between a row of squared norm d_max and one of squared norm d_min the updates of C leave rounding errors of the
// order of GS_NOISE * sqrt(d_max / d_min) in the cosine.  Sweeping on C below that level is wasted: the refresh is
// asked for as soon as the largest cosine of a sweep is under it (capped at GS_NOISE_CAP).
constexpr float GS_NOISE = 1.0e-6f;
constexpr float GS_NOISE_CAP = 3.0e-2f;

struct SvdMat {
    float* W0;               // rows_alloc x ldw: [A | T]
    float* W1;               // second buffer of the same shape, Gram-space matrices only (else null)
    float* CT;               // Gram space: rows_alloc x ldc, [C | Tgs]
    float* CT2;              // Gram space: second buffer of the same shape; its C half alternates with CT's by tick parity
    int ldw, ldc, r, M, Mp, rows_alloc;
    int nb2, R, npairs, nchg, nchu, gs, ntiles;
    int nchp;                // data space: partial Gram matrices per pair, one per work item of svd_rowgram over A
    int* idle;               // data space: [npairs] 1 if the pair problem of the running tick left its rows as they are
    float* gram;             // data space: [npairs][nchp][64*64], partial Gram matrices of the pairs of the coming tick
                             //   (the quadrant of rows 32.. x columns ..31 is not written: it mirrors the one across)
    float* gramf;            // [ntiles][nchg][64*64]: partial tiles of the Gram matrix of all rows (Gram space: the refresh;
                             //   data space: the check of DS_VERIFY, null for matrices too small for it)
    float* Q;                // data space: [npairs][64*64], the rotations of the running tick (Gram space: null)
    float* QT;               // Gram space: [2][npairs][64*64], by tick parity the rotations transposed, four entries of a row at a
                             // time: (Q^T)[row][k] at ((k / 4) * 64 + row) * 4 + k % 4 (else null)
    float* DB;               // Gram space with C one tick behind: [2][npairs][2][32*32], by tick parity the two diagonal blocks
                             // of every pair problem's rotated matrix (else null)
    int* state;              // [ST_WORDS]
    float* sig_raw;          // [rows_alloc]
    float* rowsq;            // [rows_alloc][ceil(ldw / 256)] squared norm of every row's piece of 256 columns (svd_prepare)
    float* cref;             // Gram space: [rows_alloc] reference squared norm of every row, see GS_RELIABLE
    float* cref0;            // Gram space: [rows_alloc] the same, but never measured again after the first refresh: the
                             //   scale of the row for the block weights
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
    float* src_inv;          // [capacity] what the long vector of the kept atom is multiplied by: 1 / its norm
    float* src_fold;         // [capacity] what the short vector is multiplied by: 1
                             //   (a folded message, w == null, has the weight sigma / p in the factor of its U side)
    // thin matrices (r <= THIN_R): Q = [V | rotation of the next pass], 32 x 32 each; gram = [nchg][32 x 32]
    int thin;
    int tchunk;              // positions per work item (a multiple of 256)
    float* B;                // M x r, position-major: the rotated data
    int* report;             // [2] sweeps and refreshes of this matrix, written when the message is made
    const float* X;          // the data before the first rotation, position-major with row stride r: G itself, or its copy in B
    // Gram-space matrices: the pairing of the ticks, tables indexed by tick mod 3
    int* sched;              // [3][npairs][2]: the two blocks (smaller first) of every pair
    int* pdesc;              // [npairs][3][PD_WORDS]: what a pair problem needs to know about its pair, see PD_*
    int* where;              // [3][nb2]: 2 x pair + half for every block
    float* bw;               // [2][nb2][nb2]: weight of every off-diagonal block, by parity of the tick count of its C
    float* dd;               // [2][rows_alloc]: the scale of every row for the block weights, by tick parity: cref0
                             //   after the pair problems of the tick, 0 for rows that sat out or lie under the floor
};

struct Work { int mat, a, b, c; };

// Gram space, per pair and tick (mod 3), written with the pairing by whoever plans the tick: the pair's blocks, and
// for each of the two where it sat in the tick before: the pair it was in (PD_K*), which half of that pair (PD_S*)
// and that pair's two blocks (PD_X*, PD_Y*).  One read instead of three dependent ones at the head of a pair problem.
enum { PD_BI = 0, PD_BJ, PD_K1, PD_S1, PD_X0, PD_X1, PD_K2, PD_S2, PD_Y0, PD_Y1, PD_WORDS = 12 };

// The work item of a Gram-space pair problem carries where the matrix's state words and the pair's descriptors are,
// as offsets from the descriptor table of the matrices in units of 16 bytes (b and c; 0 for data-space matrices), so
// that they are read beside the matrix's descriptor, not after it.
constexpr size_t HOT_UNIT = 16;

// Index of the pair that holds block x in `round` (inverse of pair_blocks).
__device__ inline int pair_of_block(int nb2, int round, int x)
{
    const int n1 = nb2 - 1;
    if (x == n1 || x == round) return 0;
    const int d = (x - round + n1) % n1;
    return d <= (n1 - 1) / 2 ? d : n1 - d;
}

__device__ inline void pair_blocks(int nb2, int round, int k, int& bi, int& bj)
{
    const int n1 = nb2 - 1;
    int a, b;
    if (k == 0) { a = n1; b = round; }
    else { a = (round + k) % n1; b = (round - k + n1) % n1; }
    bi = a < b ? a : b;
    bj = a < b ? b : a;
}

// The blocks of pair k in `tick`: from the table for Gram-space matrices, else the fixed tournament.
__device__ inline void tick_pair(const SvdMat& m, int tick, int k, int& bi, int& bj)
{
    if (m.gs) {
        const int* s = m.sched + ((size_t)(tick % 3) * m.npairs + k) * 2;
        bi = s[0];
        bj = s[1];
    } else {
        pair_blocks(m.nb2, tick % m.R, k, bi, bj);
    }
}

// Writes the descriptor of pair k = (bi, bj) of tick t; (w, x0, x1) for each block: its entry of the `where` table of
// tick t - 1 and the two blocks of the pair it names.
__device__ inline void write_pair_desc(const SvdMat& m, int t, int k, int bi, int bj, int wi, int xi0, int xi1, int wj,
                                       int xj0, int xj1)
{
    int* d = m.pdesc + ((size_t)k * 3 + t % 3) * PD_WORDS;
    d[PD_BI] = bi;      d[PD_BJ] = bj;
    d[PD_K1] = wi >> 1; d[PD_S1] = wi & 1; d[PD_X0] = xi0; d[PD_X1] = xi1;
    d[PD_K2] = wj >> 1; d[PD_S2] = wj & 1; d[PD_Y0] = xj0; d[PD_Y1] = xj1;
}

// exponent e such that absmax * 2^-e lies in [1, 2); 0 for an all-zero matrix
__device__ inline int scale_exponent(const SvdMat& m)
{
    const unsigned int bits = (unsigned int)m.state[ST_ABSMAX];
    if (bits == 0u) return 0;
    const int e = (int)(bits >> 23) - 127;
    return e < -126 ? -126 : e;
}

// Data-space matrices: true if work for `tick` should be skipped (finished earlier, or past the sweep limit).
__device__ inline bool skip_step(const SvdMat& m, int tick, int max_sweeps)
{
    const int done_at = m.state[ST_DONE_AT];
    if (done_at != 0 && tick >= done_at) return true;
    return tick / m.R >= max_sweeps;
}

// The buffer that currently holds [A | T].
// Both pointers are read into values before the choice: a conditional between the two fields themselves is
// an address computed at run time, which moves a by-value copy of the descriptor into scratch memory (a
// per-lane store of the whole struct at the top of every kernel).
__device__ inline float* current_w(const SvdMat& m)
{
    float* const w0 = m.W0;
    float* const w1 = m.W1;
    return (m.gs && (m.state[ST_CUR] & 1)) ? w1 : w0;
}

// Gram-space matrices: the buffer whose C half holds the Gram matrix of tick parity `parity`.
__device__ inline float* c_of_parity(const SvdMat& m, int parity)
{
    float* const c0 = m.CT;
    float* const c1 = m.CT2;
    return (parity & 1) ? c1 : c0;
}

// Data space: a pair whose largest cosine is below this fraction of stop_cosine is left alone (no Jacobi steps, and no
// row update if its rows are in order already): the sweep that only confirms convergence then costs its Gram matrices.
constexpr float DS_LEAVE = 0.1f;

// Data space: a sweep whose largest cosine (measured before rotating) is below DS_VERIFY x stop_cosine has, convergence
// being quadratic, most likely left the matrix converged.  Instead of a whole further sweep that only confirms it (R ticks
// of three launches in which nothing rotates), the Gram matrix of all rows is then formed once at the sweep boundary
// (svd_fullgram) and its largest cosine decides (svd_ds_verify): finished, or the sweeps go on.  Only for matrices of
// at least DS_VERIFY_MIN_R ticks per sweep: the check costs two launches at every sweep boundary.
constexpr float DS_VERIFY = 10.0f;
constexpr int DS_VERIFY_MIN_R = 7;

constexpr int TLD = PR + 1;      // row stride of a 64x64 tile staged in LDS

// Gram-space matrices: the two-sided update  C <- D^T C D  (D = the block rotations of the round) and
// Tgs <- D^T Tgs, one 64x64 tile at a time, by 256 threads (tid 0..255) that own the LDS tile xs:
//   kind 1: tile (pair a, pair b) of C:  Qa^T * C[rows of a, columns of b] * Qb, read from the C of this tick's
//           parity and written to the C of the other parity (svd_eig of the next tick still reads the old one)
//   kind 2: 64 rows of pair a x 64 columns of Tgs:  Qa^T * Tgs[rows of a, chunk], in place
// Every thread of the workgroup must call this (it has workgroup barriers), with item >= n_items for none.
__device__ inline void twosided_tile(const SvdMat* mats, const Work* work, int item, int n_items, int tick, float* xs,
                                     int tid)
{
    bool active = item < n_items;
    const Work wk = active ? work[item] : Work{0, 0, 0, 0};
    const SvdMat m = mats[wk.mat];
    const int kind = wk.c;
    if (active) active = m.state[(tick & 1) ? ST_QTICK_ODD : ST_QTICK] == tick + 1;   // did svd_eig rotate in this tick?
    if (!__syncthreads_or(active)) return;                       // nothing to do in this workgroup (finished matrices)
    const int lane = tid & 63, wave = tid >> 6;
    const int qi = wave >> 1, qj = wave & 1, h = lane >> 5, l32 = lane & 31;
    int ai = 0, aj = 0, bi = 0, bj = 0;
    if (active) {
        tick_pair(m, tick, wk.a, ai, aj);
        if (kind == 1) tick_pair(m, tick, wk.b, bi, bj);
    }
    // (the rotations from their transposed copies: 16 bytes of a row per load, consecutive lanes consecutive rows)
    const float* qa = m.QT + ((size_t)(tick & 1) * m.npairs + wk.a) * QSZ;
    const float* qb = m.QT + ((size_t)(tick & 1) * m.npairs + wk.b) * QSZ;
    const float* src = kind == 1 ? c_of_parity(m, tick) : m.CT;
    float* dst = kind == 1 ? c_of_parity(m, tick + 1) : m.CT;
    // column of local index j: inside C the columns of pair b, inside Tgs a plain 64-column chunk
    auto col_of = [&](int j) { return kind == 1 ? (j < BS ? bi * BS + j : bj * BS + j - BS) : m.rows_alloc + wk.b * PR + j; };
    auto row_of = [&](int i) { return i < BS ? ai * BS + i : aj * BS + i - BS; };

    // every global load is issued before the first use: the tile, and the MFMA operands from Qa and Qb
    // (instruction (u, x) of a product contracts the indices 8 u + x, lanes 0..31, and 8 u + 4 + x, lanes 32..63)
    floatx4 tile_regs[QSZ / 1024], qa_regs[PR / 8], qb_regs[PR / 8];
    // for the weight of the wave's 32x32 block of the new C: 1 / |row| of its rows and of its column (0: skip the row)
    float rrow[16], rcol = 0.0f;
    const int brow = qi ? aj : ai, bcol = qj ? bj : bi;
    if (active && kind == 1) {
        const float* d = m.dd + (size_t)(tick & 1) * m.rows_alloc;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float x = d[brow * BS + 8 * (v >> 2) + 4 * h + (v & 3)];
            rrow[v] = x > 0.0f ? __builtin_amdgcn_rsqf(x) : 0.0f;
        }
        const float x = d[bcol * BS + l32];
        rcol = x > 0.0f ? __builtin_amdgcn_rsqf(x) : 0.0f;
    }
    if (active) {
#pragma unroll
        for (int p = 0; p < QSZ / 1024; ++p) {
            const int e = tid + 256 * p, i = e >> 4, j = (e & 15) * 4;
            tile_regs[p] = *(const floatx4*)(src + (size_t)row_of(i) * m.ldc + col_of(j));
        }
#pragma unroll
        for (int u = 0; u < PR / 8; ++u) {
            qa_regs[u] = *(const floatx4*)(qa + ((2 * u + h) * PR + qi * BS + l32) * 4);      // (Qa^T)[i][8 u + 4 h ..]
            if (kind == 1) qb_regs[u] = *(const floatx4*)(qb + ((2 * u + h) * PR + qj * BS + l32) * 4);    // Qb[8 u + 4 h ..][j]
        }
#pragma unroll
        for (int p = 0; p < QSZ / 1024; ++p) {
            const int e = tid + 256 * p, i = e >> 4, j = (e & 15) * 4;
#pragma unroll
            for (int x = 0; x < 4; ++x) xs[i * TLD + j + x] = tile_regs[p][x];
        }
    }
    __syncthreads();
    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    if (active) {
#pragma unroll
        for (int u = 0; u < PR / 8; ++u)
#pragma unroll
            for (int x = 0; x < 4; ++x)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(qa_regs[u][x], xs[(8 * u + 4 * h + x) * TLD + qj * BS + l32], acc, 0, 0, 0);
    }
    __syncthreads();                                             // the tile is consumed; xs now takes Qa^T * tile
    if (active && kind == 1) {
#pragma unroll
        for (int v = 0; v < 16; ++v) xs[(qi * BS + 8 * (v >> 2) + 4 * h + (v & 3)) * TLD + qj * BS + l32] = acc[v];
    }
    __syncthreads();
    if (!active) return;
    if (kind == 1) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
        for (int u = 0; u < PR / 8; ++u)
#pragma unroll
            for (int x = 0; x < 4; ++x)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(xs[(qi * BS + l32) * TLD + 8 * u + 4 * h + x], qb_regs[u][x], acc, 0, 0, 0);
    }
    const int c = col_of(qj * BS + l32);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int i = qi * BS + 8 * (v >> 2) + 4 * h + (v & 3);
        dst[(size_t)row_of(i) * m.ldc + c] = acc[v];
    }
    if (kind == 1) {
        // the weight of this block of the C after tick + 1 ticks: sum of its squared entries, each divided by the
        // reference squared norms of its two rows (a diagonal block leaves out its diagonal), summed in a fixed order
        float sum = 0.0f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float t = acc[v] * rrow[v] * rcol;
            if (brow != bcol || 8 * (v >> 2) + 4 * h + (v & 3) != l32) sum = fmaf(t, t, sum);
        }
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
        if (lane == 0) {
            m.bw[((size_t)((tick + 1) & 1) * m.nb2 + brow) * m.nb2 + bcol] = sum;
            if (wk.a == 0 && wk.b == 0 && wave == 0) m.state[ST_WSTAMP + ((tick + 1) & 1)] = tick + 2;
        }
    }
}

// Enqueues svd_eig for one tick (defined in svd_eig.hip): n_items pair problems, plus, when n_two > 0, the
// two-sided update of tick - 1 over the n_two tiles of d_two_work.  fresh_only selects, among the Gram-space
// matrices, those whose Gram matrix was formed in this very tick (1) or all the others (0).
// With n_plan > 0 the launch also plans the pairing of tick + 1 for the Gram-space matrices of d_plan_work (one
// workgroup each): by block weight, or, with cyclic != 0, the fixed tournament.
// ask_from: a Gram-space matrix does not ask for a refresh before it has completed that many sweeps (the host enqueues
// no refresh launches at the sweep boundaries before; the sweep limit overrides it).
void launch_svd_eig(const SvdMat* d_mats, const Work* d_work, int n_items, const Work* d_two_work, int n_two,
                    const Work* d_plan_work, int n_plan, int cyclic, int tick, int max_sweeps, int ask_from,
                    float stop_cosine, int max_inner, float inner_reduction, int full_period, int fresh_only,
                    int* d_flags, hipStream_t stream);

// Thin matrices (defined in svd_thin.hip).  d_chunks lists (matrix, chunk of positions), d_list the thin matrices.
// d_direct: chunks of the matrices used in place (largest |entry| only); d_copied: chunks of those copied into B first.
void launch_thin_absmax(const SvdMat* d_mats, const Work* d_direct, int n_direct, const Work* d_copied, int n_copied,
                        hipStream_t stream);
// One pass over the data (rotate, Gram matrix) followed by the r x r problem of every thin matrix.
void launch_thin_pass(const SvdMat* d_mats, const Work* d_chunks, int n_chunks, const Work* d_list, int n_list, int pass,
                      int last_pass, float stop_cosine, int* d_flags, hipStream_t stream);
// After svd_select: the kept atoms' vectors into the message.
void launch_thin_pack(const SvdMat* d_mats, const Work* d_chunks, int n_chunks, hipStream_t stream);

}  // namespace svd
}  // namespace atomo
