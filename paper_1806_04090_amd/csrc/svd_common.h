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
constexpr int GS_MIN_BLOCKS = 8;  // matrices with at least this many row blocks iterate in Gram space

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
    ST_ARRIVE2 = 10,    // workgroups of svd_fresh_check that finished
    ST_EXP = 11,        // input was multiplied by 2^-ST_EXP before the iteration
    ST_ABSMAX = 12,     // largest |entry| of the input (float bits)
    ST_REFRESHES = 14,  // Gram-space matrices: fresh Gram matrices formed so far
    ST_QTICK = 13,      // Gram-space matrices: 1 + the tick in which svd_eig last produced rotations
    ST_WORDS = 16
};

enum { MODE_NEED_REFRESH = 0, MODE_SWEEPS = 1, MODE_DONE = 2 };

// Rows whose squared norm is below ZERO_REL * (largest squared row norm of the matrix) are rounding
// residue of the fp32 updates (about 32 ulp of the dominant rows): their directions carry no
// information, so they neither count in the convergence test nor get rotated among themselves.
constexpr float ZERO_REL = 3.64e-12f;       // (32 * 2^-24)^2

struct SvdMat {
    float* W0;               // rows_alloc x ldw: [A | T]
    float* W1;               // second buffer of the same shape, Gram-space matrices only (else null)
    float* CT;               // Gram space: rows_alloc x ldc, [C | Tgs]
    float* C2;               // Gram space: rows_alloc x rows_alloc scratch for the two-sided update
    int ldw, ldc, r, M, Mp, rows_alloc;
    int nb2, R, npairs, nchg, nchu, gs, ntiles;
    float* gram;             // data space: [npairs][nchg][64*64]; Gram space: [ntiles][nchg][64*64]
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

// Enqueues svd_eig for one tick (defined in svd_eig.hip).
void launch_svd_eig(const SvdMat* d_mats, const Work* d_work, int n_items, int tick, int max_sweeps,
                    float stop_cosine, int max_inner, float inner_reduction, int* d_flags, hipStream_t stream);

}  // namespace svd
}  // namespace atomo
