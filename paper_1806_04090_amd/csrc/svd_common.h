// Definitions shared by the translation units of the Jacobi SVD (device descriptors, schedule).
#pragma once

#include "atomo_internal.h"
#include "block_algorithm1.h"

namespace atomo {
namespace svd {

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

// Enqueues svd_eig for one Jacobi step (defined in svd_eig.hip).
void launch_svd_eig(const SvdMat* d_mats, const Work* d_work, int n_items, int step, int max_sweeps,
                    float stop_cosine, int max_inner, float inner_reduction, int* d_flags, hipStream_t stream);

}  // namespace svd
}  // namespace atomo
