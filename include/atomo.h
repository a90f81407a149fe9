/*
 * atomo.h - C ABI of the MI355X (gfx950) ATOMO gradient encoder / decoder.
 *
 * ATOMO ("ATOMO: Communication-efficient Learning via Atomic Sparsification",
 * arXiv 1806.04090) writes a stochastic gradient in an atomic decomposition
 * g = sum_i lambda_i a_i with unit-norm atoms (Section 3), draws independent
 * t_i ~ Bernoulli(p_i) and sends only the kept atoms, rescaled:
 *
 *     g_hat = sum_i (lambda_i t_i / p_i) a_i                       (eq. (vhat))
 *
 * with the p that minimises the variance under a sparsity budget sum p_i = s
 * (eq. (opt_prob1), solved by Algorithm 1).  Two decompositions are built:
 * entry-wise (a_i = e_i, lambda_i = g_i) and, for a gradient viewed as a
 * matrix, the singular value decomposition (atoms u_i v_i^T, lambda_i =
 * sigma_i; Section 5, "Spectral-ATOMO").
 *
 * Conventions for every entry point
 *  - All data pointers are DEVICE pointers (HIP global memory on the device the
 *    context was created for) unless a parameter says "host".  Descriptor
 *    structs (atomo_mat, atomo_svd_msg, atomo_ew_msg) and arrays of them are
 *    HOST memory; they are read during the call and may be freed afterwards.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Work is enqueued on it; calls do not wait for the results.  Results are
 *    valid once the stream has reached the end of the enqueued work.
 *    Descriptor tables travel to the device through a ring of eight pinned
 *    staging buffers owned by the context: a call that needs a buffer whose
 *    previous copy (eight uploads ago) has not been executed yet waits for
 *    that copy, and for nothing else.  The SVD encoder and the SVD decoder
 *    skip the upload when a call, on the same stream, describes exactly the
 *    buffers of the call before it (a training loop): the tables hold
 *    addresses and sizes, never data, and the device still has them.
 *  - The caller owns every input, output and message buffer.  Inputs are never
 *    modified.  The context owns a device workspace that grows on demand
 *    (growing it allocates, which synchronises the device; atomo_reserve
 *    pre-sizes it).  One context must not be used from two streams at once.
 *  - Return value: ATOMO_OK or a negative atomo_status.  Nothing throws, exits
 *    or prints.  Conditions that are only known on the GPU (a message that did
 *    not fit its capacity, a Jacobi run that hit the sweep limit) do not fail
 *    the call; they are latched on the device and read back by atomo_status.
 *  - Random numbers: Philox4x32-10 (Salmon et al., SC'11).  Atom i of a call
 *    with (seed, stream_id) uses output word i mod 4 of the block with counter
 *    (i div 4 [64 bit], stream_id [64 bit]) and key seed [64 bit];
 *    u = (word >> 8) * 2^-24 and the atom is kept iff u < p_i, compared in
 *    single precision.  The paper fixes only t_i ~ Bernoulli(p_i) (Section 3).
 */
#ifndef ATOMO_H
#define ATOMO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum atomo_status_code {
    ATOMO_OK = 0,
    ATOMO_EINVAL = -1,     /* null pointer, non-positive size, s <= 0 or NaN, inconsistent shapes  */
    ATOMO_ECAPACITY = -2,  /* (atomo_status only) more atoms were kept than a message could hold    */
    ATOMO_ENOCONV = -3,    /* (atomo_status only) the Jacobi SVD stopped at the sweep limit         */
    ATOMO_EHIP = -4,       /* a HIP runtime call failed; atomo_last_hip_error gives its code        */
    ATOMO_ENOMEM = -5,     /* the workspace could not be allocated                                  */
    ATOMO_ETOOLARGE = -6   /* atomo_encode_entrywise_noalloc: n exceeds what its fixed scratch holds */
} atomo_status_code;

enum { ATOMO_KIND_SVD = 0, ATOMO_KIND_ENTRYWISE = 1, ATOMO_KIND_LQ = 2 };

typedef struct atomo_ctx atomo_ctx;   /* opaque: device, workspace, latched device-side flags */

/* A gradient viewed as a matrix (Section 5; Fig. 1: a conv gradient [out,in,k,k] is the row-major
 * out x (in*k*k) matrix it already is in memory).  rows x cols, row stride ld >= cols, float32. */
typedef struct atomo_mat {
    int32_t rows, cols;
    int64_t ld;
    const float* data;               /* device */
} atomo_mat;

/* One Spectral-ATOMO message: the kept singular triplets of one matrix with their weights (what a worker
 * sends to the parameter server in Section 6).  Atom index 0 is the largest singular value.
 * All pointers are caller-owned device memory. */
typedef struct atomo_svd_msg {
    int32_t rows, cols;              /* shape of the encoded matrix                                   */
    int32_t capacity;                /* room for this many kept atoms, 1 <= capacity                 */
    int32_t* count;                  /* [1]  number of atoms kept (may exceed capacity: see status)  */
    int32_t* idx;                    /* [capacity] atom indices, ascending                           */
    float*   w;                      /* [capacity] weights sigma_i / p_i; NULL selects the folded form below */
    float*   U;                      /* [capacity][rows]  U[k*rows + i] = (u of k-th kept atom)_i, unit norm;  */
                                     /* folded form (w == NULL): (sigma_i / p_i) u, the weight carried by the   */
                                     /* left vector (Section 6), rows + cols reals per atom as in the cost      */
                                     /* s(n+m) of Table "matrix_sparse"                                         */
    float*   V;                      /* [capacity][cols]  V[k*cols + j] = (v of k-th kept atom)_j, unit norm */
} atomo_svd_msg;

/* One entry-wise ATOMO message: kept coordinates, ascending, with values g_i / p_i. */
typedef struct atomo_ew_msg {
    int64_t n;                       /* length of the encoded gradient, 0 < n < 2^32                 */
    int64_t capacity;                /* room for this many pairs                                     */
    int64_t* count;                  /* [1]  number of pairs kept (may exceed capacity: see status)  */
    uint32_t* idx;                   /* [capacity] kept coordinates, ascending                       */
    float* val;                      /* [capacity] g_i / p_i                                         */
} atomo_ew_msg;

/* One l_q-quantised gradient (Section 4: L_q(g)_i = |g|_q sign(g_i) zeta_i; q = 2 is 1-bit QSGD, q = inf
 * TernGrad): the kept coordinates with their signs, and the one magnitude they all share. */
typedef struct atomo_lq_msg {
    int64_t n;                       /* length of the encoded gradient, 0 < n < 2^31                 */
    int64_t capacity;                /* room for this many kept coordinates                          */
    int64_t* count;                  /* [1]  number kept (may exceed capacity: see status)           */
    uint32_t* idx;                   /* [capacity] kept coordinates, ascending, in bits 0..30; bit 31 is set where g_i < 0 */
    float* norm;                     /* [1]  |g|_q                                                   */
} atomo_lq_msg;

/* Tuning knobs of the Jacobi SVD; pass NULL to the encoder for the defaults. */
typedef struct atomo_svd_options {
    int32_t max_sweeps;              /* default 16 (0 = default).  Noise-dominated gradients take 8 to 10 sweeps   */
                                     /* (6 or 7 with 481 or more vectors on the shorter side, see block_order),    */
                                     /* exactly low-rank ones (rank 128 in 600 x 700) 12, singular values graded   */
                                     /* over two decades 11, three 14, five 16; a matrix half of whose rows are    */
                                     /* copies of the other half 16.  Every sweep allowed costs launches even when */
                                     /* unused (they return at once, about 0.08 ms per sweep for 512-row           */
                                     /* matrices).  Hitting the limit reports ATOMO_ENOCONV; the message is then   */
                                     /* still an exact decomposition of the input, with atoms that are not yet     */
                                     /* orthogonal to the tolerance.                                               */
                                     /* Matrices with min(rows, cols) <= 32 (the [x*y/2, 2*k*k] reshape of Section */
                                     /* 6) solve their whole r x r problem per pass over the data: they get        */
                                     /* 1 + ceil(max_sweeps / 8) passes, at least 2 and at most 8 (three by        */
                                     /* default; one or two rotate and the last confirms), and their               */
                                     /* atomo_svd_sweeps count is the number of passes that rotated                */
    float   stop_cosine;             /* default 1e-4 (0 = default): stop after the first sweep whose largest */
                                     /* |<a_i,a_j>| / (|a_i||a_j|), measured before rotating, is below; matrices   */
                                     /* that iterate on their Gram matrix stop once the Gram matrix formed afresh  */
                                     /* from the rotated data has no cosine above it                               */
    int32_t max_inner_sweeps;        /* most Jacobi sweeps per 64x64 block-pair problem; 0 = default: 1 for the   */
                                     /* matrices that iterate on their Gram matrix (481 or more vectors on the    */
                                     /* shorter side), 2 for the others                                            */
    float   inner_reduction;         /* a block-pair problem stops sweeping once its largest |cos| is below        */
                                     /* inner_reduction x the value it started at; 0 = default: 0.1 (0.01 for the  */
                                     /* matrices that iterate on their Gram matrix, which matters only with        */
                                     /* max_inner_sweeps above 1)                                                  */
    int32_t full_period;             /* default 12 (0 = default): a block-pair problem rotates all 2016 index    */
                                     /* pairs in the rounds of an outer sweep whose number is a multiple of this */
                                     /* and only the 1024 pairs that couple its two blocks in the other rounds;  */
                                     /* 1: all 2016 pairs in every round                                         */
    int32_t block_order;             /* matrices with 481 or more vectors on the shorter side (they iterate on the */
                                     /* r x r Gram matrix): 0 (default) pairs the 32-row blocks of every round by  */
                                     /* the weight of their off-diagonal blocks, heaviest first (dynamic ordering  */
                                     /* of the parallel block-Jacobi method; a matrix falls back to the tournament */
                                     /* once a row has shrunk by 1e-5, as in gradients of low rank); 1 keeps the   */
                                     /* fixed round-robin tournament that the smaller matrices use throughout.     */
                                     /* Either order gives the same result from call to call                      */
    const uint64_t* stream_ids;      /* HOST array of n_mats Philox stream ids, or NULL for stream_base + j: lets */
                                     /* one call encode the gradients of several workers (stream = worker, layer) */
                                     /* and produce the messages that separate calls would                        */
    int32_t adaptive;                /* 0 (default): the launches of all max_sweeps sweeps are enqueued.  k > 0:  */
                                     /* for a training loop that encodes the same layer set step after step. The  */
                                     /* context remembers how many sweeps the matrices of earlier calls with the  */
                                     /* same shapes took (the most recent call that has finished; at most four    */
                                     /* such calls are in flight: a fifth waits for the oldest before it is       */
                                     /* enqueued) and enqueues that many + k, at most max_sweeps, separately for  */
                                     /* the matrices that iterate on their Gram matrix and for the others; a call */
                                     /* that used up such a reduced limit is followed by one with the full limit. */
                                     /* A matrix that needs more sweeps than were enqueued is reported through    */
                                     /* ATOMO_ENOCONV exactly as at max_sweeps (its message is still an exact,    */
                                     /* unbiased decomposition); gradients change slowly from step to step, so    */
                                     /* k = 1 or 2 rarely meets that.  The matrices that iterate on their Gram     */
                                     /* matrix confirm convergence on a Gram matrix formed afresh from the rotated */
                                     /* data, at a sweep boundary; the context also remembers after how many sweeps */
                                     /* the first of them asked for that, and a call enqueues those launches only  */
                                     /* from k sweeps before: a matrix that is ready sooner sweeps on until then   */
} atomo_svd_options;

/* -------- context ------------------------------------------------------------------------------ */

/* Creates a context on HIP device `device`.  *out is set on success.
 * A context owns one workspace and (for the SVD encoder) one helper stream that is forked from and joined
 * back into the caller's stream inside every call: calls that share a context must be issued from one host
 * thread at a time and onto one stream, or onto streams the caller has ordered among themselves; use one
 * context per concurrent stream. */
int atomo_create(atomo_ctx** out, int device);
int atomo_destroy(atomo_ctx* ctx);

/* Makes sure the workspace holds at least `bytes`; atomo_svd_workspace_bytes /
 * atomo_entrywise_workspace_bytes say how much a call will need (host-side arithmetic only). */
int atomo_reserve(atomo_ctx* ctx, size_t bytes);
int atomo_svd_workspace_bytes(const atomo_mat* mats /*host*/, int n_mats, size_t* bytes /*host*/);
int atomo_entrywise_workspace_bytes(int64_t n, size_t* bytes /*host*/);

/* Waits for `stream`, then reports and clears what the GPU latched since the last call:
 * ATOMO_OK, ATOMO_ECAPACITY, ATOMO_ENOCONV or ATOMO_EHIP.  If sweeps is not NULL it receives the
 * largest number of Jacobi sweeps any matrix of the last atomo_encode_svd took. */
int atomo_status(atomo_ctx* ctx, void* stream, int32_t* sweeps /*host, optional*/);
int atomo_last_hip_error(const atomo_ctx* ctx);

/* Waits for `stream`, then copies the number of Jacobi sweeps each matrix of the last
 * atomo_encode_svd took into sweeps[0 .. n_mats) (HOST) and, if refreshes is not NULL, how many
 * times the full Gram matrix of the matrix was formed from the data (matrices of 33 .. 480 rows
 * iterate directly on the data: 0 below 225 rows, from there on the number of whole-matrix
 * convergence checks near the end).  n_mats must match that call; the counts stay readable until the
 * next atomo_encode_svd on the context. */
int atomo_svd_sweeps(atomo_ctx* ctx, void* stream, int32_t* sweeps /*host*/, int32_t* refreshes /*host, optional*/,
                     int n_mats);
const char* atomo_strerror(int status);

/* -------- the method --------------------------------------------------------------------------- */

/*
 * Algorithm 1 ("ATOMO probabilities", Section 3; closed form in the KKT appendix, eq. (p_i)).
 * For each of n_seg independent segments lambda[offsets[k] .. offsets[k+1]) computes
 *     p = argmin sum lambda_i^2 / p_i   s.t.  0 <= p_i <= 1,  sum p_i = s
 * i.e. p_i = 1 for the n_s largest |lambda_i| and p_i = |lambda_i| (s - n_s) / sum_{rest} |lambda_j|
 * for the rest, n_s the smallest count that keeps every p_i <= 1.  lambda may be in any order and
 * of any sign; p comes back in the same order.  lambda_i = 0 gets p_i = 0; if s >= #nonzeros every
 * nonzero gets 1 (then sum p < s).
 *   lambda, p : device float32 [offsets[n_seg]]      offsets : HOST int64 [n_seg + 1], ascending
 *   s > 0 (a real number, the same for every segment)
 */
int atomo_probabilities(atomo_ctx* ctx, const float* lambda, const int64_t* offsets /*host*/, int n_seg,
                        double s, float* p, void* stream);

/*
 * Spectral-ATOMO encode (Section 5; eq. (vhat) on the singular value decomposition).
 * For each matrix j: thin SVD  G_j = sum_i sigma_i u_i v_i^T  (sigma descending), p = Algorithm 1
 * on sigma with budget s, t_i ~ Bernoulli(p_i) from Philox stream (seed, stream_base + j), and the
 * message = kept atoms (index, sigma_i / p_i, u_i, v_i) in ascending index.
 *   mats, msgs : HOST arrays of n_mats descriptors; msgs[j].rows/cols must equal mats[j].rows/cols.
 *   sigma_out, p_out : optional device float32, all matrices concatenated, min(rows, cols) values
 *                      each, descending sigma order (atom order).  Pass NULL to skip.
 * Supported shapes: min(rows, cols) <= 2048, max(rows, cols) <= 2^30.
 */
int atomo_encode_svd(atomo_ctx* ctx, const atomo_mat* mats, int n_mats, double s,
                     uint64_t seed, uint64_t stream_base, const atomo_svd_options* opt /*host, optional*/,
                     const atomo_svd_msg* msgs, float* sigma_out, float* p_out, void* stream);

/*
 * Entry-wise ATOMO encode (Section 3 with the standard basis; Section 4 shows 1-bit QSGD and
 * TernGrad are this with s = |g|_1/|g|_2 and s = |g|_1/|g|_inf).  lambda_i = g_i, p = Algorithm 1,
 * coordinate i is kept iff u_i < p_i (Philox stream (seed, stream_id)) and stored as
 * (i, g_i / p_i), ascending in i.
 *   g : device float32 [msg->n];  p_out : optional device float32 [msg->n].
 */
int atomo_encode_entrywise(atomo_ctx* ctx, const float* g, double s, uint64_t seed, uint64_t stream_id,
                           const atomo_ew_msg* msg /*host*/, float* p_out, void* stream);

/*
 * atomo_encode_entrywise for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same message, bit for bit; the scratch
 * memory of the kernels (water-level search state, per-chunk counts, keep and undecided bits) is a fixed array
 * of 5 MiB that the library holds on every GPU it runs on until the process ends, instead of the context's
 * growable workspace.  The call allocates nothing (no hipMalloc, hipFree, event or stream creation), on any
 * path.
 *   n = msg->n is limited to 2^24 = 16,777,216 elements; a longer gradient returns ATOMO_ETOOLARGE and
 *   nothing is enqueued.
 *   All calls on one GPU share that GPU's array, whatever their context or stream: two such calls whose
 *   kernels overlap in time race on it.  Issue them on one stream, or order the streams.  The array keeps
 *   the previous call's contents; the call clears what it needs cleared itself, with a kernel.
 *   atomo_create looks up the array's address on the context's device, so this call does no set-up of its own.
 *   Event bracketing (atomo_profile_enable) does not cover this call.
 */
int atomo_encode_entrywise_noalloc(atomo_ctx* ctx, const float* g, double s, uint64_t seed, uint64_t stream_id,
                                   const atomo_ew_msg* msg /*host*/, float* p_out, void* stream);

/*
 * l_q quantisation (Section 4, Theorem (lqgrad)): p_i = |g_i| / |g|_q, the variance-optimal entry-wise
 * probabilities for the budget s = |g|_1 / |g|_q, computed without Algorithm 1 (every g is balanced for
 * that budget).  Coordinate i is kept iff u_i < p_i (Philox stream (seed, stream_id)); a kept coordinate
 * decodes to sign(g_i) |g|_q.  q > 0; pass INFINITY for the maximum norm (TernGrad), 2 for 1-bit QSGD.
 *   g : device float32 [msg->n];  p_out : optional device float32 [msg->n].
 */
int atomo_encode_lq(atomo_ctx* ctx, const float* g, double q, uint64_t seed, uint64_t stream_id,
                    const atomo_lq_msg* msg /*host*/, float* p_out, void* stream);

/*
 * Decode (eq. (vhat)): out = scale * sum over the n_msgs messages of sum_k w_k a_k.  With
 * scale = 1/P and the P workers' messages this is the parameter server's averaged gradient
 * (Section 2).  `out` is overwritten.
 *   kind = ATOMO_KIND_SVD:       msgs is a HOST array of n_msgs atomo_svd_msg with equal rows/cols;
 *                                out is the dense rows x cols row-major matrix with row stride ld.
 *   kind = ATOMO_KIND_ENTRYWISE: msgs is a HOST array of n_msgs atomo_ew_msg with equal n;
 *                                out is the dense vector of n floats (ld is ignored).
 *   kind = ATOMO_KIND_LQ:        msgs is a HOST array of n_msgs atomo_lq_msg with equal n; out as above.
 * A message whose count exceeds its capacity contributes its first `capacity` atoms.
 * The sum is formed in a fixed order (entry-wise and l_q messages one after the other, in the order
 * given), so the same messages decode to the same bits in every run.
 */
int atomo_decode(atomo_ctx* ctx, int kind, const void* msgs, int n_msgs, float scale,
                 float* out, int64_t ld, void* stream);

/*
 * Batched form of the SVD decode for a whole layer set: for each of n_out outputs, the messages
 * msgs[first[o] .. first[o+1]) are summed into outs[o] as atomo_decode does, in one launch.
 *   msgs : HOST array;  first : HOST int32 [n_out + 1];  outs : HOST array of n_out device pointers;
 *   lds  : HOST int64 [n_out].
 */
int atomo_decode_svd_batch(atomo_ctx* ctx, const atomo_svd_msg* msgs, const int32_t* first, int n_out,
                           float scale, float* const* outs, const int64_t* lds, void* stream);

/*
 * The parameter server's step (Section 2: w_{k+1} = w_k - gamma g_hat; Section 6: the PS combines the
 * workers' messages and updates the model with the average gradient) without materialising the gradient:
 *     params[o] += alpha * sum over msgs[first[o] .. first[o+1]) of sum_k w_k u_k v_k^T
 * for each of n_out parameter matrices, in one launch; alpha = -gamma / P for P workers.  Arguments as for
 * atomo_decode_svd_batch, except that params[o] (device, rows x cols, row stride lds[o]) is read and updated.
 */
int atomo_apply_svd_batch(atomo_ctx* ctx, const atomo_svd_msg* msgs, const int32_t* first, int n_out,
                          float alpha, float* const* params, const int64_t* lds, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ATOMO_H */
