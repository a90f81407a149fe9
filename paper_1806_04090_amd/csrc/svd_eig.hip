// svd_eig: eigen-decomposition of the 64x64 Gram matrix of one block pair (the inner problem of the
// blocked one-sided Jacobi SVD), one workgroup per pair.
//
// Two-sided Jacobi with parallel orderings, 32 disjoint rotations per step.  The matrix A and the accumulated
// rotations Q live in LDS in "slot" order: block i of the pair sits in the even slots, block j in the odd slots, and
// within a row the even slots are stored in columns 0..31 and the odd slots in columns 32..63.
//
// Cross round (most rounds).  The two diagonal 32x32 blocks of the pair only need to be diagonalised now and then
// (cyclic Jacobi rotates every index pair once per sweep); a cross round rotates only the 32 x 32 index pairs that
// couple the two blocks: at every step the rotations act on the slot pairs (0,1), (2,3), ..., (62,63), the even slots
// stay and the odd slots move on by one pair per step, 32 steps.  Matrix and rotations stay in registers for the
// whole round (see cross_sweep).
//
// Full round (every full_period-th round of an outer sweep): first the 2 x 496 index pairs inside the two blocks,
// as two round-robin ("chess tournament") schedules of 32 players side by side, 31 steps; then a cross round: all 2016
// pairs in 63 steps.  The 31 steps go through LDS: A and Q are double-buffered, a step is: read buffer X, rotate,
// write buffer Y permuted (every result goes to the place its index occupies in the next step), barrier.  Every lane
// computes the rotation of its own column pair from the diagonal 2x2 block (redundantly in every wave, so no second
// barrier) and fetches the rotation of its row pair with a lane read.
#include <cfloat>
#include <type_traits>

#include "svd_common.h"

namespace atomo {
namespace svd {

namespace {

constexpr int NT = 1024;                // threads per workgroup
constexpr int TILES_PER_WG = NT / 256;  // two-sided tiles a workgroup without a pair problem applies
constexpr int ELD = 65;                 // LDS row stride
constexpr int GROUPS = NT / 32;         // thread groups of 32 (one slot pair of columns per thread)
constexpr int QR_PER = 64 / GROUPS;     // rows of Q per thread

// A round inside the two blocks (the first 31 steps of a full round) numbers the 64 indices of the pair by positions:
// positions 0 .. 31 hold the indices of block i, 32 .. 63 those of block j, the rotations pair the positions
// (2k, 2k + 1), and between two steps the positions of either half move like a round-robin tournament of 32 players:
// position 0 stays, the odd ones move down by two (1 -> 2), the even ones up by two (30 -> 31); after 31 steps everybody
// is back.  The matrix itself stays in the layout of the cross rounds (below); within_col / within_row say where a
// position lives in it.  The columns are chosen so that the 32 lanes of a step, one per pair, read 32 different LDS
// banks: pair k of block i = the indices k and k + 16 (columns k, 16 + k), pair k of block j = the indices 16 + k and k
// (columns 48 + k, 32 + k).
__device__ inline int next_within(int v)
{
    const int s = v & 31;
    const int n = s == 0 ? 0 : (s & 1) ? (s == 1 ? 2 : s - 2) : (s == 30 ? 31 : s + 2);
    return (v & 32) | n;
}
__device__ inline int within_col(int v)
{
    const int k = (v & 31) >> 1, side = v & 1;
    return v < 32 ? 16 * side + k : 32 + (side ? k : 16 + k);
}
// (column c of the cross layout holds slot 2c, or 2(c - 32) + 1; row = slot)
__device__ inline int within_row(int v) { const int c = within_col(v); return c < 32 ? 2 * c : 2 * (c - 32) + 1; }

// column of slot s inside a row: even slots first, then odd slots
__device__ inline int mem_col(int s) { return (s >> 1) + 32 * (s & 1); }

// slot in which index i of the pair starts (and ends) a sweep
__device__ inline int home_slot(int i) { return i < 32 ? 2 * i : 2 * (i - 32) + 1; }

// Largest |A_ij| / max(sqrt(A_ii A_jj), z2) over i < j, and largest diagonal entry.  All threads call.
__device__ inline float2 max_cosine(const float* A, float z2, float* red)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float mx = 0.0f, dmax = 0.0f;
    for (int e = tid; e < QSZ; e += NT) {
        const int i = e >> 6, j = e & 63;                        // j is the memory column
        const int js = j < 32 ? 2 * j : 2 * (j - 32) + 1;        // its slot
        if (i < js) {
            const float dii = A[i * ELD + mem_col(i)], djj = A[js * ELD + j];
            if (dii > 0.0f && djj > 0.0f)
                mx = fmaxf(mx, fabsf(A[i * ELD + j]) * __builtin_amdgcn_rcpf(fmaxf(__builtin_amdgcn_sqrtf(dii * djj), z2)));
        } else if (i == js) {
            dmax = fmaxf(dmax, A[i * ELD + j]);
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        mx = fmaxf(mx, __shfl_down(mx, o));
        dmax = fmaxf(dmax, __shfl_down(dmax, o));
    }
    __syncthreads();                     // red[] may still be read from a previous call
    if (lane == 0) { red[wave] = mx; red[16 + wave] = dmax; }
    __syncthreads();
    mx = 0.0f; dmax = 0.0f;
    for (int w = 0; w < NT / 64; ++w) { mx = fmaxf(mx, red[w]); dmax = fmaxf(dmax, red[16 + w]); }
    return make_float2(mx, dmax);
}

// Rotation (c, s) that annihilates the off-diagonal entry of the slot pair (2k, 2k+1), from the
// double-angle form: with d = a_qq - a_pp and w = 2 a_pq,  cos 2t = |d| / sqrt(d^2 + w^2),
// c = sqrt((1 + cos 2t) / 2),  s = sign(d) w / (2 c sqrt(d^2 + w^2)).  Two reciprocal square roots
// (hardware approximations, 1 ulp) and no division: what a rotation misses the next sweep picks up,
// and the orthogonality of the product is restored by the Newton-Schulz step.
__device__ inline float2 rotation_of(float app, float apq, float aqq, float z2)
{
    float c = 1.0f, s = 0.0f;
    // rotate only if |a_pq| > 1e-7 * max(sqrt(a_pp a_qq), floor), compared in squares
    if (apq * apq > 1e-14f * fmaxf(fabsf(app * aqq), z2 * z2)) {
        const float d = aqq - app, w = 2.0f * apq;
        const float ir = __builtin_amdgcn_rsqf(fmaf(d, d, w * w));
        const float hc = fmaf(0.5f * fabsf(d), ir, 0.5f);        // (1 + cos 2t) / 2 = c^2
        const float ic = __builtin_amdgcn_rsqf(hc);
        c = hc * ic;
        s = copysignf(0.5f * w * ir * ic, d * w);
    }
    return make_float2(c, s);
}

// The same values without a branch; where no rotation is due the discarded operands may be NaN or infinite.
__device__ inline float2 rotation_of_select(float app, float apq, float aqq, float z2)
{
    const bool rot = apq * apq > 1e-14f * fmaxf(fabsf(app * aqq), z2 * z2);
    const float d = aqq - app, w = 2.0f * apq;
    const float ir = __builtin_amdgcn_rsqf(fmaf(d, d, w * w));
    const float hc = fmaf(0.5f * fabsf(d), ir, 0.5f);
    const float ic = __builtin_amdgcn_rsqf(hc);
    return make_float2(rot ? hc * ic : 1.0f, rot ? copysignf(0.5f * w * ir * ic, d * w) : 0.0f);
}

// (c, s) of a slot pair together with the two diagonal entries the rotation leaves behind:
// d_p' = c^2 a_pp - 2 c s a_pq + s^2 a_qq,  d_q' = s^2 a_pp + 2 c s a_pq + c^2 a_qq
__device__ inline float4 rotation_and_diagonal(float app, float apq, float aqq, float z2)
{
    const float2 r = rotation_of(app, apq, aqq, z2);
    const float cc = r.x * r.x, ss = r.y * r.y, cs2 = 2.0f * r.x * r.y * apq;
    return make_float4(r.x, r.y, fmaf(cc, app, fmaf(ss, aqq, -cs2)), fmaf(ss, app, fmaf(cc, aqq, cs2)));
}

// Plans the pairing of tick + 1 for one Gram-space matrix (all NT threads of a workgroup call).
// Dynamic order: a greedy maximum-weight matching on the block weights of the C after tick - 1 ticks (written by the
// two-sided update of the previous launch), heaviest pair first, ties to the lower block indices; the pairs of
// ticks tick - 1 and tick count as zero, their rotations are not in those weights yet.  Without such weights
// (first ticks, `cyclic`) the round of the fixed tournament.  wsh: nb2 x (nb2 + 1) floats, ptr / partner: 64 words each.
__device__ inline void plan_next_tick(const SvdMat& m, int tick, int cyclic, float* wsh, int* ptr, int* partner)
{
    if (!m.gs || m.state[ST_DONE_AT] != 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nb = m.nb2, np = m.npairs;
    int* sch = m.sched + (size_t)((tick + 1) % 3) * np * 2;
    int* whr = m.where + (size_t)((tick + 1) % 3) * nb;
    // (ST_CYCLIC_FROM may be set while this launch runs, but then to tick + 2: the answer for tick + 1 is the same)
    const int cyclic_from = m.state[ST_CYCLIC_FROM];
    const bool weighted = !cyclic && tick >= 2 && (tick + 1) / m.R < GS_DYNAMIC_SWEEPS &&
                          !(cyclic_from != 0 && tick + 1 >= cyclic_from) &&
                          m.state[ST_WSTAMP + ((tick - 1) & 1)] == tick;
    // the tables of this tick, for the descriptors of the next tick's pairs
    const int* sch_now = m.sched + (size_t)(tick % 3) * np * 2;
    const int* whr_now = m.where + (size_t)(tick % 3) * nb;
    auto describe = [&](int k, int bi, int bj) {
        const int wi = whr_now[bi], wj = whr_now[bj];
        write_pair_desc(m, tick + 1, k, bi, bj, wi, sch_now[2 * (wi >> 1)], sch_now[2 * (wi >> 1) + 1], wj,
                        sch_now[2 * (wj >> 1)], sch_now[2 * (wj >> 1) + 1]);
    };
    if (!weighted) {
        for (int k = tid; k < np; k += NT) {
            int bi, bj;
            pair_blocks(nb, (tick + 1) % m.R, k, bi, bj);
            sch[2 * k] = bi; sch[2 * k + 1] = bj;
            whr[bi] = 2 * k; whr[bj] = 2 * k + 1;
            describe(k, bi, bj);
        }
        return;
    }
    const float* W = m.bw + (size_t)((tick - 1) & 1) * nb * nb;
    auto usable = [](float w) { return (w > 0.0f && w <= FLT_MAX) ? w : 0.0f; };
    const int ld = nb + 1;                                       // odd row stride: a column is spread over the LDS banks
    for (int e = tid; e < nb * nb; e += NT) {
        const int i = e / nb, j = e - i * nb;
        wsh[i * ld + j] = i != j ? usable(W[i * nb + j]) + usable(W[j * nb + i]) : 0.0f;
    }
    if (tid < PR) { partner[tid] = -1; ptr[tid] = -1; }
    __syncthreads();
    for (int q = tid; q < 2 * np; q += NT) {
        const int* s = m.sched + ((size_t)((q < np ? tick : tick + 2) % 3) * np + (q < np ? q : q - np)) * 2;
        wsh[s[0] * ld + s[1]] = 0.0f;
        wsh[s[1] * ld + s[0]] = 0.0f;
    }
    __syncthreads();
    // The greedy matching (heaviest edge first; edges ordered by weight, then by lower block indices) is the union of
    // the locally dominant edges of successive rounds: an edge is taken when each of its two blocks is the other's
    // best free partner, which holds at least for the best free edge of all, so every round makes progress.
    // Sixteen threads per block look at four candidates each.
    const int v = tid >> 4, helper = tid & 15;
    float cw[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int j = helper + 16 * k;
        cw[k] = (v < nb && j < nb && j != v) ? wsh[v * ld + j] : -1.0f;      // -1: no candidate
    }
    for (int round = 0; round < np; ++round) {
        const bool v_free = v < nb && partner[v] < 0;
        float bw = -1.0f;
        int be = 0x7fffffff, bj = -1;
        if (v_free) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int j = helper + 16 * k;
                if (cw[k] >= 0.0f && partner[j] < 0) {
                    const int e = v < j ? v * nb + j : j * nb + v;
                    if (cw[k] > bw || (cw[k] == bw && e < be)) { bw = cw[k]; be = e; bj = j; }
                }
            }
        }
        for (int o = 8; o > 0; o >>= 1) {                        // the sixteen helpers of a block sit in one wave
            const float ow = __shfl_xor(bw, o);
            const int oe = __shfl_xor(be, o), oj = __shfl_xor(bj, o);
            if (ow > bw || (ow == bw && oe < be)) { bw = ow; be = oe; bj = oj; }
        }
        if (helper == 0 && v < nb) ptr[v] = v_free ? bj : -1;     // (last read before the barrier that ended the round before)
        __syncthreads();
        bool taken = false;
        if (helper == 0 && v_free && bj >= 0 && ptr[bj] == v) { partner[v] = bj; taken = true; }
        if (!__syncthreads_or(taken)) break;                     // (also orders the writes of partner[] before the next round)
    }
    // pair numbers in the order of each pair's lower block; blocks left over (cannot happen) pair up in order
    if (wave != 0) return;
    const int mine = lane < nb ? partner[lane] : lane;           // lanes beyond the blocks: out of the way
    const unsigned long long unmatched = __ballot(lane < nb && mine < 0);
    int mate = mine;
    if (lane < nb && mine < 0) {
        const int rank = __popcll(unmatched & ((1ull << lane) - 1ull));
        // the r-th unmatched block pairs with the (r ^ 1)-th
        int seen = 0;
        for (int b2 = 0; b2 < nb; ++b2)
            if ((unmatched >> b2) & 1ull) { if (seen == (rank ^ 1)) mate = b2; ++seen; }
    }
    const bool leader = lane < nb && mate > lane;
    const unsigned long long leaders = __ballot(leader);
    if (leader) {
        const int k = __popcll(leaders & ((1ull << lane) - 1ull));
        sch[2 * k] = lane; sch[2 * k + 1] = mate;
        whr[lane] = 2 * k; whr[mate] = 2 * k + 1;
        describe(k, lane, mate);
    }
}

// Workgroups 0 .. n_eig-1 solve block pairs.  Workgroups beyond take no pair: each applies four tiles of the
// previous tick's two-sided update (one tile per group of four waves, staged in the LDS arrays a pair problem
// would use).  The update writes the C of this tick's parity; the pair problems read the C of the previous
// parity and bring their own 64x64 block up to date themselves (step 1 below), so the two do not meet.
__global__ __launch_bounds__(NT) void svd_eig(const SvdMat* mats, const Work* work, int n_eig, const Work* two_work,
                                              int n_two, const Work* plan_work, int cyclic, int step, int max_sweeps, int ask_from,
                                              float stop_cosine, int max_inner, float inner_reduction, int full_period,
                                              int fresh_only, int* flags)
{
    __shared__ float As[2][PR * ELD];
    __shared__ float Qs[2][PR * ELD];
    __shared__ float ev[PR];
    __shared__ int dest[PR];
    __shared__ float ref[PR];            // Gram space: reference squared norm of the pair's rows (natural index)
    __shared__ float ref0[PR];           //             the same in the scaling of the first refresh (cref0)
    __shared__ int sits_out[PR];         // Gram space: by slot, rows whose diagonal entry is rounding noise
    __shared__ float red[32];
    __shared__ float rlen[PR];           // by slot: 1 / length of the row as the pair problem starts
    __shared__ unsigned int entry_bits[2];   // largest cosine and largest squared norm as the pair problem starts
    __shared__ __align__(16) float2 rotc[2][32];       // cross rounds: (c, s) of the 32 rotations of a step, by step parity
    __shared__ float2 rotd[2][32];       //               the diagonal entries (d_p', d_q') those rotations leave behind

    const int two_wgs = (n_two + TILES_PER_WG - 1) / TILES_PER_WG;
    if ((int)blockIdx.x >= n_eig + two_wgs) {                     // the last workgroups plan the next tick
        plan_next_tick(mats[plan_work[(int)blockIdx.x - n_eig - two_wgs].mat], step, cyclic, As[0], dest, sits_out);
        return;
    }
    if ((int)blockIdx.x >= n_eig) {
        const int group = threadIdx.x >> 8;
        float* tile = group == 0 ? As[0] : group == 1 ? As[1] : group == 2 ? Qs[0] : Qs[1];
        twosided_tile(mats, two_work, ((int)blockIdx.x - n_eig) * TILES_PER_WG + group, n_two, step - 1, tile,
                      (int)(threadIdx.x & 255));
        return;
    }
    const Work wk = work[blockIdx.x];
    // Gram space: the state words and the pair's descriptor are read beside the matrix's descriptor (the work item
    // says where they are), all before the first of them is looked at: one trip to memory instead of a chain of them.
    int st_fresh = 0;
    int pdw[PD_Y1 + 1];
#pragma unroll
    for (int i = 0; i <= PD_Y1; ++i) pdw[i] = 0;
    int st_done = 0, st_mode = 0;
    if (wk.c) {
        const int* hot = (const int*)((const char*)mats + (size_t)(unsigned)wk.b * HOT_UNIT);
        const int* pd = (const int*)((const char*)mats + (size_t)(unsigned)wk.c * HOT_UNIT) + (step % 3) * PD_WORDS;
        st_done = hot[ST_DONE_AT]; st_mode = hot[ST_MODE]; st_fresh = hot[ST_FRESH_AT];
#pragma unroll
        for (int i = 0; i <= PD_Y1; ++i) pdw[i] = pd[i];
    }
    const SvdMat m = mats[wk.mat];
    if (m.gs) {
        // (the same for every lane: as scalars)
        st_done = __builtin_amdgcn_readfirstlane(st_done);
        st_mode = __builtin_amdgcn_readfirstlane(st_mode);
        st_fresh = __builtin_amdgcn_readfirstlane(st_fresh);
#pragma unroll
        for (int i = 0; i <= PD_Y1; ++i) pdw[i] = __builtin_amdgcn_readfirstlane(pdw[i]);
        if (st_done != 0 || st_mode != MODE_SWEEPS) return;
        // a tick with a refresh has two launches: before it, the matrices that sweep on; after it, those
        // whose Gram matrix the refresh has just formed
        if ((st_fresh == step + 1) != (fresh_only != 0)) return;
    } else if (skip_step(m, step, max_sweeps)) {
        return;
    }
    const int round = step % m.R;
    int bi = pdw[PD_BI], bj = pdw[PD_BJ];
    if (!m.gs) pair_blocks(m.nb2, round, wk.a, bi, bj);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool cross = round % full_period != 0;

    // 1. the Gram matrix of the pair into As[0] (home slots), Q = I into Qs[0].
    //    Data-space matrices: the partial sums that svd_rowgram left, added in a fixed order.
    //    Gram-space matrices, first tick after a refresh: the pair's block of C as it is.
    //    Gram-space matrices otherwise: C (previous parity) does not contain the previous tick's rotations yet.
    //    With the pair's blocks a (then in pair k1, half s1) and b (pair k2, half s2) of the previous round,
    //        [aa ab; ba bb] = [Q1s^T C11 Q1s, Q1s^T C12 Q2s; ., Q2s^T C22 Q2s],   Qks = columns 32 s .. of Q_k,
    //    three 32x32 blocks, each two chained MFMA products (32x64x64, then 32x32x64); ba mirrors ab.
    //    Gram-space matrices of a call whose updates run as launches of their own (one C buffer, m.CT2 == m.CT):
    //    C is up to date, the pair's block as it is.
    const bool fresh = m.gs && (st_fresh == step + 1 || m.CT2 == m.CT);
    if (m.gs && tid == 0) m.state[(step & 1) ? ST_QTICK_ODD : ST_QTICK] = step + 1;
    for (int e = tid; e < QSZ; e += NT) {
        const int i = e >> 6, j = e & 63;
        Qs[0][i * ELD + mem_col(home_slot(j))] = (i == j) ? 1.0f : 0.0f;
    }
    if (tid < PR) {
        ref[tid] = m.gs ? m.cref[tid < BS ? bi * BS + tid : bj * BS + tid - BS] : 0.0f;
        ref0[tid] = m.gs ? m.cref0[tid < BS ? bi * BS + tid : bj * BS + tid - BS] : 0.0f;
    }
    if (!m.gs) {
        // one 16-byte piece of the matrix per thread; the quadrant of rows 32.. x columns ..31 is not in the partial
        // matrices: it mirrors the one across
        static_assert(NT * 4 == QSZ, "one float4 of the pair's Gram matrix per thread");
        const int i = tid >> 4, j4 = (tid & 15) * 4;
        if (i < BS || j4 >= BS) {
            const float* g = m.gram + (size_t)wk.a * m.nchp * QSZ + i * PR + j4;
            floatx4 sum = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 4
            for (int c = 0; c < m.nchp; ++c) sum += *(const floatx4*)(g + (size_t)c * QSZ);
            const int si = home_slot(i);
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int sj = home_slot(j4 + x);
                As[0][si * ELD + mem_col(sj)] = sum[x];
                if (i < BS && j4 >= BS) As[0][sj * ELD + mem_col(si)] = sum[x];
            }
        }
    } else if (fresh) {
        const float* C = c_of_parity(m, step);
        for (int e = tid; e < QSZ; e += NT) {
            const int i = e >> 6, j = e & 63;
            const int gi = i < BS ? bi * BS + i : bj * BS + i - BS;
            const int gj = j < BS ? bi * BS + j : bj * BS + j - BS;
            As[0][home_slot(i) * ELD + mem_col(home_slot(j))] = C[(size_t)gi * m.ldc + gj];
        }
    } else {
        const int pp = (step - 1) & 1;
        const float* C = c_of_parity(m, pp);
        const int k1 = pdw[PD_K1], k2 = pdw[PD_K2], s1 = pdw[PD_S1], s2 = pdw[PD_S2];
        const int x0 = pdw[PD_X0], x1 = pdw[PD_X1], y0 = pdw[PD_Y0], y1 = pdw[PD_Y1];
        // aa and bb: the pair problems of the previous tick left the two diagonal 32 x 32 blocks of their rotated
        // matrices behind (m.DB, step 4): two entries per thread, requested before the operands of ab
        float dv[2 * BS * BS / NT];
#pragma unroll
        for (int q = 0; q < 2 * BS * BS / NT; ++q) {
            const int e = tid + NT * q, blk = e >> 10;
            dv[q] = m.DB[(((size_t)pp * m.npairs + (blk ? k2 : k1)) * 2 + (blk ? s2 : s1)) * (BS * BS) + (e & (BS * BS - 1))];
        }
        // ab = Q1s^T C12 Q2s, two chained products in 16 x 16 tiles (v_mfma_f32_16x16x4f32: lane l holds A[l & 15][g]
        // and B[g][l & 15], g = l >> 4, and four results D[4 g + v][l & 15]), eight waves for the first, four for the
        // second, 16 instructions each.  Every operand is read along its contraction index k, 16 bytes at a time: lane
        // (., g) takes k = 16 u + 4 g + x, u, x = 0 .. 3, and instruction (u, x) contracts its four values of g.  The
        // rotations come from their transposed copies (m.QT: entry (row, k) at ((k / 4) * 64 + row) * 4 + k % 4, so that
        // lanes of consecutive rows read consecutive 16-byte pieces), the tile of C through its mirror image (C is
        // symmetric up to the rounding of its updates, which step 2 evens out anyway).
        const float* Q1 = m.QT + ((size_t)pp * m.npairs + k1) * QSZ;
        const float* Q2 = m.QT + ((size_t)pp * m.npairs + k2) * QSZ;
        const int g = lane >> 4, l16 = lane & 15;
        const int ti = (wave >> 2) & 1, tj = wave & 3;           // tile of the first product (waves 0 .. 7)
        float* P = As[1];                                        // the 32 x 64 intermediate, row stride ELD
        floatx4 qa[4], cb[4], qb[4];
        if (wave < 8) {
            const float* qlp = Q1 + (g * PR + s1 * BS + ti * 16 + l16) * 4;
            // column tj * 16 + l16 of the tile: in block y0 or y1; its rows 16 u + 4 g ..: in block x0 (u < 2) or x1
            const int j = tj * 16 + l16;
            const float* clp = C + (size_t)((j < BS ? y0 : y1) * BS + (j & (BS - 1))) * m.ldc + 4 * g;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                qa[u] = *(const floatx4*)(qlp + 16 * PR * u);
                cb[u] = *(const floatx4*)(clp + (u < 2 ? x0 : x1) * BS + 16 * (u & 1));
            }
        }
        if (wave < 4) {                                          // tile (wave >> 1, wave & 1) of the second product
            const float* qrp = Q2 + (g * PR + s2 * BS + (wave & 1) * 16 + l16) * 4;
#pragma unroll
            for (int u = 0; u < 4; ++u) qb[u] = *(const floatx4*)(qrp + 16 * PR * u);
        }
        if (wave < 8) {
            floatx4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int x = 0; x < 4; ++x) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[u][x], cb[u][x], acc, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 4; ++v) P[(ti * 16 + 4 * g + v) * ELD + tj * 16 + l16] = acc[v];
        }
#pragma unroll
        for (int q = 0; q < 2 * BS * BS / NT; ++q) {
            const int e = tid + NT * q, blk = e >> 10, i = (e >> 5) & (BS - 1), j = e & (BS - 1);
            As[0][home_slot(blk * BS + i) * ELD + mem_col(home_slot(blk * BS + j))] = dv[q];
        }
        __syncthreads();
        if (wave < 4) {
            const int t2i = wave >> 1, t2j = wave & 1;
            floatx4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
            const float* pr = P + (t2i * 16 + l16) * ELD + 4 * g;
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int x = 0; x < 4; ++x) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(pr[16 * u + x], qb[u][x], acc, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int si = home_slot(t2i * 16 + 4 * g + v), sj = home_slot(BS + t2j * 16 + l16);
                As[0][si * ELD + mem_col(sj)] = acc[v];
                As[0][sj * ELD + mem_col(si)] = acc[v];
            }
        }
    }
    __syncthreads();
    // 2. symmetrise (the two triangles were accumulated in different orders) and, in the same pass, the
    //    largest |cos| between two rows of the pair before rotating (rows at the rounding floor are
    //    measured against the floor instead of their own length) and the largest squared norm
    const float z2 = ZERO_REL * __int_as_float(m.state[ST_SCALE]);
    if (tid < PR) {
        const int sl = home_slot(tid);
        const float d = As[0][sl * ELD + mem_col(sl)];
        const bool out = m.gs && d < GS_RELIABLE * ref[tid];
        sits_out[sl] = out;
        // 1 / length of the row, 0 for a row without one (nothing is measured against it)
        rlen[sl] = d > 0.0f ? __builtin_amdgcn_rsqf(d) : 0.0f;
        // (rows at the rounding floor of the data are not waiting for anything: they are finished)
        if (out && ref[tid] > z2) atomicMax(&m.state[ST_SAT_OUT], 1);
    }
    if (tid == PR) { entry_bits[0] = 0u; entry_bits[1] = 0u; }
    __syncthreads();
    float2 entry;
    {
        // The 2016 slot pairs i < j, two per thread: row c of the strict upper triangle (63 - c entries) and row
        // 63 - c (c entries) together make one line of 63.
        float mx = 0.0f;
        const float floor_inv = __builtin_amdgcn_rcpf(z2);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int e = tid + NT * q;
            if (e < 63 * 32) {
                const int c = e / 63, pos = e - 63 * c;
                const int i = pos < 63 - c ? c : 63 - c;
                const int js = pos < 63 - c ? c + 1 + pos : pos + 1;     // (63 - c) + 1 + (pos - (63 - c))
                float* upper = &As[0][i * ELD + mem_col(js)];
                float* lower = &As[0][js * ELD + mem_col(i)];
                // a row that sits out is cut loose: no rotation touches it, nothing is measured against it
                const float v = (sits_out[i] | sits_out[js]) ? 0.0f : 0.5f * (*upper + *lower);
                *upper = v;
                *lower = v;
                mx = fmaxf(mx, fabsf(v) * fminf(rlen[i] * rlen[js], floor_inv));
            }
        }
        float dmax = tid < PR ? fmaxf(As[0][tid * ELD + mem_col(tid)], 0.0f) : 0.0f;
        for (int o = 32; o > 0; o >>= 1) {
            mx = fmaxf(mx, __shfl_down(mx, o));
            dmax = fmaxf(dmax, __shfl_down(dmax, o));
        }
        // (non-negative floats compare like their bit patterns)
        if (lane == 0) {
            atomicMax(&entry_bits[0], __float_as_uint(mx));
            if (wave == 0) atomicMax(&entry_bits[1], __float_as_uint(dmax));
        }
        __syncthreads();
        entry = make_float2(__uint_as_float(entry_bits[0]), __uint_as_float(entry_bits[1]));
    }
    if (tid == 0) {
        // (Gram space: the pairs of the last ticks of the sweep are the heaviest of that moment, see GS_WINDOW)
        if (!m.gs || cyclic || round >= m.R - GS_WINDOW) atomicMax((unsigned int*)&m.state[ST_OFFMAX], __float_as_uint(entry.x));
        atomicMax((unsigned int*)&m.state[ST_SCALE_NEXT], __float_as_uint(entry.y));
    }

    // 3. Jacobi sweeps.
    const int b = tid & 31, grp = tid >> 5;
    int cur = 0;
    int inner_done = 0;
    const bool leave = !m.gs && entry.x <= DS_LEAVE * stop_cosine;
    if (entry.x > 0.0f && !leave) {
        // inner target: a fixed factor below what came in is enough for the outer iteration
        const float inner_stop = fmaxf(2e-7f, inner_reduction * entry.x);
        // One step of a round inside the blocks: read buffer X, rotate, write buffer Y with the positions advanced.
        // Thread (b, g): pair b of the columns, pair g of the rows of A, rows 2g and 2g + 1 of Q; its two outputs per
        // row go to the columns of the positions next(2b), next(2b + 1).  Written as a lambda and called with the
        // buffers swapped so that every LDS address is loop-invariant.
        const int rc0 = within_col(2 * b), rc1 = within_col(2 * b + 1);
        const int wc0 = within_col(next_within(2 * b)), wc1 = within_col(next_within(2 * b + 1));
        const int rr0 = within_row(2 * grp) * ELD, rr1 = within_row(2 * grp + 1) * ELD;
        const int wr0 = within_row(next_within(2 * grp)) * ELD, wr1 = within_row(next_within(2 * grp + 1)) * ELD;
        const int dr0 = within_row(2 * b) * ELD, dr1 = within_row(2 * b + 1) * ELD;
        auto within_step = [&](const float* X, float* Y, const float* XQ, float* YQ) {
            // issue every LDS read of the step first; the rotation arithmetic overlaps their latency
            const float x00 = X[rr0 + rc0], x01 = X[rr0 + rc1], x10 = X[rr1 + rc0], x11 = X[rr1 + rc1];
            float xq[QR_PER][2];
#pragma unroll
            for (int e = 0; e < QR_PER; ++e) {
                const int i = grp * QR_PER + e;
                xq[e][0] = XQ[i * ELD + rc0];
                xq[e][1] = XQ[i * ELD + rc1];
            }
            // every lane computes the rotation of its own column pair b (both halves of the wave
            // redundantly); the rotation of the row pair is fetched from the lane of this half-wave
            // that owns it
            const float2 pb = rotation_of(X[dr0 + rc0], X[dr0 + rc1], X[dr1 + rc1], z2);
            const int from = ((lane & 32) | grp) << 2;
            const float2 pa = make_float2(__int_as_float(__builtin_amdgcn_ds_bpermute(from, __float_as_int(pb.x))),
                                          __int_as_float(__builtin_amdgcn_ds_bpermute(from, __float_as_int(pb.y))));
            const float y00 = pa.x * x00 - pa.y * x10, y01 = pa.x * x01 - pa.y * x11;
            const float y10 = pa.y * x00 + pa.x * x10, y11 = pa.y * x01 + pa.x * x11;
            Y[wr0 + wc0] = pb.x * y00 - pb.y * y01;
            Y[wr0 + wc1] = pb.y * y00 + pb.x * y01;
            Y[wr1 + wc0] = pb.x * y10 - pb.y * y11;
            Y[wr1 + wc1] = pb.y * y10 + pb.x * y11;
#pragma unroll
            for (int e = 0; e < QR_PER; ++e) {
                const int i = grp * QR_PER + e;
                const float x = xq[e][0], y = xq[e][1];
                YQ[i * ELD + wc0] = pb.x * x - pb.y * y;
                YQ[i * ELD + wc1] = pb.y * x + pb.x * y;
            }
            __syncthreads();
        };
        // A cross round keeps the matrix in registers for its 32 steps, and only one triangle of it.  The 32 x 32 grid of
        // 2x2 blocks (row pair a, column pair b) is cut into its circulant diagonals g = (a - b) mod 32; block (b, a) is
        // the mirror image of (a, b), so the diagonals 0 .. 16 hold everything.  Waves 0 .. 8 (thread groups 0 .. 17 of
        // 32 lanes) carry them: thread b of group g holds block ((b + g) mod 32, b) -- its lanes touch 32 different LDS
        // banks -- and group 17 repeats group 16 value for value (diagonal 16 is its own mirror image and holds every
        // block twice, once from either side).  Waves 9 .. 15 carry Q: a lane holds, of three (waves 9, 10) or two
        // rows, the entries in the slot pairs 2j and 2j + 1, j = lane mod 16.
        // The even slots stay and the odd slots move on by one pair per step.  After the rotation the new block (a, b)
        // keeps its entry (even, even) and takes (even, odd) from block (a, b - 1), (odd, even) from (a - 1, b) and
        // (odd, odd) from (a - 1, b - 1): the last is a lane of the same group (lane permute), the other two go through
        // LDS -- from the diagonals g + 1 and g - 1, where for g = 0 the second is the mirror image of the first and
        // for g = 16 the first is a mirror image from diagonal 15.  In Q the odd entry of pair 2j moves to pair 2j + 1
        // of the same lane and that of pair 2j + 1 to the next lane of the row of 16, a data-parallel move inside the
        // vector unit: no LDS traffic but the rotations.
        // The rotations of the next step are computed before the step's barrier by group 1 alone: its entry (even, odd)
        // is the off-diagonal entry of the next slot pair b + 1, whose diagonal entries are what this step's rotations
        // of pairs b + 1 and b leave behind (closed form, carried in rotd).  Everybody waits for that wave at the
        // barrier, so it reads the two diagonal entries together with the rotations and computes the new rotation as
        // soon as its off-diagonal entry is there.
        // Measured on one workgroup, cycles per step: 760 with every thread holding a block of the full matrix and two
        // rows of Q (24 multiply-adds and 3 lane permutes through LDS per thread); 700 with the roles; 650 with Q's
        // moves in the vector unit; 610 with the early reads.  Without the rotation arithmetic it would be 465.
        auto cross_sweep = [&](float* A0, float* Q0, float* EX) {
            // (scalar branches: every role passes the same 34 barriers, and a wave runs exactly one role)
            const int role = __builtin_amdgcn_readfirstlane(wave);
            if (role <= 8) {
                const int g = min(grp, 16);
                const int ar = (b + g) & 31;
                float x00 = A0[(2 * ar) * ELD + b],     x01 = A0[(2 * ar) * ELD + 32 + b];
                float x10 = A0[(2 * ar + 1) * ELD + b], x11 = A0[(2 * ar + 1) * ELD + 32 + b];
                if (grp == 0) {                                  // (a = b: the diagonal blocks)
                    const float4 r = rotation_and_diagonal(x00, x01, x11, z2);
                    rotc[0][b] = make_float2(r.x, r.y);
                    rotd[0][b] = make_float2(r.z, r.w);
                }
                __syncthreads();
                // exchange buffer of a step: [0, 1024) the entries (even, odd) that the blocks hand on, [1024, 2048) the
                // entries (odd, even), both indexed by block
                const int left = ((lane & 32) | ((b + 31) & 31)) << 2;  // the lane of column pair b - 1 in this group
                const int bl = (b + 31) & 31, al = (ar + 31) & 31;
                const int own = ar * 32 + b;
                const int from01 = g == 16 ? 1024 + bl * 32 + ar : ar * 32 + bl;      // (a, b - 1), or its mirror image (b - 1, a)
                const int from10 = g == 0 ? ar * 32 + bl : 1024 + al * 32 + b;        // (a - 1, b), or its mirror image (b, a - 1)
                // (two steps per trip: with the parity a constant every LDS address of a step is a loop invariant plus
                // an immediate offset)
                auto step_of_parity = [&](const int p, auto lead_tag) {
                    constexpr bool lead = decltype(lead_tag)::value;
                    const float2 ra = rotc[p][ar], rb = rotc[p][b];
                    float dpa = 0.0f, dqb = 0.0f;
                    if (lead) {
                        dpa = rotd[p][ar].x;
                        dqb = rotd[p][b].y;
                        asm volatile("" : "+v"(dpa), "+v"(dqb)); // (keeps the two reads up here, beside the rotations')
                    }
                    const float y00 = ra.x * x00 - ra.y * x10, y01 = ra.x * x01 - ra.y * x11;
                    const float y10 = ra.y * x00 + ra.x * x10, y11 = ra.y * x01 + ra.x * x11;
                    const float o01 = rb.y * y00 + rb.x * y01, o10 = rb.x * y10 - rb.y * y11, o11 = rb.y * y10 + rb.x * y11;
                    x00 = rb.x * y00 - rb.y * y01;
                    float* ex = EX + p * 2048;
                    ex[own] = o01;
                    ex[1024 + own] = o10;
                    x11 = __int_as_float(__builtin_amdgcn_ds_bpermute(left, __float_as_int(o11)));
                    if (lead && grp == 1) {                      // (a = b + 1)
                        const float2 r = rotation_of_select(dpa, o01, dqb, z2);
                        const float cc = r.x * r.x, ss = r.y * r.y, cs2 = 2.0f * r.x * r.y * o01;
                        rotc[p ^ 1][ar] = r;
                        rotd[p ^ 1][ar] = make_float2(fmaf(cc, dpa, fmaf(ss, dqb, -cs2)), fmaf(ss, dpa, fmaf(cc, dqb, cs2)));
                    }
                    __syncthreads();
                    x01 = ex[from01];
                    x10 = ex[from10];
                };
                if (role == 0) {
                    for (int t = 0; t < 32; t += 2) {
                        step_of_parity(0, std::true_type{});
                        step_of_parity(1, std::true_type{});
                    }
                } else {
                    for (int t = 0; t < 32; t += 2) {
                        step_of_parity(0, std::false_type{});
                        step_of_parity(1, std::false_type{});
                    }
                }
                // 32 steps: every index is back in its slot.  Both triangles go back to LDS.
                A0[(2 * ar) * ELD + b] = x00;     A0[(2 * ar) * ELD + 32 + b] = x01;
                A0[(2 * ar + 1) * ELD + b] = x10; A0[(2 * ar + 1) * ELD + 32 + b] = x11;
                if (g >= 1 && g <= 15) {
                    A0[(2 * b) * ELD + ar] = x00;     A0[(2 * b) * ELD + 32 + ar] = x10;
                    A0[(2 * b + 1) * ELD + ar] = x01; A0[(2 * b + 1) * ELD + 32 + ar] = x11;
                }
                __syncthreads();
            } else {
                auto rows_of_q = [&](auto n_tag) {
                    constexpr int NR = decltype(n_tag)::value;
                    const int j = lane & 15, rsub = lane >> 4;
                    const int row0 = NR == 3 ? (role - 9) * 12 + rsub * 3 : 24 + (role - 11) * 8 + rsub * 2;
                    float e0[NR], o0[NR], e1[NR], o1[NR];
#pragma unroll
                    for (int e = 0; e < NR; ++e) {
                        const float* q = Q0 + (row0 + e) * ELD;
                        e0[e] = q[2 * j];
                        e1[e] = q[2 * j + 1];
                        o0[e] = q[32 + 2 * j];
                        o1[e] = q[32 + 2 * j + 1];
                    }
                    __syncthreads();
                    auto step_of_parity = [&](const int p) {
                        const float4 r = *(const float4*)&rotc[p][2 * j];       // (c, s) of the pairs 2j and 2j + 1
#pragma unroll
                        for (int e = 0; e < NR; ++e) {
                            const float t0 = r.y * e0[e] + r.x * o0[e], t1 = r.w * e1[e] + r.z * o1[e];
                            e0[e] = r.x * e0[e] - r.y * o0[e];
                            e1[e] = r.z * e1[e] - r.w * o1[e];
                            o1[e] = t0;
                            // row_ror:1 -- every lane takes the value of the lane before it in its row of 16, lane 0 that of lane 15
                            o0[e] = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(t1), 0x121, 0xf, 0xf, false));
                        }
                        __syncthreads();
                    };
                    for (int t = 0; t < 32; t += 2) {
                        step_of_parity(0);
                        step_of_parity(1);
                    }
#pragma unroll
                    for (int e = 0; e < NR; ++e) {
                        float* q = Q0 + (row0 + e) * ELD;
                        q[2 * j] = e0[e];
                        q[2 * j + 1] = e1[e];
                        q[32 + 2 * j] = o0[e];
                        q[32 + 2 * j + 1] = o1[e];
                    }
                    __syncthreads();
                };
                if (role <= 10) rows_of_q(std::integral_constant<int, 3>{});
                else rows_of_q(std::integral_constant<int, 2>{});
            }
        };
        static_assert(NT == 1024 && PR == 64, "the roles of a cross round: 18 groups for one triangle of A, 2 x 12 + 5 x 8 rows of Q");
        static_assert(2 * 2 * 1024 <= PR * ELD, "the exchange buffers of a cross round fit the idle copy of the matrix");
        for (int isw = 0; isw < max_inner; ++isw) {
            if (!cross) {
                // a full round rotates the 2 x 496 index pairs inside the two blocks first: 31 steps through LDS, the last
                // one into the other buffer
                float* A0 = As[cur];
                float* A1 = As[cur ^ 1];
                float* Q0 = Qs[cur];
                float* Q1 = Qs[cur ^ 1];
                for (int t = 0; t < 30; t += 2) {
                    within_step(A0, A1, Q0, Q1);
                    within_step(A1, A0, Q1, Q0);
                }
                within_step(A0, A1, Q0, Q1);
                cur ^= 1;
            }
            // the 1024 pairs that couple the blocks
            cross_sweep(As[cur], Qs[cur], As[cur ^ 1]);
            ++inner_done;
            if (isw + 1 < max_inner) {
                const float2 now = max_cosine(As[cur], z2, red);
                if (now.x <= inner_stop) break;
            }
        }
    }
    const float* Acur = As[cur];
    const float* Qc = Qs[cur];                                   // Q, columns in slot order
    float* F0 = As[cur ^ 1];                                     // scratch for the Newton-Schulz factor
    // memory column of natural column j of Q
    auto qcol = [&](int j) { return mem_col(home_slot(j)); };

    // 4. eigenvalues, and where each eigenvector goes: decreasing eigenvalue over the live rows of
    //    the pair, padding rows stay padding rows
    const int nI = max(0, min(BS, m.r - bi * BS)), nJ = max(0, min(BS, m.r - bj * BS));
    if (tid < PR) {
        const bool live = tid < BS ? tid < nI : tid - BS < nJ;
        const int sl = home_slot(tid);
        ev[tid] = live ? Acur[sl * ELD + mem_col(sl)] : -FLT_MAX;
    }
    __syncthreads();
    {
        constexpr int PER_WAVE = PR / (NT / 64);                 // every wave ranks a few eigenvalues by ballot
        const float other = ev[lane];
#pragma unroll
        for (int q = 0; q < PER_WAVE; ++q) {
            const int i = wave * PER_WAVE + q;
            const float mine = ev[i];
            const int rank = __popcll(__ballot((other > mine) || (other == mine && lane < i)));
            if (lane == 0) {
                int slot;
                if (rank < nI) slot = rank;
                else if (rank < nI + nJ) slot = BS + rank - nI;
                else {
                    const int pad = rank - nI - nJ;              // padding rows, in order
                    slot = pad < BS - nI ? nI + pad : BS + nJ + pad - (BS - nI);
                }
                dest[i] = slot;
            }
        }
    }

    // Gram space: the reference values follow the rows, ref'_j = sum_i Q_ij^2 ref_i
    __syncthreads();                                             // dest[] is complete
    // Gram space: the two diagonal 32 x 32 blocks of the rotated matrix, rows and columns in their new order, for the
    // pair problems of the next tick (they would otherwise have to form them from C, which is one tick behind)
    if (m.gs && m.DB) {
        float* db = m.DB + ((size_t)(step & 1) * m.npairs + wk.a) * (2 * BS * BS);
#pragma unroll
        for (int q = 0; q < QSZ / NT; ++q) {
            const int e = tid + NT * q, ti = e >> 6, tj = e & 63;
            const int di = dest[ti], dj = dest[tj];
            if ((di ^ dj) < BS)                                  // both in the same block
                db[(di >> 5) * (BS * BS) + (di & (BS - 1)) * BS + (dj & (BS - 1))] = Acur[home_slot(ti) * ELD + mem_col(home_slot(tj))];
        }
    }
    if (!m.gs) {
        // a pair that was left alone and whose rows are in order needs no row update
        const bool in_place = leave && (tid >= PR || dest[tid] == tid);
        const int all_in_place = __syncthreads_and(in_place);
        if (tid == 0) {
            m.idle[wk.a] = all_in_place;
            // work counter: row updates that svd_rowgram will execute for this pair, in tiles of 64 rows x 64 columns
            if (!all_in_place) atomicAdd(&flags[FLAG_DS_UPDATE_UNITS], m.ldw / 64);
        }
    }
    if (m.gs && tid < PR) {
        const int cj = qcol(tid);
        float r = 0.0f, r0 = 0.0f;
#pragma unroll 8
        for (int i = 0; i < PR; ++i) {
            const float q = Qc[i * ELD + cj];
            r = fmaf(q * q, ref[i], r);
            r0 = fmaf(q * q, ref0[i], r0);
        }
        const int d = dest[tid];
        const int grow = d < BS ? bi * BS + d : bj * BS + d - BS;
        m.cref[grow] = r;
        // the scale of the row for the block weights that the two-sided update forms (rows that are not rotated: 0)
        m.cref0[grow] = r0;
        m.dd[(size_t)(step & 1) * m.rows_alloc + grow] = (ev[tid] > z2 && !sits_out[home_slot(tid)]) ? r0 : 0.0f;
    }

    // 5. one Newton-Schulz step  Q <- Q (1.5 I - 0.5 Q^T Q): removes the drift that thousands of
    //    fp32 rotations leave in the orthogonality of Q.  Every wave owns one 16x16 tile of the 64x64 result
    //    (v_mfma_f32_16x16x4f32: lane l holds A[l & 15][l >> 4] and B[l >> 4][l & 15], and four results
    //    C[4 (l >> 4) + v][l & 15]).
    {
        const int ti = wave >> 2, tj = wave & 3, lo = lane & 15, hi = lane >> 4;
        floatx4 t4 = {0.0f, 0.0f, 0.0f, 0.0f};
        const int ci = qcol(ti * 16 + lo), cj = qcol(tj * 16 + lo);
#pragma unroll
        for (int k = 0; k < PR; k += 4) {
            const float a = Qc[(k + hi) * ELD + ci];             // (Q^T)[i][k]
            const float bq = Qc[(k + hi) * ELD + cj];            // Q[k][j]
            t4 = __builtin_amdgcn_mfma_f32_16x16x4f32(a, bq, t4, 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = ti * 16 + 4 * hi + v, j = tj * 16 + lo;
            F0[i * ELD + j] = (i == j ? 1.5f : 0.0f) - 0.5f * t4[v];
        }
        __syncthreads();
        floatx4 q4 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int k = 0; k < PR; k += 4) {
            const float a = Qc[(ti * 16 + lo) * ELD + qcol(k + hi)];   // Q[i][k]
            const float bq = F0[(k + hi) * ELD + tj * 16 + lo];        // F[k][j]
            q4 = __builtin_amdgcn_mfma_f32_16x16x4f32(a, bq, q4, 0, 0, 0);
        }
        // 6. write Q with its columns permuted to their destination rows.  Gram-space matrices: only the transposed
        //    copy, which the two-sided update and the pair problems of the next tick (step 1) read; data-space
        //    matrices: Q itself, for svd_rowgram.
        const int dj = dest[tj * 16 + lo];
        if (m.gs) {
            *(floatx4*)(m.QT + ((size_t)(step & 1) * m.npairs + wk.a) * QSZ + ((ti * 4 + hi) * PR + dj) * 4) = q4;
        } else {
            float* qout = m.Q + (size_t)wk.a * QSZ;
#pragma unroll
            for (int v = 0; v < 4; ++v) qout[(ti * 16 + 4 * hi + v) * PR + dj] = q4[v];
        }
    }

    if (tid == 0) {
        atomicAdd(&flags[FLAG_EIG_VISITS], 1);
        atomicAdd(&flags[FLAG_EIG_INNER], inner_done * (cross ? 32 : 63));
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
            if (m.gs) {
                // Gram space: diagonal to the threshold (or out of sweeps) -> apply the rotations to the
                // data and look at a fresh Gram matrix at the next tick
                const bool waiting = atomicAdd(&m.state[ST_SAT_OUT], 0) != 0;
                // convergence is quadratic: a sweep that started below ten times the threshold has ended well below
                // it, which the fresh Gram matrix then confirms (or the sweeps go on)
                const float resolved = fmaxf(10.0f * stop_cosine, __int_as_float(m.state[ST_NOISE]));
                // (a call that goes by the history of the calls before it has no refresh launches at the first sweep
                // boundaries: the matrix sweeps on until there are)
                if (((worst < resolved || waiting) && sweeps >= ask_from) || sweeps >= max_sweeps) {
                    m.state[ST_MODE] = MODE_NEED_REFRESH;
                    if (m.state[ST_FIRST_ASK] == 0) m.state[ST_FIRST_ASK] = sweeps;
                }
                if (waiting && m.state[ST_CYCLIC_FROM] == 0) m.state[ST_CYCLIC_FROM] = step + 2;
                m.state[ST_SAT_OUT] = 0;
            } else if (worst < stop_cosine) {
                m.state[ST_DONE_AT] = step + 1;
            } else if (m.R >= DS_VERIFY_MIN_R && worst < DS_VERIFY * stop_cosine) {
                m.state[ST_VERIFY] = 1;                          // svd_ds_verify decides at the sweep boundary
            } else if (sweeps >= max_sweeps) {
                atomicMax(&flags[FLAG_NOCONV], 1);
            }
            m.state[ST_OFFMAX] = 0;
            m.state[ST_ARRIVE] = 0;
            const unsigned int grown = atomicAdd((unsigned int*)&m.state[ST_SCALE_NEXT], 0u);
            if (grown > (unsigned int)m.state[ST_SCALE]) m.state[ST_SCALE] = (int)grown;
        }
    }
}

}  // namespace


void launch_svd_eig(const SvdMat* d_mats, const Work* d_work, int n_items, const Work* d_two_work, int n_two,
                    const Work* d_plan_work, int n_plan, int cyclic, int step, int max_sweeps, int ask_from,
                    float stop_cosine, int max_inner, float inner_reduction, int full_period, int fresh_only,
                    int* d_flags, hipStream_t stream)
{
    static_assert(PR * ELD == PR * TLD, "the two-sided tiles are staged in the LDS arrays of the pair problem");
    static_assert((MAX_R / BS) * (MAX_R / BS) <= PR * ELD, "the block weights are staged in an LDS array of the pair problem");
    static_assert((MAX_R / BS) * (MAX_R / BS) % NT == 0 && MAX_R / BS <= 64, "candidate pairs per thread, block mask");
    const unsigned grid = (unsigned)(n_items + (n_two + TILES_PER_WG - 1) / TILES_PER_WG + n_plan);
    if (grid == 0) return;
    // A compute unit has room for two of these workgroups.  While the chip has a unit for every workgroup of
    // the launch, unused dynamic LDS keeps them apart: a pair problem is a latency chain and runs slower
    // when it shares its SIMDs.
    const size_t pad = n_items <= 200 ? 20 * 1024 : 0;
    svd_eig<<<grid, NT, pad, stream>>>(d_mats, d_work, n_items, d_two_work, n_two, d_plan_work, cyclic, step, max_sweeps,
                                     ask_from, stop_cosine, max_inner, inner_reduction, full_period, fresh_only, d_flags);
}

}  // namespace svd
}  // namespace atomo
