// Spectral-ATOMO (Section 5), matrices whose shorter side has at most 32 vectors ("thin": the
// [x*y/2, 2*k*k] reshape of Section 6 gives 18 columns for every 3x3 convolution, 2 for 1x1).
//
// The r <= 32 vectors x_c (columns of a tall G, rows of a wide one) have M entries ("positions").
// The whole Jacobi problem is one r x r eigenproblem, so a pass over the data is
//     thin_gram : B <- B * Q  (32 positions x r per wave and step, fp32 MFMA), written back in place, and in the
//                 same pass the partial Gram matrices  C = B^T B  of 1024-position chunks (MFMA, the 16 result
//                 registers of the first product are the operands of the second as they are)
//     thin_eig  : one workgroup per matrix: sums the partials, tests the cosines |C_ij| / sqrt(C_ii C_jj)
//                 measured on the data; if they are not below the threshold, diagonalises C by two-sided
//                 Jacobi (in LDS, to convergence) -> Q for the next pass, V <- V * Q
// Pass 0 reads G and only forms C (Q = I); pass 1 reads G and writes B = 2^-e G Q; later passes update B in
// place.  (A G that is not position-major and contiguous - vectors along rows, or padded rows - is first copied
// into B in that layout, thin_prepare, and the passes read the copy.)  Because every Q after the first is close to the identity, small columns are updated with small
// relative error, which an accumulated V applied to G could not give in fp32.  Two or three passes are the
// rule.  The kept atoms are then gathered from B (thin_pack); the short vectors are columns of V.
#include <cfloat>
#include <cmath>

#include "svd_common.h"

namespace atomo {
namespace svd {

namespace {

constexpr int XLD = THIN_R + 1;         // LDS row stride of a staged block (32 positions x 32 vectors)
constexpr int TNT = 512;                // threads of the streaming kernels
constexpr int TWAVES = TNT / 64;
constexpr int TSZ = THIN_R * THIN_R;

// Where lane `lane` starts in a block of 32 positions x r vectors stored position-major, and how it moves on
// when it advances by 64 elements.
struct Cursor {
    int pos, c, dq, dr;
};

__device__ inline Cursor cursor_for(int lane, int r)
{
    Cursor cu;
    cu.pos = lane / r;
    cu.c = lane % r;
    cu.dq = 64 / r;
    cu.dr = 64 % r;
    return cu;
}

__device__ inline void advance(Cursor& cu, int r)
{
    cu.c += cu.dr;
    cu.pos += cu.dq;
    if (cu.c >= r) {
        cu.c -= r;
        ++cu.pos;
    }
}

// One block = positions k0 .. k0 + 31 of a position-major source with row stride r: one contiguous run of 32 r
// floats; positions beyond M read as zero.
__device__ inline void load_block(float (&vals)[16], const float* __restrict__ src, int r, int M, int k0, int lane)
{
    const float* base = src + (long long)k0 * r;
    const int valid = min(32, M - k0) * r;
#pragma unroll
    for (int i = 0; i < 16; ++i) vals[i] = lane + 64 * i < valid ? base[lane + 64 * i] : 0.0f;
}

// The same elements into the wave's LDS block xs[position][vector], multiplied by `factor`.
__device__ inline void stage_block(float* xs, const float (&vals)[16], float factor, int r, Cursor cu)
{
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if (cu.pos < 32) xs[cu.pos * XLD + cu.c] = vals[i] * factor;
        advance(cu, r);
    }
}

struct Source {
    const float* p;
    float factor;
};

// Before the first rotation has been applied the data are X (G itself where G already is position-major and
// contiguous, else its copy in B), scaled by 2^-e on the fly; afterwards B.
__device__ inline Source source_of(const SvdMat& m, bool unrotated)
{
    Source s;
    const float* const x = m.X;
    const float* const b = m.B;
    s.p = unrotated ? x : b;
    s.factor = unrotated ? ldexpf(1.0f, -scale_exponent(m)) : 1.0f;
    return s;
}

__device__ inline void publish_absmax(const SvdMat& m, float mx, float* red)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_down(mx, o));
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < TWAVES; ++w) mx = fmaxf(mx, red[w]);
        if (mx > 0.0f && mx <= FLT_MAX) atomicMax((unsigned int*)&m.state[ST_ABSMAX], __float_as_uint(mx));
    }
}

// Largest |entry| of one chunk of a matrix that is used in place.
__global__ __launch_bounds__(TNT) void thin_absmax(const SvdMat* mats, const Work* work)
{
    __shared__ float red[TWAVES];
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    const long long lo = (long long)wk.a * m.tchunk * m.r;
    const long long hi = min((long long)m.M, (long long)(wk.a + 1) * m.tchunk) * m.r;
    float mx = 0.0f;
    const float* x = m.X + lo;
    const long long len = hi - lo;
    long long done = 0;
    if ((((size_t)x) & 15) == 0) {                                  // 16-byte loads, four in flight per thread
        const float4* x4 = (const float4*)x;
        const long long n4 = len / 4;
        for (long long q = threadIdx.x; q < n4; q += 4 * TNT) {
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = q + u * TNT < n4 ? x4[q + u * TNT] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int u = 0; u < 4; ++u)
                mx = fmaxf(fmaxf(mx, fmaxf(fabsf(v[u].x), fabsf(v[u].y))), fmaxf(fabsf(v[u].z), fabsf(v[u].w)));
        }
        done = n4 * 4;
    }
    for (long long e = done + threadIdx.x; e < len; e += TNT) mx = fmaxf(mx, fabsf(x[e]));
    publish_absmax(m, mx, red);
}

// Matrices that are not position-major and contiguous (vectors along rows, or padded rows): copy into B.
__global__ __launch_bounds__(TNT) void thin_prepare(const SvdMat* mats, const Work* work)
{
    __shared__ float red[TWAVES];
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    const int r = m.r;
    const long long lo = (long long)wk.a * m.tchunk * r;
    const long long hi = min((long long)m.M, (long long)(wk.a + 1) * m.tchunk) * r;
    float mx = 0.0f;
    for (long long e = lo + threadIdx.x; e < hi; e += TNT) {
        const long long k = e / r;
        const int c = (int)(e - k * r);
        const float v = m.transposed ? m.G[k * m.ldg + c] : m.G[c * m.ldg + k];
        m.B[e] = v;
        mx = fmaxf(mx, fabsf(v));
    }
    publish_absmax(m, mx, red);
}

// One chunk of positions of one matrix: B <- B * Q (pass >= 1) and the chunk's part of C = B^T B.
//   fp32 MFMA 32x32x2: A operand lane l = A[i = l % 32][k = l / 32], B operand lane l = B[k = l / 32][j = l % 32],
//   result register v of lane l = D[8 (v / 4) + 4 (l / 32) + v % 4][l % 32].
// For B^T B both operands of one instruction are the same register: lane l supplies entry (position of
// half l / 32, vector l % 32) of two positions, and which two positions an instruction takes does not matter
// for the sum.  Result register v of the first product holds exactly such a pair (positions 8 (v / 4) + v % 4
// and that + 4).
template <bool MATVEC>
__global__ __launch_bounds__(TNT, 4) void thin_gram(const SvdMat* mats, const Work* work, int pass)
{
    __shared__ float xs_all[TWAVES][THIN_R * XLD];
    __shared__ float qs[THIN_R * XLD];                              // the rotation, zero outside r x r
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    if (m.state[ST_MODE] == MODE_DONE) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, l32 = lane & 31;
    float* xs = xs_all[wave];
    const int r = m.r, M = m.M;
    const Source s = source_of(m, pass <= 1);
    const Cursor cu = cursor_for(lane, r);
    for (int e = lane; e < THIN_R * XLD; e += 64) xs[e] = 0.0f;     // vectors r .. 31 stay zero
    if (MATVEC)
        for (int e = tid; e < TSZ; e += TNT) qs[(e >> 5) * XLD + (e & 31)] = m.Q[TSZ + e];
    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    const int nit = m.tchunk / (32 * TWAVES);
    const int kbase = wk.a * m.tchunk;
    float vals[16];
    load_block(vals, s.p, r, M, kbase + 32 * wave, lane);
    for (int it = 0; it < nit; ++it) {
        const int k0 = kbase + 32 * (it * TWAVES + wave);
        stage_block(xs, vals, s.factor, r, cu);
        __syncthreads();
        if (it + 1 < nit) load_block(vals, s.p, r, M, k0 + 32 * TWAVES, lane);
        if (!MATVEC) {
#pragma unroll
            for (int t = 0; t < 16; ++t) {
                const float a = xs[(2 * t + h) * XLD + l32];
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, a, acc, 0, 0, 0);
            }
        } else {
            floatx16 d;
#pragma unroll
            for (int v = 0; v < 16; ++v) d[v] = 0.0f;
#pragma unroll
            for (int t = 0; t < 16; ++t)
                if (2 * t < r)
                    d = __builtin_amdgcn_mfma_f32_32x32x2f32(xs[l32 * XLD + 2 * t + h], qs[(2 * t + h) * XLD + l32], d, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 16; ++v) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(d[v], d[v], acc, 0, 0, 0);
            __syncthreads();
#pragma unroll
            for (int v = 0; v < 16; ++v) xs[(8 * (v >> 2) + 4 * h + (v & 3)) * XLD + l32] = d[v];
            __syncthreads();
            Cursor w = cu;
            float* out = m.B + (long long)k0 * r;
            const int valid = min(32, M - k0) * r;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (lane + 64 * i < valid) out[lane + 64 * i] = xs[w.pos * XLD + w.c];
                advance(w, r);
            }
        }
        __syncthreads();
    }
    // the eight waves' sums, added in a fixed order
    float* cs = &xs_all[0][0];
#pragma unroll
    for (int v = 0; v < 16; ++v) cs[wave * TSZ + (8 * (v >> 2) + 4 * h + (v & 3)) * THIN_R + l32] = acc[v];
    __syncthreads();
    for (int e = tid; e < TSZ; e += TNT) {
        float sum = 0.0f;
#pragma unroll
        for (int w = 0; w < TWAVES; ++w) sum += cs[w * TSZ + e];
        m.gram[(size_t)wk.a * TSZ + e] = sum;
    }
}

constexpr int ENT = 1024;               // threads of thin_eig: one per entry of a 32 x 32 matrix

__device__ inline float block_max(float x, float* red, int tid)
{
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = x;
    __syncthreads();
    float mx = red[0];
    for (int w = 1; w < ENT / 64; ++w) mx = fmaxf(mx, red[w]);
    return mx;
}

// One workgroup per thin matrix, after thin_gram of the same pass.
__global__ __launch_bounds__(ENT) void thin_eig(const SvdMat* mats, const Work* work, int pass, int last_pass,
                                                float stop_cosine, int* flags)
{
    __shared__ float A[THIN_R * XLD], Qs[THIN_R * XLD], T1[THIN_R * XLD], T2[THIN_R * XLD];
    __shared__ float red[ENT / 64];
    __shared__ unsigned short sched[(THIN_R - 1) * (THIN_R / 2)];   // column pair of (step, k): p | q << 8
    __shared__ float2 rot[THIN_R / 2];                              // (cos, sin) of the step's rotations
    const SvdMat m = mats[work[blockIdx.x].mat];
    if (m.state[ST_MODE] == MODE_DONE) return;
    const int tid = threadIdx.x, ei = tid >> 5, ej = tid & 31;      // this thread's entry of a 32 x 32 matrix
    const int r = m.r, n = r + (r & 1);

    // C = sum of the chunks' partial Gram matrices, in chunk order
    {
        // four interleaved running sums (chunks 0, 4, 8, ... in the first, and so on), added at the end: a fixed
        // order, and a shorter dependent chain than one sum
        float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
        for (int ch0 = 0; ch0 < m.nchg; ch0 += 32) {
            float part[32];
#pragma unroll
            for (int u = 0; u < 32; ++u) part[u] = ch0 + u < m.nchg ? m.gram[(size_t)(ch0 + u) * TSZ + tid] : 0.0f;
#pragma unroll
            for (int u = 0; u < 32; u += 4) {
                s0 += part[u];
                s1 += part[u + 1];
                s2 += part[u + 2];
                s3 += part[u + 3];
            }
        }
        const float sum = (s0 + s1) + (s2 + s3);
        A[ei * XLD + ej] = sum;
        Qs[ei * XLD + ej] = ei == ej ? 1.0f : 0.0f;
        if (tid < (n - 1) * (THIN_R / 2)) {
            int p = 0, q = 1;
            if ((tid & 15) < n / 2) pair_blocks(n, tid >> 4, tid & 15, p, q);
            sched[tid] = (unsigned short)(p | (q << 8));
        }
    }
    __syncthreads();
    float scale = 0.0f;
    for (int i = 0; i < r; ++i) scale = fmaxf(scale, A[i * XLD + i]);
    const float floor_sq = ZERO_REL * scale;                       // squared norms at or below this are rounding residue
    float worst = 0.0f;
    if (ei < ej && ej < r) {
        const float di = A[ei * XLD + ei], dj = A[ej * XLD + ej];
        if (di > floor_sq && dj > floor_sq) worst = fabsf(A[ei * XLD + ej]) * rsqrtf(di * dj);
    }
    worst = block_max(worst, red, tid);
    const bool done = worst < stop_cosine;
    if (done || pass == last_pass) {
        const int e = scale_exponent(m);
        if (tid < r) m.sig_raw[tid] = ldexpf(sqrtf(fmaxf(A[tid * XLD + tid], 0.0f)), e);
        if (pass == 0) m.Q[tid] = (ei == ej && ei < r) ? 1.0f : 0.0f;
        if (tid == 0) {
            m.state[ST_MODE] = MODE_DONE;
            m.state[ST_EXP] = e;
            atomicMax(&flags[FLAG_MAX_SWEEPS], pass);
            if (!done) atomicMax(&flags[FLAG_NOCONV], 1);
        }
        return;
    }

    // Two-sided Jacobi on the symmetric C (C <- J^T C J, Q <- Q J), round-robin pairing: n / 2 disjoint rotations
    // per step.  The cosine of a rotation is the cosine of the two data columns, the quantity the pass over the
    // data tests.  A step is two phases: thread k < n / 2 works out rotation k from C_pp, C_qq, C_pq; then one
    // thread per 2 x 2 block (rows of pair ka, columns of pair kb) applies both rotations to its block, and one
    // thread per (row, pair) rotates two entries of Q.  Every entry has one owner, which reads it before the
    // phase barrier and writes it after, so the update is in place.
    {
        const int n2 = n / 2;
        const bool blk = tid < n2 * n2;                             // owner of a 2 x 2 block of C
        const int ka = blk ? tid / n2 : 0, kb = blk ? tid % n2 : 0;
        const int t2 = tid - 256;
        const bool qit = t2 >= 0 && t2 < n * n2;                    // owner of two entries of a row of Q
        const int qi = qit ? t2 / n2 : 0, qk = qit ? t2 % n2 : 0;
        float sweep_worst = 0.0f;
        for (int sweep = 0; sweep < 10; ++sweep) {
            for (int step = 0; step < n - 1; ++step) {
                const unsigned short* sc = sched + step * (THIN_R / 2);
                float b00 = 0.0f, b01 = 0.0f, b10 = 0.0f, b11 = 0.0f, q0 = 0.0f, q1 = 0.0f;
                int pa = 0, qa = 0, pb = 0, qb = 0;
                if (blk) {
                    const int ea = sc[ka], eb = sc[kb];
                    pa = ea & 255; qa = ea >> 8; pb = eb & 255; qb = eb >> 8;
                    b00 = A[pa * XLD + pb]; b01 = A[pa * XLD + qb];
                    b10 = A[qa * XLD + pb]; b11 = A[qa * XLD + qb];
                } else if (qit) {
                    const int eb = sc[qk];
                    pb = eb & 255; qb = eb >> 8;
                    q0 = Qs[qi * XLD + pb]; q1 = Qs[qi * XLD + qb];
                }
                if (tid < n2) {
                    // here ka = 0, kb = tid: pb, qb are this rotation's columns
                    const float cpp = A[pb * XLD + pb], cqq = A[qb * XLD + qb], cpq = A[pb * XLD + qb];
                    bool rotate = cpp > floor_sq && cqq > floor_sq;
                    float cosv = 0.0f;
                    if (rotate) cosv = fabsf(cpq) * __builtin_amdgcn_rsqf(cpp * cqq);
                    rotate = rotate && cosv > 1.0e-7f;
                    // an error of a few ulp in the angle only changes which rotation is applied; (c, sn) stays a
                    // rotation to rounding because sn = c t with c = 1 / sqrt(1 + t^2)
                    float c = 1.0f, sn = 0.0f;
                    if (rotate) {
                        sweep_worst = fmaxf(sweep_worst, cosv);
                        const float zeta = (cqq - cpp) * __builtin_amdgcn_rcpf(2.0f * cpq);
                        const float t = copysignf(1.0f, zeta) *
                                        __builtin_amdgcn_rcpf(fabsf(zeta) + __builtin_amdgcn_sqrtf(fmaf(zeta, zeta, 1.0f)));
                        c = __builtin_amdgcn_rsqf(fmaf(t, t, 1.0f));
                        sn = c * t;
                    }
                    rot[tid] = make_float2(c, sn);
                }
                __syncthreads();
                if (blk) {
                    const float2 ra = rot[ka], rb = rot[kb];
                    // columns: [x, y] <- [c x - s y, s x + c y] with the rotation of pair kb
                    const float c00 = rb.x * b00 - rb.y * b01, c01 = rb.y * b00 + rb.x * b01;
                    const float c10 = rb.x * b10 - rb.y * b11, c11 = rb.y * b10 + rb.x * b11;
                    // rows, with the rotation of pair ka
                    A[pa * XLD + pb] = ra.x * c00 - ra.y * c10;
                    A[pa * XLD + qb] = ra.x * c01 - ra.y * c11;
                    A[qa * XLD + pb] = ra.y * c00 + ra.x * c10;
                    A[qa * XLD + qb] = ra.y * c01 + ra.x * c11;
                } else if (qit) {
                    const float2 rb = rot[qk];
                    Qs[qi * XLD + pb] = rb.x * q0 - rb.y * q1;
                    Qs[qi * XLD + qb] = rb.y * q0 + rb.x * q1;
                }
                __syncthreads();
            }
            // Jacobi converges quadratically: after a sweep whose largest cosine was below 1e-3 the columns are
            // orthogonal to about 1e-6, which the next pass over the data then measures
            const float w = block_max(sweep_worst, red, tid);
            sweep_worst = 0.0f;
            if (w < 1.0e-3f) break;
        }
    }
    __syncthreads();

    // one Newton-Schulz step keeps Q orthogonal to rounding:  Q <- Q (1.5 I - 0.5 Q^T Q)
    {
        float sum = 0.0f;
        for (int x = 0; x < THIN_R; ++x) sum = fmaf(Qs[x * XLD + ei], Qs[x * XLD + ej], sum);
        T1[ei * XLD + ej] = (ei == ej ? 1.5f : 0.0f) - 0.5f * sum;
        A[ei * XLD + ej] = pass == 0 ? (ei == ej ? 1.0f : 0.0f) : m.Q[tid];      // V so far
    }
    __syncthreads();
    {
        float sum = 0.0f;
        for (int x = 0; x < THIN_R; ++x) sum = fmaf(Qs[ei * XLD + x], T1[x * XLD + ej], sum);
        T2[ei * XLD + ej] = (ei < r && ej < r) ? sum : 0.0f;
    }
    __syncthreads();
    {
        float sum = 0.0f;
        for (int x = 0; x < THIN_R; ++x) sum = fmaf(A[ei * XLD + x], T2[x * XLD + ej], sum);
        m.Q[tid] = (ei < r && ej < r) ? sum : 0.0f;                // V <- V Q
        m.Q[TSZ + tid] = T2[ei * XLD + ej];                        // the rotation of the next pass
    }
    if (tid == 0) m.state[ST_SWEEPS] = pass + 1;
}

// Kept atoms of one chunk: the long vector of slot s is column src_row[s] of the data divided by its norm.
__global__ __launch_bounds__(TNT) void thin_pack(const SvdMat* mats, const Work* work)
{
    __shared__ float xs_all[TWAVES][THIN_R * XLD];
    __shared__ int col_of[THIN_R];
    __shared__ float inv_of[THIN_R], fold_of[THIN_R];
    const Work wk = work[blockIdx.x];
    const SvdMat m = mats[wk.mat];
    const int kept = min(*m.count, m.capacity);
    if (kept <= 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, l32 = lane & 31;
    float* xs = xs_all[wave];
    const int r = m.r, M = m.M;
    const Source s = source_of(m, m.state[ST_SWEEPS] == 0);
    const Cursor cu = cursor_for(lane, r);
    if (tid < kept) {
        col_of[tid] = m.src_row[tid];
        inv_of[tid] = m.src_inv[tid];
        fold_of[tid] = m.src_fold[tid];
    }
    float* const mu = m.U;
    float* const mv = m.V;
    float* long_out = m.transposed ? mu : mv;
    float* short_out = m.transposed ? mv : mu;
    const int nit = m.tchunk / (32 * TWAVES);
    for (int it = 0; it < nit; ++it) {
        const int k0 = wk.a * m.tchunk + 32 * (it * TWAVES + wave);
        float vals[16];
        load_block(vals, s.p, r, M, k0, lane);
        __syncthreads();
        stage_block(xs, vals, s.factor, r, cu);
        __syncthreads();
        const int kk = k0 + l32;
        if (kk < M)
            for (int slot = h; slot < kept; slot += 2)
                long_out[(size_t)slot * M + kk] = xs[l32 * XLD + col_of[slot]] * inv_of[slot];
    }
    if (wk.a == 0) {
        __syncthreads();
        for (int e = tid; e < kept * r; e += TNT) {
            const int slot = e / r, c = e % r;
            short_out[(size_t)slot * r + c] = m.Q[c * THIN_R + col_of[slot]] * fold_of[slot];
        }
    }
}

}  // namespace

void launch_thin_absmax(const SvdMat* d_mats, const Work* d_direct, int n_direct, const Work* d_copied, int n_copied,
                        hipStream_t stream)
{
    if (n_direct > 0) thin_absmax<<<(unsigned)n_direct, TNT, 0, stream>>>(d_mats, d_direct);
    if (n_copied > 0) thin_prepare<<<(unsigned)n_copied, TNT, 0, stream>>>(d_mats, d_copied);
}

void launch_thin_pass(const SvdMat* d_mats, const Work* d_chunks, int n_chunks, const Work* d_list, int n_list, int pass,
                      int last_pass, float stop_cosine, int* d_flags, hipStream_t stream)
{
    if (pass == 0) thin_gram<false><<<(unsigned)n_chunks, TNT, 0, stream>>>(d_mats, d_chunks, pass);
    else thin_gram<true><<<(unsigned)n_chunks, TNT, 0, stream>>>(d_mats, d_chunks, pass);
    thin_eig<<<(unsigned)n_list, ENT, 0, stream>>>(d_mats, d_list, pass, last_pass, stop_cosine, d_flags);
}

void launch_thin_pack(const SvdMat* d_mats, const Work* d_chunks, int n_chunks, hipStream_t stream)
{
    thin_pack<<<(unsigned)n_chunks, TNT, 0, stream>>>(d_mats, d_chunks);
}

}  // namespace svd
}  // namespace atomo
