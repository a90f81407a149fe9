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

#include "svd_common.h"

namespace atomo {

namespace {

using namespace svd;


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
    const int max_inner = opt && opt->max_inner_sweeps > 0 ? opt->max_inner_sweeps : 1;
    const float inner_reduction = opt && opt->inner_reduction > 0.0f ? opt->inner_reduction : 0.01f;

    Plan sizing;
    build_plan(mats, n_mats, msgs, sigma_out, p_out, stream_base, nullptr, sizing);
    int rc = ensure_workspace(ctx, sizing.bytes);
    if (rc != ATOMO_OK) return rc;

    Plan plan;
    build_plan(mats, n_mats, msgs, sigma_out, p_out, stream_base, ctx->ws, plan);

    SvdMat* d_mats = plan.d_mats;
    Work* d_work = plan.d_work;
    ctx->svd_state.clear();
    for (const SvdMat& m : plan.mats) ctx->svd_state.push_back(m.state);
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

    {
        ProfScope ps(ctx, ATOMO_K_SVD_PREPARE, stream);
        svd_prepare<<<(unsigned)plan.prep.size(), 256, 0, stream>>>(d_mats, d_work + o_prep);
        svd_norms<<<(unsigned)plan.norms.size(), 256, 0, stream>>>(d_mats, d_work + o_norms, 1);
    }
    const int n_steps = max_sweeps * plan.max_R;
    for (int step = 0; step < n_steps; ++step) {
        {
            ProfScope ps(ctx, ATOMO_K_SVD_GRAM, stream);
            svd_gram<<<(unsigned)plan.gram.size(), 256, 0, stream>>>(d_mats, d_work + o_gram, step, max_sweeps);
        }
        {
            ProfScope ps(ctx, ATOMO_K_SVD_EIG, stream);
            launch_svd_eig(d_mats, d_work + o_eig, (int)plan.eig.size(), step, max_sweeps, stop_cosine,
                           max_inner, inner_reduction, ctx->d_flags, stream);
        }
        {
            ProfScope ps(ctx, ATOMO_K_SVD_UPDATE, stream);
            svd_update<<<(unsigned)plan.upd.size(), 256, 0, stream>>>(d_mats, d_work + o_upd, step, max_sweeps);
        }
    }
    {
        ProfScope ps(ctx, ATOMO_K_SVD_FINALIZE, stream);
        svd_norms<<<(unsigned)plan.norms.size(), 256, 0, stream>>>(d_mats, d_work + o_norms, 0);
        svd_select<<<(unsigned)n_mats, 256, 0, stream>>>(d_mats, s, (unsigned long long)seed, ctx->d_flags);
        svd_pack<<<(unsigned)plan.pack.size(), 256, 0, stream>>>(d_mats, d_work + o_pack);
    }
    ATOMO_HIP(ctx, hipGetLastError());
    return ATOMO_OK;
}

int svd_sweeps(atomo_ctx* ctx, hipStream_t stream, int32_t* sweeps, int n_mats)
{
    if ((size_t)n_mats != ctx->svd_state.size()) return ATOMO_EINVAL;
    ATOMO_HIP(ctx, hipStreamSynchronize(stream));
    for (int j = 0; j < n_mats; ++j)
        ATOMO_HIP(ctx, hipMemcpy(&sweeps[j], ctx->svd_state[j] + ST_SWEEPS, sizeof(int32_t), hipMemcpyDeviceToHost));
    return ATOMO_OK;
}

}  // namespace atomo
