// Decoders (eq. (vhat) of arXiv 1806.04090): g_hat = sum over kept atoms of (lambda_i / p_i) a_i.
//
// SVD messages: out = scale * sum_msgs sum_k w_k u_k v_k^T, a dense rank-(sum k) update written once.
// Each workgroup owns a 64 x 256 tile of one output and contracts the atoms of every message summed into
// it on the matrix cores.  Few atoms (one worker, budget 3): bound by the HBM write of the tile.  Many
// (the average over 16 workers, rank ~ 48): near the ridge between the two.
// The same kernel adds the update to what `out` holds instead of overwriting it (the parameter server's step,
// params += alpha * average gradient), and takes messages in the folded form (weight inside U).
// Entry-wise messages: zero fill, then one scatter launch per message in call order (bit-identical from run to run).
#include <algorithm>
#include <vector>

#include "atomo_internal.h"

namespace atomo {

namespace {

struct DecMsg {
    const int* count;
    const float* w;
    const float* U;
    const float* V;
    int capacity;
    int pad;
};

struct DecOut {
    int rows, cols;
    int first, last;           // messages [first, last)
    long long atom_base;       // where this output's atom list starts
};

// One kept atom as the contraction reads it: its two vectors and scale * weight.
struct DecAtom {
    const float* u;
    const float* v;
    float w;
    int pad;
};

// One tile of one output; everything the tile kernel needs sits in the record it reads first.
struct DecWork {
    float* out;
    long long ld;
    const DecAtom* atoms;      // the output's atom list
    const int* natoms;         // its length (device scalar written by decode_svd_list)
    int rows, cols;
    int tile_r, tile_c;
};

constexpr int TR = 64, TC = 256;
constexpr int TALL_ROWS = 256;     // rows per workgroup for outputs of at most 32 columns
constexpr int ATOMS_MAX = 256;     // atoms staged in LDS at a time; longer lists are contracted in pieces

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Lists the kept atoms of every message summed into one output (one workgroup per output): the tile kernel then starts
// from one contiguous list instead of chasing descriptor -> count -> weight -> vectors in every tile.  Messages are
// taken 256 at a time; wave w lists messages w, w + 4, ... of the group, lane l atoms l, l + 64, ... of a message.
__global__ __launch_bounds__(256) void decode_svd_list(const DecOut* outs, const DecMsg* msgs, float scale, DecAtom* atoms,
                                                       int* natoms)
{
    __shared__ int kept_sh[256];
    __shared__ int offs_sh[256];
    const DecOut o = outs[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    DecAtom* list = atoms + o.atom_base;
    int base = 0;                                                // atoms listed so far (uniform)
    for (int m0 = o.first; m0 < o.last; m0 += 256) {
        const int q = m0 + tid;
        const int kept = q < o.last ? max(0, min(*msgs[q].count, msgs[q].capacity)) : 0;
        kept_sh[tid] = kept;
        offs_sh[tid] = kept;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {                // inclusive scan
            const int v = tid >= off ? offs_sh[tid - off] : 0;
            __syncthreads();
            offs_sh[tid] += v;
            __syncthreads();
        }
        const int group = min(256, o.last - m0);
        for (int mm = wave; mm < group; mm += 4) {
            const DecMsg m = msgs[m0 + mm];
            const int k_tot = kept_sh[mm];
            const int at = base + offs_sh[mm] - k_tot;
            for (int k = lane; k < k_tot; k += 64) {
                DecAtom a;
                a.u = m.U + (size_t)k * o.rows;
                a.v = m.V + (size_t)k * o.cols;
                a.w = m.w ? scale * m.w[k] : scale;              // folded messages carry the weight in U
                a.pad = 0;
                list[at + k] = a;
            }
        }
        base += offs_sh[255];
        __syncthreads();                                         // the scan arrays are reused by the next group
    }
    if (tid == 0) natoms[blockIdx.x] = base;
}

// out tile (64 x 256) = sum over the listed atoms of (scale w_k u_k) v_k^T as a rank-K update on the matrix cores:
// A operand (row i, atom k) = scale w_k U[k][i], B operand (atom k, column j) = V[k][j], v_mfma_f32_32x32x2f32, two
// atoms per instruction.  Wave w owns columns 64 w .. 64 w + 63 of the tile as 2 x 2 blocks of 32 x 32.  The list is
// staged in LDS ATOMS_MAX atoms at a time; operands come straight from global memory (every atom's u and v are
// contiguous rows of its message), eight atoms per trip, the loads of the next trip issued before the products of the
// current one.  An odd atom count pads with a zero weight.
// TALL: outputs of at most 32 columns (the [x*y/2, 2*k*k] reshape of Section 6).  The workgroup owns 256 rows,
// wave w rows 64 w .. 64 w + 63, one 32-column block.
template <bool TALL, bool ACCUMULATE>
__global__ __launch_bounds__(256) void decode_svd_tiles(const DecWork* work)
{
    constexpr int NCB = TALL ? 1 : 2;
    __shared__ const float* up[ATOMS_MAX];
    __shared__ const float* vp[ATOMS_MAX];
    __shared__ float wv[ATOMS_MAX];
    const DecWork wk = work[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, l32 = lane & 31;
    const int r0 = TALL ? wk.tile_r * TALL_ROWS + wave * 64 : wk.tile_r * TR;
    const int c0 = TALL ? 0 : wk.tile_c * TC + wave * 64;
    const int row_a = r0 + l32, row_b = r0 + 32 + l32;          // rows this lane feeds as A operands
    const int col_a = c0 + l32, col_b = c0 + 32 + l32;          // columns this lane feeds as B operands
    const bool ra = row_a < wk.rows, rb_ok = row_b < wk.rows, ca = col_a < wk.cols, cb_ok = !TALL && col_b < wk.cols;
    floatx16 acc[2][NCB];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[rb][cb][v] = 0.0f;

    const int n_atoms = *wk.natoms;
    for (int piece = 0; piece < n_atoms; piece += ATOMS_MAX) {
        const int total = min(ATOMS_MAX, n_atoms - piece);
        if (piece > 0) __syncthreads();                          // the previous piece is spent
        for (int k = tid; k < total; k += 256) {
            const DecAtom a = wk.atoms[piece + k];
            up[k] = a.u;
            vp[k] = a.v;
            wv[k] = a.w;
        }
        __syncthreads();
        float a0[2][4], a1[2][4], b0[2][4], b1[2][4];
        auto fetch = [&](int buf, int k0) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int kk = k0 + 2 * t + h;
                const bool live = kk < total;
                const float wgt = live ? wv[kk] : 0.0f;
                const float* u = up[live ? kk : 0];
                const float* v = vp[live ? kk : 0];
                a0[buf][t] = live && ra ? wgt * u[row_a] : 0.0f;
                a1[buf][t] = live && rb_ok ? wgt * u[row_b] : 0.0f;
                b0[buf][t] = live && ca ? v[col_a] : 0.0f;
                b1[buf][t] = live && cb_ok ? v[col_b] : 0.0f;
            }
        };
        auto contract = [&](int buf, int k0) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (k0 + 2 * t < total) {                        // uniform: skip pairs past the end
                    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[buf][t], b0[buf][t], acc[0][0], 0, 0, 0);
                    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[buf][t], b0[buf][t], acc[1][0], 0, 0, 0);
                    if (!TALL) {
                        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[buf][t], b1[buf][t], acc[0][1], 0, 0, 0);
                        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[buf][t], b1[buf][t], acc[1][1], 0, 0, 0);
                    }
                }
            }
        };
        // two trips per round so that the operand buffers are indexed by constants
        fetch(0, 0);
        for (int k0 = 0; k0 < total; k0 += 16) {
            if (k0 + 8 < total) fetch(1, k0 + 8);
            contract(0, k0);
            if (k0 + 16 < total) fetch(0, k0 + 16);
            if (k0 + 8 < total) contract(1, k0 + 8);
        }
    }
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            const int col = c0 + cb * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = r0 + rb * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                if (row < wk.rows && col < wk.cols) {
                    float* dst = wk.out + (size_t)row * wk.ld + col;
                    *dst = ACCUMULATE ? *dst + acc[rb][cb][v] : acc[rb][cb][v];
                }
            }
        }
}

__global__ __launch_bounds__(256) void fill_zero(float* __restrict__ out, long long n)
{
    const long long stride = (long long)gridDim.x * 256;
    const bool vec = (((size_t)out) & 15) == 0;
    const long long n4 = vec ? n / 4 : 0;
    for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < n4; q += stride)
        ((float4*)out)[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (long long i = n4 * 4 + (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) out[i] = 0.0f;
}

struct EwDecMsg {
    const long long* count;
    const unsigned int* idx;
    const float* val;
    long long capacity;
};

// One message per launch, in the order of the call: inside a message the kept coordinates are distinct, so plain
// stores (first message, after the zero fill) and plain read-add-write (the others) give the same bits in every run.
__global__ __launch_bounds__(256) void scatter_entrywise(const EwDecMsg* msgs, int which, float scale,
                                                         float* __restrict__ out, long long n)
{
    const EwDecMsg m = msgs[which];
    const long long kept = min(*m.count, m.capacity);
    const long long stride = (long long)gridDim.x * 256;
    for (long long k = (long long)blockIdx.x * 256 + threadIdx.x; k < kept; k += stride) {
        const unsigned int i = m.idx[k];
        if ((long long)i >= n) continue;
        const float v = scale * m.val[k];
        out[i] = which == 0 ? v : out[i] + v;
    }
}

struct LqDecMsg {
    const long long* count;
    const unsigned int* idx;
    const float* norm;
    long long capacity;
};

// l_q messages (Section 4): a kept coordinate decodes to sign * |g|_q, the sign in bit 31 of its index.
// One message per launch, like scatter_entrywise.
__global__ __launch_bounds__(256) void scatter_lq(const LqDecMsg* msgs, int which, float scale, float* __restrict__ out,
                                                  long long n)
{
    const LqDecMsg m = msgs[which];
    const long long kept = min(*m.count, m.capacity);
    const float mag = scale * *m.norm;
    const long long stride = (long long)gridDim.x * 256;
    for (long long k = (long long)blockIdx.x * 256 + threadIdx.x; k < kept; k += stride) {
        const unsigned int word = m.idx[k];
        const unsigned int i = word & 0x7FFFFFFFu;
        if ((long long)i >= n) continue;
        const float v = (word >> 31) ? -mag : mag;
        out[i] = which == 0 ? v : out[i] + v;
    }
}

}  // namespace

int decode_svd_batch(atomo_ctx* ctx, const atomo_svd_msg* msgs, const int32_t* first, int n_out, float scale,
                     float* const* outs, const int64_t* lds, bool accumulate, hipStream_t stream)
{
    const int n_msgs = first[n_out];
    // workspace: [messages | outputs | tiles] (one upload), then the atom lists and their lengths (device-made)
    size_t n_wide = 0, n_tall = 0, n_atoms_cap = 0;
    for (int o = 0; o < n_out; ++o) {
        const atomo_svd_msg& m0 = msgs[first[o]];
        if (m0.cols <= 32 && m0.rows > TR) n_tall += (size_t)(m0.rows + TALL_ROWS - 1) / TALL_ROWS;
        else n_wide += (size_t)((m0.rows + TR - 1) / TR) * (size_t)((m0.cols + TC - 1) / TC);
        for (int k = first[o]; k < first[o + 1]; ++k) n_atoms_cap += (size_t)msgs[k].capacity;
    }
    Carver size_only(nullptr);
    size_only.take<DecMsg>(n_msgs);
    size_only.take<DecOut>(n_out);
    size_only.take<DecWork>(n_wide + n_tall);
    const size_t upload_bytes = size_only.off;
    size_only.take<DecAtom>(n_atoms_cap);
    size_only.take<int>(n_out);
    int rc = ensure_workspace(ctx, size_only.off);
    if (rc != ATOMO_OK) return rc;
    Carver carve(ctx->ws);
    DecMsg* d_msgs = carve.take<DecMsg>(n_msgs);
    DecOut* d_outs = carve.take<DecOut>(n_out);
    DecWork* d_work = carve.take<DecWork>(n_wide + n_tall);
    DecAtom* d_atoms = carve.take<DecAtom>(n_atoms_cap);
    int* d_natoms = carve.take<int>(n_out);

    std::vector<char> host(upload_bytes, 0);
    DecMsg* hm = (DecMsg*)(host.data() + ((char*)d_msgs - (char*)ctx->ws));
    DecOut* ho = (DecOut*)(host.data() + ((char*)d_outs - (char*)ctx->ws));
    DecWork* hw = (DecWork*)(host.data() + ((char*)d_work - (char*)ctx->ws));
    for (int k = 0; k < n_msgs; ++k)
        hm[k] = DecMsg{msgs[k].count, msgs[k].w, msgs[k].U, msgs[k].V, msgs[k].capacity, 0};
    size_t at_wide = 0, at_tall = n_wide;
    long long atom_base = 0;
    for (int o = 0; o < n_out; ++o) {
        const atomo_svd_msg& m0 = msgs[first[o]];
        ho[o] = DecOut{m0.rows, m0.cols, first[o], first[o + 1], atom_base};
        DecWork w{outs[o], (long long)lds[o], d_atoms + atom_base, d_natoms + o, m0.rows, m0.cols, 0, 0};
        if (m0.cols <= 32 && m0.rows > TR) {
            for (int a = 0; a < (m0.rows + TALL_ROWS - 1) / TALL_ROWS; ++a) {
                w.tile_r = a;
                hw[at_tall++] = w;
            }
        } else {
            const int tr = (m0.rows + TR - 1) / TR, tc = (m0.cols + TC - 1) / TC;
            for (int a = 0; a < tr; ++a)
                for (int b = 0; b < tc; ++b) {
                    w.tile_r = a;
                    w.tile_c = b;
                    hw[at_wide++] = w;
                }
        }
        for (int k = first[o]; k < first[o + 1]; ++k) atom_base += msgs[k].capacity;
    }
    if ((rc = upload(ctx, ctx->ws, host.data(), upload_bytes, stream)) != ATOMO_OK) return rc;
    {
        ProfScope ps(ctx, ATOMO_K_DECODE_SVD, stream);
        decode_svd_list<<<(unsigned)n_out, 256, 0, stream>>>(d_outs, d_msgs, scale, d_atoms, d_natoms);
        if (n_wide > 0) {
            if (accumulate) decode_svd_tiles<false, true><<<(unsigned)n_wide, 256, 0, stream>>>(d_work);
            else decode_svd_tiles<false, false><<<(unsigned)n_wide, 256, 0, stream>>>(d_work);
        }
        if (n_tall > 0) {
            if (accumulate) decode_svd_tiles<true, true><<<(unsigned)n_tall, 256, 0, stream>>>(d_work + n_wide);
            else decode_svd_tiles<true, false><<<(unsigned)n_tall, 256, 0, stream>>>(d_work + n_wide);
        }
    }
    ATOMO_HIP(ctx, hipGetLastError());
    return ATOMO_OK;
}

int decode_entrywise(atomo_ctx* ctx, const atomo_ew_msg* msgs, int n_msgs, float scale, float* out,
                     hipStream_t stream)
{
    const int64_t n = msgs[0].n;
    std::vector<EwDecMsg> hm(n_msgs);
    for (int k = 0; k < n_msgs; ++k)
        hm[k] = EwDecMsg{(const long long*)msgs[k].count, msgs[k].idx, msgs[k].val, (long long)msgs[k].capacity};
    int rc = ensure_workspace(ctx, align_up(hm.size() * sizeof(EwDecMsg), 256));
    if (rc != ATOMO_OK) return rc;
    EwDecMsg* d_msgs = (EwDecMsg*)ctx->ws;
    if ((rc = upload(ctx, d_msgs, hm.data(), hm.size() * sizeof(EwDecMsg), stream)) != ATOMO_OK) return rc;
    const int fill_wgs = (int)std::min<int64_t>(2048, (n / 4 + 255) / 256 + 1);
    {
        ProfScope ps(ctx, ATOMO_K_EW_DECODE, stream);
        fill_zero<<<fill_wgs, 256, 0, stream>>>(out, n);
        for (int k = 0; k < n_msgs; ++k) {
            const int sc_wgs = (int)std::min<int64_t>(1024, (msgs[k].capacity + 255) / 256);
            scatter_entrywise<<<sc_wgs, 256, 0, stream>>>(d_msgs, k, scale, out, n);
        }
    }
    ATOMO_HIP(ctx, hipGetLastError());
    return ATOMO_OK;
}

int decode_lq(atomo_ctx* ctx, const atomo_lq_msg* msgs, int n_msgs, float scale, float* out, hipStream_t stream)
{
    const int64_t n = msgs[0].n;
    std::vector<LqDecMsg> hm(n_msgs);
    for (int k = 0; k < n_msgs; ++k)
        hm[k] = LqDecMsg{(const long long*)msgs[k].count, msgs[k].idx, msgs[k].norm, (long long)msgs[k].capacity};
    int rc = ensure_workspace(ctx, align_up(hm.size() * sizeof(LqDecMsg), 256));
    if (rc != ATOMO_OK) return rc;
    LqDecMsg* d_msgs = (LqDecMsg*)ctx->ws;
    if ((rc = upload(ctx, d_msgs, hm.data(), hm.size() * sizeof(LqDecMsg), stream)) != ATOMO_OK) return rc;
    const int fill_wgs = (int)std::min<int64_t>(2048, (n / 4 + 255) / 256 + 1);
    {
        ProfScope ps(ctx, ATOMO_K_EW_DECODE, stream);
        fill_zero<<<fill_wgs, 256, 0, stream>>>(out, n);
        for (int k = 0; k < n_msgs; ++k) {
            const int sc_wgs = (int)std::min<int64_t>(1024, (msgs[k].capacity + 255) / 256);
            scatter_lq<<<sc_wgs, 256, 0, stream>>>(d_msgs, k, scale, out, n);
        }
    }
    ATOMO_HIP(ctx, hipGetLastError());
    return ATOMO_OK;
}

}  // namespace atomo
