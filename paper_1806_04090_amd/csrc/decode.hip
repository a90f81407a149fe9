// Decoders (eq. (vhat) of arXiv 1806.04090): g_hat = sum over kept atoms of (lambda_i / p_i) a_i.
//
// SVD messages: out = scale * sum_msgs sum_k w_k u_k v_k^T, a dense rank-(sum k) update written once.
// Each workgroup owns a 64 x 256 tile of one output and contracts the atoms of every message summed into
// it on the matrix cores.  Few atoms (one worker, budget 3): bound by the HBM write of the tile.  Many
// (the average over 16 workers, rank ~ 48): the 2 m n K flops take as long on the fp32 matrix cores as the write,
// and the workgroups, which all start together, go through listing, products and stores in step.
// The same kernel adds the update to what `out` holds instead of overwriting it (the parameter server's step,
// params += alpha * average gradient), and takes messages in the folded form (weight inside U).
// Entry-wise messages: zero fill, then one scatter launch per message in call order (bit-identical from run to run).
#include <algorithm>
#include <cstring>
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
    float* out;
    long long ld;
    int rows, cols;
    int first, last;           // messages [first, last)
};

struct DecWork { int out, tile_r, tile_c, pad; };

constexpr int TR = 64, TC = 256;
constexpr int TALL_ROWS = 256;     // rows per workgroup for outputs of at most 32 columns
constexpr int ATOMS_MAX = 512;     // atoms listed in LDS at a time

typedef float floatx16 __attribute__((ext_vector_type(16)));

// out tile (64 x 256) = sum over messages and kept atoms of (scale w_k u_k) v_k^T as a rank-K update on the
// matrix cores: A operand (row i, atom k) = scale w_k U[k][i], B operand (atom k, column j) = V[k][j],
// v_mfma_f32_32x32x2f32, two atoms per instruction.  Wave w owns columns 64 w .. 64 w + 63 of the tile as
// 2 x 2 blocks of 32 x 32.
// The kept atoms of a batch of messages (`batch` x largest capacity <= ATOMS_MAX, chosen by the host) are first
// listed in LDS (one round trip for all counts).  The operands then come through LDS in pieces of KP atoms: all
// 256 threads fetch the piece's slices of u (64 rows) and v (256 columns) with 16-byte loads that are all in
// flight at once - every atom's u and v are contiguous rows of its message -, and the loads of the next piece
// are issued before the products of the current one.  The weight is applied on the way into LDS.
// A message with a capacity above ATOMS_MAX is a batch of its own and is listed and contracted in runs of
// ATOMS_MAX atoms.
// TALL: outputs of at most 32 columns (the [x*y/2, 2*k*k] reshape of Section 6).  The workgroup owns 256 rows,
// wave w rows 64 w .. 64 w + 63, one 32-column block.
constexpr int KP = 16;             // atoms per piece (8 and 24 measure the same; 32 leaves room for two workgroups per
                                   // compute unit instead of four and is a third slower)

template <bool TALL, bool ACCUMULATE>
__global__ __launch_bounds__(256) void decode_svd_tiles(const DecOut* outs, const DecMsg* msgs, const DecWork* work,
                                                        float scale, int batch)
{
    constexpr int NCB = TALL ? 1 : 2;
    constexpr int UROWS = TALL ? TALL_ROWS : TR;                 // rows of the tile = length of a u slice
    constexpr int VCOLS = TALL ? 32 : TC;                        // columns of the tile = length of a v slice
    constexpr int US = UROWS + 32, VS = VCOLS + 32;              // LDS strides: odd and even atoms on different banks
    constexpr int NU = (KP * UROWS / 4 + 255) / 256;             // 16-byte loads per thread and piece, u and v
    constexpr int NV = (KP * VCOLS / 4 + 255) / 256;
    __shared__ const float* up[ATOMS_MAX];
    __shared__ const float* vp[ATOMS_MAX];
    __shared__ const float* wp[ATOMS_MAX];                       // the atom's weight (nullptr: folded into u)
    __shared__ int kept_of[ATOMS_MAX];
    __shared__ int total_sh;
    __shared__ __attribute__((aligned(16))) float Us[KP * US];
    __shared__ __attribute__((aligned(16))) float Vs[KP * VS];
    const DecWork wk = work[blockIdx.x];
    const DecOut o = outs[wk.out];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, l32 = lane & 31;
    const int tile_r0 = TALL ? wk.tile_r * TALL_ROWS : wk.tile_r * TR;
    const int tile_c0 = TALL ? 0 : wk.tile_c * TC;
    const int row_off = TALL ? wave * 64 : 0, col_off = TALL ? 0 : wave * 64;    // this wave's corner inside the tile
    floatx16 acc[2][NCB];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[rb][cb][v] = 0.0f;

    // four consecutive elements of an atom's row, zero beyond `limit`; one 16-byte load where the address allows
    auto load4 = [](const float* base, int at, int limit) {
        float4 x = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        const float* p = base + at;
        if (at + 3 < limit && (((size_t)p) & 15) == 0) {
            x = *(const float4*)p;
        } else {
            if (at < limit) x.x = p[0];
            if (at + 1 < limit) x.y = p[1];
            if (at + 2 < limit) x.z = p[2];
            if (at + 3 < limit) x.w = p[3];
        }
        return x;
    };
    float4 ru[NU], rv[NV];
    // the loads of the piece that starts at list position k0 (positions from `total` on read as zero)
    auto fetch = [&](int k0, int total) {
#pragma unroll
        for (int e = 0; e < NU; ++e) {
            const int f = tid + 256 * e, atom = f / (UROWS / 4), part = f % (UROWS / 4);
            ru[e] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (atom < KP && k0 + atom < total) {
                const float* w = wp[k0 + atom];
                const float wgt = w ? scale * *w : scale;
                const float4 x = load4(up[k0 + atom], tile_r0 + 4 * part, o.rows);
                ru[e] = make_float4(wgt * x.x, wgt * x.y, wgt * x.z, wgt * x.w);
            }
        }
#pragma unroll
        for (int e = 0; e < NV; ++e) {
            const int f = tid + 256 * e, atom = f / (VCOLS / 4), part = f % (VCOLS / 4);
            rv[e] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (atom < KP && k0 + atom < total) rv[e] = load4(vp[k0 + atom], tile_c0 + 4 * part, o.cols);
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int e = 0; e < NU; ++e) {
            const int f = tid + 256 * e, atom = f / (UROWS / 4), part = f % (UROWS / 4);
            if (atom < KP) *(float4*)&Us[atom * US + 4 * part] = ru[e];
        }
#pragma unroll
        for (int e = 0; e < NV; ++e) {
            const int f = tid + 256 * e, atom = f / (VCOLS / 4), part = f % (VCOLS / 4);
            if (atom < KP) *(float4*)&Vs[atom * VS + 4 * part] = rv[e];
        }
    };

    for (int first = o.first; first < o.last; first += batch) {
        const int nm = min(batch, o.last - first);
        __syncthreads();                                         // the previous list is spent
        for (int q = tid; q < nm; q += 256) kept_of[q] = min(*msgs[first + q].count, msgs[first + q].capacity);
        __syncthreads();
        // several messages: everything fits the list by the host's choice of `batch` (one run); a message of its
        // own: runs of ATOMS_MAX atoms, `run` = first atom of the run
        const int span = nm == 1 ? kept_of[0] : 1;
        for (int run = 0; run < span; run += ATOMS_MAX) {
            if (run > 0) __syncthreads();                        // the previous run is spent
            for (int q = tid; q < nm; q += 256) {
                int at = 0;
                for (int e = 0; e < q; ++e) at += kept_of[e];
                const DecMsg m = msgs[first + q];
                const int kept = max(0, min(kept_of[q] - run, ATOMS_MAX - at));
                for (int k = 0; k < kept; ++k) {
                    up[at + k] = m.U + (size_t)(run + k) * o.rows;
                    vp[at + k] = m.V + (size_t)(run + k) * o.cols;
                    wp[at + k] = m.w ? m.w + run + k : nullptr;    // folded messages carry the weight in U
                }
                if (q == nm - 1) total_sh = at + kept;
            }
            __syncthreads();
            const int total = total_sh;
            if (total > 0) fetch(0, total);
            for (int k0 = 0; k0 < total; k0 += KP) {
                stage();
                __syncthreads();
                if (k0 + KP < total) fetch(k0 + KP, total);
                const int pairs = (min(KP, total - k0) + 1) / 2;
                for (int t = 0; t < pairs; ++t) {
                    const float* ua = &Us[(2 * t + h) * US + row_off + l32];
                    const float* vb = &Vs[(2 * t + h) * VS + col_off + l32];
                    const float a0 = ua[0], a1 = ua[32], b0 = vb[0];
                    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
                    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
                    if (!TALL) {
                        const float b1 = vb[32];
                        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
                        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
                    }
                }
                __syncthreads();                                 // the piece is spent
            }
        }
    }
    const int r0 = tile_r0 + row_off, c0 = tile_c0 + col_off;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            const int col = c0 + cb * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = r0 + rb * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                if (row < o.rows && col < o.cols) {
                    float* dst = o.out + (size_t)row * o.ld + col;
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
    std::vector<DecMsg> hm(n_msgs);
    std::vector<DecOut> ho(n_out);
    std::vector<DecWork> hw, hw_tall;
    for (int k = 0; k < n_msgs; ++k)
        hm[k] = DecMsg{msgs[k].count, msgs[k].w, msgs[k].U, msgs[k].V, msgs[k].capacity, 0};
    for (int o = 0; o < n_out; ++o) {
        const atomo_svd_msg& m0 = msgs[first[o]];
        ho[o] = DecOut{outs[o], (long long)lds[o], m0.rows, m0.cols, first[o], first[o + 1]};
        if (m0.cols <= 32 && m0.rows > TR) {
            for (int a = 0; a < (m0.rows + TALL_ROWS - 1) / TALL_ROWS; ++a) hw_tall.push_back(DecWork{o, a, 0, 0});
            continue;
        }
        const int tr = (m0.rows + TR - 1) / TR, tc = (m0.cols + TC - 1) / TC;
        for (int a = 0; a < tr; ++a)
            for (int b = 0; b < tc; ++b) hw.push_back(DecWork{o, a, b, 0});
    }
    // every die gets a contiguous run of the tiles, i.e. the tiles of a few outputs: the singular vectors of an
    // output are then fetched into one L2 instead of all eight
    deal_to_dies(hw);
    deal_to_dies(hw_tall);
    const size_t n_wide = hw.size();
    hw.insert(hw.end(), hw_tall.begin(), hw_tall.end());
    // the three tables travel in one copy, into a block of their own: a loop that decodes the same messages into the
    // same outputs call after call finds them there and uploads nothing (see atomo_ctx::dec_tables)
    Carver size_only(nullptr);
    size_only.take<DecMsg>(hm.size());
    size_only.take<DecOut>(ho.size());
    size_only.take<DecWork>(hw.size());
    int rc = ATOMO_OK;
    if (size_only.off > ctx->dec_tables_cap) {
        // (hipFree waits for the device, so no kernel still reads the old block)
        if (ctx->dec_tables_dev) ATOMO_HIP(ctx, hipFree(ctx->dec_tables_dev));
        ctx->dec_tables_dev = nullptr;
        ctx->dec_tables_cap = 0;
        ctx->dec_tables.clear();
        const size_t want = align_up(size_only.off * 2, (size_t)1 << 16);
        if (hipMalloc(&ctx->dec_tables_dev, want) != hipSuccess) return ATOMO_ENOMEM;
        ctx->dec_tables_cap = want;
    }
    Carver carve(ctx->dec_tables_dev);
    DecMsg* d_msgs = carve.take<DecMsg>(hm.size());
    DecOut* d_outs = carve.take<DecOut>(ho.size());
    DecWork* d_work = carve.take<DecWork>(hw.size());
    std::vector<char> staged(size_only.off, 0);
    memcpy(staged.data() + ((char*)d_msgs - (char*)ctx->dec_tables_dev), hm.data(), hm.size() * sizeof(DecMsg));
    memcpy(staged.data() + ((char*)d_outs - (char*)ctx->dec_tables_dev), ho.data(), ho.size() * sizeof(DecOut));
    memcpy(staged.data() + ((char*)d_work - (char*)ctx->dec_tables_dev), hw.data(), hw.size() * sizeof(DecWork));
    if (ctx->dec_tables_stream != stream || staged != ctx->dec_tables) {
        ctx->dec_tables.clear();                                 // (an upload that fails leaves nothing to match)
        if ((rc = upload(ctx, ctx->dec_tables_dev, staged.data(), staged.size(), stream)) != ATOMO_OK) return rc;
        ctx->dec_tables = staged;
        ctx->dec_tables_stream = stream;
    }
    {
        ProfScope ps(ctx, ATOMO_K_DECODE_SVD, stream);
        int max_cap = 1;
        for (int k = 0; k < n_msgs; ++k) max_cap = std::max(max_cap, (int)msgs[k].capacity);
        const int batch = std::max(1, ATOMS_MAX / max_cap);      // messages whose atoms fit the LDS list together
        const unsigned n_tall = (unsigned)hw_tall.size();
        if (n_wide > 0) {
            if (accumulate) decode_svd_tiles<false, true><<<(unsigned)n_wide, 256, 0, stream>>>(d_outs, d_msgs, d_work, scale, batch);
            else decode_svd_tiles<false, false><<<(unsigned)n_wide, 256, 0, stream>>>(d_outs, d_msgs, d_work, scale, batch);
        }
        if (n_tall > 0) {
            if (accumulate) decode_svd_tiles<true, true><<<n_tall, 256, 0, stream>>>(d_outs, d_msgs, d_work + n_wide, scale, batch);
            else decode_svd_tiles<true, false><<<n_tall, 256, 0, stream>>>(d_outs, d_msgs, d_work + n_wide, scale, batch);
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
