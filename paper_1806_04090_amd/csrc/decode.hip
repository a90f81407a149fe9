// Decoders (eq. (vhat) of arXiv 1806.04090): g_hat = sum over kept atoms of (lambda_i / p_i) a_i.
//
// SVD messages: out = scale * sum_msgs sum_k w_k u_k v_k^T, a dense rank-(sum k) update written once.
// Each workgroup owns a 64 x 256 tile of one output and walks the atoms of every message summed into
// it.  Few atoms (one worker, budget 3): the kernel is bound by the HBM write of the tile.
// Entry-wise messages: zero fill, then scatter (atomic add when several messages overlap).
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

__global__ __launch_bounds__(256) void decode_svd_tiles(const DecOut* outs, const DecMsg* msgs, const DecWork* work,
                                                        float scale)
{
    __shared__ float us[TR];
    const DecWork wk = work[blockIdx.x];
    const DecOut o = outs[wk.out];
    const int tid = threadIdx.x;
    const int r0 = wk.tile_r * TR, c0 = wk.tile_c * TC;
    const int cq = tid & 63;                    // float4 column inside the tile
    const int rg = tid >> 6;                    // row group: rows rg*16 .. rg*16+15
    const int col = c0 + cq * 4;
    float4 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);

    for (int mi = o.first; mi < o.last; ++mi) {
        const DecMsg m = msgs[mi];
        const int kept = min(*m.count, m.capacity);
        for (int k = 0; k < kept; ++k) {
            __syncthreads();
            if (tid < TR) {
                const int row = r0 + tid;
                us[tid] = row < o.rows ? scale * m.w[k] * m.U[(size_t)k * o.rows + row] : 0.0f;
            }
            __syncthreads();
            const float* v = m.V + (size_t)k * o.cols;
            float4 vv;
            vv.x = col < o.cols ? v[col] : 0.0f;
            vv.y = col + 1 < o.cols ? v[col + 1] : 0.0f;
            vv.z = col + 2 < o.cols ? v[col + 2] : 0.0f;
            vv.w = col + 3 < o.cols ? v[col + 3] : 0.0f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float u = us[rg * 16 + i];
                acc[i].x += u * vv.x;
                acc[i].y += u * vv.y;
                acc[i].z += u * vv.z;
                acc[i].w += u * vv.w;
            }
        }
    }
    const bool vec_ok = ((o.ld & 3) == 0) && ((((size_t)o.out) & 15) == 0) && (col + 3 < o.cols);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int row = r0 + rg * 16 + i;
        if (row >= o.rows) continue;
        float* dst = o.out + (size_t)row * o.ld + col;
        if (vec_ok) {
            *(float4*)dst = acc[i];
        } else {
            if (col < o.cols) dst[0] = acc[i].x;
            if (col + 1 < o.cols) dst[1] = acc[i].y;
            if (col + 2 < o.cols) dst[2] = acc[i].z;
            if (col + 3 < o.cols) dst[3] = acc[i].w;
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

// One message per blockIdx.y.  With a single message the kept coordinates are distinct: plain stores.
__global__ __launch_bounds__(256) void scatter_entrywise(const EwDecMsg* msgs, int n_msgs, float scale,
                                                         float* __restrict__ out, long long n)
{
    const EwDecMsg m = msgs[blockIdx.y];
    const long long kept = min(*m.count, m.capacity);
    const long long stride = (long long)gridDim.x * 256;
    for (long long k = (long long)blockIdx.x * 256 + threadIdx.x; k < kept; k += stride) {
        const unsigned int i = m.idx[k];
        if ((long long)i >= n) continue;
        const float v = scale * m.val[k];
        if (n_msgs == 1) out[i] = v;
        else atomicAdd(&out[i], v);
    }
}

}  // namespace

int decode_svd_batch(atomo_ctx* ctx, const atomo_svd_msg* msgs, const int32_t* first, int n_out, float scale,
                     float* const* outs, const int64_t* lds, hipStream_t stream)
{
    const int n_msgs = first[n_out];
    std::vector<DecMsg> hm(n_msgs);
    std::vector<DecOut> ho(n_out);
    std::vector<DecWork> hw;
    for (int k = 0; k < n_msgs; ++k)
        hm[k] = DecMsg{msgs[k].count, msgs[k].w, msgs[k].U, msgs[k].V, msgs[k].capacity, 0};
    for (int o = 0; o < n_out; ++o) {
        const atomo_svd_msg& m0 = msgs[first[o]];
        ho[o] = DecOut{outs[o], (long long)lds[o], m0.rows, m0.cols, first[o], first[o + 1]};
        const int tr = (m0.rows + TR - 1) / TR, tc = (m0.cols + TC - 1) / TC;
        for (int a = 0; a < tr; ++a)
            for (int b = 0; b < tc; ++b) hw.push_back(DecWork{o, a, b, 0});
    }
    Carver size_only(nullptr);
    size_only.take<DecMsg>(hm.size());
    size_only.take<DecOut>(ho.size());
    size_only.take<DecWork>(hw.size());
    int rc = ensure_workspace(ctx, size_only.off);
    if (rc != ATOMO_OK) return rc;
    Carver carve(ctx->ws);
    DecMsg* d_msgs = carve.take<DecMsg>(hm.size());
    DecOut* d_outs = carve.take<DecOut>(ho.size());
    DecWork* d_work = carve.take<DecWork>(hw.size());
    if ((rc = upload(ctx, d_msgs, hm.data(), hm.size() * sizeof(DecMsg), stream)) != ATOMO_OK) return rc;
    if ((rc = upload(ctx, d_outs, ho.data(), ho.size() * sizeof(DecOut), stream)) != ATOMO_OK) return rc;
    if ((rc = upload(ctx, d_work, hw.data(), hw.size() * sizeof(DecWork), stream)) != ATOMO_OK) return rc;
    {
        ProfScope ps(ctx, ATOMO_K_DECODE_SVD, stream);
        decode_svd_tiles<<<(unsigned)hw.size(), 256, 0, stream>>>(d_outs, d_msgs, d_work, scale);
    }
    ATOMO_HIP(ctx, hipGetLastError());
    return ATOMO_OK;
}

int decode_entrywise(atomo_ctx* ctx, const atomo_ew_msg* msgs, int n_msgs, float scale, float* out,
                     hipStream_t stream)
{
    const int64_t n = msgs[0].n;
    std::vector<EwDecMsg> hm(n_msgs);
    int64_t max_cap = 1;
    for (int k = 0; k < n_msgs; ++k) {
        hm[k] = EwDecMsg{(const long long*)msgs[k].count, msgs[k].idx, msgs[k].val, (long long)msgs[k].capacity};
        if (msgs[k].capacity > max_cap) max_cap = msgs[k].capacity;
    }
    int rc = ensure_workspace(ctx, align_up(hm.size() * sizeof(EwDecMsg), 256));
    if (rc != ATOMO_OK) return rc;
    EwDecMsg* d_msgs = (EwDecMsg*)ctx->ws;
    if ((rc = upload(ctx, d_msgs, hm.data(), hm.size() * sizeof(EwDecMsg), stream)) != ATOMO_OK) return rc;
    const int fill_wgs = (int)std::min<int64_t>(2048, (n / 4 + 255) / 256 + 1);
    const int sc_wgs = (int)std::min<int64_t>(1024, (max_cap + 255) / 256);
    {
        ProfScope ps(ctx, ATOMO_K_EW_DECODE, stream);
        fill_zero<<<fill_wgs, 256, 0, stream>>>(out, n);
        scatter_entrywise<<<dim3(sc_wgs, n_msgs), 256, 0, stream>>>(d_msgs, n_msgs, scale, out, n);
    }
    ATOMO_HIP(ctx, hipGetLastError());
    return ATOMO_OK;
}

}  // namespace atomo
