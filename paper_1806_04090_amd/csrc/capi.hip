// C ABI of libatomo: context management, argument validation, dispatch.  See include/atomo.h.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>

#include "atomo_internal.h"

namespace atomo {

int ensure_workspace(atomo_ctx* ctx, size_t bytes)
{
    ctx->svd_tables_intact = false;
    if (bytes <= ctx->ws_bytes) return ATOMO_OK;
    // Growing frees the old block; hipFree waits for the device, so no kernel still uses it.
    if (ctx->ws) {
        ATOMO_HIP(ctx, hipFree(ctx->ws));
        ctx->ws = nullptr;
        ctx->ws_bytes = 0;
    }
    size_t want = align_up(bytes + bytes / 8, (size_t)1 << 20);
    hipError_t e = hipMalloc(&ctx->ws, want);
    if (e != hipSuccess) {
        ctx->last_hip = (int)e;
        ctx->ws = nullptr;
        return ATOMO_ENOMEM;
    }
    ctx->ws_bytes = want;
    return ATOMO_OK;
}

int ensure_side_streams(atomo_ctx* ctx)
{
    if (!ctx->side) ATOMO_HIP(ctx, hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking));
    if (!ctx->side2) ATOMO_HIP(ctx, hipStreamCreateWithFlags(&ctx->side2, hipStreamNonBlocking));
    hipEvent_t* events[] = {&ctx->ev_fork, &ctx->ev_join, &ctx->ev_join2};
    for (hipEvent_t* e : events)
        if (!*e) ATOMO_HIP(ctx, hipEventCreateWithFlags(e, hipEventDisableTiming));
    return ATOMO_OK;
}

int upload(atomo_ctx* ctx, void* dst, const void* src, size_t bytes, hipStream_t stream)
{
    if (bytes == 0) return ATOMO_OK;
    const int n_slots = (int)(sizeof(ctx->ring) / sizeof(ctx->ring[0]));
    StageSlot& slot = ctx->ring[ctx->ring_next];
    ctx->ring_next = (ctx->ring_next + 1) % n_slots;
    if (slot.pending) {                       // the copy that last used this slot must have run
        ATOMO_HIP(ctx, hipEventSynchronize(slot.ev));
        slot.pending = false;
    }
    if (slot.bytes < bytes) {
        if (slot.host) ATOMO_HIP(ctx, hipHostFree(slot.host));
        slot.host = nullptr;
        slot.bytes = 0;
        // (allocating pinned memory waits for the device: every slot grows to the largest upload seen so far, so that
        // the ring settles within one round of eight uploads)
        size_t want = align_up(bytes * 2, 4096);
        for (const StageSlot& other : ctx->ring) want = std::max(want, other.bytes);
        ATOMO_HIP(ctx, hipHostMalloc(&slot.host, want, hipHostMallocDefault));
        slot.bytes = want;
    }
    if (!slot.ev) ATOMO_HIP(ctx, hipEventCreateWithFlags(&slot.ev, hipEventDisableTiming));
    memcpy(slot.host, src, bytes);
    ATOMO_HIP(ctx, hipMemcpyAsync(dst, slot.host, bytes, hipMemcpyHostToDevice, stream));
    ATOMO_HIP(ctx, hipEventRecord(slot.ev, stream));
    slot.pending = true;
    return ATOMO_OK;
}

}  // namespace atomo

using namespace atomo;

namespace {

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(atomo_ctx* ctx)
    {
        if (hipGetDevice(&prev) != hipSuccess) prev = -1;
        hipError_t e = hipSetDevice(ctx->device);
        ok = (e == hipSuccess);
        if (!ok) ctx->last_hip = (int)e;
    }
    ~DeviceGuard()
    {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

bool bad_budget(double s) { return !(s > 0.0) || std::isnan(s) || std::isinf(s); }

}  // namespace

extern "C" {

int atomo_create(atomo_ctx** out, int device)
{
    if (!out) return ATOMO_EINVAL;
    *out = nullptr;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev) return ATOMO_EHIP;
    atomo_ctx* ctx = new (std::nothrow) atomo_ctx();
    if (!ctx) return ATOMO_ENOMEM;
    ctx->device = device;
    DeviceGuard guard(ctx);
    if (!guard.ok) { delete ctx; return ATOMO_EHIP; }
    if (hipMalloc((void**)&ctx->d_flags, FLAG_COUNT * sizeof(int32_t)) != hipSuccess ||
        hipMemset(ctx->d_flags, 0, FLAG_COUNT * sizeof(int32_t)) != hipSuccess ||
        hipHostMalloc((void**)&ctx->h_flags, FLAG_COUNT * sizeof(int32_t), hipHostMallocDefault) != hipSuccess) {
        if (ctx->d_flags) (void)hipFree(ctx->d_flags);
        delete ctx;
        return ATOMO_EHIP;
    }
    // set-up for atomo_encode_entrywise_noalloc: the address of its static scratch array on this device
    if (entrywise_noalloc_setup(ctx) != ATOMO_OK) {
        (void)hipFree(ctx->d_flags);
        (void)hipHostFree(ctx->h_flags);
        delete ctx;
        return ATOMO_EHIP;
    }
    *out = ctx;
    return ATOMO_OK;
}

int atomo_destroy(atomo_ctx* ctx)
{
    if (!ctx) return ATOMO_EINVAL;
    DeviceGuard guard(ctx);
    (void)hipDeviceSynchronize();
    for (auto& slot : ctx->ring) {
        if (slot.ev) (void)hipEventDestroy(slot.ev);
        if (slot.host) (void)hipHostFree(slot.host);
    }
    for (auto& h : ctx->hints) {
        if (h.done) (void)hipEventDestroy(h.done);
        if (h.host) (void)hipHostFree(h.host);
    }
    for (hipEvent_t e : ctx->ev_pool) (void)hipEventDestroy(e);
    for (hipEvent_t e : {ctx->ev_fork, ctx->ev_join, ctx->ev_join2})
        if (e) (void)hipEventDestroy(e);
    if (ctx->side) (void)hipStreamDestroy(ctx->side);
    if (ctx->side2) (void)hipStreamDestroy(ctx->side2);
    if (ctx->ws) (void)hipFree(ctx->ws);
    if (ctx->dec_tables_dev) (void)hipFree(ctx->dec_tables_dev);
    if (ctx->ew_state) (void)hipFree(ctx->ew_state);
    if (ctx->d_report) (void)hipFree(ctx->d_report);
    if (ctx->d_flags) (void)hipFree(ctx->d_flags);
    if (ctx->h_flags) (void)hipHostFree(ctx->h_flags);
    delete ctx;
    return ATOMO_OK;
}

int atomo_reserve(atomo_ctx* ctx, size_t bytes)
{
    if (!ctx) return ATOMO_EINVAL;
    DeviceGuard guard(ctx);
    if (!guard.ok) return ATOMO_EHIP;
    return ensure_workspace(ctx, bytes);
}

int atomo_svd_workspace_bytes(const atomo_mat* mats, int n_mats, size_t* bytes)
{
    if (!mats || n_mats <= 0 || !bytes) return ATOMO_EINVAL;
    return svd_workspace_bytes(mats, n_mats, bytes);
}

int atomo_entrywise_workspace_bytes(int64_t n, size_t* bytes)
{
    if (n <= 0 || n >= ((int64_t)1 << 32) || !bytes) return ATOMO_EINVAL;
    *bytes = entrywise_workspace_bytes(n);
    return ATOMO_OK;
}

int atomo_status(atomo_ctx* ctx, void* stream, int32_t* sweeps)
{
    if (!ctx) return ATOMO_EINVAL;
    DeviceGuard guard(ctx);
    if (!guard.ok) return ATOMO_EHIP;
    hipStream_t st = (hipStream_t)stream;
    ATOMO_HIP(ctx, hipMemcpyAsync(ctx->h_flags, ctx->d_flags, FLAG_COUNT * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    ATOMO_HIP(ctx, hipMemsetAsync(ctx->d_flags, 0, FLAG_COUNT * sizeof(int32_t), st));
    ATOMO_HIP(ctx, hipStreamSynchronize(st));
    if (sweeps) *sweeps = ctx->h_flags[FLAG_MAX_SWEEPS];
    if (ctx->h_flags[FLAG_CAPACITY]) return ATOMO_ECAPACITY;
    if (ctx->h_flags[FLAG_NOCONV]) return ATOMO_ENOCONV;
    return ATOMO_OK;
}

int atomo_svd_sweeps(atomo_ctx* ctx, void* stream, int32_t* sweeps, int32_t* refreshes, int n_mats)
{
    if (!ctx || !sweeps || n_mats <= 0) return ATOMO_EINVAL;
    DeviceGuard guard(ctx);
    if (!guard.ok) return ATOMO_EHIP;
    return svd_sweeps(ctx, (hipStream_t)stream, sweeps, refreshes, n_mats);
}

int atomo_profile_enable(atomo_ctx* ctx, int enable)
{
    if (!ctx) return ATOMO_EINVAL;
    DeviceGuard guard(ctx);
    if (!guard.ok) return ATOMO_EHIP;
    ATOMO_HIP(ctx, hipDeviceSynchronize());
    ctx->profiling = enable != 0;
    ctx->ev_used = 0;
    return ATOMO_OK;
}

int atomo_profile_read(atomo_ctx* ctx, double* total_ms, int64_t* launches)
{
    if (!ctx || !total_ms || !launches) return ATOMO_EINVAL;
    DeviceGuard guard(ctx);
    if (!guard.ok) return ATOMO_EHIP;
    for (size_t k = 0; k < ctx->ev_used; ++k) {
        ATOMO_HIP(ctx, hipEventSynchronize(ctx->ev_pool[2 * k + 1]));
        float ms = 0.0f;
        ATOMO_HIP(ctx, hipEventElapsedTime(&ms, ctx->ev_pool[2 * k], ctx->ev_pool[2 * k + 1]));
        const int kind = ctx->ev_kind[k];
        if (kind >= 0 && kind < ATOMO_K_COUNT) {
            total_ms[kind] += (double)ms;
            launches[kind] += 1;
        }
    }
    ctx->ev_used = 0;
    return ATOMO_OK;
}

namespace {

typedef float probe_floatx16 __attribute__((ext_vector_type(16)));

// Nothing but fp32 matrix-core instructions: four independent accumulators per wave, `iters` rounds.
__global__ __launch_bounds__(256) void mfma_fp32_loop(float* sink, int iters)
{
    probe_floatx16 acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[q][v] = 0.0f;
    const float a = 1.0f + 1e-3f * (float)(threadIdx.x & 63), b = 1.0f - 1e-3f * (float)(threadIdx.x >> 6);
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[q], 0, 0, 0);
    }
    float sum = 0.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) sum += acc[q][v];
    if (sum == -1.0f) sink[0] = sum;                             // never true; keeps the loop alive
}

}  // namespace

int atomo_measure_mfma_fp32(atomo_ctx* ctx, double* tflops, void* stream)
{
    if (!ctx || !tflops) return ATOMO_EINVAL;
    DeviceGuard guard(ctx);
    if (!guard.ok) return ATOMO_EHIP;
    hipStream_t st = (hipStream_t)stream;
    int rc = ensure_workspace(ctx, 256);
    if (rc != ATOMO_OK) return rc;
    hipDeviceProp_t prop;
    ATOMO_HIP(ctx, hipGetDeviceProperties(&prop, ctx->device));
    const int wgs = prop.multiProcessorCount * 4, iters = 4000;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ATOMO_HIP(ctx, hipEventCreate(&e0));
    ATOMO_HIP(ctx, hipEventCreate(&e1));
    mfma_fp32_loop<<<wgs, 256, 0, st>>>((float*)ctx->ws, 16);     // warm-up
    ATOMO_HIP(ctx, hipEventRecord(e0, st));
    mfma_fp32_loop<<<wgs, 256, 0, st>>>((float*)ctx->ws, iters);
    ATOMO_HIP(ctx, hipEventRecord(e1, st));
    ATOMO_HIP(ctx, hipEventSynchronize(e1));
    float ms = 0.0f;
    ATOMO_HIP(ctx, hipEventElapsedTime(&ms, e0, e1));
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    // waves x rounds x 4 instructions x (32 x 32 x 2 multiply-adds = 4096 flop)
    *tflops = (double)wgs * 4.0 * (double)iters * 4.0 * 4096.0 / ((double)ms * 1e-3) / 1e12;
    return ATOMO_OK;
}

int atomo_last_hip_error(const atomo_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

int atomo_last_counters(const atomo_ctx* ctx, int32_t* pair_visits, int32_t* jacobi_steps, int32_t* row_update_tiles)
{
    if (!ctx || !pair_visits || !jacobi_steps || !row_update_tiles) return ATOMO_EINVAL;
    *pair_visits = ctx->h_flags[FLAG_EIG_VISITS];
    *jacobi_steps = ctx->h_flags[FLAG_EIG_INNER];
    *row_update_tiles = ctx->h_flags[FLAG_DS_UPDATE_UNITS];
    return ATOMO_OK;
}

const char* atomo_strerror(int status)
{
    switch (status) {
        case ATOMO_OK: return "ok";
        case ATOMO_EINVAL: return "invalid argument";
        case ATOMO_ECAPACITY: return "a message kept more atoms than its capacity";
        case ATOMO_ENOCONV: return "Jacobi SVD reached the sweep limit";
        case ATOMO_EHIP: return "HIP runtime error";
        case ATOMO_ENOMEM: return "out of device memory";
        case ATOMO_ETOOLARGE: return "input longer than the fixed scratch of the allocation-free entry point holds";
        default: return "unknown status";
    }
}

int atomo_probabilities(atomo_ctx* ctx, const float* lambda, const int64_t* offsets, int n_seg, double s, float* p,
                        void* stream)
{
    if (!ctx || !offsets || n_seg < 0 || bad_budget(s)) return ATOMO_EINVAL;
    if (n_seg == 0) return ATOMO_OK;
    if (offsets[0] < 0) return ATOMO_EINVAL;
    for (int k = 0; k < n_seg; ++k) {
        if (offsets[k + 1] < offsets[k]) return ATOMO_EINVAL;
        if (offsets[k + 1] - offsets[k] >= ((int64_t)1 << 32)) return ATOMO_EINVAL;
    }
    if (offsets[n_seg] == offsets[0]) return ATOMO_OK;
    if (!lambda || !p) return ATOMO_EINVAL;
    DeviceGuard guard(ctx);
    if (!guard.ok) return ATOMO_EHIP;
    return probabilities(ctx, lambda, offsets, n_seg, s, p, (hipStream_t)stream);
}

int atomo_encode_svd(atomo_ctx* ctx, const atomo_mat* mats, int n_mats, double s, uint64_t seed, uint64_t stream_base,
                     const atomo_svd_options* opt, const atomo_svd_msg* msgs, float* sigma_out, float* p_out,
                     void* stream)
{
    if (!ctx || !mats || !msgs || n_mats <= 0 || bad_budget(s)) return ATOMO_EINVAL;
    for (int j = 0; j < n_mats; ++j) {
        const atomo_mat& a = mats[j];
        const atomo_svd_msg& m = msgs[j];
        if (!a.data || a.rows <= 0 || a.cols <= 0 || a.ld < a.cols) return ATOMO_EINVAL;
        if ((a.rows < a.cols ? a.rows : a.cols) > 2048) return ATOMO_EINVAL;
        if ((a.rows > a.cols ? a.rows : a.cols) > (1 << 30)) return ATOMO_EINVAL;   // position indices stay in int32
        if (m.rows != a.rows || m.cols != a.cols || m.capacity < 1) return ATOMO_EINVAL;
        if (!m.count || !m.idx || !m.U || !m.V) return ATOMO_EINVAL;         // w may be null: folded form
    }
    if (opt && (opt->max_sweeps < 0 || !(opt->stop_cosine >= 0.0f) || opt->max_inner_sweeps < 0 ||
                !(opt->inner_reduction >= 0.0f) || opt->full_period < 0 || opt->adaptive < 0))
        return ATOMO_EINVAL;
    DeviceGuard guard(ctx);
    if (!guard.ok) return ATOMO_EHIP;
    return encode_svd(ctx, mats, n_mats, s, seed, stream_base, opt, msgs, sigma_out, p_out, (hipStream_t)stream);
}

int atomo_encode_entrywise(atomo_ctx* ctx, const float* g, double s, uint64_t seed, uint64_t stream_id,
                           const atomo_ew_msg* msg, float* p_out, void* stream)
{
    if (!ctx || !g || !msg || bad_budget(s)) return ATOMO_EINVAL;
    if (msg->n <= 0 || msg->n >= ((int64_t)1 << 32) || msg->capacity < 1) return ATOMO_EINVAL;
    if (!msg->count || !msg->idx || !msg->val) return ATOMO_EINVAL;
    DeviceGuard guard(ctx);
    if (!guard.ok) return ATOMO_EHIP;
    return encode_entrywise(ctx, g, s, seed, stream_id, msg, p_out, (hipStream_t)stream);
}

int atomo_encode_lq(atomo_ctx* ctx, const float* g, double q, uint64_t seed, uint64_t stream_id,
                    const atomo_lq_msg* msg, float* p_out, void* stream)
{
    if (!ctx || !g || !msg || !(q > 0.0)) return ATOMO_EINVAL;                      // (NaN fails the comparison)
    if (msg->n <= 0 || msg->n >= ((int64_t)1 << 31) || msg->capacity < 1) return ATOMO_EINVAL;
    if (!msg->count || !msg->idx || !msg->norm) return ATOMO_EINVAL;
    DeviceGuard guard(ctx);
    if (!guard.ok) return ATOMO_EHIP;
    return encode_lq(ctx, g, q, seed, stream_id, msg, p_out, (hipStream_t)stream);
}

static int svd_batch(atomo_ctx* ctx, const atomo_svd_msg* msgs, const int32_t* first, int n_out, float scale,
                     float* const* outs, const int64_t* lds, bool accumulate, void* stream)
{
    if (!ctx || !first || !outs || !lds || n_out <= 0) return ATOMO_EINVAL;
    if (first[0] != 0) return ATOMO_EINVAL;
    for (int o = 0; o < n_out; ++o) {
        if (first[o + 1] <= first[o] || !outs[o]) return ATOMO_EINVAL;
        if (!msgs) return ATOMO_EINVAL;
        const atomo_svd_msg& m0 = msgs[first[o]];
        if (m0.rows <= 0 || m0.cols <= 0 || lds[o] < m0.cols) return ATOMO_EINVAL;
        for (int k = first[o]; k < first[o + 1]; ++k) {
            const atomo_svd_msg& m = msgs[k];
            if (m.rows != m0.rows || m.cols != m0.cols || m.capacity < 1) return ATOMO_EINVAL;
            if (!m.count || !m.idx || !m.U || !m.V) return ATOMO_EINVAL;     // w may be null: folded form
        }
    }
    DeviceGuard guard(ctx);
    if (!guard.ok) return ATOMO_EHIP;
    return decode_svd_batch(ctx, msgs, first, n_out, scale, outs, lds, accumulate, (hipStream_t)stream);
}

int atomo_decode_svd_batch(atomo_ctx* ctx, const atomo_svd_msg* msgs, const int32_t* first, int n_out, float scale,
                           float* const* outs, const int64_t* lds, void* stream)
{
    return svd_batch(ctx, msgs, first, n_out, scale, outs, lds, false, stream);
}

int atomo_apply_svd_batch(atomo_ctx* ctx, const atomo_svd_msg* msgs, const int32_t* first, int n_out, float alpha,
                          float* const* params, const int64_t* lds, void* stream)
{
    return svd_batch(ctx, msgs, first, n_out, alpha, params, lds, true, stream);
}

int atomo_decode(atomo_ctx* ctx, int kind, const void* msgs, int n_msgs, float scale, float* out, int64_t ld,
                 void* stream)
{
    if (!ctx || !msgs || n_msgs <= 0 || !out) return ATOMO_EINVAL;
    if (kind == ATOMO_KIND_SVD) {
        const int32_t first[2] = {0, n_msgs};
        float* const outs[1] = {out};
        const int64_t lds[1] = {ld};
        return atomo_decode_svd_batch(ctx, (const atomo_svd_msg*)msgs, first, 1, scale, outs, lds, stream);
    }
    if (kind == ATOMO_KIND_ENTRYWISE) {
        const atomo_ew_msg* m = (const atomo_ew_msg*)msgs;
        for (int k = 0; k < n_msgs; ++k) {
            if (m[k].n != m[0].n || m[k].n <= 0 || m[k].n >= ((int64_t)1 << 32) || m[k].capacity < 1) return ATOMO_EINVAL;
            if (!m[k].count || !m[k].idx || !m[k].val) return ATOMO_EINVAL;
        }
        DeviceGuard guard(ctx);
        if (!guard.ok) return ATOMO_EHIP;
        return decode_entrywise(ctx, m, n_msgs, scale, out, (hipStream_t)stream);
    }
    if (kind == ATOMO_KIND_LQ) {
        const atomo_lq_msg* m = (const atomo_lq_msg*)msgs;
        for (int k = 0; k < n_msgs; ++k) {
            if (m[k].n != m[0].n || m[k].n <= 0 || m[k].n >= ((int64_t)1 << 31) || m[k].capacity < 1) return ATOMO_EINVAL;
            if (!m[k].count || !m[k].idx || !m[k].norm) return ATOMO_EINVAL;
        }
        DeviceGuard guard(ctx);
        if (!guard.ok) return ATOMO_EHIP;
        return decode_lq(ctx, m, n_msgs, scale, out, (hipStream_t)stream);
    }
    return ATOMO_EINVAL;
}

}  // extern "C"
