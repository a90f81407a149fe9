// Internal declarations shared by the translation units of libatomo (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "../../include/atomo.h"
#include "../../include/atomo_bench.h"

namespace atomo {

// ---------------------------------------------------------------------------------------------
// Context
// ---------------------------------------------------------------------------------------------

// Device-side latched flags (int32 each).
enum { FLAG_CAPACITY = 0, FLAG_NOCONV = 1, FLAG_MAX_SWEEPS = 2, FLAG_EIG_VISITS = 3, FLAG_EIG_INNER = 4, FLAG_DS_UPDATE_UNITS = 5, FLAG_COUNT = 8 };

// What an SVD encode learnt about its own sweep counts, for the calls after it (atomo_svd_options.adaptive).
struct SweepHint {
    int32_t* host = nullptr;     // pinned, device-visible: [0] most sweeps of a Gram-space matrix, [1] of a data-space one,
                                 // [2] 1 once written
    int32_t* dev = nullptr;      // the same memory as the device addresses it
    hipEvent_t done = nullptr;   // recorded after the kernel that writes `host`
    bool pending = false;        // the event has not been seen complete yet
    uint64_t sig = 0;            // shapes of the call
    uint64_t seq = 0;            // order of the calls (0 = unused)
    int limit_gs = 0, limit_ds = 0;   // the sweep limits that call ran with
};

struct StageSlot {
    void* host = nullptr;        // pinned
    size_t bytes = 0;
    hipEvent_t ev = nullptr;     // recorded after the last copy out of `host`
    bool pending = false;
};

}  // namespace atomo

struct atomo_ctx {
    int device = 0;
    void* ws = nullptr;          // device workspace
    size_t ws_bytes = 0;
    int32_t* d_flags = nullptr;  // [FLAG_COUNT] device
    int32_t* h_flags = nullptr;  // pinned readback buffer
    int last_hip = 0;
    atomo::StageSlot ring[8];
    int ring_next = 0;
    // sweep and refresh counts of the last SVD encode, [2 * report_n] on the device, outside the workspace (which the
    // next call of any kind overwrites)
    int32_t* d_report = nullptr;
    size_t report_cap = 0;               // pairs allocated
    size_t report_n = 0;                 // matrices of the last SVD encode
    // streams and events of the SVD encoder's internal fork/join (created on first use, default priority)
    void* ew_state = nullptr;            // entry-wise encoder: search state kept from call to call (histograms zero between calls)
    atomo::SweepHint hints[4];
    int hint_next = 0;
    uint64_t hint_seq = 0;
    size_t rowgram_lds = 0;        // dynamic LDS that svd_rowgram has been allowed on this context's device
    // Descriptor tables of the last SVD encode (at the start of the workspace) and of the last SVD decode (in a block
    // of their own): a training loop passes the same layer set and buffers step after step, so a call whose tables
    // come out byte for byte the same, on the same stream, with the device copy untouched since, uploads nothing.
    std::vector<char> svd_tables;        // host copy of what the workspace holds
    bool svd_tables_intact = false;      // nothing has asked for the workspace since they were uploaded
    hipStream_t svd_tables_stream = nullptr;
    void* dec_tables_dev = nullptr;
    size_t dec_tables_cap = 0;
    std::vector<char> dec_tables;        // host copy of what dec_tables_dev holds
    hipStream_t dec_tables_stream = nullptr;
    hipStream_t side = nullptr, side2 = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr, ev_join2 = nullptr;
    // optional event bracketing of kernel launches (atomo_profile_*)
    bool profiling = false;
    std::vector<hipEvent_t> ev_pool;     // pairs: [2k] start, [2k+1] stop
    std::vector<int> ev_kind;            // kernel class of pair k
    size_t ev_used = 0;                  // pairs in use
};

namespace atomo {

#define ATOMO_HIP(ctx, call)                                   \
    do {                                                       \
        hipError_t e__ = (call);                               \
        if (e__ != hipSuccess) {                               \
            (ctx)->last_hip = (int)e__;                        \
            return ATOMO_EHIP;                                 \
        }                                                      \
    } while (0)

// Grows the workspace to at least `bytes` (contents are not preserved).  Every user of the workspace asks for it here
// first, so this is also where the SVD encoder's tables stop counting as intact.
int ensure_workspace(atomo_ctx* ctx, size_t bytes);

// Creates ctx->side, ctx->side2 and the fork/join events if they do not exist yet.
int ensure_side_streams(atomo_ctx* ctx);

// Copies `bytes` of host data to device address `dst` on `stream` through a pinned staging slot,
// so the caller's host buffer may be reused as soon as this returns.
int upload(atomo_ctx* ctx, void* dst, const void* src, size_t bytes, hipStream_t stream);

// Brackets the launches issued during its lifetime with two events when profiling is on.
struct ProfScope {
    atomo_ctx* ctx;
    hipStream_t stream;
    hipEvent_t stop = nullptr;
    ProfScope(atomo_ctx* c, int kind, hipStream_t s) : ctx(c), stream(s)
    {
        if (!ctx->profiling) return;
        if (ctx->ev_used * 2 >= ctx->ev_pool.size()) {
            hipEvent_t a = nullptr, b = nullptr;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return;
            ctx->ev_pool.push_back(a);
            ctx->ev_pool.push_back(b);
            ctx->ev_kind.push_back(kind);
        }
        ctx->ev_kind[ctx->ev_used] = kind;
        (void)hipEventRecord(ctx->ev_pool[ctx->ev_used * 2], stream);
        stop = ctx->ev_pool[ctx->ev_used * 2 + 1];
        ++ctx->ev_used;
    }
    ~ProfScope()
    {
        if (stop) (void)hipEventRecord(stop, stream);
    }
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// A bump allocator over the workspace; first pass with base == nullptr only measures.
struct Carver {
    char* base;
    size_t off = 0;
    size_t last = 0;                     // offset of what the last take returned
    explicit Carver(void* b) : base((char*)b) {}
    template <typename T>
    T* take(size_t count) {
        off = align_up(off, 256);
        last = off;
        T* p = base ? (T*)(base + off) : nullptr;
        off += count * sizeof(T);
        return p;
    }
};

// Workgroups go to the chip's eight dies in turn (workgroup b to die b mod 8), and each die has its own L2.  Reorders a
// work list so that every die gets one contiguous run of it: neighbours in the list, which read the same operands,
// then find them in the same L2 instead of fetching them into all eight.
template <typename T>
inline void deal_to_dies(std::vector<T>& list)
{
    constexpr size_t DIES = 8;
    const size_t n = list.size();
    std::vector<T> dealt(n);
    size_t start[DIES + 1] = {0};
    for (size_t x = 0; x < DIES; ++x) start[x + 1] = start[x] + (n + DIES - 1 - x) / DIES;
    for (size_t b = 0; b < n; ++b) dealt[b] = list[start[b % DIES] + b / DIES];
    list.swap(dealt);
}

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): device + host inline so every kernel draws the same stream
// ---------------------------------------------------------------------------------------------

struct u32x4 { uint32_t x, y, z, w; };

__host__ __device__ inline u32x4 philox4x32_10(uint64_t block, uint64_t stream_id, uint64_t seed)
{
    uint32_t c0 = (uint32_t)block, c1 = (uint32_t)(block >> 32);
    uint32_t c2 = (uint32_t)stream_id, c3 = (uint32_t)(stream_id >> 32);
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return u32x4{c0, c1, c2, c3};
}

// 24 random bits -> [0,1), exact in float32.
__host__ __device__ inline float u01(uint32_t word) { return (float)(word >> 8) * 5.9604644775390625e-08f; }

// ---------------------------------------------------------------------------------------------
// Entry points implemented per translation unit
// ---------------------------------------------------------------------------------------------

int svd_workspace_bytes(const atomo_mat* mats, int n_mats, size_t* bytes);
int encode_svd(atomo_ctx* ctx, const atomo_mat* mats, int n_mats, double s, uint64_t seed, uint64_t stream_base,
               const atomo_svd_options* opt, const atomo_svd_msg* msgs, float* sigma_out, float* p_out,
               hipStream_t stream);

int svd_sweeps(atomo_ctx* ctx, hipStream_t stream, int32_t* sweeps, int32_t* refreshes, int n_mats);

size_t entrywise_workspace_bytes(int64_t n);
int encode_entrywise(atomo_ctx* ctx, const float* g, double s, uint64_t seed, uint64_t stream_id,
                     const atomo_ew_msg* msg, float* p_out, hipStream_t stream);
int entrywise_noalloc_setup(atomo_ctx* ctx);   // device address of the static scratch array, once per device
int encode_lq(atomo_ctx* ctx, const float* g, double q, uint64_t seed, uint64_t stream_id, const atomo_lq_msg* msg,
              float* p_out, hipStream_t stream);
int probabilities(atomo_ctx* ctx, const float* lambda, const int64_t* offsets, int n_seg, double s, float* p,
                  hipStream_t stream);

// accumulate: outs[o] += ... instead of outs[o] = ...
int decode_svd_batch(atomo_ctx* ctx, const atomo_svd_msg* msgs, const int32_t* first, int n_out, float scale,
                     float* const* outs, const int64_t* lds, bool accumulate, hipStream_t stream);
int decode_entrywise(atomo_ctx* ctx, const atomo_ew_msg* msgs, int n_msgs, float scale, float* out,
                     hipStream_t stream);
int decode_lq(atomo_ctx* ctx, const atomo_lq_msg* msgs, int n_msgs, float scale, float* out, hipStream_t stream);

}  // namespace atomo
