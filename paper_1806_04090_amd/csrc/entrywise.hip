// Entry-wise ATOMO (Section 3 of arXiv 1806.04090 with the standard basis: lambda_i = g_i, a_i = e_i)
// and the stand-alone Algorithm 1 entry point.
//
// Algorithm 1 without a sort.  The KKT appendix shows the optimum has the water-filling form
// p_i = min(1, |lambda_i| / tau) with one level tau, tau = (sum of the uncapped |lambda|) / (s - n_s)
// (eq. (p_i)).  With N(v) = #{|lambda| > v} and T(v) = sum of the |lambda| <= v, the function
//     h(v) = v * (s - N(v)) - T(v)
// is continuous, has h <= 0 below tau and h > 0 above it, and an element is capped (p = 1) exactly
// when h(|lambda_i|) > 0 - the same test Algorithm 1 applies along the sorted order.  h can be
// evaluated exactly at bucket edges from a histogram that stores, per bucket of the float bit
// pattern, the element count and the sum of the 24-bit significands (all elements of a bucket share
// their exponent, so this integer sum is exact and independent of summation order).  Three levels of
// 11 + 10 + 10 key bits pin tau down to a single float value; each level is one pass over the data
// that only histograms elements inside the bucket chosen by the previous level.  A level whose
// chosen bucket holds zero or one element already decides everything and the remaining levels are
// skipped on the device.
//
// Sampling and packing.  Coordinate i is kept iff u_i < p_i (Philox stream, float32 compare) and is
// stored as (i, g_i / p_i) in ascending i.  The encoder reads the gradient twice ("the two-read encoder"
// below): once for the level-0 histogram, once to draw every uniform and settle it against the bracket
// that level 0 leaves for p_i; the few draws that fall inside the bracket wait for the exact water level.
// The l_q encoder (Section 4), whose probabilities need only a norm, uses the plain form: a counting pass
// per 4096-element chunk, a scan of the chunk counts, and a writing pass that reads the keep bits.
#include <cmath>
#include <vector>

#include "atomo_internal.h"
#include "block_algorithm1.h"

namespace atomo {

namespace {

constexpr int L0_BITS = 11, L1_BITS = 10, L2_BITS = 10;
constexpr int NBUCKET = 1 << L0_BITS;        // the largest level
constexpr int HIST_WGS = 1024;
constexpr int CHUNK = 4096;                  // elements per sampling workgroup (256 threads x 4 float4)

// What a level leaves behind: either the final answer or the path to continue on.
struct SolveOut {
    int done;                     // n_s and tail are final
    unsigned int prefix;          // key bits chosen so far (not done)
    unsigned long long n_above;   // elements above the chosen bucket
    double sum_below;             // sum of the elements below it
    unsigned long long n_s;       // done: number of capped elements
    double tail;                  // done: sum of the uncapped magnitudes
    double lo, hi;                // level 0: the edges of the chosen bucket; the water level lies in [lo, hi]
};

struct EwState {
    unsigned int cnt[3][NBUCKET];
    unsigned long long sig[3][NBUCKET];
    SolveOut lvl[3];              // what each level found (written by one kernel, read by the kernels after it);
                                  // lvl[k].done also when an earlier level already settled everything
    unsigned int ticket[3][65];   // per pass: workgroups that have finished (the last one solves the level); zero between calls
    unsigned long long n_s;       // final: number of capped elements
    double tail;                  // final: sum of the uncapped magnitudes
    double budget;                // final: s - n_s
    double ratio;                 // final: budget / tail, +inf if tail == 0
    unsigned long long total_kept;
};


// value of an integer significand sum for elements whose biased exponent is e
__device__ inline double sig_value(unsigned long long sigsum, unsigned int e)
{
    return ldexp((double)sigsum, (int)(e == 0 ? 1 : e) - 150);
}

__device__ inline unsigned int significand(unsigned int key)
{
    const unsigned int e = key >> 23, mant = key & 0x7FFFFFu;
    return e ? (mant | 0x800000u) : mant;
}

__global__ __launch_bounds__(256) void ew_clear(EwState* st)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < 3 * NBUCKET) { (&st->cnt[0][0])[i] = 0u; (&st->sig[0][0])[i] = 0ull; }
    if (i == 0) {
        for (int k = 0; k < 3 * 65; ++k) (&st->ticket[0][0])[k] = 0u;
        for (int k = 0; k < 3; ++k) { st->lvl[k].done = 0; st->lvl[k].prefix = 0u; st->lvl[k].n_above = 0ull; st->lvl[k].sum_below = 0.0; }
        st->n_s = 0ull; st->tail = 0.0; st->budget = 0.0; st->ratio = 0.0; st->total_kept = 0ull;
    }
}

// Level-LEVEL histogram of the elements on the path `prefix`, by the TPB threads of a workgroup (all call):
// accumulated in the LDS array acc (COPIES x NB packed words), then added to the global histogram.
template <int LEVEL, int TPB>
__device__ inline void hist_body(const float* __restrict__ g, long long n, EwState* st, unsigned long long* acc, unsigned int prefix)
{
    // Level 0 sees every element and most of them fall into a few dozen buckets: four copies of the
    // histogram (one per lane mod 4) keep lanes of a wave from queueing on the same LDS word.
    // One 64-bit word per bucket: element count in bits 40.., sum of 24-bit significands below.  A
    // workgroup visits fewer than 2^16 elements (checked by the launcher), so neither field overflows.
    constexpr int COPIES = LEVEL == 0 ? 4 : 1;
    constexpr int NB = LEVEL == 0 ? (1 << L0_BITS) : (1 << L1_BITS);
    constexpr int SHIFT = LEVEL == 0 ? 20 : LEVEL == 1 ? 10 : 0;
    const unsigned int copy = LEVEL == 0 ? (threadIdx.x & (COPIES - 1)) * NB : 0u;
    for (int b = threadIdx.x; b < COPIES * NB; b += TPB) acc[b] = 0ull;
    __syncthreads();

    auto visit = [&](float x) {
        const unsigned int key = __float_as_uint(x) & 0x7FFFFFFFu;
        const unsigned long long word = (1ull << 40) | (unsigned long long)significand(key);
        if (LEVEL == 0) {
            atomicAdd(&acc[copy + (key >> SHIFT)], word);
        } else {
            if ((key >> (SHIFT + (LEVEL == 1 ? L1_BITS : L2_BITS))) == prefix)
                atomicAdd(&acc[(key >> SHIFT) & (NB - 1)], word);
        }
    };

    const bool vec = (((size_t)g) & 15) == 0;
    const long long n4 = vec ? n / 4 : 0;
    const long long stride = (long long)gridDim.x * TPB;
    // four loads in flight per thread: one at a time, the pass is a chain of memory latencies
    for (long long q0 = (long long)blockIdx.x * TPB + threadIdx.x; q0 < n4; q0 += 4 * stride) {
        float4 x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const long long q = q0 + u * stride;
            if (q < n4) x[u] = ((const float4*)g)[q];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (q0 + u * stride < n4) { visit(x[u].x); visit(x[u].y); visit(x[u].z); visit(x[u].w); }
        }
    }
    for (long long i = n4 * 4 + (long long)blockIdx.x * TPB + threadIdx.x; i < n; i += stride) visit(g[i]);
    __syncthreads();
    for (int b = threadIdx.x; b < NB; b += TPB) {
        unsigned int c = 0u;
        unsigned long long sg = 0ull;
#pragma unroll
        for (int k = 0; k < COPIES; ++k) {
            const unsigned long long w = acc[k * NB + b];
            c += (unsigned int)(w >> 40);
            sg += w & ((1ull << 40) - 1);
        }
        if (c) {
            atomicAdd(&st->cnt[LEVEL][b], c);
            atomicAdd(&st->sig[LEVEL][b], sg);
        }
    }
}

// Histogram of one level.  Elements are visited as float4 where the pointer allows.
template <int LEVEL>
__global__ __launch_bounds__(LEVEL == 0 ? 1024 : 256) void ew_hist(const float* __restrict__ g, long long n, EwState* st)
{
    constexpr int TPB = LEVEL == 0 ? 1024 : 256;
    __shared__ unsigned long long acc[(LEVEL == 0 ? 4 : 1) * (LEVEL == 0 ? (1 << L0_BITS) : (1 << L1_BITS))];
    if (LEVEL > 0 && st->lvl[LEVEL > 0 ? LEVEL - 1 : 0].done) return;
    hist_body<LEVEL, TPB>(g, n, st, acc, LEVEL == 0 ? 0u : st->lvl[LEVEL > 0 ? LEVEL - 1 : 0].prefix);
}

// One level of the search, by the T threads of a workgroup (all must call).
// Reads the level's histogram from st, and the path chosen so far from `in` (level 0: nothing).  The result goes
// to `out` (LDS or global, visible to the workgroup after the call's last barrier).
// T threads (256 or 1024); COHERENT: the histogram was written by other workgroups of the running kernel (atomics), so it
// is read with device-scope atomic loads instead of plain ones.
// scratch: LDS, (2 T + 1) x 8 bytes.
template <int LEVEL, int T = 256, bool COHERENT = false>
__device__ inline void solve_level(const EwState* st, double s, unsigned int prefix, unsigned long long n_above0,
                                   double sum_below0, SolveOut* out, unsigned long long* scratch)
{
    unsigned long long* cpart = scratch;
    double* spart = (double*)(scratch + T);
    int& best = *(int*)(scratch + 2 * T);
    constexpr int NB = LEVEL == 0 ? (1 << L0_BITS) : (1 << L1_BITS);
    constexpr int SHIFT = LEVEL == 0 ? 20 : LEVEL == 1 ? 10 : 0;
    constexpr int PER = NB / T;
    static_assert(PER >= 1, "one bucket per thread at least");
    const int tid = threadIdx.x;
    auto bucket_key = [&](int b) -> unsigned int {
        return ((LEVEL == 0 ? 0u : prefix << (LEVEL == 1 ? L1_BITS : L2_BITS)) | (unsigned int)b) << SHIFT;
    };
    // exponent shared by every element on the chosen path (level 0: part of the bucket index)
    auto bucket_exp = [&](int b) -> unsigned int { return bucket_key(b) >> 23; };
    auto bucket_lo = [&](int b) -> double { return (double)__uint_as_float(bucket_key(b)); };

    // this thread's PER consecutive buckets stay in registers
    unsigned int cnt_r[PER];
    double sum_r[PER];
    unsigned long long c_mine = 0ull;
    double s_mine = 0.0;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        const int b = tid * PER + e;
        if (COHERENT) {                                          // (both loads in flight at once)
            cnt_r[e] = __hip_atomic_load(&st->cnt[LEVEL][b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const unsigned long long sg = __hip_atomic_load(&st->sig[LEVEL][b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            sum_r[e] = cnt_r[e] ? sig_value(sg, bucket_exp(b)) : 0.0;
        } else {
            cnt_r[e] = st->cnt[LEVEL][b];
            sum_r[e] = cnt_r[e] ? sig_value(st->sig[LEVEL][b], bucket_exp(b)) : 0.0;    // (most buckets are empty)
        }
        c_mine += cnt_r[e];
        s_mine += sum_r[e];
    }
    __syncthreads();                                             // (the scratch may still be read from a previous call)
    cpart[tid] = c_mine;
    spart[tid] = s_mine;
    if (tid == 0) best = 0;
    __syncthreads();
    // suffix scan of the counts and prefix scan of the sums over the 256 threads (log-step, in LDS)
    for (int off = 1; off < T; off <<= 1) {
        const unsigned long long cv = tid + off < T ? cpart[tid + off] : 0ull;
        const double sv = tid >= off ? spart[tid - off] : 0.0;
        __syncthreads();
        cpart[tid] += cv;
        spart[tid] += sv;
        __syncthreads();
    }
    const unsigned long long c_after = tid < T - 1 ? cpart[tid + 1] : 0ull; // count in buckets owned by later threads
    const double s_before = tid > 0 ? spart[tid - 1] : 0.0;                 // sum in buckets owned by earlier threads

    // h at the lower edge of bucket b:  lo_b * (s - #{elements in buckets >= b}) - sum(buckets < b)
    {
        unsigned long long at_or_above = c_after + c_mine;
        double below = s_before;
        int mine_best = -1;
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            const int b = tid * PER + e;
            const double h = bucket_lo(b) * (s - (double)(n_above0 + at_or_above)) - (sum_below0 + below);
            if (h <= 0.0) mine_best = b;
            at_or_above -= cnt_r[e];
            below += sum_r[e];
        }
        if (mine_best >= 0) atomicMax(&best, mine_best);
    }
    __syncthreads();
    const int bs = best;
    if (tid == bs / PER) {                      // the owner of the chosen bucket finishes from its registers
        unsigned long long above = c_after;
        double below = s_before;
        unsigned int c = 0;
        double bucket_sum = 0.0;
#pragma unroll
        for (int e = 0; e < PER; ++e) {
            const int b = tid * PER + e;
            if (b > bs) above += cnt_r[e];
            if (b < bs) below += sum_r[e];
            if (b == bs) { c = cnt_r[e]; bucket_sum = sum_r[e]; }
        }
        const unsigned long long n_above = n_above0 + above;
        const double sum_below = sum_below0 + below;
        bool done = false;
        unsigned long long n_s = n_above;
        double tail = sum_below;
        if (c == 0) {
            done = true;
        } else if (c == 1) {
            const double x = bucket_sum;                       // the element itself
            if (x * (s - (double)n_above) - sum_below - x > 0.0) n_s = n_above + 1;
            else tail = sum_below + x;
            done = true;
        } else if (LEVEL == 2) {
            tail = sum_below + bucket_sum;                     // equal elements at the level: uncapped
            done = true;
        }
        out->done = done ? 1 : 0;
        out->n_s = n_s;
        out->tail = tail;
        out->n_above = n_above;
        out->sum_below = sum_below;
        out->prefix = (LEVEL == 0 ? 0u : prefix << (LEVEL == 1 ? L1_BITS : L2_BITS)) | (unsigned int)bs;
        out->lo = bucket_lo(bs);
        out->hi = bs + 1 < NB ? bucket_lo(bs + 1) : __longlong_as_double(0x7FF0000000000000LL);
    }
    __syncthreads();
}

// (s - n_s) / tail, or +inf when nothing is left uncapped
__device__ inline double final_ratio(double s, unsigned long long n_s, double tail)
{
    return tail > 0.0 ? (s - (double)n_s) / tail : __longlong_as_double(0x7FF0000000000000LL);
}

// Records what level `level` found; the final quantities once they are known.
__device__ inline void publish(EwState* st, int level, const SolveOut& r, double s)
{
    st->lvl[level] = r;
    if (r.done) {
        st->n_s = r.n_s;
        st->tail = r.tail;
        st->budget = s - (double)r.n_s;
        st->ratio = final_ratio(s, r.n_s, r.tail);
    }
}

template <int LEVEL>
__global__ __launch_bounds__(256) void ew_solve(EwState* st, double s)
{
    __shared__ SolveOut out;
    __shared__ unsigned long long scratch[2 * 256 + 1];
    unsigned int prefix = 0u;
    unsigned long long n_above = 0ull;
    double sum_below = 0.0;
    if (LEVEL > 0) {
        const SolveOut& in = st->lvl[LEVEL > 0 ? LEVEL - 1 : 0];
        if (in.done) {                                           // settled earlier: hand the mark on
            if (threadIdx.x == 0) st->lvl[LEVEL].done = 1;
            return;
        }
        prefix = in.prefix; n_above = in.n_above; sum_below = in.sum_below;
    }
    solve_level<LEVEL>(st, s, prefix, n_above, sum_below, &out, scratch);
    if (threadIdx.x == 0) publish(st, LEVEL, out, s);
}

// True in every thread of the workgroup that finishes last among the launch's workgroups (all threads of every
// workgroup call, at their very end).  The last workgroup may then read what the others added to the global
// histograms, with device-scope atomic loads: every wave first waits until its own atomics have been performed
// (s_waitcnt vmcnt(0): on gfx9 stores and atomics count in vmcnt, and a workgroup barrier alone does not wait for memory
// operations in flight), and device-scope atomics are performed where every compute unit sees them, so no cache
// maintenance is involved.  Nobody waits for anybody: the others simply leave.
// Tickets in two levels (thousands of atomic adds on one address are performed one after the other, about ten
// nanoseconds each): a workgroup counts on word blockIdx.x mod 64, the last one of a word counts on word 64.
// ticket: [65] words, zero on entry and zero again when the last workgroup returns.
__device__ inline bool last_workgroup(unsigned int* ticket)
{
    __shared__ int last_sh;
    __builtin_amdgcn_s_waitcnt(0x0F70);                          // vmcnt(0), other counters untouched
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int slots = min(64u, gridDim.x), slot = blockIdx.x % slots;
        const unsigned int members = (gridDim.x - slot + slots - 1) / slots;
        int last = 0;
        if (__hip_atomic_fetch_add(&ticket[slot], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == members - 1)
            last = __hip_atomic_fetch_add(&ticket[64], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == slots - 1;
        last_sh = last;
    }
    __syncthreads();
    if (last_sh && threadIdx.x < 65)                             // for the next call
        __hip_atomic_store(&ticket[threadIdx.x], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return last_sh != 0;
}

// ew_hist<0> whose last workgroup solves level 0 at once: one launch and one chain of dependent loads less than with
// ew_solve<0> behind it.
__global__ __launch_bounds__(1024) void ew_hist0_solve0(const float* __restrict__ g, long long n, EwState* st, double s)
{
    __shared__ unsigned long long acc[4 * NBUCKET];
    __shared__ SolveOut out;
    hist_body<0, 1024>(g, n, st, acc, 0u);
    if (!last_workgroup(st->ticket[0])) return;
    solve_level<0, 1024, true>(st, s, 0u, 0ull, 0.0, &out, acc);            // (acc is spent: scratch)
    if (threadIdx.x == 0) publish(st, 0, out, s);
}

// p = min(1, |x| (s - n_s) / tail) (eq. (p_i), KKT appendix); `ratio` = (s - n_s) / tail in double,
// or +inf when nothing is left uncapped.  One double multiply and one rounding to float per element.
__device__ inline float ew_probability(float x, double ratio)
{
    const float a = fabsf(x);
    if (a == 0.0f) return 0.0f;
    return fminf(1.0f, (float)((double)a * ratio));
}

// p for a large segment of atomo_probabilities
__global__ __launch_bounds__(256) void ew_write_p(const float* __restrict__ lam, long long n, const EwState* st,
                                                  float* __restrict__ p)
{
    const double ratio = st->ratio;
    const long long stride = (long long)gridDim.x * 256;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += stride)
        p[i] = ew_probability(lam[i], ratio);
}

// Draws for the four coordinates 4q .. 4q+3 (one Philox block).  Returns the keep bits.
__device__ inline unsigned int draw4(const float4 x, long long q, unsigned long long stream_id, unsigned long long seed,
                                     double ratio, float4& p)
{
    const u32x4 rnd = philox4x32_10((unsigned long long)q, stream_id, seed);
    p.x = ew_probability(x.x, ratio);
    p.y = ew_probability(x.y, ratio);
    p.z = ew_probability(x.z, ratio);
    p.w = ew_probability(x.w, ratio);
    return (u01(rnd.x) < p.x ? 1u : 0u) | (u01(rnd.y) < p.y ? 2u : 0u) | (u01(rnd.z) < p.z ? 4u : 0u) |
           (u01(rnd.w) < p.w ? 8u : 0u);
}

__device__ inline float4 load4(const float* g, long long q, long long n, bool vec)
{
    const long long i = q * 4;
    if (vec && i + 3 < n) return ((const float4*)g)[q];
    float4 x;
    x.x = i < n ? g[i] : 0.0f;
    x.y = i + 1 < n ? g[i + 1] : 0.0f;
    x.z = i + 2 < n ? g[i + 2] : 0.0f;
    x.w = i + 3 < n ? g[i + 3] : 0.0f;
    return x;
}

// Kept coordinates per chunk, and their keep bits.  Wave w of a chunk owns float4 [w*256, (w+1)*256) of the
// chunk, in four iterations of 64 lanes: order inside a chunk is (wave, iteration, lane, component) =
// ascending index.  keep[((chunk*4 + wave)*4 + iteration)*4 + component] holds one bit per lane, so that the
// writer neither draws the random numbers again nor reads the gradient outside the kept coordinates.
__global__ __launch_bounds__(256) void ew_count(const float* __restrict__ g, long long n, const EwState* st,
                                                unsigned long long stream_id, unsigned long long seed,
                                                unsigned int* __restrict__ chunk_count,
                                                unsigned long long* __restrict__ keep)
{
    __shared__ unsigned int wsum[4];
    const double ratio = st->ratio;
    const bool vec = (((size_t)g) & 15) == 0;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long q0 = (long long)blockIdx.x * (CHUNK / 4) + wave * 256;
    unsigned long long* kw = keep + ((long long)blockIdx.x * 4 + wave) * 16;
    unsigned int kept = 0;                                   // wave-uniform
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const long long q = q0 + j * 64 + lane;
        unsigned int bits = 0;
        if (q * 4 < n) {
            float4 p;
            bits = draw4(load4(g, q, n, vec), q, stream_id, seed, ratio, p);
        }
        unsigned long long mine = 0ull;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const unsigned long long ballot = __ballot((bits >> c) & 1u);
            kept += __popcll(ballot);
            if (lane == c) mine = ballot;
        }
        if (lane < 4) kw[j * 4 + lane] = mine;
    }
    if (lane == 0) wsum[wave] = kept;
    __syncthreads();
    if (threadIdx.x == 0) chunk_count[blockIdx.x] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

// Exclusive scan of the chunk counts (single workgroup).
__global__ __launch_bounds__(256) void ew_scan(const unsigned int* __restrict__ chunk_count, long long n_chunks,
                                               unsigned long long* __restrict__ chunk_base, EwState* st,
                                               long long* count_out, long long capacity, int* flags)
{
    __shared__ unsigned long long part[256];
    const int tid = threadIdx.x;
    const long long per = (n_chunks + 255) / 256;
    const long long lo = min(n_chunks, tid * per), hi = min(n_chunks, lo + per);
    unsigned long long mine = 0ull;
    for (long long c = lo; c < hi; ++c) mine += chunk_count[c];
    part[tid] = mine;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        const unsigned long long v = tid >= off ? part[tid - off] : 0ull;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    unsigned long long base = tid > 0 ? part[tid - 1] : 0ull;
    for (long long c = lo; c < hi; ++c) {
        chunk_base[c] = base;
        base += chunk_count[c];
    }
    if (tid == 255) {
        st->total_kept = base;
        *count_out = (long long)base;
        if ((long long)base > capacity) atomicMax(&flags[FLAG_CAPACITY], 1);
    }
}

// Writes the kept coordinates of one chunk in ascending order.  The keep bits give every kept coordinate
// its rank inside the chunk; the coordinates are first listed in LDS by rank, then thread t takes the t-th
// one, so the gradient is read and the message written in one batch of loads and coalesced stores.
__global__ __launch_bounds__(256) void ew_write(const float* __restrict__ g, const EwState* st,
                                                const unsigned long long* __restrict__ keep,
                                                const unsigned long long* __restrict__ chunk_base, long long capacity,
                                                unsigned int* __restrict__ idx, float* __restrict__ val /* null: signs in idx */)
{
    __shared__ unsigned int wsum[4];
    __shared__ unsigned short local[CHUNK];    // coordinate offsets inside the chunk, by rank
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long* kw = keep + ((long long)blockIdx.x * 4 + wave) * 16;
    const unsigned long long lt_mask = lane == 0 ? 0ull : (~0ull >> (64 - lane));

    unsigned int bits[4], before[4];           // keep bits; kept coordinates of this wave ahead of this lane's float4
    unsigned int running = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        unsigned int ahead = 0, all = 0;
        bits[j] = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const unsigned long long ballot = kw[j * 4 + c];
            bits[j] |= (unsigned int)((ballot >> lane) & 1ull) << c;
            ahead += __popcll(ballot & lt_mask);
            all += __popcll(ballot);
        }
        before[j] = running + ahead;
        running += all;
    }
    if (lane == 0) wsum[wave] = running;
    __syncthreads();
    unsigned int wave_base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        if (w < wave) wave_base += wsum[w];
        total += wsum[w];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        unsigned int pos = wave_base + before[j];
        const unsigned int off = (unsigned int)(wave * 256 + j * 64 + lane) * 4u;
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if ((bits[j] >> c) & 1u) local[pos++] = (unsigned short)(off + c);
    }
    __syncthreads();
    const double ratio = st->ratio;
    const unsigned long long base = chunk_base[blockIdx.x];
    const long long i0 = (long long)blockIdx.x * CHUNK;
    for (unsigned int t = threadIdx.x; t < total; t += 256) {
        const unsigned long long pos = base + t;
        if ((long long)pos < capacity) {
            const long long i = i0 + local[t];
            const float x = g[i];
            if (val) {
                idx[pos] = (unsigned int)i;
                val[pos] = x / ew_probability(x, ratio);
            } else {                                             // l_q message: the sign rides in bit 31
                idx[pos] = (unsigned int)i | (x < 0.0f ? 0x80000000u : 0u);
            }
        }
    }
}

// ---- the two-read encoder -----------------------------------------------------------------------------
// After the level-0 histogram the water level tau = tail / (s - n_s) is known to lie inside one bucket [lo, hi] of the
// float bit pattern (12.5 % wide), so p_i = min(1, |g_i| / tau) is bracketed for every element, and because rounding
// is monotone,  fl(|g_i| / hi) <= p_i <= fl(|g_i| / lo)  holds for the float32 p_i that the final ratio will give.
// The second pass over g therefore draws every element's uniform once and settles it at once wherever the bracket
// allows: kept for sure if u < p_lo, dropped for sure if u >= p_hi.  What lies between (about 0.12 s elements) is
// marked undecided and settled by ew_settle once the remaining levels have fixed tau exactly.  The same pass forms
// the level-1 histogram of the elements inside the chosen bucket, so g is read twice in all unless a third level
// is needed.

constexpr int SUPER = 256;                   // chunks per entry of the coarse count table

// Second pass, one chunk per workgroup; the level-0 result is read from st->lvl[0] (the launch before left it there).
// Layout of the keep / undecided bits: see ew_count.
__global__ __launch_bounds__(256) void ew_pass_b(const float* __restrict__ g, long long n, long long n_chunks, EwState* st,
                                                 double s, unsigned long long stream_id, unsigned long long seed,
                                                 unsigned int* __restrict__ chunk_count,
                                                 unsigned long long* __restrict__ keep,
                                                 unsigned long long* __restrict__ und)
{
    __shared__ unsigned int l1cnt[1 << L1_BITS];
    __shared__ unsigned long long l1sig[1 << L1_BITS];
    __shared__ unsigned int wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const SolveOut so = st->lvl[0];
    const bool done = so.done != 0;
    const double inf = __longlong_as_double(0x7FF0000000000000LL);
    // Single-precision brackets of the p that the final ratio will give, p = fl32(|g| ratio): with
    // r_lo <= ratio (1 - 2^-22) and r_hi >= ratio (1 + 2^-22),  fl32(|g| r_lo) (1 - 2^-22) <= p <= fl32(|g| r_hi) (1 + 2^-22)
    // (each rounding moves a value by at most 2^-24 of itself).  A bracket that is a little wide only sends a few more
    // coordinates to ew_settle, which decides with the exact formula.
    double ratio_lo, ratio_hi;
    if (done) {
        ratio_lo = ratio_hi = final_ratio(s, so.n_s, so.tail);
    } else {
        ratio_lo = so.hi < inf ? 1.0 / so.hi : 0.0;              // 1 / hi <= ratio <= 1 / lo
        ratio_hi = so.lo > 0.0 ? 1.0 / so.lo : inf;
    }
    const float down = 1.0f - 2.384185791015625e-07f, up = 1.0f + 2.384185791015625e-07f;    // 1 -+ 2^-22
    // (1 - 2^-21): covers its own rounding; a ratio beyond the float range is bounded from below by the largest float
    const float r_lo = ratio_lo < 3.0e38 ? (float)(ratio_lo * (1.0 - 4.76837158203125e-07)) : 3.0e38f;
    const float r_hi = ratio_hi < 3.0e38 ? (float)(ratio_hi * (1.0 + 4.76837158203125e-07)) : __int_as_float(0x7f800000);
    const unsigned int bucket = so.prefix;
    if (!done) {
        for (int b = tid; b < (1 << L1_BITS); b += 256) { l1cnt[b] = 0u; l1sig[b] = 0ull; }
        __syncthreads();
    }

    const bool vec = (((size_t)g) & 15) == 0;
    {
        const long long c = blockIdx.x;
        const long long q0 = c * (CHUNK / 4) + wave * 256;
        unsigned long long* kw = keep + (c * 4 + wave) * 16;
        unsigned long long* uw = und + (c * 4 + wave) * 16;
        unsigned int kept = 0;                                   // wave-uniform
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const long long q = q0 + j * 64 + lane;
            unsigned int sure = 0, open = 0;
            if (q * 4 < n) {
                const float4 x = load4(g, q, n, vec);
                const u32x4 rnd = philox4x32_10((unsigned long long)q, stream_id, seed);
                const float xs[4] = {x.x, x.y, x.z, x.w};
                const float us[4] = {u01(rnd.x), u01(rnd.y), u01(rnd.z), u01(rnd.w)};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float a = fabsf(xs[e]);
                    // (a = 0: both are 0, never kept.  The floor 2^-24 under p_hi keeps the draw u = 0 undecided for
                    // an element whose bound underflows.)
                    const float p_lo = a > 0.0f ? fminf(1.0f, a * r_lo) * down : 0.0f;
                    const float p_hi = a > 0.0f ? fmaxf(fminf(1.0f, a * r_hi * up), 5.9604644775390625e-08f) : 0.0f;
                    if (us[e] < p_lo) sure |= 1u << e;
                    else if (us[e] < p_hi) open |= 1u << e;
                    if (!done) {
                        const unsigned int key = __float_as_uint(xs[e]) & 0x7FFFFFFFu;
                        if ((key >> 20) == bucket && (q * 4 + e) < n) {
                            atomicAdd(&l1cnt[(key >> 10) & ((1 << L1_BITS) - 1)], 1u);
                            atomicAdd(&l1sig[(key >> 10) & ((1 << L1_BITS) - 1)], (unsigned long long)significand(key));
                        }
                    }
                }
            }
            unsigned long long mine = 0ull, mine_open = 0ull;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const unsigned long long ballot = __ballot((sure >> e) & 1u);
                const unsigned long long ballot_open = __ballot((open >> e) & 1u);
                kept += __popcll(ballot);
                if (lane == e) { mine = ballot; mine_open = ballot_open; }
            }
            if (lane < 4) { kw[j * 4 + lane] = mine; uw[j * 4 + lane] = mine_open; }
        }
        if (lane == 0) wsum[wave] = kept;
        __syncthreads();
        if (tid == 0) chunk_count[c] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
    }
    if (done) {
        if (blockIdx.x == 0 && tid == 0) st->lvl[1].done = 1;    // nothing left for the levels below
        return;
    }
    for (int b = tid; b < (1 << L1_BITS); b += 256) {
        const unsigned int cnt = l1cnt[b];
        if (cnt) {
            atomicAdd(&st->cnt[1][b], cnt);
            atomicAdd(&st->sig[1][b], l1sig[b]);
        }
    }
    // the last workgroup to finish solves level 1 from the merged histogram
    if (!last_workgroup(st->ticket[1])) return;
    __shared__ SolveOut out;
    solve_level<1, 256, true>(st, s, so.prefix, so.n_above, so.sum_below, &out, l1sig);     // (l1sig is spent: scratch)
    if (tid == 0) publish(st, 1, out, s);
}

// Level-2 histogram of the elements on the path that level 1 chose (nothing to do if level 1 settled everything, the
// usual case); its last workgroup solves level 2.
__global__ __launch_bounds__(256) void ew_hist2_solve2(const float* __restrict__ g, long long n, EwState* st, double s)
{
    __shared__ unsigned long long acc[1 << L2_BITS];
    __shared__ SolveOut out;
    const SolveOut in = st->lvl[1];
    if (in.done) return;
    hist_body<2, 256>(g, n, st, acc, in.prefix);
    if (!last_workgroup(st->ticket[2])) return;
    solve_level<2, 256, true>(st, s, in.prefix, in.n_above, in.sum_below, &out, acc);
    if (threadIdx.x == 0) publish(st, 2, out, s);
}

// Settles the undecided coordinates of one chunk with the final ratio (the draws are repeated for the float4s that
// hold one), completes the chunk's keep bits and count, and adds the count to the coarse table.  Also leaves the
// three histograms zeroed for the next call (their last reader has run).
__global__ __launch_bounds__(256) void ew_settle(const float* __restrict__ g, long long n, const EwState* st,
                                                 unsigned long long stream_id, unsigned long long seed,
                                                 unsigned int* __restrict__ chunk_count,
                                                 unsigned long long* __restrict__ keep,
                                                 const unsigned long long* __restrict__ und)
{
    __shared__ unsigned int wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const double ratio = st->ratio;                              // final since the last solve
    const bool vec = (((size_t)g) & 15) == 0;
    const long long c = blockIdx.x;
    const long long q0 = c * (CHUNK / 4) + wave * 256;
    unsigned long long* kw = keep + (c * 4 + wave) * 16;
    const unsigned long long* uw = und + (c * 4 + wave) * 16;
    unsigned int added = 0;                                      // wave-uniform
    const unsigned long long word = lane < 16 ? uw[lane] : 0ull;
    if (__ballot(word != 0ull)) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            unsigned int open = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const unsigned long long w = __shfl(word, j * 4 + e);
                open |= (unsigned int)((w >> lane) & 1ull) << e;
            }
            if (__ballot(open != 0u) == 0ull) continue;          // (uniform)
            const long long q = q0 + j * 64 + lane;
            unsigned int now = 0;
            if (open) {
                float4 p;
                now = draw4(load4(g, q, n, vec), q, stream_id, seed, ratio, p) & open;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const unsigned long long ballot = __ballot((now >> e) & 1u);
                added += __popcll(ballot);
                if (lane == e && ballot) kw[j * 4 + e] |= ballot;
            }
        }
    }
    if (lane == 0) wsum[wave] = added;
    __syncthreads();
    const unsigned int more = wsum[0] + wsum[1] + wsum[2] + wsum[3];
    if (tid == 0 && more) chunk_count[c] += more;
}

// Sums of the chunk counts per group of SUPER chunks, for gradients so long that a workgroup of ew_write2 could not
// add up all the counts before its own (one workgroup per group).
__global__ __launch_bounds__(256) void ew_super(const unsigned int* __restrict__ chunk_count, long long n_chunks,
                                                unsigned long long* __restrict__ super_count)
{
    __shared__ unsigned long long part[4];
    const long long i = (long long)blockIdx.x * SUPER + threadIdx.x;
    unsigned long long v = i < n_chunks ? chunk_count[i] : 0u;
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) super_count[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

// ew_write with the chunk's offset summed up by the workgroup itself: the counts of all chunks before it (for very
// long gradients: the coarse table up to the chunk's group of SUPER chunks, then the counts inside the group).  The
// last chunk also reports the total.  Leaves the three histograms zeroed for the next call.
__global__ __launch_bounds__(256) void ew_write2(const float* __restrict__ g, EwState* st,
                                                 const unsigned long long* __restrict__ keep,
                                                 const unsigned int* __restrict__ chunk_count,
                                                 const unsigned long long* __restrict__ super_count /* null: add up chunk_count */,
                                                 long long capacity,
                                                 unsigned int* __restrict__ idx, float* __restrict__ val /* null: signs in idx */,
                                                 long long* count_out, int* flags)
{
    __shared__ unsigned int wsum[4];
    __shared__ unsigned long long bsum[4];
    __shared__ unsigned short local[CHUNK];    // coordinate offsets inside the chunk, by rank
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long* kw = keep + ((long long)blockIdx.x * 4 + wave) * 16;
    const unsigned long long lt_mask = lane == 0 ? 0ull : (~0ull >> (64 - lane));

    // offset of the chunk in the message
    unsigned long long part = 0ull;
    {
        const long long sup = super_count ? (long long)blockIdx.x / SUPER : 0;
        for (long long i = threadIdx.x; i < sup; i += 256) part += super_count[i];
        for (long long i = sup * SUPER + threadIdx.x; i < (long long)blockIdx.x; i += 256) part += chunk_count[i];
        for (int o = 32; o > 0; o >>= 1) part += __shfl_down(part, o);
    }

    unsigned int bits[4], before[4];           // keep bits; kept coordinates of this wave ahead of this lane's float4
    unsigned int running = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        unsigned int ahead = 0, all = 0;
        bits[j] = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const unsigned long long ballot = kw[j * 4 + c];
            bits[j] |= (unsigned int)((ballot >> lane) & 1ull) << c;
            ahead += __popcll(ballot & lt_mask);
            all += __popcll(ballot);
        }
        before[j] = running + ahead;
        running += all;
    }
    if (lane == 0) { wsum[wave] = running; bsum[wave] = part; }
    __syncthreads();
    unsigned int wave_base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        if (w < wave) wave_base += wsum[w];
        total += wsum[w];
    }
    const unsigned long long base = bsum[0] + bsum[1] + bsum[2] + bsum[3];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        unsigned int pos = wave_base + before[j];
        const unsigned int off = (unsigned int)(wave * 256 + j * 64 + lane) * 4u;
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if ((bits[j] >> c) & 1u) local[pos++] = (unsigned short)(off + c);
    }
    __syncthreads();
    const double ratio = st->ratio;
    const long long i0 = (long long)blockIdx.x * CHUNK;
    for (unsigned int t = threadIdx.x; t < total; t += 256) {
        const unsigned long long pos = base + t;
        if ((long long)pos < capacity) {
            const long long i = i0 + local[t];
            const float x = g[i];
            if (val) {
                idx[pos] = (unsigned int)i;
                val[pos] = x / ew_probability(x, ratio);
            } else {                                             // l_q message: the sign rides in bit 31
                idx[pos] = (unsigned int)i | (x < 0.0f ? 0x80000000u : 0u);
            }
        }
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) {
        const unsigned long long all = base + total;
        st->total_kept = all;
        *count_out = (long long)all;
        if ((long long)all > capacity) atomicMax(&flags[FLAG_CAPACITY], 1);
    }
    // the histograms have had their last reader: zero again for the next call
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < 3 * NBUCKET; i += (long long)gridDim.x * 256) {
        (&st->cnt[0][0])[i] = 0u;
        (&st->sig[0][0])[i] = 0ull;
    }
}

// Small segments of atomo_probabilities: sort-based Algorithm 1, one workgroup per segment.
struct SmallSeg { long long begin; int n; int pad; };

__global__ __launch_bounds__(256) void prob_small(const float* __restrict__ lam, const SmallSeg* segs, double s,
                                                  float* __restrict__ p)
{
    __shared__ float key[ALG1_MAX];
    __shared__ int src[ALG1_MAX];
    __shared__ Alg1Scratch sc;
    const SmallSeg seg = segs[blockIdx.x];
    const int n = seg.n, tid = threadIdx.x;
    if (n <= 0) return;
    int P = 1;
    while (P < n) P <<= 1;
    for (int i = tid; i < P; i += 256) {
        key[i] = i < n ? fabsf(lam[seg.begin + i]) : -1.0f;
        src[i] = i;
    }
    __syncthreads();
    block_sort_desc(key, src, P);
    const int ns = block_algorithm1(key, n, s, sc);
    const double tail_ns = sc.tail_ns;
    for (int i = tid; i < n; i += 256) p[seg.begin + src[i]] = alg1_probability(key[i], i, ns, s, tail_ns);
}

// ---- l_q quantisation (Section 4) -------------------------------------------------------------------
enum { LQ_MAX = 0, LQ_TWO = 1, LQ_ONE = 2, LQ_POW = 3 };
constexpr int LQ_WGS = 1024;

// Per-workgroup part of |g|_q: max |g_i|, or the sum of g_i^2, |g_i| or |g_i|^q in double (fixed thread ->
// element map and fixed reduction tree, so the norm is the same bits in every run).
__global__ __launch_bounds__(256) void lq_norm_partial(const float* __restrict__ g, long long n, int mode, double q,
                                                       double* __restrict__ partial)
{
    __shared__ double wpart[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    double acc = 0.0;
    auto visit = [&](float x) {
        const double a = (double)fabsf(x);
        if (mode == LQ_MAX) acc = fmax(acc, a);
        else if (mode == LQ_TWO) acc = fma(a, a, acc);
        else if (mode == LQ_ONE) acc += a;
        else if (a > 0.0) acc += pow(a, q);
    };
    const bool vec = (((size_t)g) & 15) == 0;
    const long long n4 = vec ? n / 4 : 0;
    const long long stride = (long long)gridDim.x * 256;
    for (long long q0 = (long long)blockIdx.x * 256 + tid; q0 < n4; q0 += 4 * stride) {
        float4 x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const long long qq = q0 + u * stride;
            x[u] = qq < n4 ? ((const float4*)g)[qq] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) { visit(x[u].x); visit(x[u].y); visit(x[u].z); visit(x[u].w); }
    }
    for (long long i = n4 * 4 + (long long)blockIdx.x * 256 + tid; i < n; i += stride) visit(g[i]);
    for (int o = 32; o > 0; o >>= 1) {
        const double other = __shfl_down(acc, o);
        acc = mode == LQ_MAX ? fmax(acc, other) : acc + other;
    }
    if (lane == 0) wpart[wave] = acc;
    __syncthreads();
    if (tid == 0) {
        double t = wpart[0];
        for (int w = 1; w < 4; ++w) t = mode == LQ_MAX ? fmax(t, wpart[w]) : t + wpart[w];
        partial[blockIdx.x] = t;
    }
}

// |g|_q from the partial results (one workgroup), 1 / |g|_q as the sampler's ratio, and the message's norm.
__global__ __launch_bounds__(256) void lq_norm_final(const double* __restrict__ partial, int n_partial, int mode, double q,
                                                     EwState* st, float* norm_out)
{
    __shared__ double tree[256];
    const int tid = threadIdx.x;
    double t = 0.0;
    for (int k = tid; k < n_partial; k += 256) t = mode == LQ_MAX ? fmax(t, partial[k]) : t + partial[k];
    tree[tid] = t;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (tid < off) tree[tid] = mode == LQ_MAX ? fmax(tree[tid], tree[tid + off]) : tree[tid] + tree[tid + off];
        __syncthreads();
    }
    if (tid == 0) {
        const double acc = tree[0];
        const double norm = mode == LQ_MAX || mode == LQ_ONE ? acc : mode == LQ_TWO ? sqrt(acc) : pow(acc, 1.0 / q);
        st->ratio = norm > 0.0 ? 1.0 / norm : 0.0;               // p_i = min(1, |g_i| / |g|_q)
        st->n_s = 0ull; st->tail = norm; st->budget = 1.0; st->total_kept = 0ull;
        for (int k = 0; k < 3; ++k) st->lvl[k].done = 1;
        *norm_out = (float)norm;
    }
}

struct EwLayout {
    EwState* st;
    unsigned int* chunk_count;
    unsigned long long* chunk_base;
    unsigned long long* keep;     // [n_chunks][64] keep bits, see ew_count
    unsigned long long* und;      // [n_chunks][64] coordinates the second pass could not settle, same layout
    unsigned long long* super_count;   // [ceil(n_chunks / SUPER)] kept coordinates per group of SUPER chunks
    double* lq_partial;           // [LQ_WGS] per-workgroup parts of |g|_q
    size_t bytes;
};

EwLayout ew_layout(void* base, int64_t n)
{
    Carver carve(base);
    EwLayout l;
    const size_t n_chunks = (size_t)((n + CHUNK - 1) / CHUNK);
    l.st = carve.take<EwState>(1);
    l.chunk_count = carve.take<unsigned int>(n_chunks);
    l.chunk_base = carve.take<unsigned long long>(n_chunks);
    l.keep = carve.take<unsigned long long>(n_chunks * 64);
    l.und = carve.take<unsigned long long>(n_chunks * 64);
    l.super_count = carve.take<unsigned long long>((n_chunks + SUPER - 1) / SUPER);
    l.lq_partial = carve.take<double>(LQ_WGS);
    l.bytes = carve.off;
    return l;
}

// Enqueues the three histogram / solve levels; afterwards st->{n_s, tail, budget} are final.
void enqueue_water_level(atomo_ctx* ctx, const float* x, int64_t n, double s, EwState* st, hipStream_t stream)
{
    // No workgroup may visit 2^16 elements or more (field widths of the packed histogram word).
    const int64_t floor_wgs = (n + 49151) / 49152;
    const int wgs = (int)std::max<int64_t>(std::min<int64_t>(HIST_WGS, (n + 1023) / 1024), floor_wgs);
    const int wgs0 = (int)std::max<int64_t>(std::min<int64_t>(256, (n + 4095) / 4096), floor_wgs);
    { ProfScope ps(ctx, ATOMO_K_EW_SOLVE, stream); ew_clear<<<(3 * NBUCKET + 255) / 256, 256, 0, stream>>>(st); }
    { ProfScope ps(ctx, ATOMO_K_EW_HIST, stream); ew_hist<0><<<wgs0, 1024, 0, stream>>>(x, n, st); }
    { ProfScope ps(ctx, ATOMO_K_EW_SOLVE, stream); ew_solve<0><<<1, 256, 0, stream>>>(st, s); }
    { ProfScope ps(ctx, ATOMO_K_EW_HIST, stream); ew_hist<1><<<wgs, 256, 0, stream>>>(x, n, st); }
    { ProfScope ps(ctx, ATOMO_K_EW_SOLVE, stream); ew_solve<1><<<1, 256, 0, stream>>>(st, s); }
    { ProfScope ps(ctx, ATOMO_K_EW_HIST, stream); ew_hist<2><<<wgs, 256, 0, stream>>>(x, n, st); }
    { ProfScope ps(ctx, ATOMO_K_EW_SOLVE, stream); ew_solve<2><<<1, 256, 0, stream>>>(st, s); }
}

}  // namespace

size_t entrywise_workspace_bytes(int64_t n) { return ew_layout(nullptr, n).bytes; }

namespace {

// The encoder proper: every buffer it needs beyond the caller's lies in `l`.  The histograms in l.st must be zero on
// entry and are zero again when the last kernel has run (clear_first: do not rely on that, clear them first).
int enqueue_encode_entrywise(atomo_ctx* ctx, const float* g, double s, uint64_t seed, uint64_t stream_id,
                             const atomo_ew_msg* msg, float* p_out, const EwLayout& l, bool clear_first, hipStream_t stream)
{
    const int64_t n = msg->n;
    const long long n_chunks = (n + CHUNK - 1) / CHUNK;
    const int n_super = (int)((n_chunks + SUPER - 1) / SUPER);
    // No workgroup of the level-0 pass may visit 2^16 elements or more (field widths of its packed histogram word).
    const int64_t floor_wgs = (n + 49151) / 49152;
    const int wgs = (int)std::max<int64_t>(std::min<int64_t>(HIST_WGS, (n + 1023) / 1024), floor_wgs);
    const int wgs0 = (int)std::max<int64_t>(std::min<int64_t>(256, (n + 4095) / 4096), floor_wgs);
    if (clear_first) { ProfScope ps(ctx, ATOMO_K_EW_SOLVE, stream); ew_clear<<<(3 * NBUCKET + 255) / 256, 256, 0, stream>>>(l.st); }
    { ProfScope ps(ctx, ATOMO_K_EW_HIST, stream); ew_hist0_solve0<<<wgs0, 1024, 0, stream>>>(g, n, l.st, s); }
    {
        ProfScope ps(ctx, ATOMO_K_EW_SAMPLE, stream);
        ew_pass_b<<<(unsigned)n_chunks, 256, 0, stream>>>(g, n, n_chunks, l.st, s, stream_id, seed, l.chunk_count, l.keep,
                                                          l.und);
    }
    { ProfScope ps(ctx, ATOMO_K_EW_HIST, stream); ew_hist2_solve2<<<wgs, 256, 0, stream>>>(g, n, l.st, s); }
    {
        ProfScope ps(ctx, ATOMO_K_EW_SAMPLE, stream);
        ew_settle<<<(unsigned)n_chunks, 256, 0, stream>>>(g, n, l.st, stream_id, seed, l.chunk_count, l.keep, l.und);
        const bool coarse = n_chunks > 16384;                    // (above 2^26 elements)
        if (coarse) ew_super<<<(unsigned)n_super, 256, 0, stream>>>(l.chunk_count, n_chunks, l.super_count);
        ew_write2<<<(unsigned)n_chunks, 256, 0, stream>>>(g, l.st, l.keep, l.chunk_count, coarse ? l.super_count : nullptr,
                                                          (long long)msg->capacity, msg->idx, msg->val,
                                                          (long long*)msg->count, ctx->d_flags);
        if (p_out) ew_write_p<<<(int)std::min<int64_t>(4096, (n + 255) / 256), 256, 0, stream>>>(g, n, l.st, p_out);
    }
    ATOMO_HIP(ctx, hipGetLastError());
    return ATOMO_OK;
}

}  // namespace

int encode_entrywise(atomo_ctx* ctx, const float* g, double s, uint64_t seed, uint64_t stream_id,
                     const atomo_ew_msg* msg, float* p_out, hipStream_t stream)
{
    const int64_t n = msg->n;
    int rc = ensure_workspace(ctx, entrywise_workspace_bytes(n));
    if (rc != ATOMO_OK) return rc;
    // The search state lives outside the shared workspace: its histograms are handed from call to call zeroed (the
    // last kernel of a call clears them), which saves the clearing launch at the head of every call.
    if (!ctx->ew_state) {
        ATOMO_HIP(ctx, hipMalloc(&ctx->ew_state, sizeof(EwState)));
        ATOMO_HIP(ctx, hipMemsetAsync(ctx->ew_state, 0, sizeof(EwState), stream));
    }
    EwLayout l = ew_layout(ctx->ws, n);
    l.st = (EwState*)ctx->ew_state;
    return enqueue_encode_entrywise(ctx, g, s, seed, stream_id, msg, p_out, l, false, stream);
}

int encode_lq(atomo_ctx* ctx, const float* g, double q, uint64_t seed, uint64_t stream_id, const atomo_lq_msg* msg,
              float* p_out, hipStream_t stream)
{
    const int64_t n = msg->n;
    int rc = ensure_workspace(ctx, entrywise_workspace_bytes(n));
    if (rc != ATOMO_OK) return rc;
    const EwLayout l = ew_layout(ctx->ws, n);
    const long long n_chunks = (n + CHUNK - 1) / CHUNK;
    const int mode = std::isinf(q) ? LQ_MAX : q == 2.0 ? LQ_TWO : q == 1.0 ? LQ_ONE : LQ_POW;
    const int wgs = (int)std::min<int64_t>(LQ_WGS, (n + 4095) / 4096);
    {
        ProfScope ps(ctx, ATOMO_K_EW_HIST, stream);              // the norm pass takes the place of the histograms
        lq_norm_partial<<<wgs, 256, 0, stream>>>(g, n, mode, q, l.lq_partial);
    }
    { ProfScope ps(ctx, ATOMO_K_EW_SOLVE, stream); lq_norm_final<<<1, 256, 0, stream>>>(l.lq_partial, wgs, mode, q, l.st, msg->norm); }
    {
        ProfScope ps(ctx, ATOMO_K_EW_SAMPLE, stream);
        ew_count<<<(unsigned)n_chunks, 256, 0, stream>>>(g, n, l.st, stream_id, seed, l.chunk_count, l.keep);
        ew_scan<<<1, 256, 0, stream>>>(l.chunk_count, n_chunks, l.chunk_base, l.st, (long long*)msg->count,
                                       (long long)msg->capacity, ctx->d_flags);
        ew_write<<<(unsigned)n_chunks, 256, 0, stream>>>(g, l.st, l.keep, l.chunk_base, (long long)msg->capacity,
                                                         msg->idx, nullptr);
        if (p_out) ew_write_p<<<(int)std::min<int64_t>(4096, (n + 255) / 256), 256, 0, stream>>>(g, n, l.st, p_out);
    }
    ATOMO_HIP(ctx, hipGetLastError());
    return ATOMO_OK;
}

int probabilities(atomo_ctx* ctx, const float* lambda, const int64_t* offsets, int n_seg, double s, float* p,
                  hipStream_t stream)
{
    std::vector<SmallSeg> small;
    std::vector<int> large;
    for (int k = 0; k < n_seg; ++k) {
        const int64_t len = offsets[k + 1] - offsets[k];
        if (len == 0) continue;
        if (len <= ALG1_MAX) small.push_back(SmallSeg{(long long)offsets[k], (int)len, 0});
        else large.push_back(k);
    }
    size_t need = align_up(small.size() * sizeof(SmallSeg), 256) + 256;
    if (!large.empty()) need += align_up(sizeof(EwState), 256);
    int rc = ensure_workspace(ctx, need);
    if (rc != ATOMO_OK) return rc;
    Carver carve(ctx->ws);
    SmallSeg* d_small = carve.take<SmallSeg>(small.size());
    EwState* st = large.empty() ? nullptr : carve.take<EwState>(1);
    if (!small.empty()) {
        rc = upload(ctx, d_small, small.data(), small.size() * sizeof(SmallSeg), stream);
        if (rc != ATOMO_OK) return rc;
        prob_small<<<(unsigned)small.size(), 256, 0, stream>>>(lambda, d_small, s, p);
    }
    for (int k : large) {
        const int64_t len = offsets[k + 1] - offsets[k];
        const float* x = lambda + offsets[k];
        enqueue_water_level(ctx, x, len, s, st, stream);
        const int wgs = (int)std::min<int64_t>(4096, (len + 255) / 256);
        ew_write_p<<<wgs, 256, 0, stream>>>(x, len, st, p + offsets[k]);
    }
    ATOMO_HIP(ctx, hipGetLastError());
    return ATOMO_OK;
}

}  // namespace atomo

// ---------------------------------------------------------------------------------------------------------
// atomo_encode_entrywise_noalloc: the entry-wise encoder for callers that cannot allocate (see include/atomo.h).
// Its scratch memory (the state of the water-level search, per-chunk counts, offsets and keep bits) is the
// file-scope device array below instead of the context's growable workspace.  Every GPU the library runs on
// holds its own copy of the array, at its own address, until the process ends; the address on a device is
// looked up once, with that device current (atomo_create does it, so that no call made later has to).
// ---------------------------------------------------------------------------------------------------------
namespace {

constexpr long long NOALLOC_MAX_N = 1ll << 24;                   // 16,777,216 elements (64 MiB of gradient)
constexpr size_t NOALLOC_SCRATCH_BYTES = (size_t)5 << 20;        // 5 MiB per GPU
constexpr int NOALLOC_MAX_DEVICES = 64;

static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];

// Device address of `scratch` per HIP device (the array's name is only a host-side handle for the symbol).
void* scratch_ptr[NOALLOC_MAX_DEVICES];

}  // namespace

namespace atomo {

// Called with ctx->device current.  Looks the address up on the first call for a device.
int entrywise_noalloc_setup(atomo_ctx* ctx)
{
    const int dev = ctx->device;
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return ATOMO_EINVAL;
    if (__atomic_load_n(&scratch_ptr[dev], __ATOMIC_ACQUIRE)) return ATOMO_OK;
    if (ew_layout(nullptr, NOALLOC_MAX_N).bytes > NOALLOC_SCRATCH_BYTES) return ATOMO_EINVAL;   // (a build-time fact)
    void* ptr = nullptr;
    ATOMO_HIP(ctx, hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return ATOMO_EHIP;
    __atomic_store_n(&scratch_ptr[dev], ptr, __ATOMIC_RELEASE);   // (two threads racing here store the same address)
    return ATOMO_OK;
}

}  // namespace atomo

extern "C" int atomo_encode_entrywise_noalloc(atomo_ctx* ctx, const float* g, double s, uint64_t seed, uint64_t stream_id,
                                              const atomo_ew_msg* msg, float* p_out, void* stream)
{
    using namespace atomo;
    if (!ctx || !g || !msg || !(s > 0.0) || std::isinf(s)) return ATOMO_EINVAL;
    if (msg->n <= 0 || msg->capacity < 1 || !msg->count || !msg->idx || !msg->val) return ATOMO_EINVAL;
    if (msg->n > NOALLOC_MAX_N) return ATOMO_ETOOLARGE;
    int prev = -1;
    if (hipGetDevice(&prev) != hipSuccess) prev = -1;
    if (prev != ctx->device) ATOMO_HIP(ctx, hipSetDevice(ctx->device));
    int rc = entrywise_noalloc_setup(ctx);                        // a table look-up after atomo_create
    if (rc == ATOMO_OK) {
        // event bracketing of launches creates events on demand: not on this path
        const bool profiling = ctx->profiling;
        ctx->profiling = false;
        void* base = __atomic_load_n(&scratch_ptr[ctx->device], __ATOMIC_ACQUIRE);
        // (the array keeps what the previous call left: the histograms are cleared first, by a kernel)
        rc = enqueue_encode_entrywise(ctx, g, s, seed, stream_id, msg, p_out, ew_layout(base, msg->n), true, (hipStream_t)stream);
        ctx->profiling = profiling;
    }
    if (prev >= 0 && prev != ctx->device) (void)hipSetDevice(prev);
    return rc;
}

