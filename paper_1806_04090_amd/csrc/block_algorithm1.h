// Algorithm 1 ("ATOMO probabilities", Section 3 of arXiv 1806.04090) for one workgroup of 256
// threads on up to 2048 magnitudes held in LDS.  HIP side only.
#pragma once

#include <hip/hip_runtime.h>

namespace atomo {

constexpr int ALG1_MAX = 2048;

struct Alg1Scratch {
    double part[2][256];
    double tail_ns;
    int first_true;
};

// Bitonic sort of (key, src) pairs, descending by key, ties by ascending src.  P = power of two
// >= count; entries beyond the data must hold keys below every real key.  All 256 threads call, after a
// workgroup barrier behind the writes of key and src; the sorted arrays are visible to all on return.
// Thread t takes the compare-exchanges t, t + 256, ... of a stage; exchange q pairs the elements i and i + j with
// i = 2 (q - q mod j) + q mod j.  For j <= 64 the 64 exchanges of a wave stay inside 128 consecutive elements
// that are the same at every such stage, and the LDS operations of a wave are performed in program order: only
// the stages with j >= 128 (three of the 45 for 512 keys) need workgroup barriers around them.
__device__ inline void block_sort_desc(float* key, int* src, int P)
{
    const int tid = threadIdx.x;
    bool across = false;                                         // the stage before paired elements of different waves
    for (int k = 2; k <= P; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            if (j >= 128 || across) {
                __syncthreads();
            } else {
                // same wave: nothing to wait for, but the compiler must keep the stages apart
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
            across = j >= 128;
            for (int q = tid; q < (P >> 1); q += 256) {
                const int i = ((q & ~(j - 1)) << 1) | (q & (j - 1)), o = i | j;
                const float ki = key[i], ko = key[o];
                const int si = src[i], so = src[o];
                const bool i_first = (ki > ko) || (ki == ko && si < so);
                const bool desc = (i & k) == 0;
                if (desc ? !i_first : i_first) {
                    key[i] = ko; key[o] = ki;
                    src[i] = so; src[o] = si;
                }
            }
        }
    }
    __syncthreads();
}

// key[0..n) holds magnitudes sorted descending.  Finds n_s = the first sorted index i with
// key_i * (s - i) <= sum_{j >= i} key_j (the test of Algorithm 1 with the budget that remains; it
// is monotone in i, so "first true" can be searched in parallel) and the tail sum at that index.
// Thread t owns the slice [t*per, min(n,(t+1)*per)).  After the call every thread may evaluate
//     p_i = 1                                   for i <  n_s
//     p_i = key_i * (s - n_s) / tail            for i >= n_s and tail > 0      (eq. (p_i), KKT appendix)
//     p_i = 0                                   otherwise (only zeros remain)
// All 256 threads call; returns n_s, and the tail sum through sc.tail_ns (valid if n_s < n).
__device__ inline int block_algorithm1(const float* key, int n, double s, Alg1Scratch& sc)
{
    const int tid = threadIdx.x;
    const int per = (n + 255) / 256;
    const int lo = min(n, tid * per), hi = min(n, lo + per);
    double mine = 0.0;
    for (int i = hi - 1; i >= lo; --i) mine += (double)key[i];
    sc.part[0][tid] = mine;
    if (tid == 0) { sc.first_true = n; sc.tail_ns = 0.0; }
    __syncthreads();
    // after = the sum of the slices behind this one: suffix sums over the 256 slice sums in eight doubling steps
    // (sums of non-negative numbers in a fixed order; empty slices hold 0)
    int cur = 0;
    for (int d = 1; d < 256; d <<= 1) {
        sc.part[cur ^ 1][tid] = sc.part[cur][tid] + (tid + d < 256 ? sc.part[cur][tid + d] : 0.0);
        cur ^= 1;
        __syncthreads();
    }
    const double after = tid + 1 < 256 ? sc.part[cur][tid + 1] : 0.0;
    {
        // tail sums of the slice, each accumulated from the small end: subtracting the large leading values from
        // one total instead would cancel (a slice that holds 1e30 and 1 would lose the 1)
        double suffix[ALG1_MAX / 256];
        double run = after;
#pragma unroll
        for (int k = ALG1_MAX / 256 - 1; k >= 0; --k) {
            if (lo + k < hi) run += (double)key[lo + k];
            suffix[k] = run;
        }
        int found = n;
#pragma unroll
        for (int k = ALG1_MAX / 256 - 1; k >= 0; --k)
            if (lo + k < hi && (double)key[lo + k] * (s - (double)(lo + k)) <= suffix[k]) found = lo + k;
        if (found < n) atomicMin(&sc.first_true, found);
    }
    __syncthreads();
    const int ns = sc.first_true;
    if (ns < n && ns >= lo && ns < hi) {
        double tail = after;
        for (int i = hi - 1; i >= ns; --i) tail += (double)key[i];
        sc.tail_ns = tail;
    }
    __syncthreads();
    return ns;
}

__device__ inline float alg1_probability(float key, int i, int ns, double s, double tail_ns)
{
    if (i < ns) return 1.0f;
    if (tail_ns > 0.0) return fminf(1.0f, (float)((double)key * (s - (double)ns) / tail_ns));
    return 0.0f;
}

}  // namespace atomo
