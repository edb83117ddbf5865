// Device helpers shared by the selection kernels: order-preserving float bits, a bitonic sort
// in LDS, rank counting, and the R-th smallest of a long list of distinct 64-bit values.
#pragma once
#include "freeze_internal.h"

namespace fz {

// fp32 -> unsigned with the same order (so that (key, index) packs into one u64)
__device__ __forceinline__ uint32_t ordered_bits(float x)
{
    uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float from_ordered_bits(uint32_t u)
{
    return __uint_as_float((u & 0x80000000u) ? (u & 0x7fffffffu) : ~u);
}

constexpr int kThrThreads = 1024;
constexpr int kThrGroups = 256;
constexpr int kThrRegs = 32;      // values per thread kept in registers between the two rounds
constexpr int kThrList = 8192;    // capacity of the gathered list; callers check V * R <= kThrList

__device__ inline void bitonic_sort_lds(uint64_t *a, int n_pow2, int tid, int nthreads)
{
    for (int size = 2; size <= n_pow2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int i = tid; i < (n_pow2 >> 1); i += nthreads) {
                const int lo = ((i & ~(stride - 1)) << 1) | (i & (stride - 1));   // stride is a power of two
                const int hi = lo + stride;
                const bool up = ((lo & size) == 0);
                const uint64_t x = a[lo], y = a[hi];
                if ((x > y) == up) {
                    a[lo] = y;
                    a[hi] = x;
                }
            }
            __syncthreads();
        }
    }
}

// The element of a[0..n) with exactly `rank` smaller elements (all distinct), n <= blockDim.x.
__device__ __forceinline__ void select_by_rank_counting(const uint64_t *a, int n, int rank, int tid, uint64_t *out)
{
    if (tid < n) {
        const uint64_t mine = a[tid];
        int c = 0;
        for (int j = 0; j < n; ++j) c += (a[j] < mine);
        if (c == rank) *out = mine;
    }
}

// Ascending sort of one value per lane across the 64 lanes of a wave (bitonic network on
// register shuffles: no LDS, no barrier).
__device__ __forceinline__ uint64_t wave_sort64(uint64_t x, int lane)
{
#pragma unroll
    for (int size = 2; size <= 64; size <<= 1) {
#pragma unroll
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)x, stride, 64);
            const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(x >> 32), stride, 64);
            const uint64_t y = ((uint64_t)hi << 32) | lo;
            const bool up = (lane & size) == 0 || size == 64;
            const bool lower = (lane & stride) == 0;
            const uint64_t mn = x < y ? x : y, mx = x < y ? y : x;
            x = (lower == up) ? mn : mx;
        }
    }
    return x;
}

// The `keep` smallest of a[0..cnt), sorted ascending, by the whole workgroup (nthreads a multiple
// of 64): rounds of wave-local sorts of 64 values that each pass on their `keep` smallest, until
// one wave holds the rest.  Needs keep <= 32 (each round at least halves the count) and a second
// buffer b of the same capacity; returns the buffer whose first min(keep, cnt) entries are the
// result.  Every thread must call it; a and b are LDS.
__device__ inline uint64_t *smallest_sorted(uint64_t *a, uint64_t *b, int cnt, int keep, int tid, int nthreads)
{
    const int lane = tid & 63, wave = tid >> 6, nwaves = nthreads >> 6;
    while (true) {
        const int chunks = (cnt + 63) >> 6;
        for (int c = wave; c < chunks; c += nwaves) {
            const int i = c * 64 + lane;
            const uint64_t x = wave_sort64(i < cnt ? a[i] : kSentinel, lane);
            if (chunks == 1) {
                if (lane < 64) b[lane] = x;
            } else if (lane < keep) {
                b[c * keep + lane] = x;
            }
        }
        __syncthreads();
        uint64_t *t = a;
        a = b;
        b = t;
        if (chunks == 1) return a;
        cnt = chunks * keep;   // sentinels may pad the tail: they sort last
    }
}

// T = the r_sel-th smallest of src[0..nb) (distinct values; r_sel < nb), by a workgroup of
// kThrThreads threads, in two rounds: the values are dealt into 256 groups (value j belongs to
// group j mod 256); the r_sel-th smallest group minimum T1 bounds T from above, and at most
// V * r_sel values are <= T1 (V = values per group); those are gathered into `list` (LDS,
// kThrList entries) and the r_sel-th of them is T.  The r_sel-th smallest of a short list is
// found by rank counting, with a bitonic sort only for an unusually long list.  On return
// list[0 .. *list_n) still holds the gathered values, in no particular order (sorted when the
// sort ran): exactly r_sel of them are <= T.  Every thread of the workgroup must call it.
__device__ inline uint64_t rth_smallest_of(const uint64_t *src, int64_t nb, int r_sel, uint64_t *list, uint64_t *sel_s,
                                           int *list_n, int tid)
{
    if (tid == 0) *list_n = 0;
    // first pass: thread minima -> 256 group minima -> T1 = the r_sel-th smallest group minimum
    uint64_t v[kThrRegs];
    uint64_t m = kSentinel;
#pragma unroll
    for (int i = 0; i < kThrRegs; ++i) {
        const int64_t j = (int64_t)i * kThrThreads + tid;
        v[i] = j < nb ? src[j] : kSentinel;
        m = v[i] < m ? v[i] : m;
    }
    for (int64_t j = (int64_t)kThrRegs * kThrThreads + tid; j < nb; j += kThrThreads) {
        const uint64_t x = src[j];
        m = x < m ? x : m;
    }
    list[tid] = m;
    __syncthreads();
    if (tid < kThrGroups) {
        uint64_t g = list[tid];
#pragma unroll
        for (int i = 1; i < kThrThreads / kThrGroups; ++i) {
            const uint64_t x = list[tid + i * kThrGroups];
            g = x < g ? x : g;
        }
        list[kThrThreads + tid] = g;   // group minima live in list[1024 .. 1280)
    }
    __syncthreads();
    // sentinels (groups with no value) are equal to each other; they rank last and r_sel < nb real values exist
    select_by_rank_counting(list + kThrThreads, kThrGroups, r_sel - 1, tid, sel_s);
    __syncthreads();
    const uint64_t t1 = *sel_s;
    __syncthreads();
    // second pass: gather the values <= T1 (at least r_sel, at most V * r_sel of them)
#pragma unroll
    for (int i = 0; i < kThrRegs; ++i) {
        if (v[i] <= t1 && v[i] != kSentinel) {
            const int pos = atomicAdd(list_n, 1);
            if (pos < kThrList) list[pos] = v[i];
        }
    }
    for (int64_t j = (int64_t)kThrRegs * kThrThreads + tid; j < nb; j += kThrThreads) {
        const uint64_t x = src[j];
        if (x <= t1) {
            const int pos = atomicAdd(list_n, 1);
            if (pos < kThrList) list[pos] = x;
        }
    }
    __syncthreads();
    const int cnt = *list_n < kThrList ? *list_n : kThrList;
    if (cnt <= kThrThreads) {
        select_by_rank_counting(list, cnt, r_sel - 1, tid, sel_s);
        __syncthreads();
        return *sel_s;
    }
    int n2 = 2;
    while (n2 < cnt) n2 <<= 1;
    for (int i = cnt + tid; i < n2; i += kThrThreads) list[i] = kSentinel;
    __syncthreads();
    bitonic_sort_lds(list, n2, tid, kThrThreads);
    return list[r_sel - 1];
}

}  // namespace fz
