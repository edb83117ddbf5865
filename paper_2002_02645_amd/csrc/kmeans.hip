// k-means cache (paper Sec. 4, "k-means"): the intermediate points of a layer are clustered
// and each cluster is represented by its centre; a cache item is the centre, the majority
// label of the cluster and the fraction of the cluster that carries it.
//
// The assignment step of Lloyd's iterations is the batched look-up itself (every point against
// the centres, k = 1) and is driven from the API file; this file holds what is left: the update
// of the centres, the majority label and fraction of every cluster, and a read-out.  gfx950 only.
#include "freeze_internal.h"

namespace fz {

// Update step of Lloyd's iterations.  The points are first grouped by the centre they were
// assigned to, each group in point order (integer work only: the grouping is the same in every
// run): sizes by a histogram, offsets by a scan, and one workgroup per centre that walks the
// assignment list and writes its members' ids in order (ballot / popcount compaction; the list is
// n ints and stays in L2).  Then one workgroup per (centre, 256 dimensions) adds up its members'
// rows in that order in fp64 and rounds the mean once to fp32, so the result does not depend on
// scheduling; every point row is read exactly once, in 1 KiB pieces, eight rows in flight per
// thread.  A cluster without points keeps its centre.
__global__ __launch_bounds__(256) void kmeans_count_kernel(const int32_t *assign, int64_t n, int64_t k, int32_t *sizes)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) {
        const int32_t c = assign[i];
        if ((uint32_t)c < (uint64_t)k) atomicAdd(&sizes[c], 1);
    }
}

// offsets[c] = sizes[0] + .. + sizes[c-1], offsets[k] = total; one workgroup
__global__ __launch_bounds__(1024) void kmeans_offsets_kernel(const int32_t *sizes, int64_t k, int32_t *offsets)
{
    __shared__ int wave_tot[16];
    __shared__ int base_s;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    if (tid == 0) base_s = 0;
    __syncthreads();
    for (int64_t start = 0; start < k; start += 1024) {
        const int64_t c = start + tid;
        const int v = c < k ? sizes[c] : 0;
        int incl = v;   // inclusive scan within the wave
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(incl, off, 64);
            if (lane >= off) incl += o;
        }
        if (lane == 63) wave_tot[w] = incl;
        __syncthreads();
        int before = base_s;
        for (int i = 0; i < w; ++i) before += wave_tot[i];
        if (c < k) offsets[c] = before + incl - v;
        __syncthreads();
        if (tid == 1023) base_s = before + incl;
        __syncthreads();
    }
    if (tid == 0) offsets[k] = base_s;
}

// members[offsets[c] ..) = the ids of the points assigned to centre c = blockIdx.x, ascending
__global__ __launch_bounds__(1024) void kmeans_members_kernel(const int32_t *assign, int64_t n, const int32_t *offsets,
                                                              int32_t *members)
{
    __shared__ int wave_tot[16];
    const int c = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    int base = offsets[c];
    if (offsets[c + 1] == base) return;   // uniform: an empty cluster
    for (int64_t start = 0; start < n; start += 1024) {
        const int64_t i = start + tid;
        const bool mine = i < n && assign[i] == c;
        const uint64_t bal = __ballot(mine);
        if (lane == 0) wave_tot[w] = __builtin_popcountll(bal);
        __syncthreads();
        int before = 0, all = 0;
        for (int j = 0; j < 16; ++j) {
            before += j < w ? wave_tot[j] : 0;
            all += wave_tot[j];
        }
        if (mine) members[base + before + __builtin_popcountll(bal & ((1ull << lane) - 1ull))] = (int32_t)i;
        base += all;
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void kmeans_update_kernel(const float *points, const int32_t *offsets, const int32_t *members,
                                                            int64_t d, const float *old_centers, float *new_centers)
{
    const int c = blockIdx.x;
    const int64_t dim = (int64_t)blockIdx.y * 256 + threadIdx.x;
    if (dim >= d) return;
    const int m0 = offsets[c], m1 = offsets[c + 1];
    double acc = 0.0;
    int j = m0;
    for (; j + 8 <= m1; j += 8) {
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = points[(int64_t)members[j + e] * d + dim];   // eight rows in flight
#pragma unroll
        for (int e = 0; e < 8; ++e) acc += (double)v[e];                                 // ... added in point order
    }
    for (; j < m1; ++j) acc += (double)points[(int64_t)members[j] * d + dim];
    new_centers[(int64_t)c * d + dim] = m1 > m0 ? (float)(acc / (double)(m1 - m0)) : old_centers[(int64_t)c * d + dim];
}

hipError_t launch_kmeans_update(const float *points, const int32_t *assign, int64_t n, int64_t d, int64_t k,
                                const float *old_centers, float *new_centers, int32_t *sizes, int32_t *offsets,
                                int32_t *members, hipStream_t s)
{
    hipError_t e = launch_fill_i32(sizes, 0, k, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kmeans_count_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, assign, n, k, sizes);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(kmeans_offsets_kernel, dim3(1), dim3(1024), 0, s, sizes, k, offsets);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(kmeans_members_kernel, dim3((unsigned)k), dim3(1024), 0, s, assign, n, offsets, members);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(kmeans_update_kernel, dim3((unsigned)k, (unsigned)((d + 255) / 256)), dim3(256), 0, s, points,
                       offsets, members, d, old_centers, new_centers);
    return hipGetLastError();
}

// Majority label (equal counts -> the smaller label), its share of the cluster, and the cluster
// size, one block per cluster, by a histogram of the members' labels in LDS (integer counts:
// no dependence on the order of the atomic additions).  An empty cluster gets label 0, share 0.
constexpr int kKmeansMaxClasses = 8192;

__global__ __launch_bounds__(256) void kmeans_majority_kernel(const int32_t *assign, const int32_t *labels, int64_t n,
                                                              int num_classes, int32_t *majority, float *fraction,
                                                              int64_t *sizes)
{
    __shared__ int hist[kKmeansMaxClasses];
    __shared__ int best_s[256], bestl_s[256], size_s;
    const int c = blockIdx.x, tid = threadIdx.x;
    for (int l = tid; l < num_classes; l += 256) hist[l] = 0;
    if (tid == 0) size_s = 0;
    __syncthreads();
    int mine = 0;
    for (int64_t i = tid; i < n; i += 256) {
        if (assign[i] == c) {
            const int l = labels[i];
            if ((unsigned)l < (unsigned)num_classes) atomicAdd(&hist[l], 1);   // labels outside the contract are not counted
            ++mine;
        }
    }
    atomicAdd(&size_s, mine);
    __syncthreads();
    int best = -1, bestl = 0;
    for (int l = tid; l < num_classes; l += 256) {   // ascending l per thread: the first maximum is the smallest label
        if (hist[l] > best) {
            best = hist[l];
            bestl = l;
        }
    }
    best_s[tid] = best;
    bestl_s[tid] = bestl;
    __syncthreads();
    if (tid == 0) {
        int b = -1, bl = 0;
        for (int t = 0; t < 256; ++t)
            if (best_s[t] > b || (best_s[t] == b && bestl_s[t] < bl)) {
                b = best_s[t];
                bl = bestl_s[t];
            }
        const int size = size_s;
        majority[c] = size ? bl : 0;
        fraction[c] = size ? (float)((double)b / (double)size) : 0.f;
        if (sizes) sizes[c] = size;
    }
}

hipError_t launch_kmeans_majority(const int32_t *assign, const int32_t *labels, int64_t n, int num_classes, int64_t k,
                                  int32_t *majority, float *fraction, int64_t *sizes, hipStream_t s)
{
    if (num_classes < 1 || num_classes > kKmeansMaxClasses) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kmeans_majority_kernel, dim3((unsigned)k), dim3(256), 0, s, assign, labels, n, num_classes,
                       majority, fraction, sizes);
    return hipGetLastError();
}

// dst[i] = src[i] for float arrays; rows of a [rows, d] matrix out of a [rows, d_pad] one
__global__ void copy_rows_f32_kernel(const float *src, int64_t src_stride, float *dst, int64_t rows, int64_t d)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows * d) dst[i] = src[(i / d) * src_stride + i % d];
}

hipError_t launch_copy_rows_f32(const float *src, int64_t src_stride, float *dst, int64_t rows, int64_t d, hipStream_t s)
{
    const int64_t total = rows * d;
    if (total <= 0) return hipSuccess;
    hipLaunchKernelGGL(copy_rows_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, src, src_stride, dst,
                       rows, d);
    return hipGetLastError();
}

__global__ void copy_i32_plain_kernel(const int32_t *src, int32_t *dst, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

hipError_t launch_copy_i32(const int32_t *src, int32_t *dst, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(copy_i32_plain_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, src, dst, n);
    return hipGetLastError();
}

__global__ void fill_i32_kernel(int32_t *dst, int32_t v, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = v;
}

hipError_t launch_fill_i32(int32_t *dst, int32_t v, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, dst, v, n);
    return hipGetLastError();
}

}  // namespace fz
