// k-means cache (paper Sec. 4, "k-means"): the intermediate points of a layer are clustered
// and each cluster is represented by its centre; a cache item is the centre, the majority
// label of the cluster and the fraction of the cluster that carries it.
//
// The assignment step of Lloyd's iterations is the batched look-up itself (every point against
// the centres, k = 1) and is driven from the API file; this file holds what is left: the update
// of the centres, the majority label and fraction of every cluster, and a read-out.  gfx950 only.
#include "freeze_internal.h"

namespace fz {

// New centre of cluster c = blockIdx.x, dimensions blockIdx.y * 256 + threadIdx.x: the mean of
// the points assigned to it, summed in point order in fp64 and rounded once to fp32 (so the
// result does not depend on scheduling); a cluster without points keeps its centre.
// The block walks the assignment list in LDS-sized pieces; whether a point belongs to the
// cluster is uniform over the block, so the row reads are whole coalesced pieces.
__global__ __launch_bounds__(256) void kmeans_update_kernel(const float *points, const int32_t *assign, int64_t n,
                                                            int64_t d, const float *old_centers, float *new_centers)
{
    __shared__ int32_t a_s[2048];
    const int c = blockIdx.x;
    const int64_t dim = (int64_t)blockIdx.y * 256 + threadIdx.x;
    double acc = 0.0;
    int64_t count = 0;
    for (int64_t base = 0; base < n; base += 2048) {
        const int len = (int)(n - base < 2048 ? n - base : 2048);
        __syncthreads();
        for (int i = threadIdx.x; i < len; i += 256) a_s[i] = assign[base + i];
        __syncthreads();
        for (int i = 0; i < len; ++i) {
            if (a_s[i] == c) {
                ++count;
                if (dim < d) acc += (double)points[(base + i) * d + dim];
            }
        }
    }
    if (dim < d) new_centers[(int64_t)c * d + dim] = count ? (float)(acc / (double)count) : old_centers[(int64_t)c * d + dim];
}

hipError_t launch_kmeans_update(const float *points, const int32_t *assign, int64_t n, int64_t d, int64_t k,
                                const float *old_centers, float *new_centers, hipStream_t s)
{
    hipLaunchKernelGGL(kmeans_update_kernel, dim3((unsigned)k, (unsigned)((d + 255) / 256)), dim3(256), 0, s, points,
                       assign, n, d, old_centers, new_centers);
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
