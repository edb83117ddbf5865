// Kernels around the distance pass: cache ingest, query preparation, the finishing
// kernels (merge of per-split candidate lists, exact fp32 re-scoring, final top-k, the
// certificate that no entry outside the candidates can be nearer, label vote, hit decision;
// the wider re-scoring and the exact fp32 scan for queries the certificate does not confirm;
// the one-launch finish of the small-batch path), miss compaction, the cascade's scatter, the
// row gather and the threshold calibration.  gfx950 only.
#include "freeze_internal.h"
#include "select_common.h"

namespace fz {

typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// Sum over the 256 threads of a block in a fixed order; result valid in every thread.
__device__ __forceinline__ float block_sum_256(float v, float *scratch4)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch4[w] = v;
    __syncthreads();
    return (scratch4[0] + scratch4[1]) + (scratch4[2] + scratch4[3]);
}

// ---------------------------------------------------------------------------------------
// Cache ingest (Pseudocode 1, ConstructCache: the layer's list of <output, label>).
// One block per padded cache row: bf16 copy (round to nearest even when given fp32) into the
// tiled layout, zero padding, |c|^2 of the bf16 row in fp32, and a row-major copy of the stored
// values for exact re-scoring (fp32 rows when the cache was given in fp32, else bf16 rows): the
// re-scoring gathers whole rows, which the tiled layout would serve in half-used cache lines.
// ---------------------------------------------------------------------------------------
// Centring of the matrix-core copy.  Distances do not change when the same vector is subtracted
// from entries and queries, but the coarse key |c|^2 - 2 q.c does: for a cache that sits far from
// the origin both of its terms are huge next to the distance and their bf16 / fp32 rounding swamps
// the differences between neighbours.  So the bf16 copy the matrix cores read (and the queries'
// bf16 copy) may be taken relative to the cache's mean vector mu; the stored values, which the exact
// re-scoring reads, stay as they are.  Whether to do so is decided on the device from the column
// statistics: only when the mean dominates the spread (|mu|^2 > 4 * total variance); otherwise mu is
// all zeros, the subtraction is exact and the copy is the plain rounding of the stored values (for
// a cache stored in bf16 centring adds a rounding error the plain copy does not have).
//
// The statistics come from a sample of at most kStatRows rows, evenly spaced over the cache (all
// rows of a smaller cache): mu may be any vector, the results never depend on it, and the
// decision needs no more precision than that.
//
// Column sums and sums of squares of the sampled rows in fp64: block (x, y) takes 512 columns (eight
// per lane, so that a wave reads 1 KiB, or 2 KiB of fp32, of a row at a time) and a range of the
// sample; its four waves take every fourth row of that range.
constexpr int kStatRows = 8192;
__global__ __launch_bounds__(256) void col_stats_kernel(const void *entries, int dtype, int64_t n, int64_t d, int64_t d_pad,
                                                        int64_t ns, double *stats)
{
    __shared__ double comb[3][64][16];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t col = ((int64_t)blockIdx.x * 64 + lane) * 8;
    const int64_t per = (ns + gridDim.y - 1) / gridDim.y;
    const int64_t i0 = (int64_t)blockIdx.y * per, i1 = i0 + per < ns ? i0 + per : ns;
    const bool vec = (reinterpret_cast<uintptr_t>(entries) % 16) == 0 && (dtype == 0 ? d % 4 == 0 : d % 8 == 0) && col + 8 <= d;
    double s1[8], s2[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) s1[e] = s2[e] = 0.0;
    if (col < d) {
        for (int64_t i = i0 + w; i < i1; i += 4) {
            const int64_t r = i * n / ns;   // sample i of ns (distinct rows: ns <= n)
            float v[8];
            if (vec && dtype == 0) {
                const float *src = reinterpret_cast<const float *>(entries) + r * d + col;
                const f32x4 v0 = *reinterpret_cast<const f32x4 *>(src), v1 = *reinterpret_cast<const f32x4 *>(src + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[e] = v0[e];
                    v[4 + e] = v1[e];
                }
            } else if (vec) {
                const uint4 u = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(entries) + r * d + col);
                const uint32_t wv[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[2 * e] = __uint_as_float(wv[e] << 16);
                    v[2 * e + 1] = __uint_as_float(wv[e] & 0xffff0000u);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    v[e] = col + e >= d ? 0.f
                                        : (dtype == 0 ? reinterpret_cast<const float *>(entries)[r * d + col + e]
                                                      : bf16_to_f32(reinterpret_cast<const uint16_t *>(entries)[r * d + col + e]));
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                s1[e] += (double)v[e];
                s2[e] += (double)v[e] * (double)v[e];
            }
        }
    }
    if (w > 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            comb[w - 1][lane][e] = s1[e];
            comb[w - 1][lane][8 + e] = s2[e];
        }
    }
    __syncthreads();
    if (w == 0 && col < d) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (col + e < d) {
                atomicAdd(&stats[col + e], s1[e] + (comb[0][lane][e] + comb[1][lane][e] + comb[2][lane][e]));
                atomicAdd(&stats[d_pad + col + e], s2[e] + (comb[0][lane][8 + e] + comb[1][lane][8 + e] + comb[2][lane][8 + e]));
            }
        }
    }
}

// mu[i] = column mean (or 0 everywhere when the cache is not worth centring); one workgroup
__global__ __launch_bounds__(1024) void col_mean_kernel(const double *stats, int64_t n, int64_t d, int64_t d_pad, int mode,
                                                        float *mu)
{
    __shared__ double red_m[16], red_v[16];
    __shared__ int centre_s;
    const int tid = threadIdx.x;
    double m2 = 0.0, var = 0.0;
    for (int64_t i = tid; i < d; i += 1024) {
        const double mean = stats[i] / (double)n;
        const double v = stats[d_pad + i] / (double)n - mean * mean;
        m2 += mean * mean;
        var += v > 0.0 ? v : 0.0;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        m2 += __shfl_xor(m2, off, 64);
        var += __shfl_xor(var, off, 64);
    }
    if ((tid & 63) == 0) {
        red_m[tid >> 6] = m2;
        red_v[tid >> 6] = var;
    }
    __syncthreads();
    if (tid == 0) {
        double a = 0.0, b = 0.0;
        for (int w = 0; w < 16; ++w) {
            a += red_m[w];
            b += red_v[w];
        }
        centre_s = mode == 2 || (mode == 1 && a > 4.0 * b);
    }
    __syncthreads();
    const bool centre = centre_s != 0;
    for (int64_t i = tid; i < d_pad; i += 1024) mu[i] = (centre && i < d) ? (float)(stats[i] / (double)n) : 0.f;
}

// RB rows per workgroup (16; 4 for caches of few rows, which would otherwise leave most CUs without work)
template <int RB>
__global__ __launch_bounds__(256) void cache_build_kernel(const void *entries, int dtype, int64_t n, int64_t d,
                                                          int64_t d_pad, uint16_t *c_bf, float *norm, float *c_f32,
                                                          uint16_t *c_rows, const float *mu)
{
    // the matrix cores' copy of the block's rows, 64 chunks (512 elements) of every row at a time, on its
    // way from row order to the tiled order (rows padded by one chunk against bank conflicts)
    static_assert(RB == 4 || RB == 16, "rows per workgroup");
    __shared__ uint4 stage[RB][65];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t row0 = (int64_t)blockIdx.x * RB;
    const int64_t tile = row0 / kTileN;
    const int rit0 = (int)(row0 % kTileN);
    uint4 *tile_base = reinterpret_cast<uint4 *>(c_bf + tile * kTileN * d_pad);
    const int64_t chunks = d_pad / 8;
    // rows start 16-byte aligned when the batch does and d is a multiple of 8 (bf16) or 4 (fp32):
    // whole chunks are then fetched with 16-byte loads
    const bool vec = (reinterpret_cast<uintptr_t>(entries) % 16) == 0 && (dtype == 0 ? d % 4 == 0 : d % 8 == 0);
    constexpr int RPW = RB / 4;   // rows per wave
    float ss[RPW];
#pragma unroll
    for (int q = 0; q < RPW; ++q) ss[q] = 0.f;
    for (int64_t c0 = 0; c0 < chunks; c0 += 64) {
        const int64_t j = c0 + lane;   // this lane's chunk (elements 8 j .. 8 j + 7) of each of the wave's rows
        if (j < chunks) {
            float mv[8];
            if (mu) {
                const f32x4 m0 = *reinterpret_cast<const f32x4 *>(mu + j * 8), m1 = *reinterpret_cast<const f32x4 *>(mu + j * 8 + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    mv[e] = m0[e];
                    mv[4 + e] = m1[e];
                }
            }
#pragma unroll
            for (int q = 0; q < RPW; ++q) {
                const int rl = w * RPW + q;
                const int64_t row = row0 + rl;
                uint16_t h[8];
                float f[8];
                if (row >= n) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        h[e] = 0;
                        f[e] = 0.f;
                    }
                } else if (vec && j * 8 + 8 <= d) {
                    if (dtype == 0) {
                        const float *src = reinterpret_cast<const float *>(entries) + row * d + j * 8;
                        const f32x4 v0 = *reinterpret_cast<const f32x4 *>(src), v1 = *reinterpret_cast<const f32x4 *>(src + 4);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            f[e] = v0[e];
                            f[4 + e] = v1[e];
                        }
#pragma unroll
                        for (int e = 0; e < 8; ++e) h[e] = bf16_rne(f[e]);
                    } else {
                        const uint4 v = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(entries) + row * d + j * 8);
                        const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            h[2 * e] = (uint16_t)(wv[e] & 0xffffu);
                            h[2 * e + 1] = (uint16_t)(wv[e] >> 16);
                        }
#pragma unroll
                        for (int e = 0; e < 8; ++e) f[e] = 0.f;   // (fp32 rows are kept only for fp32 input)
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int64_t i = j * 8 + e;
                        f[e] = 0.f;
                        h[e] = 0;
                        if (i < d) {
                            if (dtype == 0) {
                                f[e] = reinterpret_cast<const float *>(entries)[row * d + i];
                                h[e] = bf16_rne(f[e]);
                            } else {
                                h[e] = reinterpret_cast<const uint16_t *>(entries)[row * d + i];
                            }
                        }
                    }
                }
                uint4 v;   // the stored values (bf16 input) for the row-major copy
                v.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
                v.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
                v.z = (uint32_t)h[4] | ((uint32_t)h[5] << 16);
                v.w = (uint32_t)h[6] | ((uint32_t)h[7] << 16);
                if (row < n) {
                    if (c_rows) reinterpret_cast<uint4 *>(c_rows + row * d_pad)[j] = v;
                    if (c_f32) {
                        f32x4 o0, o1;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            o0[e] = f[e];
                            o1[e] = f[4 + e];
                        }
                        *reinterpret_cast<f32x4 *>(c_f32 + row * d_pad + j * 8) = o0;
                        *reinterpret_cast<f32x4 *>(c_f32 + row * d_pad + j * 8 + 4) = o1;
                    }
                    if (mu) {
                        // the matrix cores' copy relative to mu (all zeros unless the cache is centred: then exact)
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float stored = dtype == 0 ? f[e] : bf16_to_f32(h[e]);
                            h[e] = j * 8 + e < d ? bf16_rne(stored - mv[e]) : (uint16_t)0;
                        }
                        v.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
                        v.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
                        v.z = (uint32_t)h[4] | ((uint32_t)h[5] << 16);
                        v.w = (uint32_t)h[6] | ((uint32_t)h[7] << 16);
                    }
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float x = bf16_to_f32(h[e]);
                    ss[q] = __builtin_fmaf(x, x, ss[q]);
                }
                stage[rl][lane] = v;
            }
        }
        __syncthreads();
        // out in tiled order: for one k-block (4 chunks) the RB rows of the block are RB * 64 bytes in a
        // row; a wave writes 64 / (4 RB) k-blocks at a time
        const int64_t kb0 = c0 / 4;
        constexpr int KPW = 64 / (4 * RB);
        for (int qb = w * KPW + lane / (4 * RB); qb < 16 && (kb0 + qb) * 4 < chunks; qb += 4 * KPW) {
            const int rl = (lane >> 2) % RB, c = lane & 3;
            tile_base[tiled_chunk_offset(rit0 + rl, (kb0 + qb) * 4 + c, kTileN)] = stage[rl][qb * 4 + c];
        }
        __syncthreads();
    }
    // |c|^2 of the bf16 row: the lanes' partial sums in a fixed order
#pragma unroll
    for (int q = 0; q < RPW; ++q) {
        float v = ss[q];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
        const int64_t row = row0 + w * RPW + q;
        if (lane == 0) norm[row] = (row < n) ? v : __builtin_inff();
    }
}

__global__ void copy_i32_kernel(const int32_t *src, int32_t *dst, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

hipError_t launch_cache_build(const void *entries, int dtype, int64_t n, int64_t d, int64_t n_pad, int64_t d_pad,
                              uint16_t *c_bf, float *norm, float *c_f32, uint16_t *c_rows, const int32_t *labels_in,
                              int32_t *labels_out, float *mu, double *stats, int centre_mode, hipStream_t s)
{
    hipError_t e;
    if (mu) {
        // column statistics -> mu (zeros unless the cache is to be centred)
        if ((e = launch_fill_i32(reinterpret_cast<int32_t *>(stats), 0, 4 * d_pad, s)) != hipSuccess) return e;
        const int64_t ns = n < kStatRows ? n : kStatRows;   // sampled rows
        const int64_t col_blocks = (d + 511) / 512;
        int64_t row_chunks = 2048 / col_blocks;
        if (row_chunks > (ns + 31) / 32) row_chunks = (ns + 31) / 32;
        if (row_chunks < 1) row_chunks = 1;
        if (row_chunks > 65535) row_chunks = 65535;
        hipLaunchKernelGGL(col_stats_kernel, dim3((unsigned)col_blocks, (unsigned)row_chunks), dim3(256), 0, s, entries,
                           dtype, n, d, d_pad, ns, stats);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(col_mean_kernel, dim3(1), dim3(1024), 0, s, stats, ns, d, d_pad, centre_mode, mu);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    static_assert(kTileN % 16 == 0, "a workgroup's rows lie in one tile");
    if (n_pad / 16 >= 512)
        hipLaunchKernelGGL(cache_build_kernel<16>, dim3((unsigned)(n_pad / 16)), dim3(256), 0, s, entries, dtype, n, d, d_pad,
                           c_bf, norm, c_f32, c_rows, mu);
    else
        hipLaunchKernelGGL(cache_build_kernel<4>, dim3((unsigned)(n_pad / 4)), dim3(256), 0, s, entries, dtype, n, d, d_pad,
                           c_bf, norm, c_f32, c_rows, mu);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(copy_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, labels_in, labels_out, n);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Query preparation: bf16 copy (round to nearest even) of the live queries for the matrix
// cores in the tiled layout (tiles of bm rows), gathered through the miss list when there is
// one; rows up to the next tile boundary are zero filled.  One block per pair of rows: in the
// tiled layout the 64-byte pieces of two neighbouring rows share a 128-byte line, so eight
// consecutive threads (two rows x four 16-byte chunks of one k-block) write a whole line.
// With few rows and long activations the grid's second dimension cuts the row pair into ranges
// of chunks, so that a batch of 256 rows still fills the chip.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void query_prep_kernel(const float *queries, const int32_t *sel, const int32_t *count,
                                                         int b, int bm, int64_t d, int64_t d_pad, uint16_t *q_bf,
                                                         int32_t *flag_count, int32_t *tickets, const float *mu)
{
    const int nq = count ? *count : b;
    const int row0 = blockIdx.x * 2;   // bm is even: both rows lie in one tile
    // counters of the kernels that follow in this look-up (the list of flagged queries, the exact
    // scan's tickets) start at zero
    if (blockIdx.y == 0 && threadIdx.x < 2) {
        if (tickets && row0 + (int)threadIdx.x < b) tickets[row0 + threadIdx.x] = 0;
        if (flag_count && blockIdx.x == 0) flag_count[threadIdx.x] = 0;   // both lists' counts
    }
    const int live_pad = ((nq + bm - 1) / bm) * bm;
    if (row0 >= live_pad) return;
    uint4 *tile_base = reinterpret_cast<uint4 *>(q_bf + (int64_t)(row0 / bm) * bm * d_pad);
    const int rsel = (threadIdx.x >> 2) & 1;
    const int row = row0 + rsel, rit = row % bm;
    const float *src = (row < nq) ? queries + (int64_t)(sel ? sel[row] : row) * d : nullptr;
    const bool vec = (d % 4) == 0;     // rows are then 16-byte aligned (the batch pointer is)
    const int64_t pair_chunks = d_pad / 4;   // 16-byte chunks of the two rows together
    const int64_t per = ((pair_chunks + gridDim.y - 1) / gridDim.y + 255) / 256 * 256;   // chunks per block of the pair
    const int64_t jj_end = (blockIdx.y + 1) * per < pair_chunks ? (blockIdx.y + 1) * per : pair_chunks;
    // one 16-byte chunk of the bf16 copy from 8 fp32 values
    // (relative to the cache's mean vector when the cache is centred; mu is zero past d and all zeros
    // when it is not)
    auto convert_store = [&](int64_t j, const float (&x)[8]) {
        uint16_t h[8];
        if (mu && src) {
            const f32x4 m0 = *reinterpret_cast<const f32x4 *>(mu + j * 8);
            const f32x4 m1 = *reinterpret_cast<const f32x4 *>(mu + j * 8 + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                h[e] = bf16_rne(x[e] - m0[e]);
                h[4 + e] = bf16_rne(x[4 + e] - m1[e]);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = bf16_rne(x[e]);
        }
        uint4 v;
        v.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
        v.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
        v.z = (uint32_t)h[4] | ((uint32_t)h[5] << 16);
        v.w = (uint32_t)h[6] | ((uint32_t)h[7] << 16);
        tile_base[tiled_chunk_offset(rit, j, bm)] = v;
    };
    int64_t jj = blockIdx.y * per + threadIdx.x;
    // whole rows of 16-byte aligned values: four steps' loads are issued before the first is
    // converted, so that a thread keeps 128 bytes of reads in flight
    if (src && vec && d == d_pad) {
        for (; jj + 3 * 256 < jj_end; jj += 4 * 256) {
            f32x4 v0[4], v1[4];
            int64_t jc[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t ju = jj + u * 256;
                jc[u] = (ju >> 3) * 4 + (ju & 3);
                v0[u] = *reinterpret_cast<const f32x4 *>(src + jc[u] * 8);
                v1[u] = *reinterpret_cast<const f32x4 *>(src + jc[u] * 8 + 4);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float x[8] = {v0[u][0], v0[u][1], v0[u][2], v0[u][3], v1[u][0], v1[u][1], v1[u][2], v1[u][3]};
                convert_store(jc[u], x);
            }
        }
    }
    for (; jj < jj_end; jj += 256) {
        const int64_t j = (jj >> 3) * 4 + (jj & 3);   // chunk of 8 elements within the row
        const int64_t i0 = j * 8;
        float x[8];
        if (src && vec && i0 + 8 <= d) {
            const f32x4 v0 = *reinterpret_cast<const f32x4 *>(src + i0);
            const f32x4 v1 = *reinterpret_cast<const f32x4 *>(src + i0 + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                x[e] = v0[e];
                x[4 + e] = v1[e];
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = (src && i0 + e < d) ? src[i0 + e] : 0.f;
        }
        convert_store(j, x);
    }
}

hipError_t launch_query_prep(const float *queries, const int32_t *sel, const int32_t *count, int64_t b,
                             int64_t b_pad, int bm, int64_t d, int64_t d_pad, uint16_t *q_bf, int32_t *flag_count,
                             int32_t *tickets, const float *mu, hipStream_t s)
{
    if (bm % 2 != 0 || b_pad % 2 != 0) return hipErrorInvalidValue;
    // about 2048 blocks in all, at least four rounds of 256 chunks each
    const int64_t pairs = b_pad / 2, rounds = d_pad / 4 / 256;
    int64_t ysplit = pairs > 0 ? 2048 / pairs : 1;
    if (ysplit > rounds / 4) ysplit = rounds / 4;
    if (ysplit < 1) ysplit = 1;
    hipLaunchKernelGGL(query_prep_kernel, dim3((unsigned)pairs, (unsigned)ysplit), dim3(256), 0, s, queries, sel, count,
                       (int)b, bm, d, d_pad, q_bf, flag_count, tickets, mu);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Finishing kernel, one block per live query:
//  1. gather the query's n_splits * r packed (ordered key, index) candidates and sort them
//     (bitonic, in LDS); the first r are the coarse candidates;
//  2. exact re-scoring: dist = sum_i (q_i - c_i)^2 in fp32 against the stored cache values
//     (bf16 rows widen exactly; fp32 rows when the cache was given in fp32);
//  3. rank the r candidates by (dist, index), emit the first k (Sec. 3: the k (label,
//     distance) tuples);
//  4. vote: occurrences m of each label among the k, winner = most occurrences, smaller
//     label id on equal counts; hit iff m >= vote_threshold (Sec. 2.1 / Sec. 3).
//     With the distance-weighted rule of Sec. 3 instead: C_i = (m_i / k) * sum_j 1/d_j over the
//     label's neighbours (d = square root of the reported squared distance, sums in fp64 in
//     neighbour order), winner = largest C_i, smaller label id on equality; the confidence is
//     reported in fp32 and the look-up is a hit iff it is strictly greater than the layer's
//     threshold (Pseudocode 1, FreezeInference).  A zero distance gives +inf, i.e. a hit.
// ---------------------------------------------------------------------------------------
// Exact re-scoring by one wave of `nwaves`: candidates c0 .. c0+G-1 (c0 = wave * G, stepping nwaves * G), the 64
// lanes striding over the activation 8 elements at a time; dist = sum (q_i - c_i)^2 in fp32,
// per-lane partial sums in index order, then a butterfly over the lanes (fixed order).
template <int G>
__device__ __forceinline__ void rescore_wave(const FinishArgs &a, const float *qrow, const int32_t *idx_s,
                                             float *dist_s, int r, int wave, int lane, int nwaves = 4)
{
    const bool vec = (a.d % 8) == 0;
    for (int c0 = wave * G; c0 < r; c0 += nwaves * G) {
        float acc[G];
        int64_t cand[G];
#pragma unroll
        for (int j = 0; j < G; ++j) {
            acc[j] = 0.f;
            cand[j] = idx_s[(c0 + j < r) ? c0 + j : r - 1];
        }
        if (vec) {
            for (int64_t i = (int64_t)lane * 8; i < a.d; i += 64 * 8) {
                const f32x4 q0 = *reinterpret_cast<const f32x4 *>(qrow + i);
                const f32x4 q1 = *reinterpret_cast<const f32x4 *>(qrow + i + 4);
                const float qv[8] = {q0[0], q0[1], q0[2], q0[3], q1[0], q1[1], q1[2], q1[3]};
                if (a.c_f32) {
#pragma unroll
                    for (int j = 0; j < G; ++j) {
                        const float *c = a.c_f32 + cand[j] * a.d_pad + i;
                        const f32x4 c0v = *reinterpret_cast<const f32x4 *>(c);
                        const f32x4 c1v = *reinterpret_cast<const f32x4 *>(c + 4);
                        const float cv[8] = {c0v[0], c0v[1], c0v[2], c0v[3], c1v[0], c1v[1], c1v[2], c1v[3]};
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float df = qv[e] - cv[e];
                            acc[j] = __builtin_fmaf(df, df, acc[j]);
                        }
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < G; ++j) {
                        const uint4 cb = *reinterpret_cast<const uint4 *>(a.c_rows + cand[j] * a.d_pad + i);
                        const uint32_t wv[4] = {cb.x, cb.y, cb.z, cb.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float c_lo = __uint_as_float(wv[e] << 16);
                            const float c_hi = __uint_as_float(wv[e] & 0xffff0000u);
                            const float d0 = qv[2 * e] - c_lo;
                            acc[j] = __builtin_fmaf(d0, d0, acc[j]);
                            const float d1 = qv[2 * e + 1] - c_hi;
                            acc[j] = __builtin_fmaf(d1, d1, acc[j]);
                        }
                    }
                }
            }
        } else {
            for (int64_t i = lane; i < a.d; i += 64) {
                const float qv = qrow[i];
#pragma unroll
                for (int j = 0; j < G; ++j) {
                    float cv;
                    if (a.c_f32) {
                        cv = a.c_f32[cand[j] * a.d_pad + i];
                    } else {
                        cv = bf16_to_f32(a.c_rows[cand[j] * a.d_pad + i]);
                    }
                    const float df = qv - cv;
                    acc[j] = __builtin_fmaf(df, df, acc[j]);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
            float v = acc[j];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
            if (lane == 0 && c0 + j < r) dist_s[c0 + j] = v;
        }
    }
}

// Exact re-scoring of many candidates against a short activation (d_pad <= 1024, d a multiple
// of 8) by one wave of `nwaves`: the query stays in registers (a lane owns elements 8 l .. 8 l + 7
// and 512 + 8 l .. 512 + 8 l + 7), and G candidate rows are fetched at a time, all loads issued
// before the first is used.  Same per-lane order of additions and the same butterfly as
// rescore_wave, so the same distances bit for bit.
template <int G, bool F32>
__device__ __forceinline__ void rescore_short(const FinishArgs &a, const float *qrow, const int32_t *idx_s,
                                              float *dist_s, int m, int wave, int lane, int nwaves)
{
    const int64_t i0 = (int64_t)lane * 8, i1 = i0 + 512;
    const bool h0 = i0 < a.d, h1 = i1 < a.d;
    float qv[2][8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        qv[0][e] = h0 ? qrow[i0 + e] : 0.f;
        qv[1][e] = h1 ? qrow[i1 + e] : 0.f;
    }
    for (int c0 = wave * G; c0 < m; c0 += nwaves * G) {
        float acc[G];
        if constexpr (F32) {
            f32x4 cv[G][2][2];
#pragma unroll
            for (int j = 0; j < G; ++j) {
                const float *row = a.c_f32 + (int64_t)idx_s[(c0 + j < m) ? c0 + j : m - 1] * a.d_pad;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const bool live = h ? h1 : h0;
                    const float *src = row + (h ? i1 : i0);
                    cv[j][h][0] = live ? *reinterpret_cast<const f32x4 *>(src) : f32x4{0.f, 0.f, 0.f, 0.f};
                    cv[j][h][1] = live ? *reinterpret_cast<const f32x4 *>(src + 4) : f32x4{0.f, 0.f, 0.f, 0.f};
                }
            }
#pragma unroll
            for (int j = 0; j < G; ++j) {
                acc[j] = 0.f;
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float df = qv[h][e] - cv[j][h][e >> 2][e & 3];
                        acc[j] = __builtin_fmaf(df, df, acc[j]);
                    }
            }
        } else {
            uint4 cb[G][2];
#pragma unroll
            for (int j = 0; j < G; ++j) {
                const uint16_t *row = a.c_rows + (int64_t)idx_s[(c0 + j < m) ? c0 + j : m - 1] * a.d_pad;
                cb[j][0] = h0 ? *reinterpret_cast<const uint4 *>(row + i0) : uint4{0, 0, 0, 0};
                cb[j][1] = h1 ? *reinterpret_cast<const uint4 *>(row + i1) : uint4{0, 0, 0, 0};
            }
#pragma unroll
            for (int j = 0; j < G; ++j) {
                acc[j] = 0.f;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const uint32_t wv[4] = {cb[j][h].x, cb[j][h].y, cb[j][h].z, cb[j][h].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float c_lo = __uint_as_float(wv[e] << 16);
                        const float c_hi = __uint_as_float(wv[e] & 0xffff0000u);
                        const float d0 = qv[h][2 * e] - c_lo;
                        acc[j] = __builtin_fmaf(d0, d0, acc[j]);
                        const float d1 = qv[h][2 * e + 1] - c_hi;
                        acc[j] = __builtin_fmaf(d1, d1, acc[j]);
                    }
                }
            }
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
            float v = acc[j];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
            if (lane == 0 && c0 + j < m) dist_s[c0 + j] = v;
        }
    }
}

// Exact re-scoring by the whole block of NT threads for long activations, up to RG candidates at
// once (r <= RG, RG a multiple of 8).  The loop over the activation is the outer one: a thread
// reads its 8-element pieces of the query row once and applies each to all candidates (a 256 KB
// query row of a 64 x 32 x 32 activation does not survive in L2 between passes while the candidate
// rows stream through it: with the row re-read per eight candidates a tenth of the traffic was
// those re-reads), at the price of RG accumulators per thread.  Small batches use 1024-thread
// blocks so that a block per query still fills the memory system.  Same arithmetic as
// rescore_wave: per-thread partial sums in index order, a butterfly over the lanes, then the waves'
// sums combined in a fixed order.
template <int NT, int RG>
__device__ __forceinline__ void rescore_block_all(const FinishArgs &a, const float *qrow, const int32_t *idx_s,
                                                  float *dist_s, float (*red)[8], int r, int tid)
{
    float acc[RG];
#pragma unroll
    for (int j = 0; j < RG; ++j) acc[j] = 0.f;
    for (int64_t i = (int64_t)tid * 8; i < a.d; i += NT * 8) {
        const f32x4 q0 = *reinterpret_cast<const f32x4 *>(qrow + i);
        const f32x4 q1 = *reinterpret_cast<const f32x4 *>(qrow + i + 4);
        const float qv[8] = {q0[0], q0[1], q0[2], q0[3], q1[0], q1[1], q1[2], q1[3]};
#pragma unroll
        for (int g = 0; g < RG; g += 8) {
            if (g < r) {   // uniform
                if (a.c_f32) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float *c = a.c_f32 + (int64_t)idx_s[(g + j < r) ? g + j : r - 1] * a.d_pad + i;
                        const f32x4 c0v = *reinterpret_cast<const f32x4 *>(c);
                        const f32x4 c1v = *reinterpret_cast<const f32x4 *>(c + 4);
                        const float cv[8] = {c0v[0], c0v[1], c0v[2], c0v[3], c1v[0], c1v[1], c1v[2], c1v[3]};
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const float df = qv[e] - cv[e];
                            acc[g + j] = __builtin_fmaf(df, df, acc[g + j]);
                        }
                    }
                } else {
                    uint4 cb[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        cb[j] = *reinterpret_cast<const uint4 *>(a.c_rows + (int64_t)idx_s[(g + j < r) ? g + j : r - 1] * a.d_pad + i);
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const uint32_t wv[4] = {cb[j].x, cb[j].y, cb[j].z, cb[j].w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float c_lo = __uint_as_float(wv[e] << 16);
                            const float c_hi = __uint_as_float(wv[e] & 0xffff0000u);
                            const float d0 = qv[2 * e] - c_lo;
                            acc[g + j] = __builtin_fmaf(d0, d0, acc[g + j]);
                            const float d1 = qv[2 * e + 1] - c_hi;
                            acc[g + j] = __builtin_fmaf(d1, d1, acc[g + j]);
                        }
                    }
                }
            }
        }
    }
#pragma unroll
    for (int g = 0; g < RG; g += 8) {
        if (g < r) {   // uniform
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float v = acc[g + j];
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
                if ((tid & 63) == 0) red[tid >> 6][j] = v;
            }
            __syncthreads();
            if (tid < 8 && g + tid < r) {
                float t = 0.f;
#pragma unroll
                for (int wv = 0; wv < NT / 64; wv += 4)   // fixed order: groups of four waves
                    t += (red[wv][tid] + red[wv + 1][tid]) + (red[wv + 2][tid] + red[wv + 3][tid]);
                dist_s[g + tid] = t;
            }
            __syncthreads();
        }
    }
}

// Label and hit decision from the k nearest neighbours (labels lab_s[k], squared distances
// dsel_s[k], nearest first), by the first k threads of the block; cnt_s / conf_s are scratch.
// Plurality rule: occurrences m of each label, winner = most occurrences, smaller label id on
// equal counts, hit iff m >= vote_threshold.  Distance-weighted rule of Sec. 3: C_i = (m_i / k) *
// sum_j 1 / d_j in fp64 in neighbour order, winner = largest C_i (smaller id on equality), the
// confidence rounded once to fp32, hit iff confidence > threshold (Pseudocode 1).
// k-means cache (Sec. 4; k = 1): the label is the nearest centre's majority label and the
// confidence its majority share over the distance (zero distance: +inf, or 0 for an empty cluster).
__device__ __forceinline__ void decide_and_write(const FinishArgs &a, int q, int tid, const int32_t *lab_s,
                                                 const float *dsel_s, int32_t *cnt_s, double *conf_s, int32_t nearest)
{
    if (a.weighted == 2) {
        if (tid == 0) {
            const double fr = (double)a.fraction[nearest], dd = (double)dsel_s[0];
            const float conf = dd > 0.0 ? (float)(fr / __builtin_sqrt(dd)) : (fr > 0.0 ? __builtin_inff() : 0.f);
            a.out_labels[q] = lab_s[0];
            a.out_votes[q] = 1;
            a.out_conf[q] = conf;
            a.out_hit[q] = (uint8_t)(conf > a.conf_threshold);
        }
        return;
    }
    if (tid < a.k) {
        const int32_t lm = lab_s[tid];
        int c = 0;
        for (int j = 0; j < a.k; ++j) c += (lab_s[j] == lm);
        cnt_s[tid] = c;
        if (a.weighted == 1) {
            double inv = 0.0;
            for (int j = 0; j < a.k; ++j)
                if (lab_s[j] == lm) inv += 1.0 / __builtin_sqrt((double)dsel_s[j]);
            conf_s[tid] = ((double)c / (double)a.k) * inv;
        }
    }
    __syncthreads();
    if (tid == 0 && a.weighted == 1) {
        double best_conf = -1.0;
        int best_c = 0;
        int32_t best_l = 0;
        for (int j = 0; j < a.k; ++j) {
            const double cf = conf_s[j];
            const int32_t l = lab_s[j];
            if (cf > best_conf || (cf == best_conf && l < best_l)) {
                best_conf = cf;
                best_l = l;
                best_c = cnt_s[j];
            }
        }
        const float conf = (float)best_conf;
        a.out_labels[q] = best_l;
        a.out_votes[q] = best_c;
        a.out_conf[q] = conf;
        a.out_hit[q] = (uint8_t)(conf > a.conf_threshold);
    } else if (tid == 0) {
        int best_c = 0;
        int32_t best_l = 0;
        for (int j = 0; j < a.k; ++j) {
            const int c = cnt_s[j];
            const int32_t l = lab_s[j];
            if (c > best_c || (c == best_c && l < best_l)) {
                best_c = c;
                best_l = l;
            }
        }
        a.out_labels[q] = best_l;
        a.out_votes[q] = best_c;
        a.out_hit[q] = (uint8_t)(best_c >= a.vote_threshold);
    }
}

// Rank of each of the m re-scored candidates under (distance, index); the first k go to the
// outputs and to lab_s / dsel_s.  Also counts the candidates that are not preceded by one at the
// same distance (*distinct_s, zero on entry): how many different samples the certificate has.
__device__ __forceinline__ void rank_and_emit(const FinishArgs &a, int q, int m, int tid, int nthreads, const float *dist_s,
                                              const int32_t *idx_s, int32_t *lab_s, float *dsel_s, int32_t *nearest_s,
                                              int *distinct_s)
{
    for (int c = tid; c < m; c += nthreads) {
        const float dm = dist_s[c];
        const int32_t im = idx_s[c];
        int rank = 0, twin = 0;
        for (int j = 0; j < m; ++j) {
            const float dj = dist_s[j];
            const int32_t ij = idx_s[j];
            rank += (dj < dm) || (dj == dm && ij < im);
            twin |= (dj == dm && ij < im);
        }
        if (!twin) atomicAdd(distinct_s, 1);
        if (rank < a.k) {
            a.out_nbr_idx[(int64_t)q * a.k + rank] = im;
            a.out_nbr_dist[(int64_t)q * a.k + rank] = dm;
            lab_s[rank] = a.labels[im];
            dsel_s[rank] = dm;
            if (rank == 0) *nearest_s = im;
        }
    }
}

struct FinishKernelArgs {
    FinishArgs a;
    int sort_cap;   // power of two >= the largest number of entries gathered per query (LDS allocation)
};

// Exactness certificate of the bf16 pre-filter, by the first wave of the block (every thread
// calls; the verdict is valid in every thread after the call).
//
// The m candidates ent[0 .. m) (coarse key kappa_j in the upper half) were re-scored exactly
// (dist_s[j]); dk is the k-th smallest of those exact distances.  Every entry that was NOT
// re-scored has a coarse key >= the float behind excl_bits (+inf or the "no entry" marker: there is
// no such entry).
// The coarse key is the exact distance minus |q|^2 plus an error (bf16 rounding of the query, and of
// the entries when the cache is stored in fp32; fp32 accumulation), so e_j = kappa_j - dist_j
// samples (error - |q|^2) on entries as near to the query as any that could have been missed.  With
// mean and standard deviation sd of the e_j, an excluded entry has, under that error distribution,
//     distance >= kappa_excl - mean - z (1 + 4/m) sd sqrt(1 + 1/m),
// and when this exceeds dk no excluded entry can be among the k nearest: the result is the exact
// one.  z = kCertZ; the estimate needs kCertMinSamples samples from as many distinct distances
// (duplicated rows repeat one sample).  Otherwise the verdict is "unconfirmed" and the caller
// widens the candidate set or hands the query to the exact scan.
__device__ __forceinline__ bool certificate(const uint64_t *ent, const float *dist_s, int m, float dk, uint32_t excl_bits,
                                            int distinct, int tid, int *verdict_s)
{
    if (tid < 64) {
        const double e0 = (double)from_ordered_bits((uint32_t)(ent[0] >> 32)) - (double)dist_s[0];
        double s1 = 0.0, s2 = 0.0;
        for (int j = tid; j < m; j += 64) {
            const double e = ((double)from_ordered_bits((uint32_t)(ent[j] >> 32)) - (double)dist_s[j]) - e0;
            s1 += e;
            s2 += e * e;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            s1 += __shfl_xor(s1, off, 64);
            s2 += __shfl_xor(s2, off, 64);
        }
        if (tid == 0) {
            int ok;
            if (excl_bits >= 0xff800000u) {
                ok = 1;   // nothing was left out (marker), or only padding rows (their keys are +inf)
            } else if (m < kCertMinSamples || distinct < kCertMinSamples) {
                ok = 0;
            } else {
                const double mean_rel = s1 / m;
                double var = (s2 - m * mean_rel * mean_rel) / (m - 1);
                var = var > 0.0 ? var : 0.0;
                const double mean = e0 + mean_rel;
                const double kex = (double)from_ordered_bits(excl_bits);
                // z standard deviations of (an excluded entry's error minus the sample mean), widened by
                // 1 + 4/m for the uncertainty of a standard deviation estimated from m samples
                double margin = kCertZ * (1.0 + 4.0 / m) * __builtin_sqrt(var * (1.0 + 1.0 / m));
                const double floor_ = 4.0 * 5.9604644775390625e-8 * (__builtin_fabs(kex) + __builtin_fabs(mean) + (double)dk);
                margin = margin > floor_ ? margin : floor_;
                ok = (kex - mean - margin > (double)dk) ? 1 : 0;   // false for NaN
            }
            *verdict_s = ok;
        }
    }
    __syncthreads();
    return *verdict_s != 0;
}

// 256-thread blocks are held to four waves per SIMD, i.e. at most 128 registers: the compiler
// would take 169 and leave two blocks per CU, too few to cover one block's merge and final
// phases with the other blocks' re-scoring loads (0.55 -> 0.45 ms on 10,000 queries x 8,192).
//
// WIDER = false: one block per live query, the r best by the coarse key are re-scored; a query
// the certificate does not confirm goes on list 0 (or straight on list 1 when no further
// entries were gathered for it).  WIDER = true (a launch of its own, so that its code and registers
// stay out of the kernel every query runs through; usually it finds list 0 empty): the blocks
// share the queries of list 0 and re-score up to kTier1 of the gathered entries; what is still
// unconfirmed goes on list 1, the exact scan's.
template <int NT, bool WIDER>
__global__ __launch_bounds__(NT, NT == 256 ? 4 : 1) void finish_kernel(FinishKernelArgs fa)
{
    const FinishArgs &a = fa.a;
    constexpr int MAXC = WIDER ? kTier1 : kMaxRescore;   // candidates re-scored per query at most
    extern __shared__ uint64_t ent[];   // sort_cap entries (dynamic: small merges keep occupancy high)
    __shared__ float red[NT / 64][8];
    __shared__ float dist_s[MAXC];
    __shared__ int32_t idx_s[MAXC];
    __shared__ int32_t lab_s[kMaxK];
    __shared__ int32_t cnt_s[kMaxK];
    __shared__ float dsel_s[kMaxK];
    __shared__ double conf_s[kMaxK];
    __shared__ int32_t nearest_s;
    __shared__ int real_s, distinct_s, verdict_s;
    __shared__ uint32_t excl_s;

    const int nq = a.count ? *a.count : a.b;
    const int todo = WIDER ? a.flag_count[0] : nq;   // queries this launch works on
    const int tid = threadIdx.x;
    const int r = a.r;
    auto one_query = [&](int job) {
        const int q = WIDER ? a.flag_list[job] : job;

        // 1. merge the per-split lists (or sort the query's candidate list)
        int n_splits = a.n_splits;
        if (a.count && !a.part_count)   // cascade: the distance pass derived its splits from the live count
            n_splits = splits_for((nq + a.bm - 1) / a.bm, a.n_tiles, a.num_cus, a.max_splits);
        int total = n_splits * r, stride = a.alloc_splits * r;
        if (a.part_count) {
            stride = a.part_stride;
            total = a.part_count[q] < stride ? a.part_count[q] : stride;
        }
        int sort_n = 2;
        while (sort_n < total) sort_n <<= 1;   // <= fa.sort_cap, the LDS allocation
        const uint64_t *src = a.part + (size_t)q * stride;
        if (tid == 0) {
            real_s = 0;
            excl_s = 0xffffffffu;
            distinct_s = 0;
        }
        __syncthreads();
        int mine = 0;
        for (int i = tid; i < sort_n; i += NT) {
            const uint64_t x = (i < total) ? src[i] : kSentinel;
            ent[i] = x;
            mine += (uint32_t)x < (uint32_t)a.n;   // a real cache entry (the "no entry" marker carries index 2^32 - 1)
        }
        if (mine) atomicAdd(&real_s, mine);
        __syncthreads();
        if (!a.part_count) {
            // Per-split lists: a split that filled its list kept its r smallest keys, so every entry
            // of its range that it dropped has a key >= the list's largest.  The smallest of these
            // bounds every entry outside the gathered lists.  (Slots rotate with the thread
            // number so that neighbouring threads read different LDS banks.)
            for (int sp = tid; sp < n_splits; sp += NT) {
                uint32_t mx = 0;
                int jj = sp % r;
                for (int j = 0; j < r; ++j) {
                    const uint32_t kb = (uint32_t)(ent[sp * r + jj] >> 32);
                    mx = kb > mx ? kb : mx;
                    jj = jj + 1 == r ? 0 : jj + 1;
                }
                atomicMin(&excl_s, mx);   // a list with an empty slot dropped nothing: its largest is the marker
            }
            __syncthreads();
        }
        for (int size = 2; size <= sort_n; size <<= 1) {
            for (int stride2 = size >> 1; stride2 > 0; stride2 >>= 1) {
                for (int i = tid; i < (sort_n >> 1); i += NT) {
                    const int lo = ((i & ~(stride2 - 1)) << 1) | (i & (stride2 - 1));   // stride2 is a power of two
                    const int hi = lo + stride2;
                    const bool up = ((lo & size) == 0);
                    const uint64_t x = ent[lo], y = ent[hi];
                    if ((x > y) == up) {
                        ent[lo] = y;
                        ent[hi] = x;
                    }
                }
                __syncthreads();
            }
        }
        const float *qrow = a.queries + (int64_t)(a.sel ? a.sel[q] : q) * a.d;
        // candidates of this round: the best by the coarse key (real entries sort in front of the markers)
        int m = WIDER ? (real_s < kTier1 ? real_s : kTier1) : r;
        // Long activations, a width of 16 (or 32) that leaves room: the last quarter of the candidates
        // is re-scored only when the certificate over the first twelve (24), which then counts the
        // others among the excluded entries, does not confirm the result; most queries are spared a
        // quarter of the rows (C2: 92 % of the queries, 0.42 -> 0.36 ms for the batch).
        const bool two_steps = !WIDER && (r == 16 || r == 32) && a.k <= r / 2 + r / 8 && a.d >= 4096 && a.d % 8 == 0;
        const int m_first = two_steps ? r - r / 4 : m;

        for (int c = tid; c < m; c += NT) {
            // With finite inputs every one of the first r entries is a real cache row.  Non-finite
            // inputs (outside the contract) can leave "no entry" markers here: map them to row 0 so
            // that nothing is read out of bounds.
            const uint32_t ci = (uint32_t)(ent[c] & 0xffffffffu);
            idx_s[c] = ci < (uint32_t)a.n ? (int32_t)ci : 0;
        }
        __syncthreads();

        // 2. exact fp32 re-scoring: each wave takes a group of candidates and needs no block barrier
        if (a.d >= 4096 && a.d % 8 == 0) {
            // long activations: the whole block per candidate, the query row read once
            if (WIDER) {
                for (int c0 = 0; c0 < m; c0 += 32)
                    rescore_block_all<NT, 32>(a, qrow, idx_s + c0, dist_s + c0, red, m - c0 < 32 ? m - c0 : 32, tid);
            } else if (m <= 16) {
                rescore_block_all<NT, 16>(a, qrow, idx_s, dist_s, red, m_first, tid);
            } else if (m <= 32) {
                rescore_block_all<NT, 32>(a, qrow, idx_s, dist_s, red, m_first, tid);
            } else {
                // (two passes of 32: 64 accumulators per thread spill, and the pass is 8 % slower for it)
                rescore_block_all<NT, 32>(a, qrow, idx_s, dist_s, red, 32, tid);
                rescore_block_all<NT, 32>(a, qrow, idx_s + 32, dist_s + 32, red, m - 32, tid);
            }
        } else if (tid < 256) {   // short activations: four waves, one group of candidates each
            if (m <= 16)
                rescore_wave<4>(a, qrow, idx_s, dist_s, m, tid >> 6, tid & 63);
            else if (m <= 32)
                rescore_wave<8>(a, qrow, idx_s, dist_s, m, tid >> 6, tid & 63);
            else
                rescore_wave<16>(a, qrow, idx_s, dist_s, m, tid >> 6, tid & 63);
        }
        __syncthreads();

        // 3. final order (dist, index) and the first k
        const int real = real_s;   // real entries gathered
        const int wider = real < kTier1 ? real : kTier1;
        // the certificate: is any entry that was not re-scored possibly nearer than the k-th?
        // (a candidate list of the keys-out selection holds every entry up to its largest pair)
        const uint32_t excl0 = a.part_count ? (real >= a.n || real < 1 ? 0xffffffffu : (uint32_t)(ent[real - 1] >> 32)) : excl_s;
        bool ok = false;
        if (two_steps) {
            rank_and_emit(a, q, m_first, tid, NT, dist_s, idx_s, lab_s, dsel_s, &nearest_s, &distinct_s);
            __syncthreads();
            const uint32_t nxt = (uint32_t)(ent[m_first] >> 32);   // (real >= r > m_first with finite inputs; else the marker)
            ok = certificate(ent, dist_s, m_first, dsel_s[a.k - 1], nxt < excl0 ? nxt : excl0, distinct_s, tid, &verdict_s);
            if (!ok) {   // uniform
                rescore_block_all<NT, 16>(a, qrow, idx_s + m_first, dist_s + m_first, red, m - m_first, tid);
                if (tid == 0) distinct_s = 0;
                __syncthreads();
            }
        }
        if (!ok) {
            rank_and_emit(a, q, m, tid, NT, dist_s, idx_s, lab_s, dsel_s, &nearest_s, &distinct_s);
            __syncthreads();
            uint32_t excl = excl0;
            if (real > m) {
                const uint32_t nxt = (uint32_t)(ent[m] >> 32);
                excl = nxt < excl ? nxt : excl;
            }
            ok = certificate(ent, dist_s, m, dsel_s[a.k - 1], excl, distinct_s, tid, &verdict_s);
        }
        if (tid == 0) {
            // unconfirmed: the wider round, or the exact scan, redoes this query (the outputs written
            // here stand until then)
            const int next = (WIDER || wider <= r) ? 1 : 0;
            if (!ok) {
                const int pos = atomicAdd(a.flag_count + next, 1);
                (next ? a.flag_list2 : a.flag_list)[pos] = q;
            }
            if (a.stats && (ok || next == 1)) atomicAdd(a.stats + (ok ? (WIDER ? 1 : 0) : 2), 1ull);
        }

        // 4. vote and hit decision
        decide_and_write(a, q, tid, lab_s, dsel_s, cnt_s, conf_s, nearest_s);
    };
    if constexpr (WIDER) {
        for (int job = blockIdx.x; job < todo; job += gridDim.x) {
            one_query(job);
            __syncthreads();   // the next job reuses the shared arrays
        }
    } else {
        if ((int)blockIdx.x < todo) one_query(blockIdx.x);
    }
}

// ---------------------------------------------------------------------------------------
// Finishing kernel of the small-batch path (short activations, at most 16 queries), from the
// block minima alone.  One launch, grid (pairs of blocks, queries), 1024 threads:
//  1. selection (every workgroup of a query repeats it: a few thousand L2-resident reads): T =
//     the R-th smallest block minimum; the R blocks whose minimum is <= T hold every entry that is
//     <= T, hence the R best by the coarse key.  It starts from the per-workgroup minima of the
//     streaming kernel, so only the block minima of the R groups that can matter are read.  The
//     selected blocks are put in ascending order of their minima, the same in every workgroup.
//  2. workgroup x re-scores blocks 2 x and 2 x + 1 of that order exactly in fp32 (64 entries, the
//     same arithmetic as above), sorts them in one wave and leaves the `keep` nearest, and for
//     each block the (coarse key, exact distance) of its minimum entry: samples of the coarse
//     key's error for the certificate.
//  3. the last workgroup of a query to arrive (a ticket per query) takes the k nearest by
//     (distance, index) of what was left, decides label and hit, and checks the certificate:
//     every entry outside the selected blocks has a coarse key >= T.  Unconfirmed queries go on
//     the list of the exact scan.
// ---------------------------------------------------------------------------------------
struct SkinnyTailArgs {
    FinishArgs a;            // queries, cache rows, n, d, d_pad, outputs, flag list (a.r = blocks to take)
    const uint64_t *bmin;    // [b, nb] smallest (ordered key, index) of every block of 32 entries
    const uint64_t *wgmin;   // [b, n_groups] smallest value of each group of blocks
    int64_t nb;
    int n_groups, n_tiles;   // group j = the blocks of cache tiles [j n_tiles / n_groups, (j+1) n_tiles / n_groups)
    uint64_t *cand;          // [b, pairs * keep] packed (ordered distance, index), marker-padded
    uint64_t *samp;          // [b, 2 pairs] (coarse key bits << 32 | distance bits) of each block's minimum entry
    int32_t *tickets;        // [b], zero on entry (the streaming kernel clears them); left zero
    int keep;                // entries each workgroup passes on (<= 64)
    int pairs;               // workgroups per query
};

// The R-th smallest of list[0..cnt) (distinct values), cnt <= kThrList, by the whole workgroup.
__device__ inline uint64_t rth_of_list(uint64_t *list, int cnt, int r_sel, uint64_t *sel_s, int tid)
{
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

__global__ __launch_bounds__(kThrThreads) void skinny_tail_kernel(SkinnyTailArgs sa)
{
    const FinishArgs &a = sa.a;
    __shared__ uint64_t list[kThrList];
    __shared__ uint64_t gm_s[kThrThreads];
    __shared__ uint64_t pick_s[kMaxRescore];   // minima (pairs) of the selected blocks, ascending
    __shared__ uint64_t sel_s;
    __shared__ int list_n, blk_n, grp_n, last_s, distinct_s, verdict_s;
    __shared__ int32_t grp_s[kMaxRescore];
    __shared__ int32_t idx_s[64], row_s[64];
    __shared__ float dist_s[64];
    __shared__ int32_t lab_s[kMaxK], cnt_s[kMaxK];
    __shared__ float dsel_s[kMaxK];
    __shared__ double conf_s[kMaxK];
    __shared__ int32_t nearest_s;
    const int q = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
    const int64_t nb = sa.nb;
    const int r = a.r;

    // ---- 1. selection ----
    int nblk;
    if (r >= nb) {   // fewer blocks than wanted: take them all, in index order
        if (tid < (int)nb) pick_s[tid] = sa.bmin[(size_t)q * nb + tid];
        nblk = (int)nb;
        __syncthreads();
    } else {
        // 1a. the groups that can hold one of the r smallest block minima: those whose own minimum
        //     is among the r smallest group minima (T1 = the r-th of them bounds the answer above)
        const int ng = sa.n_groups;
        if (tid == 0) {
            list_n = 0;
            blk_n = 0;
            grp_n = 0;
        }
        const uint64_t my_gm = tid < ng ? sa.wgmin[(size_t)q * ng + tid] : kSentinel;
        gm_s[tid] = my_gm;
        __syncthreads();
        uint64_t t1 = kSentinel;
        if (r < ng) {
            if (r <= 32) {
                t1 = smallest_sorted(gm_s, list, ng, r, tid, kThrThreads)[r - 1];
            } else {
                select_by_rank_counting(gm_s, ng, r - 1, tid, &sel_s);
                __syncthreads();
                t1 = sel_s;
            }
            __syncthreads();
        }
        if (tid < ng && my_gm <= t1) {
            const int pos = atomicAdd(&grp_n, 1);
            if (pos < kMaxRescore) grp_s[pos] = tid;
        }
        __syncthreads();
        const int ngrp = grp_n < kMaxRescore ? grp_n : kMaxRescore;   // min(r, ng) groups
        // 1b. gather their block minima <= T1: at least r, at most r * (blocks per group)
        const int bpg = ((sa.n_tiles + ng - 1) / ng) * (kTileN / 32);
        const uint64_t *src = sa.bmin + (size_t)q * nb;
        for (int c = tid; c < ngrp * bpg; c += kThrThreads) {
            const int gidx = grp_s[c / bpg];
            const int64_t b0 = ((int64_t)gidx * sa.n_tiles / ng) * (kTileN / 32);
            const int64_t b1 = ((int64_t)(gidx + 1) * sa.n_tiles / ng) * (kTileN / 32);
            const int64_t bi = b0 + c % bpg;
            if (bi < b1) {
                const uint64_t x = src[bi];
                if (x <= t1) {
                    const int pos = atomicAdd(&list_n, 1);
                    if (pos < kThrList) list[pos] = x;
                }
            }
        }
        __syncthreads();
        const int cnt = list_n < kThrList ? list_n : kThrList;
        // 1c. the r smallest of them, ascending, are the minima of the blocks to take (distinct values)
        if (r <= 32 && cnt <= kThrList / 2) {
            const uint64_t *res = smallest_sorted(list, list + kThrList / 2, cnt, r, tid, kThrThreads);
            if (tid < r) pick_s[tid] = res[tid];
        } else {
            const uint64_t t = rth_of_list(list, cnt, r, &sel_s, tid);
            __syncthreads();
            for (int i = tid; i < cnt; i += kThrThreads) {
                const uint64_t x = list[i];
                if (x <= t) {
                    const int pos = atomicAdd(&blk_n, 1);
                    if (pos < kMaxRescore) pick_s[pos] = x;
                }
            }
            __syncthreads();
            if (tid < 64) {   // exactly r <= 64 values: one wave puts them in order
                const uint64_t v = wave_sort64(lane < r ? pick_s[lane] : kSentinel, lane);
                if (lane < r) pick_s[lane] = v;
            }
        }
        nblk = r;
        __syncthreads();
    }

    // ---- 2. exact re-scoring of this workgroup's two blocks ----
    uint64_t *out = sa.cand + ((size_t)q * sa.pairs + blockIdx.x) * sa.keep;
    uint64_t *samp = sa.samp + (size_t)q * 2 * sa.pairs + 2 * blockIdx.x;
    const int first = blockIdx.x * 2;
    const int here = nblk - first < 2 ? nblk - first : 2;   // blocks of this workgroup
    if (here <= 0) {
        if (tid < sa.keep) out[tid] = kSentinel;
        if (tid < 2) samp[tid] = kSentinel;
    } else {
        const int m = here * 32;
        // entries past the cache (padding rows of the last tile) are re-scored as row 0 and dropped below
        if (tid < m) {
            const int e = (int)((uint32_t)pick_s[first + (tid >> 5)] >> 5) * 32 + (tid & 31);
            idx_s[tid] = e < a.n ? e : -1 - e;
            row_s[tid] = e < a.n ? e : 0;
        }
        __syncthreads();
        const float *qrow = a.queries + (int64_t)q * a.d;
        if (a.d % 8 != 0)
            rescore_wave<4>(a, qrow, row_s, dist_s, m, tid >> 6, lane, kThrThreads / 64);
        else if (a.c_f32)
            rescore_short<4, true>(a, qrow, row_s, dist_s, m, tid >> 6, lane, kThrThreads / 64);
        else
            rescore_short<4, false>(a, qrow, row_s, dist_s, m, tid >> 6, lane, kThrThreads / 64);
        __syncthreads();
        if (tid < 64) {
            uint64_t x = kSentinel;
            if (tid < m && idx_s[tid] >= 0) x = ((uint64_t)ordered_bits(dist_s[tid]) << 32) | (uint32_t)idx_s[tid];
            x = wave_sort64(x, lane);
            if (lane < sa.keep) out[lane] = x;
        } else if (tid < 66) {
            const int hb = tid - 64;
            uint64_t sv = kSentinel;
            if (hb < here) {
                const uint64_t pr = pick_s[first + hb];   // (coarse key, index) of the block's minimum entry
                sv = (pr & 0xffffffff00000000ull) | __float_as_uint(dist_s[hb * 32 + ((uint32_t)pr & 31u)]);
            }
            samp[hb] = sv;
        }
    }

    // ---- 3. the last workgroup of the query finishes it ----
    // (the barrier orders every thread's stores before thread 0's fence, which publishes them to the
    // device before the ticket is taken; the last workgroup reads them with device-coherent loads)
    __syncthreads();
    if (tid == 0) {
        __threadfence();
        last_s = (atomicAdd(&sa.tickets[q], 1) == sa.pairs - 1);
        __threadfence();
    }
    __syncthreads();
    if (!last_s) return;   // uniform
    const int mcand = sa.pairs * sa.keep;   // <= kThrList / 2
    for (int c = tid; c < mcand; c += kThrThreads)
        list[c] = __hip_atomic_load(sa.cand + (size_t)q * mcand + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tid == 0) {
        sa.tickets[q] = 0;
        distinct_s = 0;
    }
    __syncthreads();
    const uint64_t *res;
    if (a.k <= 32) {
        res = smallest_sorted(list, list + kThrList / 2, mcand, a.k, tid, kThrThreads);
    } else {
        int n2 = 2;
        while (n2 < mcand) n2 <<= 1;
        for (int c = mcand + tid; c < n2; c += kThrThreads) list[c] = kSentinel;
        __syncthreads();
        bitonic_sort_lds(list, n2, tid, kThrThreads);
        res = list;
    }
    if (tid < a.k) {
        const uint64_t x = res[tid];
        // with finite inputs the first k are real entries; a "no entry" marker maps to row 0
        const int32_t im = x == kSentinel ? 0 : (int32_t)(uint32_t)x;
        const float dm = from_ordered_bits((uint32_t)(x >> 32));
        a.out_nbr_idx[(int64_t)q * a.k + tid] = im;
        a.out_nbr_dist[(int64_t)q * a.k + tid] = dm;
        lab_s[tid] = a.labels[im];
        dsel_s[tid] = dm;
        if (tid == 0) nearest_s = im;
    }
    __syncthreads();
    // certificate from the block minima: gm_s = the samples' coarse keys (upper halves), dist_s = their distances
    if (tid < nblk) {
        const uint64_t sv = __hip_atomic_load(sa.samp + (size_t)q * 2 * sa.pairs + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        gm_s[tid] = sv & 0xffffffff00000000ull;
        dist_s[tid] = __uint_as_float((uint32_t)sv);
    }
    __syncthreads();
    if (tid < nblk) {
        int twin = 0;
        for (int j = 0; j < tid; ++j) twin |= (dist_s[j] == dist_s[tid]);
        if (!twin) atomicAdd(&distinct_s, 1);
    }
    __syncthreads();
    const uint32_t excl = r >= nb ? 0xffffffffu : (uint32_t)(pick_s[nblk - 1] >> 32);
    const bool ok = certificate(gm_s, dist_s, nblk, dsel_s[a.k - 1], excl, distinct_s, tid, &verdict_s);
    if (tid == 0) {
        if (!ok) {
            const int pos = atomicAdd(a.flag_count + 1, 1);
            a.flag_list2[pos] = q;
        }
        if (a.stats) atomicAdd(a.stats + (ok ? 0 : 2), 1ull);
    }
    decide_and_write(a, q, tid, lab_s, dsel_s, cnt_s, conf_s, nearest_s);
}

size_t skinny_finish_workspace_bytes(int r, size_t align)
{
    auto up = [&](size_t x) { return (x + align - 1) / align * align; };
    const size_t pairs = (size_t)(r + 1) / 2;
    return up((size_t)kSkinnyRows * pairs * 64 * 8) + up((size_t)kSkinnyRows * pairs * 2 * 8);
}

hipError_t launch_skinny_finish(const FinishArgs &a, const uint64_t *bmin, const uint64_t *wgmin, int64_t nb,
                                int n_groups, int n_tiles, uint64_t *cand, uint64_t *samp, int32_t *tickets, hipStream_t s)
{
    if (a.r < 1 || a.r > kMaxRescore || a.k > kMaxK || a.k > a.r || a.b < 1 || a.b > kSkinnyRows || a.sel || a.count)
        return hipErrorInvalidValue;
    if (n_groups < 1 || n_groups > kThrThreads || n_groups > n_tiles) return hipErrorInvalidValue;
    if (!a.flag_count || !a.flag_list2 || !tickets) return hipErrorInvalidValue;
    const int64_t bpg = ((int64_t)(n_tiles + n_groups - 1) / n_groups) * (kTileN / 32);
    if (a.r < nb && bpg * a.r > kThrList) return hipErrorInvalidValue;
    const int pairs = (a.r + 1) / 2;   // a.r >= the number of blocks selected
    const int keep = a.k <= 32 ? a.k : 64;
    SkinnyTailArgs ta{a, bmin, wgmin, nb, n_groups, n_tiles, cand, samp, tickets, keep, pairs};
    hipLaunchKernelGGL(skinny_tail_kernel, dim3((unsigned)pairs, (unsigned)a.b), dim3(kThrThreads), 0, s, ta);
    return hipGetLastError();
}

hipError_t launch_finish(const FinishArgs &a, int num_cus, hipStream_t s)
{
    const int total = a.part_count ? a.part_stride : a.alloc_splits * a.r;
    if (total > kMaxMergeEntries || a.r > kMaxRescore || a.k > kMaxK || a.k > a.r) return hipErrorInvalidValue;
    if (!a.flag_count || !a.flag_list || !a.flag_list2) return hipErrorInvalidValue;
    FinishKernelArgs fa{a, 2};
    while (fa.sort_cap < total) fa.sort_cap <<= 1;
    const size_t lds = (size_t)fa.sort_cap * sizeof(uint64_t);
    // a block per query: with few queries and long activations use 1024-thread blocks
    if (a.b <= 1024 && a.d >= 16384 && a.d % 8 == 0)
        hipLaunchKernelGGL((finish_kernel<1024, false>), dim3((unsigned)a.b), dim3(1024), lds, s, fa);
    else
        hipLaunchKernelGGL((finish_kernel<256, false>), dim3((unsigned)a.b), dim3(256), lds, s, fa);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // the wider round for the queries on list 0: a fixed grid shares them (usually there are none)
    const int grid = a.b < 2 * num_cus ? a.b : 2 * num_cus;
    hipLaunchKernelGGL((finish_kernel<256, true>), dim3((unsigned)grid), dim3(256), lds, s, fa);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Exact scan of the queries whose result the certificate did not confirm (Sec. 3: the look-up
// returns THE k nearest neighbours): brute-force fp32 distances sum (q_i - c_i)^2 to every
// stored entry, the same arithmetic as the re-scoring above, no bf16 anywhere.  A fixed grid of
// workgroups shares the flagged queries: with nf of them, each is cut into S = grid / nf
// ranges of at least 16 entries (at least one range, at most max_splits); a workgroup scans its range 256 entries
// at a time and keeps the k nearest by (distance, index); the last workgroup of a query to finish
// (a ticket per query) merges the S lists and writes the neighbours, the label and the hit
// decision over that query's outputs.  Nothing is flagged on the paper's kind of data, and then
// the kernel reads one counter and returns.
// ---------------------------------------------------------------------------------------
struct ScanArgs {
    FinishArgs a;
    int32_t *tickets;    // [b], zero on entry; left zero
    uint64_t *part_x;    // [items, k] the k nearest of each (query, range), packed (ordered distance, index)
    int max_splits;
};

__global__ __launch_bounds__(256) void exact_scan_kernel(ScanArgs sa)
{
    const FinishArgs &a = sa.a;
    extern __shared__ uint64_t ent[];   // >= 512 entries and >= max_splits * k
    __shared__ float red[4][8];
    __shared__ float dist_s[256];
    __shared__ int32_t idx_s[256];
    __shared__ uint64_t best_s[kMaxK];
    __shared__ int32_t lab_s[kMaxK];
    __shared__ int32_t cnt_s[kMaxK];
    __shared__ float dsel_s[kMaxK];
    __shared__ double conf_s[kMaxK];
    __shared__ int32_t nearest_s;
    __shared__ int surv_s, last_s;

    const int nf = a.flag_count[1];
    if (nf <= 0) return;   // the usual case
    const int tid = threadIdx.x;
    const int grid = (int)gridDim.x, k = a.k;
    int S = grid / nf;
    const int by_size = (a.n + 15) / 16;   // a range holds at least 16 entries
    S = S > sa.max_splits ? sa.max_splits : S;
    S = S > by_size ? by_size : S;
    S = S < 1 ? 1 : S;
    const int64_t items = (int64_t)nf * S;
    for (int64_t item = blockIdx.x; item < items; item += grid) {
        const int j = (int)(item / S), sp = (int)(item - (int64_t)j * S);
        const int q = a.flag_list2[j];
        const float *qrow = a.queries + (int64_t)(a.sel ? a.sel[q] : q) * a.d;
        const int row0 = (int)((int64_t)a.n * sp / S), row1 = (int)((int64_t)a.n * (sp + 1) / S);
        if (tid < kMaxK) best_s[tid] = kSentinel;
        __syncthreads();
        for (int base = row0; base < row1; base += 256) {
            const int m = row1 - base < 256 ? row1 - base : 256;
            if (tid < m) idx_s[tid] = base + tid;
            if (tid == 0) surv_s = 0;
            __syncthreads();
            if (a.d >= 4096 && a.d % 8 == 0) {
                for (int c0 = 0; c0 < m; c0 += 32)
                    rescore_block_all<256, 32>(a, qrow, idx_s + c0, dist_s + c0, red, m - c0 < 32 ? m - c0 : 32, tid);
            } else
                rescore_wave<16>(a, qrow, idx_s, dist_s, m, tid >> 6, tid & 63);
            __syncthreads();
            // entries that beat the k-th best so far, then the k best of those and the list
            const uint64_t tau = best_s[k - 1];
            if (tid < m) {
                const uint64_t x = ((uint64_t)ordered_bits(dist_s[tid]) << 32) | (uint32_t)(base + tid);
                if (x < tau) ent[atomicAdd(&surv_s, 1)] = x;
            }
            __syncthreads();
            const int c = surv_s;
            if (c > 0) {   // uniform
                int n2 = 2;
                while (n2 < c + k) n2 <<= 1;   // <= 512
                for (int i = c + tid; i < n2; i += 256) ent[i] = i < c + k ? best_s[i - c] : kSentinel;
                __syncthreads();
                bitonic_sort_lds(ent, n2, tid, 256);
                if (tid < k) best_s[tid] = ent[tid];
                __syncthreads();
            }
        }
        if (tid < k) sa.part_x[(size_t)item * k + tid] = best_s[tid];
        __syncthreads();
        if (tid == 0) {
            __threadfence();   // the list is visible to the whole device before the ticket is taken
            last_s = (atomicAdd(&sa.tickets[j], 1) == S - 1);
            __threadfence();
        }
        __syncthreads();
        if (last_s) {   // uniform: this workgroup finished the query's last range
            const int total = S * k;
            int n2 = 2;
            while (n2 < total) n2 <<= 1;
            const uint64_t *src = sa.part_x + (size_t)j * S * k;
            for (int i = tid; i < n2; i += 256)
                ent[i] = i < total ? __hip_atomic_load(src + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : kSentinel;
            __syncthreads();
            bitonic_sort_lds(ent, n2, tid, 256);
            if (tid < k) {
                const uint64_t x = ent[tid];
                const int32_t im = (uint32_t)x < (uint32_t)a.n ? (int32_t)(uint32_t)x : 0;   // (non-finite inputs only)
                const float dm = from_ordered_bits((uint32_t)(x >> 32));
                a.out_nbr_idx[(int64_t)q * k + tid] = im;
                a.out_nbr_dist[(int64_t)q * k + tid] = dm;
                lab_s[tid] = a.labels[im];
                dsel_s[tid] = dm;
                if (tid == 0) {
                    nearest_s = im;
                    sa.tickets[j] = 0;
                }
            }
            __syncthreads();
            decide_and_write(a, q, tid, lab_s, dsel_s, cnt_s, conf_s, nearest_s);
        }
        __syncthreads();
    }
}

static int scan_max_splits(int k) { return kMaxMergeEntries / k < kScanMaxSplits ? kMaxMergeEntries / k : kScanMaxSplits; }
// (an empty launch costs the same 4 us whatever its grid: no smaller grid for small batches, whose
// flagged queries then get all the workgroups)
static int scan_grid(int num_cus, int64_t) { return 2 * num_cus; }

size_t scan_scratch_entries(int64_t b, int k, int num_cus)
{
    // items = flagged queries x ranges <= max(b, grid)
    const int64_t items = b > scan_grid(num_cus, b) ? b : scan_grid(num_cus, b);
    return (size_t)items * (size_t)k;
}

hipError_t launch_exact_scan(const FinishArgs &a, int32_t *tickets, uint64_t *part_x, int num_cus, hipStream_t s)
{
    if (!a.flag_count || !a.flag_list2 || !tickets || !part_x || a.k < 1 || a.k > kMaxK) return hipErrorInvalidValue;
    const int grid = scan_grid(num_cus, a.b);
    ScanArgs sa{a, tickets, part_x, scan_max_splits(a.k) < grid ? scan_max_splits(a.k) : grid};
    int cap = 512;
    while (cap < sa.max_splits * a.k) cap <<= 1;
    hipLaunchKernelGGL(exact_scan_kernel, dim3((unsigned)grid), dim3(256), (size_t)cap * sizeof(uint64_t), s, sa);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Miss compaction (Sec. 5, "Freeze Inference on GPUs": the batch is rebuilt without the
// frozen items).  Stable: misses keep their order.  One block; ballot-based scan.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void compact_kernel(const uint8_t *hit, const int32_t *sel_in, const int32_t *count_in,
                                                       int count_max, int32_t *sel_out, int32_t *count_out,
                                                       int64_t *hits_out)
{
    __shared__ int wave_tot[16];
    __shared__ int base_s;
    const int cnt = count_in ? *count_in : count_max;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    if (tid == 0) base_s = 0;
    __syncthreads();
    for (int start = 0; start < cnt; start += 1024) {
        const int j = start + tid;
        const bool miss = (j < cnt) && (hit[j] == 0);
        const uint64_t bal = __ballot(miss);
        const int before = __builtin_popcountll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) wave_tot[w] = __builtin_popcountll(bal);
        __syncthreads();
        int off = base_s;
        for (int i = 0; i < w; ++i) off += wave_tot[i];
        if (miss) sel_out[off + before] = sel_in ? sel_in[j] : j;
        __syncthreads();
        if (tid == 0) {
            int t = 0;
            for (int i = 0; i < 16; ++i) t += wave_tot[i];
            base_s += t;
        }
        __syncthreads();
    }
    if (tid == 0) {
        *count_out = base_s;
        if (hits_out) *hits_out = (int64_t)cnt - (int64_t)base_s;
    }
}

hipError_t launch_compact(const uint8_t *hit, const int32_t *sel_in, const int32_t *count_in, int64_t count_max,
                          int32_t *sel_out, int32_t *count_out, int64_t *hits_out, hipStream_t s)
{
    hipLaunchKernelGGL(compact_kernel, dim3(1), dim3(1024), 0, s, hit, sel_in, count_in, (int)count_max, sel_out,
                       count_out, hits_out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Cascade bookkeeping (Pseudocode 1, FreezeInference): start with "no layer hit", then
// after each layer record (label, layer position) for the requests that hit there.
// ---------------------------------------------------------------------------------------
__global__ void cascade_init_kernel(int32_t *out_labels, int32_t *out_exit, int64_t b)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < b) {
        out_labels[i] = -1;
        out_exit[i] = -1;
    }
}

hipError_t launch_cascade_init(int32_t *out_labels, int32_t *out_exit, int64_t b, hipStream_t s)
{
    hipLaunchKernelGGL(cascade_init_kernel, dim3((unsigned)((b + 255) / 256)), dim3(256), 0, s, out_labels, out_exit, b);
    return hipGetLastError();
}

__global__ void cascade_scatter_kernel(const int32_t *labels, const uint8_t *hit, const int32_t *sel, const int32_t *count,
                                       int b, int layer_pos, int32_t *out_labels, int32_t *out_exit)
{
    const int nq = count ? *count : b;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < nq && hit[j]) {
        const int orig = sel ? sel[j] : j;
        out_labels[orig] = labels[j];
        out_exit[orig] = layer_pos;
    }
}

hipError_t launch_cascade_scatter(const int32_t *labels, const uint8_t *hit, const int32_t *sel,
                                  const int32_t *count, int64_t b, int layer_pos, int32_t *out_labels,
                                  int32_t *out_exit, hipStream_t s)
{
    hipLaunchKernelGGL(cascade_scatter_kernel, dim3((unsigned)((b + 255) / 256)), dim3(256), 0, s, labels, hit, sel,
                       count, (int)b, layer_pos, out_labels, out_exit);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Batch reconstruction of a tensor (Sec. 5, "Freeze Inference on GPUs"): the rows of the missed
// requests, in miss-list order, so that the next layer of the model runs on a dense smaller
// batch.  One block per output row; nothing is done past the device-side count.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gather_rows_kernel(const float *x, int64_t d, const int32_t *sel, const int32_t *count,
                                                          int64_t max_count, float *out)
{
    const int64_t nq = count ? *count : max_count;
    const int64_t j = blockIdx.x;
    if (j >= nq) return;
    const float *src = x + (int64_t)sel[j] * d;
    float *dst = out + j * d;
    if ((d % 4) == 0 && (reinterpret_cast<uintptr_t>(x) % 16) == 0 && (reinterpret_cast<uintptr_t>(out) % 16) == 0) {
        for (int64_t i = threadIdx.x; i < d / 4; i += 256)
            reinterpret_cast<f32x4 *>(dst)[i] = reinterpret_cast<const f32x4 *>(src)[i];
    } else {
        for (int64_t i = threadIdx.x; i < d; i += 256) dst[i] = src[i];
    }
}

hipError_t launch_gather_rows(const float *x, int64_t d, const int32_t *sel, const int32_t *count, int64_t max_count,
                              float *out, hipStream_t s)
{
    if (max_count <= 0) return hipSuccess;
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)max_count), dim3(256), 0, s, x, d, sel, count, max_count, out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Per-layer threshold (Pseudocode 1, ComputeThresholds): the largest confidence among the
// validation items whose look-up disagrees with the model's label; 0 when none disagrees.
// Confidences are >= 0 (or +inf), so their fp32 bit patterns order like unsigned integers.
// ---------------------------------------------------------------------------------------
__global__ void threshold_init_kernel(float *thr, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) thr[i] = 0.f;
}

__global__ void threshold_max_kernel(const int32_t *pred, const float *conf, const int32_t *model_labels, int64_t b,
                                     float *thr)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t v = 0;
    if (i < b && pred[i] != model_labels[i]) v = __float_as_uint(conf[i]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)v, off, 64);
        v = o > v ? o : v;
    }
    if ((threadIdx.x & 63) == 0 && v != 0) atomicMax(reinterpret_cast<unsigned int *>(thr), v);
}

hipError_t launch_threshold_init(float *thr, int n, hipStream_t s)
{
    hipLaunchKernelGGL(threshold_init_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, thr, n);
    return hipGetLastError();
}

hipError_t launch_threshold_max(const int32_t *pred, const float *conf, const int32_t *model_labels, int64_t b,
                                float *thr, hipStream_t s)
{
    if (b <= 0) return hipSuccess;
    hipLaunchKernelGGL(threshold_max_kernel, dim3((unsigned)((b + 255) / 256)), dim3(256), 0, s, pred, conf,
                       model_labels, b, thr);
    return hipGetLastError();
}

}  // namespace fz
