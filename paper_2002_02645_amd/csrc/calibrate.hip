// Calibration microbenchmarks (measurement aids, not part of the look-up): what this GPU
// sustains on the two roofs the look-up kernels are priced against.
//  - pure MFMA: every wave issues back-to-back, independent v_mfma_f32_16x16x32_bf16 (the shape
//    the distance kernel uses) from registers, no memory traffic at all, rotating through four
//    operand pairs of pseudo-random bf16 values: the chip runs matrix work against its power
//    limit, and the clock it holds depends on how much the operands toggle (constant operands
//    read about 20 % higher).  Also reports that shader clock (shader-clock counter against the
//    100 MHz real-time counter);
//  - pure read: every byte of a buffer is read once with 16-byte loads (grid-stride).
// Both synchronise the device: they are for benchmarks, not for the serving path.
#include "../../include/freeze.h"

#include <hip/hip_runtime.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int kCalAcc = 32;   // independent accumulators per wave (128 registers, as in the distance kernel)

// 8 bf16 values in [0.125, 1) with random sign and mantissa, from a hash of (thread, slot)
__device__ inline bf16x8 random_operand(unsigned seed)
{
    u32x4 w;
    for (int i = 0; i < 4; ++i) {
        seed = seed * 1664525u + 1013904223u;
        unsigned x = seed ^ (seed >> 15);
        const unsigned lo = ((x >> 3) & 0x80ffu) | (0x3e00u + ((x >> 1) & 0x180u));
        const unsigned hi = ((x >> 17) & 0x80ffu) | (0x3e00u + ((x >> 12) & 0x180u));
        w[i] = lo | (hi << 16);
    }
    return __builtin_bit_cast(bf16x8, w);
}

__global__ __launch_bounds__(512) void mfma_peak_kernel(float *out, unsigned long long *clk, int iters)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        clk[0] = clock64();
        clk[1] = wall_clock64();
    }
    bf16x8 a[4], b[4];
    for (int i = 0; i < 4; ++i) {
        a[i] = random_operand(threadIdx.x * 8u + i);
        b[i] = random_operand(threadIdx.x * 8u + 4u + i);
    }
    f32x4 acc[kCalAcc];
    for (int j = 0; j < kCalAcc; ++j)
        for (int e = 0; e < 4; ++e) acc[j][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < kCalAcc; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j % 4], b[(j / 4) % 4], acc[j], 0, 0, 0);
    }
    float s = 0.f;
    for (int j = 0; j < kCalAcc; ++j)
        for (int e = 0; e < 4; ++e) s += acc[j][e];
    out[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        clk[2] = clock64();
        clk[3] = wall_clock64();
    }
}

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// Every byte is read once, so the loads carry the non-temporal hint, like the library's own
// read-once streams (on this chip such a stream runs about a tenth faster than with plain loads).
__global__ __launch_bounds__(256) void read_kernel(const u32x4 *__restrict__ p, size_t n16)
{
    // each workgroup walks one contiguous share of the buffer, eight 4 KiB rows per round in flight
    unsigned s = 0;
    const size_t share = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t begin = (size_t)blockIdx.x * share;
    const size_t end = begin + share < n16 ? begin + share : n16;
    size_t i = begin + threadIdx.x;
    for (; i + 7 * 256 < end; i += 8 * 256) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + i + u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u][u & 3];
    }
    for (; i < end; i += 256) s += __builtin_nontemporal_load(p + i)[0];
    asm volatile("" ::"v"(s));   // keeps the loads alive; nothing is written
}

}  // namespace

extern "C" {

int freeze_calibrate_mfma(void *scratch, size_t scratch_bytes, double *tflops, double *shader_mhz)
{
    int dev = 0;
    hipDeviceProp_t prop;
    if (!scratch || !tflops || !shader_mhz) return FREEZE_EINVAL;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return FREEZE_EHIP;
    const int cus = prop.multiProcessorCount;
    const size_t need = (size_t)cus * 512 * sizeof(float) + 4 * sizeof(unsigned long long);
    if (scratch_bytes < need || (reinterpret_cast<uintptr_t>(scratch) % 8) != 0) return FREEZE_EWORKSPACE;
    unsigned long long *clk = static_cast<unsigned long long *>(scratch);
    float *out = reinterpret_cast<float *>(clk + 4);
    const int iters = 5000;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return FREEZE_EHIP;
    hipLaunchKernelGGL(mfma_peak_kernel, dim3(cus), dim3(512), 0, nullptr, out, clk, 200);   // warm-up
    (void)hipEventRecord(e0, nullptr);
    hipLaunchKernelGGL(mfma_peak_kernel, dim3(cus), dim3(512), 0, nullptr, out, clk, iters);
    (void)hipEventRecord(e1, nullptr);
    int rc = FREEZE_OK;
    float ms = 0.f;
    unsigned long long h[4] = {0, 0, 0, 0};
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess ||
        hipMemcpy(h, clk, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess)
        rc = FREEZE_EHIP;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != FREEZE_OK) return rc;
    const double flops = (double)cus * 8.0 /*waves*/ * iters * (double)kCalAcc /*mfma*/ * 16384.0;
    *tflops = flops / (ms * 1e-3) / 1e12;
    *shader_mhz = (h[3] > h[1]) ? (double)(h[2] - h[0]) / ((double)(h[3] - h[1]) / 100.0) : 0.0;
    return FREEZE_OK;
}

int freeze_calibrate_hbm_read(const void *buffer, size_t bytes, double *gbytes_per_s)
{
    if (!buffer || !gbytes_per_s || bytes < (1u << 20) || (reinterpret_cast<uintptr_t>(buffer) % 16) != 0)
        return FREEZE_EINVAL;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return FREEZE_EHIP;
    const size_t n16 = bytes / 16;
    hipLaunchKernelGGL(read_kernel, dim3(2048), dim3(256), 0, nullptr, static_cast<const u32x4 *>(buffer), n16);
    (void)hipEventRecord(e0, nullptr);
    const int reps = 5;
    for (int i = 0; i < reps; ++i)
        hipLaunchKernelGGL(read_kernel, dim3(2048), dim3(256), 0, nullptr, static_cast<const u32x4 *>(buffer), n16);
    (void)hipEventRecord(e1, nullptr);
    float ms = 0.f;
    int rc = FREEZE_OK;
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = FREEZE_EHIP;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != FREEZE_OK) return rc;
    *gbytes_per_s = (double)(n16 * 16) * reps / (ms * 1e-3) / 1e9;
    return FREEZE_OK;
}

}  // extern "C"
