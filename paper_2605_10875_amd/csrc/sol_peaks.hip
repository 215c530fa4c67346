// Two microbenchmarks that measure what this GPU actually reaches on the two rooflines the path is priced against:
// a register-only bf16 MFMA loop (no memory traffic at all) and a plain device-to-device copy. The benchmark prints
// them beside the published peaks; nothing on the product path calls them.
#include "../../include/sol.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// Every wave issues `iters` rounds of eight independent 32x32x16 bf16 MFMAs on registers (eight accumulators, so a
// result is never waited for); the sums are stored once at the end so the loop cannot be dropped.
__global__ __launch_bounds__(256) void k_peak_mfma(float *out, int iters)
{
    const uint32_t lane = threadIdx.x;
    const u32x4_t au = {0x3f803f80u + lane, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};      // bf16 ones (and a lane mark)
    const u32x4_t bu = {0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
    const bf16x8_t a = __builtin_bit_cast(bf16x8_t, au), b = __builtin_bit_cast(bf16x8_t, bu);
    f32x16_t acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[j][r];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// dst[i] = src[i], 16 bytes per lane and step, grid-stride
__global__ __launch_bounds__(256) void k_peak_copy(const u32x4_t *__restrict__ src, u32x4_t *__restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        dst[i] = __builtin_nontemporal_load(src + i);
}

// read-only: four independent 16-byte loads per lane and step, folded into one word that is stored at the end
__global__ __launch_bounds__(256) void k_peak_read(const u32x4_t *__restrict__ src, uint32_t *__restrict__ out, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const size_t n4 = n16 / (4 * stride) * (4 * stride);
    u32x4_t acc = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += 4 * stride) {
        const u32x4_t a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride);
        const u32x4_t c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
        acc ^= a ^ b ^ c ^ d;
    }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

}  // namespace

extern "C" int sol_measure_peaks(void *scratch, size_t scratch_bytes, int reps, float *mfma_tflops_out, float *copy_gbs_out,
                                 float *read_gbs_out, void *stream)
{
    if (!scratch || !mfma_tflops_out || !copy_gbs_out || !read_gbs_out || reps <= 0) return SOL_ERR_INVALID_ARG;
    if (scratch_bytes < ((size_t)64 << 20)) return SOL_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return SOL_ERR_HIP;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return SOL_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return SOL_ERR_HIP; }
    int rc = SOL_OK;
    float ms = 0.f;
    // MFMA: two workgroups of four waves per CU (two waves per SIMD), 4096 rounds of 8 MFMAs of 32 * 32 * 16 * 2 flops
    const int blocks = 2 * cus, iters = 4096;
    hipLaunchKernelGGL(k_peak_mfma, dim3(blocks), dim3(256), 0, st, (float *)scratch, 64);      // warm-up
    (void)hipEventRecord(e0, st);
    for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(k_peak_mfma, dim3(blocks), dim3(256), 0, st, (float *)scratch, iters);
    (void)hipEventRecord(e1, st);
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = SOL_ERR_HIP;
    const double flops = (double)reps * blocks * 4.0 * iters * 8.0 * (32.0 * 32.0 * 16.0 * 2.0);
    *mfma_tflops_out = rc ? 0.f : (float)(flops / (ms * 1e-3) / 1e12);
    // copy: half of the scratch into the other half (read + written bytes counted)
    const size_t half = (scratch_bytes / 2) & ~(size_t)255, n16 = half / 16;
    const u32x4_t *src = (const u32x4_t *)scratch;
    u32x4_t *dst = (u32x4_t *)((char *)scratch + half);
    const int cblocks = cus * 16;
    hipLaunchKernelGGL(k_peak_copy, dim3(cblocks), dim3(256), 0, st, src, dst, n16);            // warm-up
    (void)hipEventRecord(e0, st);
    for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(k_peak_copy, dim3(cblocks), dim3(256), 0, st, src, dst, n16);
    (void)hipEventRecord(e1, st);
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = SOL_ERR_HIP;
    *copy_gbs_out = rc ? 0.f : (float)(2.0 * half * reps / (ms * 1e-3) / 1e9);
    // read: the first half of the scratch, results into the start of the second half
    const int rblocks = cus * 8;
    const size_t rstride = (size_t)rblocks * 256, rbytes = n16 / (4 * rstride) * (4 * rstride) * 16;
    hipLaunchKernelGGL(k_peak_read, dim3(rblocks), dim3(256), 0, st, src, (uint32_t *)dst, n16);   // warm-up
    (void)hipEventRecord(e0, st);
    for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(k_peak_read, dim3(rblocks), dim3(256), 0, st, src, (uint32_t *)dst, n16);
    (void)hipEventRecord(e1, st);
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = SOL_ERR_HIP;
    *read_gbs_out = rc ? 0.f : (float)((double)rbytes * reps / (ms * 1e-3) / 1e9);
    if (hipGetLastError() != hipSuccess) rc = SOL_ERR_HIP;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}
