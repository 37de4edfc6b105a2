// Two measured ceilings of the chip, for benchmarks (no part of the method): what a plain copy
// kernel moves through HBM and what a register-only loop of bf16 MFMAs sustains.  The published
// peaks (8 TB/s, 2.5 PFLOP/s) are what the benchmark prices against; these say how much of them
// simple code reaches on the machine at hand.
#include "mfma.h"

namespace moba {

__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                   int64_t n16)
{
    // four 16-byte loads in flight per lane
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}

// eight independent accumulation chains per wave, operands never change: nothing but MFMA issue
__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, float* sink)
{
    Frag a, b;
#pragma unroll
    for (int i = 0; i < 4; ++i) { a.u[i] = 0x3c003c00u + threadIdx.x; b.u[i] = 0x3c003c00u + i; }
    f32x4_t acc[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] = mfma16(a, b, acc[c]);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) s += acc[c][0] + acc[c][1] + acc[c][2] + acc[c][3];
    if (s == 12345.678f) sink[threadIdx.x] = s;         // never true for these operands; keeps the loop
}

}  // namespace moba

using namespace moba;

extern "C" {

int moba_microbench_copy(void* dst, const void* src, size_t bytes, int reps, float* ms, void* stream)
{
    if (!dst || !src || !ms || reps <= 0 || bytes < 16 || (bytes & 15)) return MOBA_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return MOBA_EHIP;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return MOBA_EHIP;}
    const int64_t n16 = (int64_t)(bytes / 16);
    const unsigned grid = 256 * 16;                        // 16 workgroups per CU, grid-stride
    hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, n16);   // warm-up
    (void)hipEventRecord(e0, st);
    for (int r = 0; r < reps; ++r)
        hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, n16);
    (void)hipEventRecord(e1, st);
    hipError_t e = hipEventSynchronize(e1);
    float t = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&t, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return MOBA_EHIP;
    *ms = t / reps;
    return MOBA_OK;
}

int moba_microbench_mfma(int waves_per_simd, int iters, void* sink, float* ms, double* flop, void* stream)
{
    if (!sink || !ms || !flop || waves_per_simd <= 0 || waves_per_simd > 8 || iters <= 0) return MOBA_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return MOBA_EHIP;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return MOBA_EHIP;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return MOBA_EHIP;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return MOBA_EHIP; }
    const unsigned grid = (unsigned)(cus * waves_per_simd);    // 4 waves per workgroup: one per SIMD
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(grid), dim3(256), 0, st, 64, (float*)sink);      // warm-up
    (void)hipEventRecord(e0, st);
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(grid), dim3(256), 0, st, iters, (float*)sink);
    (void)hipEventRecord(e1, st);
    hipError_t e = hipEventSynchronize(e1);
    float t = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&t, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return MOBA_EHIP;
    *ms = t;
    *flop = (double)grid * 4.0 * (double)iters * 8.0 * (2.0 * 16 * 16 * 32);
    return MOBA_OK;
}

}  // extern "C"
