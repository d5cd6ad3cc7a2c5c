// Practical-ceiling probes: what this GPU sustains on a plain device-to-device copy and on a
// back-to-back bf16 MFMA issue loop, measured with HIP events.  The benchmark prices its
// kernels against the published peaks and reports these beside them.
#include <hip/hip_runtime.h>

#include "common.hpp"

namespace rpo {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void probe_copy_kernel(const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst,
                                                         size_t n_vec) {
    for (size_t i = blockIdx.x * (size_t)256 + threadIdx.x; i < n_vec; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// Eight independent 32x32x16 accumulations per wave, operands that differ per lane and change
// every iteration (constant operands would flatter the clock the chip sustains).
__global__ __launch_bounds__(256) void probe_mfma_kernel(float* __restrict__ out, int iters) {
    bf16x8_t a, b;
    unsigned h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        h = h * 1664525u + 1013904223u;
        a[j] = (__bf16)((float)((int)(h >> 16 & 0xff) - 128) * (1.0f / 128.0f));
        h = h * 1664525u + 1013904223u;
        b[j] = (__bf16)((float)((int)(h >> 16 & 0xff) - 128) * (1.0f / 128.0f));
    }
    f32x16_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
        // rotate the operands' elements so that the inputs toggle like real data
        const __bf16 t = a[0];
#pragma unroll
        for (int j = 0; j < 7; ++j) a[j] = a[j + 1];
        a[7] = b[0];
#pragma unroll
        for (int j = 0; j < 7; ++j) b[j] = b[j + 1];
        b[7] = t;
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// reps timed launches after one warm-up; returns the best launch's rate
hipError_t probe_copy(const void* src, void* dst, size_t bytes, int reps, double* gbps, hipStream_t s) {
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&e1);
    if (e != hipSuccess) return e;
    const size_t n_vec = bytes / 16;
    float best = 0.f;
    for (int r = 0; r <= reps; ++r) {
        (void)hipEventRecord(e0, s);
        probe_copy_kernel<<<4096, 256, 0, s>>>((const u32x4_t*)src, (u32x4_t*)dst, n_vec);
        (void)hipEventRecord(e1, s);
        e = hipEventSynchronize(e1);
        if (e != hipSuccess) break;
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        if (r > 0 && (best == 0.f || ms < best)) best = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e == hipSuccess) e = hipGetLastError();
    *gbps = best > 0.f ? 2.0 * (double)(n_vec * 16) / (best * 1e-3) / 1e9 : 0.0;  // read + write
    return e;
}

// scratch: 512 * 256 floats.  512 workgroups of 4 waves (two per CU), `iters` x 8 MFMAs per wave.
hipError_t probe_mfma(float* scratch, int iters, int reps, double* tflops, hipStream_t s) {
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&e1);
    if (e != hipSuccess) return e;
    const int wgs = 512;
    float best = 0.f;
    for (int r = 0; r <= reps; ++r) {
        (void)hipEventRecord(e0, s);
        probe_mfma_kernel<<<wgs, 256, 0, s>>>(scratch, iters);
        (void)hipEventRecord(e1, s);
        e = hipEventSynchronize(e1);
        if (e != hipSuccess) break;
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        if (r > 0 && (best == 0.f || ms < best)) best = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e == hipSuccess) e = hipGetLastError();
    *tflops = best > 0.f ? (double)wgs * 4 * iters * 8 * 32768.0 / (best * 1e-3) / 1e12 : 0.0;
    return e;
}

}  // namespace rpo
