// Micro-benchmarks of the three machine rates the kernels are measured against (csrk_microbench in include/csrk.h):
// device-to-device copy (HBM), a loop of independent plain FP32 multiply-adds acc += x * y (vector ALU without packed
// FP32),
// and a loop of conflict-free 128-bit LDS reads with 16 wavefronts per CU (the tiled kernels' launch shape).
// They follow the paper's practice of quoting its kernels against measured device peaks (section "Performance
// Analysis": the roofline's ceilings are what the profiler measured on the device, not datasheet figures).
#include "../../include/csrk.h"

#include <hip/hip_runtime.h>

#include <cstdio>

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void copy_kernel(const f32x4 *__restrict__ src, f32x4 *__restrict__ dst, size_t n) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

// 32 independent accumulators per lane, each the target of a multiply-add whose two factors are run-time values
// (acc += x * y, the form the kernels' inner loops have: the accumulator is both addend and result, which the
// hardware encodes in the short two-operand multiply-add); the factors change from round to round so that nothing
// folds.  2 * 32 * iters flops per lane.
__global__ __launch_bounds__(256) void fma_kernel(float *out, int iters, float scale, float addend) {
    float acc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = (float)(threadIdx.x + i);
    float x = scale, y = addend;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 32; ++i) acc[i] = fmaf(x, y, acc[i]);
        x = -x;
        y += 1e-3f;
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 32; ++i) s += acc[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Every wavefront reads rows of 2 KB (64 lanes x two 128-bit reads, the layout of the 512-column tiled kernels) at
// changing row offsets of a 128 KB LDS tile, 8 reads in flight per lane; nothing else happens.  The reads are
// volatile asm so that none is dropped or merged; the waits are written out because the compiler does not count
// LDS operations it did not issue itself.
__global__ __launch_bounds__(1024) void lds_read_kernel(float *out, int iters) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    constexpr int kRows = 64;
    for (int i = threadIdx.x; i < kRows * 512; i += blockDim.x) lds[i] = 1e-6f * (float)i;
    __syncthreads();
    const unsigned lane_b = (threadIdx.x & 63) * 16u;
    const unsigned wave = threadIdx.x >> 6;
    f32x4 c[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) c[u] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const unsigned row = (unsigned)__builtin_amdgcn_readfirstlane((int)((wave * 7 + blockIdx.x + u * 13 + it * 5) & (kRows - 1)));
            const unsigned addr = lane_b + row * 2048u;
            asm volatile("ds_read_b128 %0, %1" : "=v"(c[2 * u]) : "v"(addr));
            asm volatile("ds_read_b128 %0, %1 offset:1024" : "=v"(c[2 * u + 1]) : "v"(addr));
        }
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(c[0]), "+v"(c[1]), "+v"(c[2]), "+v"(c[3]), "+v"(c[4]), "+v"(c[5]), "+v"(c[6]), "+v"(c[7]));
    }
    f32x4 t = c[0];
#pragma unroll
    for (int u = 1; u < 8; ++u) t += c[u];
    out[blockIdx.x * blockDim.x + threadIdx.x] = t.x + t.y + t.z + t.w;
}

template <typename F>
hipError_t best_of(int reps, float *best_ms, F launch) {
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&e1);
    if (e != hipSuccess) {
        (void)hipEventDestroy(e0);
        return e;
    }
    launch();
    e = hipDeviceSynchronize();
    *best_ms = 1e30f;
    for (int i = 0; i < reps && e == hipSuccess; ++i) {
        (void)hipEventRecord(e0, 0);
        launch();
        (void)hipEventRecord(e1, 0);
        e = hipEventSynchronize(e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e == hipSuccess && ms < *best_ms) *best_ms = ms;
    }
    if (e == hipSuccess) e = hipGetLastError();
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return e;
}

}  // namespace

extern "C" csrk_status csrk_microbench(int kind, double *value) {
    if (!value) return CSRK_INVALID_ARG;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return CSRK_HIP_ERROR;
    float ms = 0.f;
    hipError_t e = hipSuccess;
    if (kind == CSRK_BENCH_HBM_COPY) {
        const size_t bytes = size_t(1) << 30;
        f32x4 *src = nullptr, *dst = nullptr;
        if (hipMalloc((void **)&src, bytes) != hipSuccess) return CSRK_WORKSPACE;
        if (hipMalloc((void **)&dst, bytes) != hipSuccess) {
            (void)hipFree(src);
            return CSRK_WORKSPACE;
        }
        e = hipMemset(src, 1, bytes);
        if (e == hipSuccess)
            e = best_of(5, &ms, [&] { hipLaunchKernelGGL(copy_kernel, dim3(cus * 16), dim3(256), 0, 0, src, dst, bytes / 16); });
        (void)hipFree(src);
        (void)hipFree(dst);
        if (e != hipSuccess) return CSRK_HIP_ERROR;
        *value = 2.0 * (double)bytes / (ms * 1e-3) / 1e9;          // GB/s, bytes read + bytes written
        return CSRK_OK;
    }
    float *out = nullptr;
    if (hipMalloc((void **)&out, (size_t)cus * 8 * 1024 * sizeof(float)) != hipSuccess) return CSRK_WORKSPACE;
    if (kind == CSRK_BENCH_FMA_F32) {
        const int iters = 4000, blocks = cus * 8;
        e = best_of(5, &ms, [&] { hipLaunchKernelGGL(fma_kernel, dim3(blocks), dim3(256), 0, 0, out, iters, 1.0001f, 0.5f); });
        *value = 2.0 * 32.0 * iters * (double)blocks * 256.0 / (ms * 1e-3) / 1e12;       // TFLOP/s
    } else if (kind == CSRK_BENCH_LDS_READ) {
        const int iters = 2000, lds_bytes = 64 * 2048;
        e = hipFuncSetAttribute((const void *)lds_read_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e == hipSuccess)
            e = best_of(5, &ms, [&] { hipLaunchKernelGGL(lds_read_kernel, dim3(cus), dim3(1024), lds_bytes, 0, out, iters); });
        *value = (double)cus * 1024.0 * iters * 8.0 * 16.0 / (ms * 1e-3) / 1e12;          // TB/s
    } else {
        (void)hipFree(out);
        return CSRK_INVALID_ARG;
    }
    (void)hipFree(out);
    return e == hipSuccess ? CSRK_OK : CSRK_HIP_ERROR;
}
