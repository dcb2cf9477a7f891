// hbm_probe: plain copy and read kernels of known size and a plain arithmetic kernel of known instruction count,
// timed with HIP events.
// Two uses: (1) the practical HBM ceiling of this GPU, to put the row sweep's GB/s in context;
// (2) a reference dispatch of known byte count for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE
// counters (run it under `rocprofv3 --pmc FETCH_SIZE` and compare with the bytes printed here);
// (3) the vector-ALU issue rate this GPU sustains, the practical ceiling for the one ALU-bound kernel.
//
// Measurement tool, not part of the library: build with
//   hipcc -O3 -std=c++17 --offload-arch=gfx950 -o tests/hbm_probe tests/hbm_probe.hip
// usage: tests/hbm_probe [MiB per buffer = 2048] [repeats = 10]
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#define CHECK(x)                                                                         \
    do {                                                                                 \
        hipError_t e_ = (x);                                                             \
        if (e_ != hipSuccess) {                                                          \
            fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));               \
            return 1;                                                                    \
        }                                                                                \
    } while (0)

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void probe_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4* __restrict__ src, unsigned* __restrict__ sink, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    unsigned acc = 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const u32x4 v = src[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x12345678u) sink[0] = acc;  // practically never: keeps the loads alive
}

// the same read with non-temporal loads (the form the row sweep uses for data it reads once)
__global__ __launch_bounds__(256) void probe_read_nt_kernel(const u32x4* __restrict__ src, unsigned* __restrict__ sink, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    unsigned acc = 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const u32x4 v = __builtin_nontemporal_load(src + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x12345678u) sink[0] = acc;
}

// Vector-ALU issue rate: every lane runs `iters` rounds of 16 independent fused multiply-adds (full-rate fp32
// instructions, no memory access).  wave instructions = waves x iters x 16.
__global__ __launch_bounds__(256) void probe_valu_kernel(float* sink, int iters, float seed)
{
    float a[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) a[i] = seed + (float)(threadIdx.x + i);
    const float m = 1.0000001f, c = 1e-7f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) a[i] = __builtin_fmaf(a[i], m, c);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += a[i];
    if (s == 12345.678f) sink[0] = s;   // practically never: keeps the arithmetic alive
}

int main(int argc, char** argv)
{
    const size_t mib = argc > 1 ? (size_t)atoll(argv[1]) : 2048;
    const int reps = argc > 2 ? atoi(argv[2]) : 10;
    const size_t bytes = mib << 20, n = bytes / 16;
    u32x4 *a = nullptr, *b = nullptr;
    unsigned* sink = nullptr;
    CHECK(hipMalloc(&a, bytes));
    CHECK(hipMalloc(&b, bytes));
    CHECK(hipMalloc(&sink, 4));
    CHECK(hipMemset(a, 1, bytes));
    CHECK(hipMemset(b, 2, bytes));
    hipDeviceProp_t prop;
    CHECK(hipGetDeviceProperties(&prop, 0));
    const int grid = prop.multiProcessorCount * 16;
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    printf("device %s, %d CUs, LDS/block %zu B, buffer %zu MiB, %d repeats\n", prop.name, prop.multiProcessorCount,
           (size_t)prop.sharedMemPerBlock, mib, reps);
    float ms = 0.f;
    hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(256), 0, 0, a, b, n);
    CHECK(hipEventRecord(e0));
    for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(256), 0, 0, a, b, n);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    printf("copy: %zu B read + %zu B written per launch, %.1f us, %.1f GB/s (read+write)\n", bytes, bytes,
           ms * 1e3 / reps, 2.0 * bytes / (ms * 1e-3 / reps) / 1e9);
    hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(256), 0, 0, a, sink, n);
    CHECK(hipEventRecord(e0));
    for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(256), 0, 0, a, sink, n);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    printf("read: %zu B read per launch, %.1f us, %.1f GB/s\n", bytes, ms * 1e3 / reps, bytes / (ms * 1e-3 / reps) / 1e9);
    hipLaunchKernelGGL(probe_read_nt_kernel, dim3(grid), dim3(256), 0, 0, a, sink, n);
    CHECK(hipEventRecord(e0));
    for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(probe_read_nt_kernel, dim3(grid), dim3(256), 0, 0, a, sink, n);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    printf("read, non-temporal loads: %zu B read per launch, %.1f us, %.1f GB/s\n", bytes, ms * 1e3 / reps,
           bytes / (ms * 1e-3 / reps) / 1e9);
    {   // vector-ALU issue rate with every SIMD holding 8 waves
        const int iters = 4096, wgs = prop.multiProcessorCount * 8;
        hipLaunchKernelGGL(probe_valu_kernel, dim3(wgs), dim3(256), 0, 0, (float*)sink, iters, 1.0f);
        CHECK(hipEventRecord(e0));
        for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(probe_valu_kernel, dim3(wgs), dim3(256), 0, 0, (float*)sink, iters, 1.0f);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        const double insts = (double)wgs * 4.0 * iters * 16.0;
        printf("valu: %.0f wave instructions (fma) per launch, %.1f us, %.1f G wave instructions/s = %.1f TFLOP/s fp32\n", insts,
               ms * 1e3 / reps, insts / (ms * 1e-3 / reps) / 1e9, insts * 128.0 / (ms * 1e-3 / reps) / 1e12);
    }
    CHECK(hipDeviceSynchronize());
    return 0;
}
