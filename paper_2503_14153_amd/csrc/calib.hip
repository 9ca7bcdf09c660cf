// sd_calib: plain copy / read kernels of known size, used to calibrate the HBM byte counters
// (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) and to measure what a long streaming kernel
// reaches on this machine.   usage: sd_calib copy|read|stream <MiB> [reps]
//   read:   every load instruction of the grid covers one contiguous span (waves interleaved)
//   stream: every wave walks its own contiguous region, 16 loads of 1 KiB in flight (the access
//           pattern of the weight and KV streams of the library)
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstring>

typedef __attribute__((ext_vector_type(4))) unsigned u4;

__global__ void k_calib_copy(const u4* __restrict__ src, u4* __restrict__ dst, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = src[i];
}

// every wave keeps eight 1 KiB loads in flight
__global__ void k_calib_read(const u4* __restrict__ src, size_t n, unsigned* __restrict__ sink) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
    u4 acc = {0, 0, 0, 0};
    for (; i + 7 * stride < n; i += 8 * stride) {
        u4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = 1;
}

// every wave streams its own contiguous region with sixteen 1 KiB loads in flight
__global__ void k_calib_stream(const u4* __restrict__ src, size_t units_per_wave, unsigned* __restrict__ sink) {
    const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const u4* q = src + wave * units_per_wave + (threadIdx.x & 63);
    u4 acc = {0, 0, 0, 0};
    for (size_t i = 0; i + 15 * 64 < units_per_wave; i += 16 * 64) {
        u4 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = __builtin_nontemporal_load(q + i + u * 64);
#pragma unroll
        for (int u = 0; u < 16; ++u) acc ^= v[u];
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = 1;
}

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)

int main(int argc, char** argv) {
    if (argc < 3) { fprintf(stderr, "usage: sd_calib copy|read|stream <MiB> [reps]\n"); return 2; }
    const bool copy = !strcmp(argv[1], "copy"), stream = !strcmp(argv[1], "stream");
    const size_t bytes = (size_t)atol(argv[2]) << 20, n = bytes / 16;
    const int reps = argc > 3 ? atoi(argv[3]) : 5;
    u4 *a, *b;
    unsigned* sink;
    CK(hipMalloc(&a, bytes)); CK(hipMalloc(&b, copy ? bytes : 16)); CK(hipMalloc(&sink, 4));
    CK(hipMemset(a, 1, bytes));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const int blocks = copy ? 4096 : 1024;
    for (int pass = 0; pass < 2; ++pass) {               // pass 0 warms up
        CK(hipEventRecord(e0));
        for (int r = 0; r < reps; ++r) {
            if (copy) hipLaunchKernelGGL(k_calib_copy, dim3(blocks), dim3(256), 0, 0, a, b, n);
            else if (stream) hipLaunchKernelGGL(k_calib_stream, dim3(256), dim3(256), 0, 0, a, (n / 1024) & ~(size_t)1023, sink);
            else hipLaunchKernelGGL(k_calib_read, dim3(blocks), dim3(256), 0, 0, a, n, sink);
        }
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    }
    float ms = 0;
    CK(hipEventElapsedTime(&ms, e0, e1));
    const double moved = (copy ? 2.0 : 1.0) * bytes * reps;
    printf("%s %zu MiB x %d: %.1f us per launch, %.0f GB/s (%s bytes)\n", argv[1], bytes >> 20, reps,
           ms * 1e3 / reps, moved / ms / 1e6, copy ? "read + written" : "read");
    return 0;
}
