// sd_calib: plain copy / read kernels of known size, used to calibrate the HBM byte counters
// (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) and to measure what a long streaming kernel
// reaches on this machine.   usage: sd_calib copy|read|stream|ldsstream <MiB> [reps]
//   read:   every load instruction of the grid covers one contiguous span (waves interleaved)
//   stream: every wave walks its own contiguous region, 16 loads of 1 KiB in flight (the access
//           pattern of the weight and KV streams of the library)
//   ldsstream: the same per-wave streams as `stream` (256 workgroups of 4 waves), but every 1 KiB goes straight
//           from memory into a per-wave ring of four 8 KiB slots in LDS (global_load_lds_dwordx4) and is read
//           from there: the other way to stage K/V or weight tiles; 32 KiB in flight per wave, twice `stream`'s
// and what the ingredients of the weight-streaming GEMM cost beside the bare weight stream:
//   sd_calib parts <NB> <KB> [reps]   a projection with NB column blocks of 32 and KB contraction blocks of 16, in
//           the GEMM's launch shape and unit walk (256 workgroups of 8 waves, ring of 16 fragments per wave),
//           weights never touched before (a fresh region per launch): the stream alone, + the partial-tile
//           stores of a 64-row pass at every segment end, + the activation chunks (L2 -> registers -> LDS, a
//           barrier per chunk), + both. No arithmetic: the figures bound what the real kernel can reach.
//   sd_calib ratio [reps]             the weight stream of a 384 MiB matrix while every thread also reads x:w
//           times as many bytes from a 1 MiB buffer that stays in L2 (x:w = 0 .. 4): what an operand costs that
//           is shared by fewer waves
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

// ---- ldsstream ------------------------------------------------------------------------------------------------
static __device__ __forceinline__ void calib_lds_dma16(const u4* src_lane, uint32_t lds_byte_addr) {
    // lane i's 16 bytes land at lds_byte_addr + 16 * i; M0 (the LDS base of the load) is put back
    uint32_t saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0) : "s"(lds_byte_addr), "v"(src_lane) : "memory");
}
__global__ __launch_bounds__(256) void k_calib_ldsstream(const u4* __restrict__ src, size_t units_per_wave,
                                                         unsigned* __restrict__ sink) {
    constexpr int SLOTS = 4;                             // 8 KiB each
    __shared__ __attribute__((aligned(1024))) u4 lds[4 * SLOTS * 512];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const u4* q = src + ((size_t)blockIdx.x * 4 + wave) * units_per_wave + lane;
    const uint32_t base = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(__attribute__((address_space(3))) u4*)(lds + wave * SLOTS * 512));
    const int steps = (int)(units_per_wave / 512);       // 8 KiB per step
    if (steps < 1) return;
#pragma unroll
    for (int s = 0; s < SLOTS; ++s)
#pragma unroll
        for (int u = 0; u < 8; ++u)
            calib_lds_dma16(q + (size_t)(s < steps ? s : steps - 1) * 512 + u * 64, base + (s * 512 + u * 64) * 16);
    unsigned acc = 0;
    for (int i = 0; i < steps; i += SLOTS) {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            asm volatile("s_waitcnt vmcnt(%0)" :: "n"((SLOTS - 1) * 8) : "memory");      // slot s has landed
#pragma unroll
            for (int u = 0; u < 8; ++u) acc ^= lds[wave * SLOTS * 512 + s * 512 + u * 64 + lane].x;
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                            // read before it is refilled
            int nx = i + s + SLOTS;
            nx = nx < steps ? nx : steps - 1;
#pragma unroll
            for (int u = 0; u < 8; ++u) calib_lds_dma16(q + (size_t)nx * 512 + u * 64, base + (s * 512 + u * 64) * 16);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (acc == 0x9e3779b9u) sink[0] = 1;
}

// ---- parts ---------------------------------------------------------------------------------------------------
template <int STORES, int XCHUNKS>
__global__ __launch_bounds__(512) void k_calib_parts(const u4* __restrict__ w, int NB, int KB, const u4* __restrict__ x,
                                                     float* __restrict__ out, int ldo, size_t slot_stride, int nslots,
                                                     unsigned* __restrict__ sink) {
    __shared__ u4 xs[2][1024];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = blockIdx.x;
    const int U = NB / 8 * KB;                           // units: (column group of 8 blocks, contraction block)
    const int u0 = (int)((long long)g * U / 256), u1 = (int)((long long)(g + 1) * U / 256);
    auto addr = [&](int u) {                             // fragment of this wave in unit u ([kb][nb] layout)
        if (u >= u1) u = u1 - 1;
        const int ng = u / KB, kb = u - ng * KB;
        return w + ((size_t)kb * NB + ng * 8 + wave) * 64 + lane;
    };
    u4 ring[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) ring[i] = __builtin_nontemporal_load(addr(u0 + i));
    u4 acc = {0, 0, 0, 0};
    int slot = g % nslots;
    for (int u = u0; u < u1; u += 16) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            if (XCHUNKS) {                               // a chunk of 8 contraction blocks of a 64-row operand: 16 KiB
                const int kb = (u + c * 8) % KB;
                u4 a = x[(size_t)kb * 128 + tid], b = x[(size_t)kb * 128 + 512 + tid];
                xs[c][tid] = a;
                xs[c][512 + tid] = b;
                __syncthreads();
                acc ^= xs[c][(tid * 7) & 1023];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int i = c * 8 + j;
                acc ^= ring[i];
                ring[i] = __builtin_nontemporal_load(addr(u + 16 + i));
            }
        }
        const int ng_now = u / KB, ng_next = (u + 16 < u1) ? (u + 16) / KB : -1;
        if (STORES && ng_now != ng_next) {               // a segment ends: this wave's 64 x 32 floats, write-through
            float* o = out + (size_t)slot * slot_stride + (size_t)(ng_now * 8 + wave) * 32 + (lane & 31);
            const int gq = lane >> 5;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = mt * 32 + 8 * (v >> 2) + 4 * gq + (v & 3);
                    __hip_atomic_store(&o[(size_t)m * ldo], (float)(acc.x + v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            slot = 0;
        }
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = 1;
}

// ---- ratio ---------------------------------------------------------------------------------------------------
template <int XP>
__global__ __launch_bounds__(512) void k_calib_ratio(const u4* __restrict__ w, size_t frags_per_wave,
                                                     const u4* __restrict__ x, unsigned x_mask16,
                                                     unsigned* __restrict__ sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const u4* wp = w + ((size_t)blockIdx.x * 8 + wave) * frags_per_wave * 64 + lane;
    u4 ring[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) ring[i] = __builtin_nontemporal_load(wp + (size_t)i * 64);
    u4 acc = {0, 0, 0, 0};
    unsigned xo = (blockIdx.x * 977u + threadIdx.x) & x_mask16;
    for (size_t f = 16; f + 16 <= frags_per_wave; f += 16) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            acc ^= ring[i];
            ring[i] = __builtin_nontemporal_load(wp + (f + i) * 64);
#pragma unroll
            for (int p = 0; p < XP; ++p) {
                acc ^= x[xo];
                xo = (xo + 512) & x_mask16;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) acc ^= ring[i];
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = 1;
}

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)

static int run_parts(int NB, int KB, int reps) {
    if (NB < 8 || NB % 8 || KB < 16 || KB > 4096 || (size_t)NB * KB > (1u << 20)) {
        fprintf(stderr, "parts: NB must be a multiple of 8, 16 <= KB <= 4096, NB * KB <= 2^20\n");
        return 2;
    }
    const size_t bytes = (size_t)NB * KB * 1024, step = (bytes + (2u << 20)) & ~((size_t)(2u << 20) - 1);
    const size_t pool = step * (size_t)(reps + 2) < (12ull << 30) ? step * (size_t)(reps + 2) : (12ull << 30);
    const int nslots = 16, ldo = NB * 32;
    const size_t slot_stride = (size_t)64 * ldo;
    char *wbuf, *xbuf;
    float* out;
    unsigned* sink;
    CK(hipMalloc(&wbuf, pool)); CK(hipMalloc(&xbuf, 9u << 20)); CK(hipMalloc(&out, nslots * slot_stride * 4));
    CK(hipMalloc(&sink, 4));
    CK(hipMemset(wbuf, 1, pool)); CK(hipMemset(xbuf, 2, 9u << 20)); CK(hipMemset(out, 0, nslots * slot_stride * 4));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const char* names[4] = {"weight stream alone", "+ partial-tile stores", "+ activation chunks", "+ stores + chunks"};
    for (int var = 0; var < 4; ++var) {
        float sum = 0;
        size_t off = 0;
        for (int r = 0; r < reps + 2; ++r) {             // the first two launches warm up
            if (off + bytes > pool) off = 0;
            const u4* wp = (const u4*)(wbuf + off);
            CK(hipEventRecord(e0));
#define PARTS(S, X) hipLaunchKernelGGL((k_calib_parts<S, X>), dim3(256), dim3(512), 0, 0, wp, NB, KB, (const u4*)xbuf, out, ldo, slot_stride, nslots, sink)
            if (var == 0) PARTS(0, 0); else if (var == 1) PARTS(1, 0); else if (var == 2) PARTS(0, 1); else PARTS(1, 1);
#undef PARTS
            CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
            float ms;
            CK(hipEventElapsedTime(&ms, e0, e1));
            if (r >= 2) sum += ms;
            off += step;
        }
        const double us = sum / reps * 1e3;
        printf("parts NB=%d KB=%d (%.1f MB of weights) %-24s %7.1f us per launch between events, %5.0f GB/s\n", NB, KB,
               bytes / 1e6, names[var], us, bytes / us / 1e3);
    }
    return 0;
}

static int run_ratio(int reps) {
    const size_t frags = 192, W = 2048 * frags * 1024;   // 384 MiB over 2048 waves
    char *wbuf, *xbuf;
    unsigned* sink;
    CK(hipMalloc(&wbuf, W)); CK(hipMalloc(&xbuf, 1u << 20)); CK(hipMalloc(&sink, 4));
    CK(hipMemset(wbuf, 1, W)); CK(hipMemset(xbuf, 2, 1u << 20));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const unsigned mask = (1u << 20) / 16 - 1;
    for (int xp = 0; xp <= 4; ++xp) {
        float best = 1e30f;
        for (int r = 0; r < reps + 1; ++r) {
            CK(hipEventRecord(e0));
#define RATIO(N) hipLaunchKernelGGL(k_calib_ratio<N>, dim3(256), dim3(512), 0, 0, (const u4*)wbuf, frags, (const u4*)xbuf, mask, sink)
            if (xp == 0) RATIO(0); else if (xp == 1) RATIO(1); else if (xp == 2) RATIO(2); else if (xp == 3) RATIO(3); else RATIO(4);
#undef RATIO
            CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
            float ms;
            CK(hipEventElapsedTime(&ms, e0, e1));
            if (r && ms < best) best = ms;
        }
        printf("ratio x:w = %d:1   %7.1f us   weights %5.0f GB/s   operand from L2 %5.0f GB/s\n", xp, best * 1e3,
               W / best / 1e6, (double)W * xp / best / 1e6);
    }
    return 0;
}

int main(int argc, char** argv) {
    if (argc >= 4 && !strcmp(argv[1], "parts")) return run_parts(atoi(argv[2]), atoi(argv[3]), argc > 4 ? atoi(argv[4]) : 10);
    if (argc >= 2 && !strcmp(argv[1], "ratio")) return run_ratio(argc > 2 ? atoi(argv[2]) : 4);
    if (argc < 3) {
        fprintf(stderr, "usage: sd_calib copy|read|stream|ldsstream <MiB> [reps] | parts <NB> <KB> [reps] | ratio [reps]\n");
        return 2;
    }
    const bool copy = !strcmp(argv[1], "copy"), stream = !strcmp(argv[1], "stream"), ldsstream = !strcmp(argv[1], "ldsstream");
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
            else if (ldsstream) hipLaunchKernelGGL(k_calib_ldsstream, dim3(256), dim3(256), 0, 0, a, (n / 1024) & ~(size_t)1023, sink);
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
