// Weight-streaming GEMM for the verifying forward pass: out[m][n] = sum_k X[m][k] * W[n][k].
//
// The tree has T <= 256 rows, so every projection of the step (QKV, O, gate/up, down, LM
// head, draft heads) multiplies a few 32-row blocks of activations by a weight matrix that is
// read exactly once: the kernel is bound by the HBM read of W, not by the matrix cores. The
// design therefore (1) stores W pre-tiled so each wave streams one contiguous run of 1 KiB
// MFMA fragments with 16-byte-per-lane loads, (2) keeps many such loads in flight per wave
// (a chunk of KC fragments is fetched while the previous chunk is multiplied), (3) shares the
// small activation operand between the waves of a workgroup through LDS, and (4) splits the
// contraction across workgroups when N alone gives too few workgroups for 256 CUs; the
// consumer kernel sums the split partial results (deterministic, no atomics).
//
// Precision: the weights are bf16 by definition, the activations are not. Since the matrix
// cores idle most of the time in an HBM-bound kernel, each activation enters as a two-term
// bf16 expansion x = hi + lo (two MFMAs per weight fragment), which keeps ~16 mantissa bits
// of x and makes the product exact up to fp32 accumulation.
#include "sd_internal.h"

// ------------------------------------------------------------------------------------------
// Re-tile a row-major bf16 matrix W[N][K] into fragment order (see sd_internal.h).
__global__ void k_pack_weight(const uint4* __restrict__ src, uint4* __restrict__ dst, int N, int K,
                              int nb_offset, int KB, int NBsrc) {
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // one 16-byte piece each
    size_t total = (size_t)NBsrc * KB * 64;
    if (idx >= total) return;
    int lane = (int)(idx & 63);
    size_t t = idx >> 6;
    int kb = (int)(t % KB);
    int nb = (int)(t / KB);
    int n = nb * 32 + (lane & 31);
    int k0 = kb * 16 + (lane >> 5) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (n < N) v = src[((size_t)n * K + k0) >> 3];
    dst[((size_t)(nb + nb_offset) * KB + kb) * 64 + lane] = v;
}

void launch_pack_weight(const void* src, void* dst, int N, int K, int nb_offset, int KB, hipStream_t s) {
    int NBsrc = (N + 31) / 32;
    size_t total = (size_t)NBsrc * KB * 64;
    int threads = 256;
    unsigned blocks = (unsigned)((total + threads - 1) / threads);
    hipLaunchKernelGGL(k_pack_weight, dim3(blocks), dim3(threads), 0, s, (const uint4*)src, (uint4*)dst, N, K,
                       nb_offset, KB, NBsrc);
}

// ------------------------------------------------------------------------------------------
// MT  = number of 32-row activation blocks (all of them: W is read once for every row)
// KC  = fragments (16 contraction elements each) per pipeline chunk
// NW  = waves per workgroup; wave w owns output columns [32*(NW*blockIdx.x + w), +32)
template <int MT, int KC, int NW>
__global__ __launch_bounds__(NW * 64) void k_gemm_stream(const bf16x8* __restrict__ Xp,
                                                          const bf16x8* __restrict__ Wp,
                                                          float* __restrict__ out, int KB, int NB, int ldo,
                                                          int chunks_per_split, size_t split_stride) {
    constexpr int XF = KC * MT * 2;                  // X fragments per chunk (hi and lo parts)
    constexpr int XR = (XF * 64) / (NW * 64);        // 16-byte pieces of X per thread per chunk
    static_assert(XF % NW == 0, "chunk must divide evenly over the workgroup");
    __shared__ bf16x8 xs[2][XF * 64];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    int nb = blockIdx.x * NW + wave;
    const bool owns = nb < NB;
    if (!owns) nb = NB - 1;                           // keep the wave in the barriers
    const int nchunks = (KB + KC - 1) / KC;
    const int c0 = blockIdx.y * chunks_per_split;
    int c1 = c0 + chunks_per_split;
    if (c1 > nchunks) c1 = nchunks;

    const bf16x8* wrow = Wp + (size_t)nb * KB * 64 + lane;
    f32x16 acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    bf16x8 wA[KC], wB[KC], xr[XR];
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};

    auto load_w = [&](bf16x8(&w)[KC], int c) {
#pragma unroll
        for (int kk = 0; kk < KC; ++kk) {
            int kb = c * KC + kk;
            w[kk] = (kb < KB) ? __builtin_nontemporal_load(wrow + (size_t)kb * 64) : zero;
        }
    };
    auto load_x = [&](int c) {
        const bf16x8* base = Xp + (size_t)c * XF * 64;
        const int limit = (KB - c * KC) * MT * 2 * 64;   // pieces that exist in this chunk
#pragma unroll
        for (int r = 0; r < XR; ++r) {
            int i = r * (NW * 64) + tid;
            xr[r] = (i < limit) ? base[i] : zero;
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int r = 0; r < XR; ++r) xs[buf][r * (NW * 64) + tid] = xr[r];
    };
    auto compute = [&](const bf16x8(&w)[KC], int buf) {
#pragma unroll
        for (int kk = 0; kk < KC; ++kk)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                bf16x8 hi = xs[buf][((kk * MT + mt) * 2) * 64 + lane];
                bf16x8 lo = xs[buf][((kk * MT + mt) * 2 + 1) * 64 + lane];
                acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi, w[kk], acc[mt], 0, 0, 0);
                acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo, w[kk], acc[mt], 0, 0, 0);
            }
    };

    if (c0 < c1) {
        load_w(wA, c0);
        load_x(c0);
        store_x(0);
        __syncthreads();
        for (int c = c0; c < c1; c += 2) {
            const bool more1 = c + 1 < c1;
            if (more1) { load_w(wB, c + 1); load_x(c + 1); }
            compute(wA, 0);
            if (more1) store_x(1);
            __syncthreads();
            if (!more1) break;
            const bool more2 = c + 2 < c1;
            if (more2) { load_w(wA, c + 2); load_x(c + 2); }
            compute(wB, 1);
            if (more2) store_x(0);
            __syncthreads();
        }
    }

    if (!owns) return;
    float* o = out + (size_t)blockIdx.y * split_stride + (size_t)nb * 32 + (lane & 31);
    const int g = lane >> 5;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int m = mt * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
            o[(size_t)m * ldo] = acc[mt][v];
        }
}

// How many ways to split the contraction so that the launch has enough workgroups.
int gemm_choose_split(int MB, int KB, int NB) {
    const int NW = 4;
    int KC = 16 / MB; if (KC < 2) KC = 2;
    int groups = (NB + NW - 1) / NW;
    int nchunks = (KB + KC - 1) / KC;
    int split = 1;
    // aim for >= 2 workgroups per CU (512) while keeping each slice >= 256 contraction elements
    while (groups * split < 512 && split < 16 && nchunks / (split * 2) * KC * 16 >= 256) split *= 2;
    if (split > nchunks) split = nchunks;
    return split < 1 ? 1 : split;
}

template <int MT, int KC>
static void launch_gemm_t(const void* Xp, const void* Wp, float* out, int KB, int NB, int ldo, int nsplit,
                          size_t split_stride, hipStream_t s) {
    constexpr int NW = 4;
    int groups = (NB + NW - 1) / NW;
    int nchunks = (KB + KC - 1) / KC;
    int cps = (nchunks + nsplit - 1) / nsplit;
    hipLaunchKernelGGL((k_gemm_stream<MT, KC, NW>), dim3(groups, nsplit), dim3(NW * 64), 0, s,
                       (const bf16x8*)Xp, (const bf16x8*)Wp, out, KB, NB, ldo, cps, split_stride);
}

void launch_gemm(const void* Xp, const void* Wp, float* out, int MB, int KB, int NB, int ldo, int nsplit,
                 size_t split_stride, hipStream_t s) {
    switch (MB) {
        case 1: launch_gemm_t<1, 16>(Xp, Wp, out, KB, NB, ldo, nsplit, split_stride, s); break;
        case 2: launch_gemm_t<2, 8>(Xp, Wp, out, KB, NB, ldo, nsplit, split_stride, s); break;
        case 4: launch_gemm_t<4, 4>(Xp, Wp, out, KB, NB, ldo, nsplit, split_stride, s); break;
        case 8: launch_gemm_t<8, 2>(Xp, Wp, out, KB, NB, ldo, nsplit, split_stride, s); break;
        default: break;   // validated by the caller: MB in {1,2,4,8}
    }
}
