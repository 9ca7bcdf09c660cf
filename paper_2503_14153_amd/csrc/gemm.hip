// Weight-streaming GEMM for the verifying forward pass: out[m][n] = sum_k X[m][k] * W[n][k].
//
// The tree has T <= 256 rows, so every projection of the step (QKV, O, gate/up, down, LM
// head, draft heads) multiplies a few 32-row blocks of activations by a weight matrix that is
// read exactly once: the kernel is bound by the HBM read of W, not by the matrix cores. The
// design therefore (1) stores W pre-tiled as 1 KiB MFMA fragments, contraction-block-major
// ([kb][nb]): a wave fetches a fragment with one 16-byte-per-lane load, and at any moment the
// waves of the whole grid read one contiguous region of HBM, (2) keeps a ring of such loads in
// flight per wave, refilled as it is consumed, (3) shares the small activation operand between
// the waves of a workgroup through LDS, and (4) splits the contraction across workgroups so
// that every one of 256 CUs streams the same number of weight bytes; the consumer kernel sums
// the split partial results (deterministic, no atomics).
//
// Precision: the weights are bf16 by definition, the activations are not. Since the matrix
// cores idle most of the time in an HBM-bound kernel, each activation enters as a two-term
// bf16 expansion x = hi + lo (two MFMAs per weight fragment), which keeps ~16 mantissa bits
// of x and makes the product exact up to fp32 accumulation.
#include "sd_internal.h"
#include "sk_gemm.h"

// ------------------------------------------------------------------------------------------
// Re-tile a row-major bf16 matrix W[N][K] into fragment order (see sd_internal.h).
__global__ void k_pack_weight(const uint4* __restrict__ src, uint4* __restrict__ dst, int N, int K,
                              int nb_offset, int KB, int NBsrc, int NBdst) {
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
    dst[((size_t)kb * NBdst + nb + nb_offset) * 64 + lane] = v;
}

void launch_pack_weight(const void* src, void* dst, int N, int K, int nb_offset, int NBdst, int KB, hipStream_t s) {
    int NBsrc = (N + 31) / 32;
    size_t total = (size_t)NBsrc * KB * 64;
    int threads = 256;
    unsigned blocks = (unsigned)((total + threads - 1) / threads);
    hipLaunchKernelGGL(k_pack_weight, dim3(blocks), dim3(threads), 0, s, (const uint4*)src, (uint4*)dst, N, K,
                       nb_offset, KB, NBsrc, NBdst);
}

// ------------------------------------------------------------------------------------------
// Balanced streaming ("stream-K") over MT = 1, 2 or 8 row blocks of 32 rows (this kernel) or four (the
// kernel after it).
//
// The work of one GEMM is the list of units (column group of 256 outputs, contraction block),
// contraction block fastest; workgroup g of G takes the contiguous range [g*U/G, (g+1)*U/G),
// so every workgroup streams the same number of weight bytes whatever N and K are (one
// workgroup per CU: no tail round). A range touches at most a few column groups
// ("segments"); each segment's partial tile goes to slot = ordinal of the workgroup among
// the contributors of that column group, and the consumer sums cnt[group] slots in slot
// order (deterministic, no atomics).
//
// Eight waves, wave w owns columns [32*(8*group + w), +32). Every wave keeps a ring of R
// weight fragments in flight and refills a slot the moment it is consumed, across segment
// boundaries, so the HBM stream of a wave never drains before its last fragment. Segments
// are padded to a multiple of R steps with zero fragments (no loads, idle MFMA work only),
// which keeps every ring slot a compile-time register.
//
// The shared activation operand is double-buffered in LDS in chunks of XK contraction blocks.
// Loads of one wave return in order, so an activation load queues behind the HBM loads issued
// before it: chunks are therefore fetched one ring-length (R steps) ahead, by all threads, and
// parked in registers until the chunk before them has been consumed.
template <int MT>
__global__ __launch_bounds__(512, MT == 8 ? 1 : 2) void k_gemm_sk(const bf16x8* __restrict__ Xp, const bf16x8* __restrict__ Wp,
                                                    const bf16x8* __restrict__ zfrag, float* __restrict__ out,
                                                    int KB, int NB, int ldo, size_t slot_stride, int upw, int rem,
                                                    uint32_t kb_magic, const int32_t* __restrict__ slot0_tab) {
    __shared__ bf16x8 xs[SK_LDS_UNITS];
    SkGemm<MT> gm;
    gm.setup(Xp, Wp, zfrag, out, KB, NB, ldo, slot_stride, upw, rem, kb_magic, slot0_tab, blockIdx.x, gridDim.x);
    gm.issue_x();                                      // the short L2 loads first: a wave's loads return in order
    gm.issue_ring();
    gm.template run<false>(xs, SkRowScale{nullptr, 0, 0.f, 0.f}, nullptr);
}

// ------------------------------------------------------------------------------------------
// Four row blocks (128 rows). The kernel above at four row blocks issues eight LDS fragment reads and
// eight MFMAs per weight fragment and is bound by those, not by HBM; the form below measured a little
// faster there (54.1 against 54.8 us per launch at the 13B shape), the one above at eight row blocks.
// Here a workgroup is four waves, one per SIMD, so that a wave may hold up to 512 registers; wave
// w owns column blocks 2w and 2w+1 of the same 256-column group, every activation fragment read
// from LDS feeds two weight fragments (half the LDS traffic per weight byte), and the four MFMAs
// of a row block alternate between its two accumulators, so that none waits for the one before
// it. Units, ring, segments, zero page and slots exactly as above.
#define SKW_THREADS 256
#ifndef SKW_R
#define SKW_R 6
#endif
__global__ __launch_bounds__(SKW_THREADS, 1) void k_gemm_sk_wide(const bf16x8* __restrict__ Xp,
                                                                 const bf16x8* __restrict__ Wp,
                                                                 const bf16x8* __restrict__ zfrag,
                                                                 float* __restrict__ out, int KB, int NB, int ldo,
                                                                 size_t slot_stride, int upw, int rem, uint32_t kb_magic,
                                                                 const int32_t* __restrict__ slot0_tab) {
    constexpr int MT = 4, CB = 2, R = SKW_R, XK = 2, CPI = R / XK, XF = XK * MT * 2, XP = XF * 64 / SKW_THREADS;
    static_assert(CPI == 3, "three chunks per ring length, three LDS buffers");
    __shared__ bf16x8 xs[3][XF * 64];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = blockIdx.x;
    SkWalk walk = sk_walk_init(g, upw, rem, KB, kb_magic);
    const int slot0 = slot0_tab[g];                    // slot of this workgroup's first segment (later ones: 0)
    int nseg = 0;
    // the wave's two fragments of a contraction block lie side by side (2 KiB)
    auto wptr = [&](const SkIter& I, int cb) {
        int nb = I.ng * 8 + wave * CB + cb;
        if (nb >= NB) nb = NB - 1;
        return Wp + ((size_t)I.kb * NB + nb) * 64 + lane;
    };
    const size_t wstep = (size_t)NB * 64;
    const bf16x8* zl = zfrag + lane;
    auto xload = [&](bf16x8(&dst)[XP], const SkIter& I, int c) {
        int steps = I.valid - c * XK;
        steps = steps < 0 ? 0 : (steps > XK ? XK : steps);
        constexpr int PER_KB = MT * 2 * 64;
        const int limit = steps * PER_KB;
        const bf16x8* base = Xp + (size_t)(I.kb + c * XK) * PER_KB;
#pragma unroll
        for (int p = 0; p < XP; ++p) {
            const int i = p * SKW_THREADS + tid;
            dst[p] = *((i < limit) ? base + i : zl);
        }
    };
    auto xstore = [&](const bf16x8(&src)[XP], int buf) {
#pragma unroll
        for (int p = 0; p < XP; ++p) xs[buf][p * SKW_THREADS + tid] = src[p];
    };

    SkIter cur = sk_walk_next<R>(walk, KB), nxt = sk_walk_next<R>(walk, KB), nx2 = sk_walk_next<R>(walk, KB);
    if (cur.valid == 0) return;

    f32x16 acc[MT][CB];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][cb][v] = 0.f;

    bf16x8 w[R][CB], xr[CPI][XP];
#pragma unroll
    for (int c = 0; c < CPI; ++c) xload(xr[c], cur, c);
    {
        const bf16x8* wc[CB];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) wc[cb] = wptr(cur, cb);
#pragma unroll
        for (int i = 0; i < R; ++i)
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
                w[i][cb] = __builtin_nontemporal_load((i < cur.valid) ? wc[cb] + (size_t)i * wstep : zl);
    }
    // LDS holds three chunks: the one in use and the next two. Chunk t+2 is written at the start of
    // chunk t (its buffer was last read during chunk t-1, which every wave left through a barrier),
    // so the first fragments of chunk t+1 can be read before the barrier that ends chunk t, and
    // neither the LDS writes nor those reads sit on the critical path behind a barrier.
    xstore(xr[0], 0);
    xstore(xr[1], 1);
    xload(xr[0], nxt, 0);
    xload(xr[1], nxt, 1);
    __syncthreads();
    bf16x8 ph[2], pl[2];
    ph[0] = xs[0][lane];
    pl[0] = xs[0][64 + lane];

    for (;;) {
        const bf16x8* wn[CB];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) wn[cb] = wptr(nxt, cb);
#pragma unroll
        for (int c = 0; c < CPI; ++c) {
            // chunk t+2 -> LDS; its staging slot is refilled with the chunk one ring length further on
            constexpr int XQ = XK * MT;                            // (hi, lo) pairs per chunk, even
            const int sl = (c + 2) % CPI;
            xstore(xr[sl], sl);
            if (c == 0) xload(xr[sl], nxt, 2);
            else xload(xr[sl], nx2, c - 1);
            // the pairs are read one ahead of the MFMAs that use them (pair 0 was read before the barrier)
#pragma unroll
            for (int q = 0; q < XQ; ++q) {
                const int j = q / MT, mt = q % MT;
                const int i = c * XK + j;                         // ring slot (compile-time)
                if (q + 1 < XQ) {
                    ph[(q + 1) & 1] = xs[c][((q + 1) * 2) * 64 + lane];
                    pl[(q + 1) & 1] = xs[c][((q + 1) * 2 + 1) * 64 + lane];
                } else {
                    ph[0] = xs[(c + 1) % CPI][lane];
                    pl[0] = xs[(c + 1) % CPI][64 + lane];
                }
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
                    acc[mt][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph[q & 1], w[i][cb], acc[mt][cb], 0, 0, 0);
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
                    acc[mt][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pl[q & 1], w[i][cb], acc[mt][cb], 0, 0, 0);
                if (mt == MT - 1) {
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb)
                        w[i][cb] = __builtin_nontemporal_load((i < nxt.valid) ? wn[cb] + (size_t)i * wstep : zl);
                }
            }
            __syncthreads();
        }
        if (cur.last) {
            const int slot = nseg == 0 ? slot0 : 0;
            ++nseg;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const int nb = cur.ng * 8 + wave * CB + cb;
                if (nb < NB) {
                    float* o = out + (size_t)slot * slot_stride + (size_t)nb * 32 + (lane & 31);
                    int gq = lane >> 5, ldo_here = ldo;            // opaque, as in k_gemm_sk: no hoisted row offsets
                    asm volatile("" : "+v"(gq), "+s"(ldo_here));
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            int m = mt * 32 + 8 * (v >> 2) + 4 * gq + (v & 3);
                            __hip_atomic_store(&o[(size_t)m * ldo_here], acc[mt][cb][v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        }
                }
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[mt][cb][v] = 0.f;
        }
        if (nxt.valid == 0) break;
        cur = nxt;
        nxt = nx2;
        nx2 = sk_walk_next<R>(walk, KB);
    }
}

// ------------------------------------------------------------------------------------------
// dst[m][c] = sum of the slots of column c (used where the consumer wants dense rows: logits)
__global__ void k_reduce_slots(PartView pv, float* __restrict__ dst, int rows) {
    const int c4 = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
    const int m = blockIdx.y;
    if (c4 >= pv.ld || m >= rows) return;
    const int n = part_count(pv, c4);
    float4 a = make_float4(0, 0, 0, 0);
    for (int sp = 0; sp < n; ++sp) {
        float4 v = *(const float4*)(pv.base + (size_t)sp * pv.slot_stride + (size_t)m * pv.ld + c4);
        a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
    }
    *(float4*)(dst + (size_t)m * pv.ld + c4) = a;
}
void launch_reduce_slots(PartView pv, float* dst, int rows, hipStream_t s) {
    hipLaunchKernelGGL(k_reduce_slots, dim3((pv.ld / 4 + 255) / 256, rows), dim3(256), 0, s, pv, dst, rows);
}

// Sums the slots of selected rows only: output row (i, b), i < H, b < B, is row i*M + sel[b] of a
// row-chunked GEMM sequence; this launch covers the chunk holding rows [row0, row0 + rows) and
// writes dst row i*B + b when that row lies in it.
__global__ void k_reduce_selected(PartView pv, float* __restrict__ dst, const int32_t* __restrict__ sel, int B, int M,
                                  int row0, int rows) {
    const int c4 = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
    const int i = blockIdx.y / B, b = blockIdx.y % B;
    const int s = sel[b];
    if (c4 >= pv.ld || s < 0 || s >= M) return;
    const int m = i * M + s - row0;
    if (m < 0 || m >= rows) return;
    const int n = part_count(pv, c4);
    float4 a = make_float4(0, 0, 0, 0);
    for (int sp = 0; sp < n; ++sp) {
        float4 v = *(const float4*)(pv.base + (size_t)sp * pv.slot_stride + (size_t)m * pv.ld + c4);
        a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
    }
    *(float4*)(dst + (size_t)blockIdx.y * pv.ld + c4) = a;
}
void launch_reduce_selected(PartView pv, float* dst, const int32_t* sel, int B, int H, int M, int row0, int rows,
                            hipStream_t s) {
    hipLaunchKernelGGL(k_reduce_selected, dim3((pv.ld / 4 + 255) / 256, H * B), dim3(256), 0, s, pv, dst, sel, B, M, row0,
                       rows);
}

// ------------------------------------------------------------------------------------------
#define SK_MAX_WG 256       // one workgroup of 8 waves per CU
#ifndef SK_SMALL_U
#define SK_SMALL_U (16 * SK_MAX_WG * 2)   // (column groups x contraction blocks) up to which half the workgroups are used
#endif

void gemm_plan_make(GemmPlan* p, int MB, int KB, int NB, int32_t* cnt_host, int32_t* slot0_host) {
    p->MB = MB; p->KB = KB; p->NB = NB;
    p->cnt_dev = nullptr;
    p->slot0_dev = nullptr;
    p->NG = (NB + 7) / 8;
    const int U = p->NG * KB;
    int G = U / 16;                                   // at least one ring length of steps each
    if (G > SK_MAX_WG) G = SK_MAX_WG;
    // A small matrix (the O projection: 33 MB at the 7B shape) gains nothing from the last
    // doubling of workgroups but pays for it in partial tiles (measured 13.5 us with 128
    // workgroups / 8 slots against 14.9 us with 256 / 16, and the consumer reads half as much).
    if (G == SK_MAX_WG && U <= SK_SMALL_U) G = SK_MAX_WG / 2;
    if (G < 1) G = 1;
    p->G = G;
    // workgroup g takes upw units, the first `rem` workgroups one more (the kernels compute the same)
    p->upw = U / G;
    p->rem = U % G;
    for (int ng = 0; ng < p->NG; ++ng) cnt_host[ng] = 0;
    for (int g = 0; g < G; ++g) {
        const int u0 = g * p->upw + (g < p->rem ? g : p->rem), u1 = u0 + p->upw + (g < p->rem ? 1 : 0);
        const int ng0 = u0 / KB, ng1 = (u1 - 1) / KB;
        slot0_host[g] = cnt_host[ng0];                // contributors of its first column group before it
        for (int ng = ng0; ng <= ng1; ++ng) ++cnt_host[ng];
    }
    int slots = 1;
    for (int ng = 0; ng < p->NG; ++ng) slots = cnt_host[ng] > slots ? cnt_host[ng] : slots;
    p->slots = slots;
    p->uniform = 1;                                   // every column group has the same number of contributors?
    for (int ng = 0; ng < p->NG; ++ng) p->uniform &= (cnt_host[ng] == slots);
}

PartView launch_gemm(const GemmPlan& p, const void* Xp, const void* Wp, const void* zfrag, float* out, hipStream_t s,
                     hipEvent_t ev0, hipEvent_t ev1) {
    PartView pv;
    pv.base = out;
    pv.ld = p.NB * 32;
    pv.slot_stride = (size_t)p.MB * 32 * pv.ld;
    pv.cnt = p.uniform ? nullptr : p.cnt_dev;         // NULL: nmax slots everywhere, the consumer need not look it up
    pv.nmax = p.slots;
    const uint32_t kb_magic = (uint32_t)((0x100000000ull + (uint64_t)p.KB - 1) / (uint64_t)p.KB);
#define SK_ARGS (const bf16x8*)Xp, (const bf16x8*)Wp, (const bf16x8*)zfrag, out, p.KB, p.NB, pv.ld, pv.slot_stride, p.upw, p.rem, kb_magic, p.slot0_dev
#define SK_LAUNCH(KERNEL_, THREADS_, ...)                                                                  \
    do {                                                                                                   \
        if (ev0 || ev1)                                                                                    \
            hipExtLaunchKernelGGL(KERNEL_, dim3(p.G), dim3(THREADS_), 0, s, ev0, ev1, 0, SK_ARGS, ##__VA_ARGS__); \
        else                                                                                               \
            hipLaunchKernelGGL(KERNEL_, dim3(p.G), dim3(THREADS_), 0, s, SK_ARGS, ##__VA_ARGS__);          \
    } while (0)
    switch (p.MB) {                                    // the plan's row blocks: 1, 2, 4 or 8, one pass each
    case 1: SK_LAUNCH(k_gemm_sk<1>, 512); break;
    case 2: SK_LAUNCH(k_gemm_sk<2>, 512); break;
    case 4: SK_LAUNCH(k_gemm_sk_wide, SKW_THREADS); break;
    case 8: SK_LAUNCH(k_gemm_sk<8>, 512); break;
    default:                                           // plans are only ever made for 1, 2, 4 or 8 row blocks
        pv.nmax = 0;                                   // nothing launched, nothing for a consumer to read
        pv.cnt = nullptr;
        break;
    }
#undef SK_LAUNCH
#undef SK_ARGS
    return pv;
}
