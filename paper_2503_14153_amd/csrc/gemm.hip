// Weight-streaming GEMM for the verifying forward pass: out[m][n] = sum_k X[m][k] * W[n][k].
//
// The tree has T <= 256 rows, so every projection of the step (QKV, O, gate/up, down, LM
// head, draft heads) multiplies a few 32-row blocks of activations by a weight matrix that is
// read exactly once: the kernel is bound by the HBM read of W, not by the matrix cores. The
// design therefore (1) stores W pre-tiled as 1 KiB MFMA fragments, contraction-block-major
// ([kb][nb]): a wave fetches a fragment with one 16-byte-per-lane load, and at any moment the
// waves of the whole grid (all nb, similar kb) read one contiguous region of HBM, which
// spreads over every channel instead of marching through power-of-two strides in step, (2) keeps many such loads in flight per wave
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
// MT  = number of 32-row activation blocks (all of them: W is read once for every row)
// NW  = consumer waves per workgroup; wave w owns output columns [32*(NW*blockIdx.x + w), +32)
// R   = depth of the per-wave ring of weight fragments: R 1-KiB loads stay in flight per wave;
//       a ring slot is refilled with the fragment R steps ahead as soon as it is consumed
// XK  = contraction blocks per LDS chunk of the shared activation operand (double-buffered)
//
// Wave NW is a producer: it alone fetches the activation chunks (L2 hits) and stores them to
// LDS. Vector loads of one wave return in order, so an activation load issued by a consumer
// would queue behind the R HBM loads of its ring and every chunk would cost a full HBM
// latency; the producer's queue holds only the short L2 loads.
template <int MT, int NW>
__global__ __launch_bounds__((NW + 1) * 64, (MT <= 2 ? 3 : 1)) void k_gemm_stream(
    const bf16x8* __restrict__ Xp, const bf16x8* __restrict__ Wp, float* __restrict__ out, int KB, int NB, int ldo,
    int kb_per_split, size_t split_stride) {
    constexpr int R = 16;
    constexpr int XK = (MT >= 8) ? 1 : 8 / MT;
    constexpr int XF = XK * MT * 2;                  // X fragments per chunk (hi and lo parts) = 16
    constexpr int CPI = R / XK;                      // chunks per outer iteration (even)
    constexpr int D = 2;                             // chunks the producer keeps in flight
    static_assert(R % XK == 0 && CPI % 2 == 0 && XF == 16, "bad tiling");
    __shared__ bf16x8 xs[2][XF * 64];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int kb0 = blockIdx.y * kb_per_split;
    int kb1 = kb0 + kb_per_split;
    if (kb1 > KB) kb1 = KB;
    const int nsteps = kb1 - kb0;                     // may be <= 0 for a trailing split
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};

    if (wave == NW) {
        // ---------------- producer: chunk c = contraction blocks [c*XK, (c+1)*XK) of the slice
        if (nsteps <= 0) return;
        const bf16x8* xbase = Xp + (size_t)kb0 * MT * 2 * 64 + lane;
        const int nfrag = nsteps * MT * 2;            // fragments in the slice
        bf16x8 st[D][XF];
        auto fetch = [&](bf16x8(&dst)[XF], int c) {
#pragma unroll
            for (int f = 0; f < XF; ++f) {
                int fi = c * XF + f;
                dst[f] = (fi < nfrag) ? xbase[(size_t)fi * 64] : zero;
            }
        };
        auto put = [&](const bf16x8(&src)[XF], int buf) {
#pragma unroll
            for (int f = 0; f < XF; ++f) xs[buf][f * 64 + lane] = src[f];
        };
        fetch(st[0], 0);
        put(st[0], 0);
        fetch(st[1], 1);                              // stage (c+1)&1 holds chunk c+1
        fetch(st[0], 2);
        __syncthreads();
        for (int base = 0; base < nsteps; base += R) {
#pragma unroll
            for (int c = 0; c < CPI; ++c) {
                const int step0 = base + c * XK;
                if (step0 >= nsteps) break;
                const int ci = step0 / XK;            // chunk being consumed; CPI even => parity of ci == c & 1
                if (step0 + XK < nsteps) {
                    put(st[(c + 1) & 1], (c + 1) & 1);
                    fetch(st[(c + 1) & 1], ci + 1 + D);
                }
                __syncthreads();
            }
        }
        return;
    }

    // -------------------- consumers
    int nb = blockIdx.x * NW + wave;
    const bool owns = nb < NB;
    if (!owns) nb = NB - 1;                           // keep the wave in the barriers
    const bf16x8* wrow = Wp + ((size_t)kb0 * NB + nb) * 64 + lane;     // fragment (kb, nb); next kb is NB further
    const size_t wstep = (size_t)NB * 64;
    f32x16 acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    if (nsteps > 0) {
        bf16x8 w[R];
#pragma unroll
        for (int i = 0; i < R; ++i) w[i] = (i < nsteps) ? __builtin_nontemporal_load(wrow + (size_t)i * wstep) : zero;
        __syncthreads();
        for (int base = 0; base < nsteps; base += R) {
#pragma unroll
            for (int c = 0; c < CPI; ++c) {
                const int step0 = base + c * XK;
                if (step0 >= nsteps) break;           // uniform over the workgroup
#pragma unroll
                for (int j = 0; j < XK; ++j) {
                    const int i = c * XK + j;         // ring slot (compile-time)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        bf16x8 hi = xs[c & 1][((j * MT + mt) * 2) * 64 + lane];
                        bf16x8 lo = xs[c & 1][((j * MT + mt) * 2 + 1) * 64 + lane];
                        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi, w[i], acc[mt], 0, 0, 0);
                        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo, w[i], acc[mt], 0, 0, 0);
                    }
                    const int nxt = base + i + R;
                    w[i] = (nxt < nsteps) ? __builtin_nontemporal_load(wrow + (size_t)nxt * wstep) : zero;
                }
                __syncthreads();
            }
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

// ------------------------------------------------------------------------------------------
// Balanced streaming ("stream-K") variant for MT <= 2, the shapes of batch-1 decoding.
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
struct SkIter { int kb, ng, valid, last; };

template <int MT>
__global__ __launch_bounds__(512, 2) void k_gemm_sk(const bf16x8* __restrict__ Xp, const bf16x8* __restrict__ Wp,
                                                    const bf16x8* __restrict__ zfrag, float* __restrict__ out,
                                                    int KB, int NB, int NG, int ldo, size_t slot_stride) {
    constexpr int R = MT >= 4 ? 8 : 16;              // ring depth: with four row blocks the accumulators need the registers
    constexpr int XK = 8 / MT;                       // contraction blocks per chunk
    constexpr int CPI = R / XK;                      // chunks per outer iteration (2 or 4)
    constexpr int XF = 16;                           // fragments per chunk = XK * MT * 2
    constexpr int XP = XF * 64 / 512;                // 16-byte pieces per thread per chunk = 2
    __shared__ bf16x8 xs[2][XF * 64];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int G = gridDim.x, g = blockIdx.x;
    const int U = NG * KB;
    auto ustart = [&](int gg) { return (int)(((long long)gg * U) / G); };
    const int u0 = ustart(g), u1 = ustart(g + 1);

    // k-th outer iteration (R steps) of this workgroup's padded segment list
    auto iter_info = [&](int k) {
        SkIter r = {0, 0, 0, 0};
        int u = u0;
        while (u < u1) {
            const int ng = u / KB, kb = u - ng * KB;
            int send = (ng + 1) * KB;
            if (send > u1) send = u1;
            const int len = send - u, nit = (len + R - 1) / R;
            if (k < nit) {
                r.kb = kb + k * R;
                r.ng = ng;
                r.valid = len - k * R < R ? len - k * R : R;
                r.last = (k == nit - 1);
                return r;
            }
            k -= nit;
            u = send;
        }
        return r;
    };
    auto wptr = [&](const SkIter& I) {
        int nb = I.ng * 8 + wave;
        if (nb >= NB) nb = NB - 1;
        return Wp + ((size_t)I.kb * NB + nb) * 64 + lane;
    };
    const size_t wstep = (size_t)NB * 64;
    // Every load below is unconditional and its result is used as loaded: a fragment past the
    // end of a segment is fetched from a 1 KiB page of zeros (zfrag) by selecting the ADDRESS.
    // A branch around a load, or a select on its result, makes the compiler wait for the whole
    // ring (s_waitcnt vmcnt(0)) in every iteration; straight-line loads are counted exactly.
    const bf16x8* zl = zfrag + lane;
    auto xload = [&](bf16x8(&dst)[XP], const SkIter& I, int c) {
        int steps = I.valid - c * XK;
        steps = steps < 0 ? 0 : (steps > XK ? XK : steps);
        const int limit = steps * MT * 2 * 64;
        const bf16x8* base = Xp + (size_t)(I.kb + c * XK) * MT * 2 * 64;
#pragma unroll
        for (int p = 0; p < XP; ++p) {
            const int i = p * 512 + tid;
            dst[p] = *((i < limit) ? base + i : zl);
        }
    };
    auto xstore = [&](const bf16x8(&src)[XP], int buf) {
#pragma unroll
        for (int p = 0; p < XP; ++p) xs[buf][p * 512 + tid] = src[p];
    };

    SkIter cur = iter_info(0), nxt = iter_info(1), nx2 = iter_info(2);
    if (cur.valid == 0) return;

    f32x16 acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    bf16x8 w[R], xr[CPI][XP];
#pragma unroll
    for (int c = 0; c < CPI; ++c) xload(xr[c], cur, c);           // short L2 loads first
    {
        const bf16x8* wc = wptr(cur);
#pragma unroll
        for (int i = 0; i < R; ++i) w[i] = __builtin_nontemporal_load((i < cur.valid) ? wc + (size_t)i * wstep : zl);
    }
    xstore(xr[0], 0);
    xload(xr[0], nxt, 0);
    __syncthreads();

    for (int k = 0;; ++k) {
        const bf16x8* wn = wptr(nxt);
#pragma unroll
        for (int c = 0; c < CPI; ++c) {
#pragma unroll
            for (int j = 0; j < XK; ++j) {
                const int i = c * XK + j;                         // ring slot (compile-time)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    bf16x8 hi = xs[c & 1][((j * MT + mt) * 2) * 64 + lane];
                    bf16x8 lo = xs[c & 1][((j * MT + mt) * 2 + 1) * 64 + lane];
                    acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi, w[i], acc[mt], 0, 0, 0);
                    acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo, w[i], acc[mt], 0, 0, 0);
                }
                w[i] = __builtin_nontemporal_load((i < nxt.valid) ? wn + (size_t)i * wstep : zl);
            }
            // the chunk consumed next goes to the other buffer; its register slot is refilled
            // with the chunk one outer iteration further on
            const int nc = (c + 1) % CPI;
            xstore(xr[nc], (c + 1) & 1);
            if (c + 1 < CPI) xload(xr[nc], nxt, c + 1);
            else xload(xr[nc], nx2, 0);
            __syncthreads();
        }
        if (cur.last) {
            // slot = ordinal of this workgroup among those whose ranges meet column group cur.ng
            const int first_unit = cur.ng * KB;
            int gf = (int)(((long long)first_unit * G) / U);
            while (gf + 1 < G && ustart(gf + 1) <= first_unit) ++gf;
            while (gf > 0 && ustart(gf) > first_unit) --gf;
            const int nb = cur.ng * 8 + wave;
            if (nb < NB) {
                float* o = out + (size_t)(g - gf) * slot_stride + (size_t)nb * 32 + (lane & 31);
                const int gq = lane >> 5;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        int m = mt * 32 + 8 * (v >> 2) + 4 * gq + (v & 3);
                        o[(size_t)m * ldo] = acc[mt][v];
                    }
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mt][v] = 0.f;
        }
        if (nxt.valid == 0) break;
        cur = nxt;
        nxt = nx2;
        nx2 = iter_info(k + 3);
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

// ------------------------------------------------------------------------------------------
// Uniform split-K (kind 0): enough workgroups to fill 256 CUs a few times over, slices of at
// least 256 contraction elements, and partial sums (which the consumer re-reads) kept to a
// fraction of the weight bytes.
static int gemm_choose_split(int MB, int KB, int NB) {
    const int NW = 4;
    int groups = (NB + NW - 1) / NW;
    int split = 1;
    const double w_bytes = (double)NB * 32 * KB * 16 * 2;
    while (groups * split < 512 && split < 16 && KB / (split * 2) >= 16) {
        double part_bytes = (double)(split * 2) * (MB * 32) * (NB * 32) * 4 * 2;   // written, then read
        if (part_bytes > 0.5 * w_bytes) break;
        split *= 2;
    }
    return split;
}

#define SK_MAX_WG 256       // one workgroup of 8 waves per CU
#ifndef SK_MAX_MB
#define SK_MAX_MB 4          // row blocks (of 32 rows) up to which the stream-K kernel is used
#endif
#ifndef SK_SMALL_U
#define SK_SMALL_U (16 * SK_MAX_WG * 2)   // (column groups x contraction blocks) up to which half the workgroups are used
#endif

void gemm_plan_make(GemmPlan* p, int MB, int KB, int NB, int32_t* cnt_host) {
    p->MB = MB; p->KB = KB; p->NB = NB;
    p->cnt_dev = nullptr;
    if (MB > SK_MAX_MB) {
        p->kind = 0;
        p->nsplit = gemm_choose_split(MB, KB, NB);
        p->G = 0; p->NG = 0;
        p->slots = p->nsplit;
        return;
    }
    p->kind = 1;
    p->nsplit = 0;
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
    auto ustart = [&](int gg) { return (int)(((long long)gg * U) / G); };
    int slots = 1;
    for (int ng = 0; ng < p->NG; ++ng) {
        int first = ng * KB, last = (ng + 1) * KB - 1;
        int gf = (int)(((long long)first * G) / U);
        while (gf + 1 < G && ustart(gf + 1) <= first) ++gf;
        while (gf > 0 && ustart(gf) > first) --gf;
        int gl = (int)(((long long)last * G) / U);
        while (gl + 1 < G && ustart(gl + 1) <= last) ++gl;
        while (gl > 0 && ustart(gl) > last) --gl;
        cnt_host[ng] = gl - gf + 1;
        if (cnt_host[ng] > slots) slots = cnt_host[ng];
    }
    p->slots = slots;
}

template <int MT>
static void launch_gemm_t(const void* Xp, const void* Wp, float* out, int KB, int NB, int ldo, int nsplit,
                          size_t split_stride, hipStream_t s) {
    constexpr int NW = 4;
    int groups = (NB + NW - 1) / NW;
    int kps = (KB + nsplit - 1) / nsplit;
    hipLaunchKernelGGL((k_gemm_stream<MT, NW>), dim3(groups, nsplit), dim3((NW + 1) * 64), 0, s,
                       (const bf16x8*)Xp, (const bf16x8*)Wp, out, KB, NB, ldo, kps, split_stride);
}

PartView launch_gemm(const GemmPlan& p, const void* Xp, const void* Wp, const void* zfrag, float* out, hipStream_t s) {
    PartView pv;
    pv.base = out;
    pv.ld = p.NB * 32;
    pv.slot_stride = (size_t)p.MB * 32 * pv.ld;
    pv.group_cols = 256;
    if (p.kind == 1) {
        pv.cnt = p.cnt_dev;
        pv.nmax = p.slots;
        if (p.MB == 1)
            hipLaunchKernelGGL((k_gemm_sk<1>), dim3(p.G), dim3(512), 0, s, (const bf16x8*)Xp, (const bf16x8*)Wp,
                               (const bf16x8*)zfrag, out, p.KB, p.NB, p.NG, pv.ld, pv.slot_stride);
        else if (p.MB == 2)
            hipLaunchKernelGGL((k_gemm_sk<2>), dim3(p.G), dim3(512), 0, s, (const bf16x8*)Xp, (const bf16x8*)Wp,
                               (const bf16x8*)zfrag, out, p.KB, p.NB, p.NG, pv.ld, pv.slot_stride);
        else
            hipLaunchKernelGGL((k_gemm_sk<4>), dim3(p.G), dim3(512), 0, s, (const bf16x8*)Xp, (const bf16x8*)Wp,
                               (const bf16x8*)zfrag, out, p.KB, p.NB, p.NG, pv.ld, pv.slot_stride);
        return pv;
    }
    pv.cnt = nullptr;
    pv.nmax = p.nsplit;
    if (p.MB == 4) launch_gemm_t<4>(Xp, Wp, out, p.KB, p.NB, pv.ld, p.nsplit, pv.slot_stride, s);
    else launch_gemm_t<8>(Xp, Wp, out, p.KB, p.NB, pv.ld, p.nsplit, pv.slot_stride, s);
    return pv;
}
