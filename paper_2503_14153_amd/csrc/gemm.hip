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
// that every workgroup streams the same number of weight bytes (over all 256 CUs, or over fewer
// when that lets every workgroup stay inside one column group: gemm_plan_make); the consumer
// kernel sums the split partial results (deterministic, no atomics).
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
// Balanced streaming ("stream-K") over MT = 1 or 2 row blocks of 32 rows (this kernel; also the GEMM body of the
// persistent layer kernel, there with eight row blocks as well) or four and eight (the kernel after it).
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
// Eight (or four) row blocks with the operand roles swapped: the WEIGHT fragments of a step go through LDS and the
// activations stay in registers. With many row blocks the kernel above reads every activation fragment from LDS
// once per column block (16 one-KiB reads and 16 MFMAs per wave and step at eight row blocks: the LDS port and
// the matrix cores are both needed all the time, and neither gets it). Here wave w owns ROW block w % MT and MT
// column blocks of the group: its two activation fragments of a step (hi, lo) come straight from L2 into registers
// (nobody else needs them), every wave still streams one weight fragment per step through its ring and drops it
// into LDS, and each weight fragment read from LDS feeds two MFMAs: half the LDS bytes per MFMA, the MFMAs of a
// step go to MT different accumulators. Units, segments, zero page, slots and partial tiles exactly as above.
template <int MT>
__global__ __launch_bounds__(512, 2) void k_gemm_sk_rows(const bf16x8* __restrict__ Xp, const bf16x8* __restrict__ Wp,
                                                         const bf16x8* __restrict__ zfrag, float* __restrict__ out,
                                                         int KB, int NB, int ldo, size_t slot_stride, int upw, int rem,
                                                         uint32_t kb_magic, const int32_t* __restrict__ slot0_tab) {
    static_assert(MT == 4 || MT == 8, "row blocks");
    constexpr int R = 4;       // ring depth in steps; even (the LDS buffer of a step is i & 1); 6 measured slower
    constexpr int CPW = MT;                             // column blocks per wave: 8 waves cover MT rows x 8 columns
    __shared__ bf16x8 ws[2][8 * 64];                    // the eight weight fragments of two consecutive steps
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int r = wave % MT, ch = wave / MT;
    SkWalk walk = sk_walk_init(blockIdx.x, upw, rem, KB, kb_magic);
    const int slot0 = slot0_tab[blockIdx.x];
    int nseg = 0;
    SkIter cur = sk_walk_next<R>(walk, KB), nxt = sk_walk_next<R>(walk, KB);
    if (cur.valid == 0) return;
    const bf16x8* zl = zfrag + lane;
    const size_t wstep = (size_t)NB * 64, xstep = (size_t)MT * 2 * 64;
    auto wptr = [&](const SkIter& I) {
        int nb = I.ng * 8 + wave;
        if (nb >= NB) nb = NB - 1;
        return Wp + ((size_t)I.kb * NB + nb) * 64 + lane;
    };
    auto xptr = [&](const SkIter& I) { return Xp + ((size_t)I.kb * MT + r) * 2 * 64 + lane; };

    f32x16 acc[CPW];
#pragma unroll
    for (int j = 0; j < CPW; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    bf16x8 w[R], xh[R], xl[R];
    {
        const bf16x8* wc = wptr(cur);
        const bf16x8* xc = xptr(cur);
#pragma unroll
        for (int i = 0; i < R; ++i) {
            w[i] = __builtin_nontemporal_load((i < cur.valid) ? wc + (size_t)i * wstep : zl);
            xh[i] = *((i < cur.valid) ? xc + (size_t)i * xstep : zl);
            xl[i] = *((i < cur.valid) ? xc + (size_t)i * xstep + 64 : zl);
        }
    }
    for (;;) {
        const bf16x8* wn = wptr(nxt);
        const bf16x8* xn = xptr(nxt);
#pragma unroll
        for (int i = 0; i < R; ++i) {
            // Buffer i & 1 was last read in step i - 2; every wave has passed the barrier of step i - 1 since, and
            // its reads of step i - 2 come before that barrier in program order.
            ws[i & 1][wave * 64 + lane] = w[i];
            __syncthreads();
#pragma unroll
            for (int j = 0; j < CPW; ++j) {
                const bf16x8 b = ws[i & 1][(ch * CPW + j) * 64 + lane];
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh[i], b, acc[j], 0, 0, 0);
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xl[i], b, acc[j], 0, 0, 0);
            }
            w[i] = __builtin_nontemporal_load((i < nxt.valid) ? wn + (size_t)i * wstep : zl);
            xh[i] = *((i < nxt.valid) ? xn + (size_t)i * xstep : zl);
            xl[i] = *((i < nxt.valid) ? xn + (size_t)i * xstep + 64 : zl);
        }
        if (cur.last) {
            const int slot = nseg == 0 ? slot0 : 0;
            ++nseg;
            int gq = lane >> 5, ldo_here = ldo;            // opaque, as in k_gemm_sk: no hoisted row offsets
            asm volatile("" : "+v"(gq), "+s"(ldo_here));
#pragma unroll
            for (int j = 0; j < CPW; ++j) {
                const int nb = cur.ng * 8 + ch * CPW + j;
                if (nb < NB) {
                    float* o = out + (size_t)slot * slot_stride + (size_t)nb * 32 + (lane & 31);
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int m = r * 32 + 8 * (v >> 2) + 4 * gq + (v & 3);
                        __hip_atomic_store(&o[(size_t)m * ldo_here], acc[j][v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < CPW; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
        }
        if (nxt.valid == 0) break;
        cur = nxt;
        nxt = sk_walk_next<R>(walk, KB);
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
    // Prefer a split in which no workgroup's range crosses a column group: s workgroups per group with s a divisor
    // of KB. Every workgroup then has ONE segment, writes its partial tile once, at the end of its stream, and a
    // group has exactly s slots. With ranges that straddle groups a workgroup stores a tile in the middle of its
    // stream and the groups get one or two slots more (measured at the 7B shape, 64 rows: QKV 256 -> 192
    // workgroups, gate/up 256 -> 172, LM head 256 -> 252: step 5.23 -> 5.00 ms on one box; gate/up alone 5.08).
    // Taken when it keeps at least five eighths of the workgroups (seven eighths at eight row blocks, where the
    // matrix cores are short: there 192 of 256 workgroups made the GEMMs 5 % slower and the step no faster);
    // otherwise the balanced split stays.
    int aligned = 0;
    for (int sp = 1; p->NG * sp <= G; ++sp)
        if (KB % sp == 0) aligned = p->NG * sp;
    if (aligned * 8 >= G * (MB >= 8 ? 7 : 5)) G = aligned;
    // A small matrix (the O projection: 33 MB at the 7B shape) gains nothing from the last
    // doubling of workgroups but pays for it in partial tiles (measured 13.5 us with 128
    // workgroups / 8 slots against 14.9 us with 256 / 16, and the consumer reads half as much).
    if (G > SK_MAX_WG / 2 && U <= SK_SMALL_U) {
        const int sp = G / p->NG;                     // (aligned splits stay aligned when s is even)
        G = (G == aligned && sp % 2 == 0) ? G / 2 : SK_MAX_WG / 2;
    }
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
    case 4: SK_LAUNCH(k_gemm_sk_rows<4>, 512); break;
    case 8: SK_LAUNCH(k_gemm_sk_rows<8>, 512); break;
    default:                                           // plans are only ever made for 1, 2, 4 or 8 row blocks
        pv.nmax = 0;                                   // nothing launched, nothing for a consumer to read
        pv.cnt = nullptr;
        break;
    }
#undef SK_LAUNCH
#undef SK_ARGS
    return pv;
}
