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
// the matrix cores are both needed all the time, and neither gets it). Here wave w owns ROW block w % MT and
// CPW = CG * MT / 8 column blocks of a column group of CG blocks: its two activation fragments of a step (hi, lo)
// come straight from L2 into registers (nobody else needs them), the first CG waves stream one weight fragment per
// step through their rings and drop it into LDS, and each weight fragment read from LDS feeds two MFMAs.
//
// At these row counts the matrix cores, not the weight stream, set the pace, and what a step costs beyond its
// MFMAs is the hand-over through LDS. So the split is always the aligned one (workgroup g = column group g / S,
// segment g % S of the contraction: one partial tile per workgroup, slot = segment), the width of a column group is
// chosen with the split (gemm_plan_rows: narrower groups mean more workgroups and fewer slots), and a step is
// software-pipelined around its one barrier:
//   write the NEXT step's fragment to the other LDS buffer (its last readers passed the previous barrier);
//   MFMAs of the first half of the column blocks (fragments already in registers), the ring's weight load among them;
//   barrier; read the next step's first-half fragments;
//   MFMAs of the second half, the two activation loads among them; read the next step's second-half fragments.
// A wave that arrives at the barrier has its MFMAs queued and the reads it needs next already in flight; the
// global loads are spread over the step because a wave cannot issue past a vector-memory instruction the address
// unit has not taken yet (24 loads of 1 KiB per step at once held every wave's next MFMAs back).
// Measured per step at 256 rows, column groups of six blocks (768 MFMA cycles): 1230 cycles with write, barrier,
// read, MFMA in sequence; 1075 with the hand-over pipelined; 1030 with the loads spread as well.
template <int MT, int CG>
__global__ __launch_bounds__(512, 2) void k_gemm_rows(const bf16x8* __restrict__ Xp, const bf16x8* __restrict__ Wp,
                                                      const bf16x8* __restrict__ zfrag, float* __restrict__ out,
                                                      int KB, int NB, int ldo, size_t slot_stride, int S) {
    static_assert((MT == 4 || MT == 8) && (CG * MT) % 16 == 0 && CG <= 8, "row blocks / column group");
    constexpr int R = 4;                                // ring depth in steps; even (the LDS buffer of step i is i & 1)
    constexpr int CPW = CG * MT / 8;                    // column blocks per wave: 8 waves cover MT rows x CG columns
    constexpr int H = CPW / 2;                          // first half
    __shared__ bf16x8 ws[2][CG * 64];                   // the weight fragments of two consecutive steps
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int r = wave % MT, ch = wave / MT;
    const int ng = blockIdx.x / S, seg = blockIdx.x - ng * S;
    const int n = KB / S, kb0 = seg * n;                // this workgroup's steps: contraction blocks [kb0, kb0 + n)
    const bool loader = wave < CG;
    int nbw = ng * CG + wave;
    if (nbw >= NB) nbw = NB - 1;                        // (a ragged last group: a duplicate fragment, never stored)
    const size_t wstep = (size_t)NB * 64, xstep = (size_t)MT * 2 * 64;
    const bf16x8* wp = Wp + ((size_t)kb0 * NB + nbw) * 64 + lane;
    const bf16x8* xp = Xp + ((size_t)kb0 * MT + r) * 2 * 64 + lane;
    const bf16x8* zl = zfrag + lane;                    // steps past n read zeros (no weight bytes, idle MFMA work)

    f32x16 acc[CPW];
#pragma unroll
    for (int j = 0; j < CPW; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
    bf16x8 w[R], xh[R], xl[R], b[CPW];
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const bool ok = i < n;
        if (loader) w[i] = __builtin_nontemporal_load(ok ? wp + (size_t)i * wstep : zl);
        xh[i] = *(ok ? xp + (size_t)i * xstep : zl);
        xl[i] = *(ok ? xp + (size_t)i * xstep + 64 : zl);
    }
    wp += R * wstep;
    xp += R * xstep;
    // step 0's fragments; its ring slot takes step R
    if (loader) ws[0][wave * 64 + lane] = w[0];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < CPW; ++j) b[j] = ws[0][(ch * CPW + j) * 64 + lane];
    if (loader) w[0] = __builtin_nontemporal_load(R < n ? wp : zl);
    for (int s0 = 0; s0 < n; s0 += R) {
#pragma unroll
        for (int i = 0; i < R; ++i) {
            // entering step s0 + i: b holds its fragments (read from buffer i & 1), buffer (i + 1) & 1 is free
            const bf16x8* wn = (s0 + R + i + 1 < n) ? wp + (size_t)(i + 1) * wstep : zl;   // step s0 + i + 1 + R
            const bool xok = s0 + R + i < n;                                               // step s0 + i + R
            const bf16x8* xhn = xok ? xp + (size_t)i * xstep : zl;
            const bf16x8* xln = xok ? xp + (size_t)i * xstep + 64 : zl;
            if (loader) ws[(i + 1) & 1][wave * 64 + lane] = w[(i + 1) % R];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < H; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh[i], b[j], acc[j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (loader) w[(i + 1) % R] = __builtin_nontemporal_load(wn);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < H; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xl[i], b[j], acc[j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
#pragma unroll
            for (int j = 0; j < H; ++j) b[j] = ws[(i + 1) & 1][(ch * CPW + j) * 64 + lane];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = H; j < CPW; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh[i], b[j], acc[j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            xh[i] = *xhn;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = H; j < CPW; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xl[i], b[j], acc[j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            xl[i] = *xln;
#pragma unroll
            for (int j = H; j < CPW; ++j) b[j] = ws[(i + 1) & 1][(ch * CPW + j) * 64 + lane];
            __builtin_amdgcn_sched_barrier(0);
        }
        wp += R * wstep;
        xp += R * xstep;
    }
    int gq = lane >> 5, ldo_here = ldo;                // opaque, as in k_gemm_sk: no hoisted row offsets
    asm volatile("" : "+v"(gq), "+s"(ldo_here));
#pragma unroll
    for (int j = 0; j < CPW; ++j) {
        const int nb = ng * CG + ch * CPW + j;
        if (nb < NB) {
            float* o = out + (size_t)seg * slot_stride + (size_t)nb * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = r * 32 + 8 * (v >> 2) + 4 * gq + (v & 3);
                __hip_atomic_store(&o[(size_t)m * ldo_here], acc[j][v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
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

// Four and eight row blocks (k_gemm_rows): the width of a column group, CG blocks, and the number of segments S the
// contraction is split into, S a divisor of KB, at most 16. Cost of a candidate in shader cycles, from the kernel's
// measured pace: a step costs its MFMAs (two waves per SIMD, 2 x CPW MFMAs of 32 cycles each) plus about 300 cycles
// of hand-over; a workgroup runs KB / S steps (rounded up to the ring), the grid ceil(groups x S / 256) rounds; the S
// partial tiles are written at the end of the kernel and read by the consumer at about 2500 bytes per cycle each
// way. Narrow groups buy workgroups and few slots for the matrices with few columns (O and down projection at the
// 7B shape, 256 rows: 4 blocks x 8 segments instead of 8 x 16: 22 us against 26, 41 against 43, and the consumer
// reads half as much); six-block groups fill the chip where eight-block ones leave a quarter of it idle (QKV: 64
// groups x 4 = 256 workgroups, 45 us against 55 with 48 x 4; gate/up 115 x 2 = 230 against 86 x 2 = 172: 76 against 89).
static void gemm_plan_rows(GemmPlan* p) {
    const int MT = p->MB;
    static const int widths8[] = {8, 6, 4}, widths4[] = {8, 4};
    const int* widths = MT == 8 ? widths8 : widths4;
    const int n_widths = MT == 8 ? 3 : 2;
    double best = 0;
    for (int wi = 0; wi < n_widths; ++wi) {
        const int CG = widths[wi], groups = (p->NB + CG - 1) / CG;
        for (int S = 1; S <= 16 && S <= p->KB; ++S) {
            if (p->KB % S) continue;
            const int G = groups * S, rounds = (G + SK_MAX_WG - 1) / SK_MAX_WG;
            const int steps = (p->KB / S + 3) / 4 * 4;
            const double step_cycles = 16.0 * CG * MT + 300.0;
            const double tile_bytes = (double)S * MT * 32 * p->NB * 32 * 4;
            const double cost = rounds * steps * step_cycles + 2.0 * tile_bytes / 2500.0;
            if (p->CG == 0 || cost < best) { best = cost; p->CG = CG; p->S = S; }
        }
    }
    if (p->S > p->slots_max) p->slots_max = p->S;
}

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
    p->CG = 0;
    p->S = 0;
    p->slots_max = slots;
    if (MB >= 4) gemm_plan_rows(p);
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
    if (p.CG) {                                        // four / eight row blocks: the aligned split of k_gemm_rows
        const int G = (p.NB + p.CG - 1) / p.CG * p.S;
        pv.cnt = nullptr;
        pv.nmax = p.S;
#define ROWS_LAUNCH(MT_, CG_)                                                                              \
    do {                                                                                                   \
        if (ev0 || ev1)                                                                                    \
            hipExtLaunchKernelGGL((k_gemm_rows<MT_, CG_>), dim3(G), dim3(512), 0, s, ev0, ev1, 0, (const bf16x8*)Xp, \
                                  (const bf16x8*)Wp, (const bf16x8*)zfrag, out, p.KB, p.NB, pv.ld, pv.slot_stride, p.S); \
        else                                                                                               \
            hipLaunchKernelGGL((k_gemm_rows<MT_, CG_>), dim3(G), dim3(512), 0, s, (const bf16x8*)Xp, (const bf16x8*)Wp, \
                               (const bf16x8*)zfrag, out, p.KB, p.NB, pv.ld, pv.slot_stride, p.S);         \
    } while (0)
        const int key = p.MB * 10 + p.CG;
        if (key == 88) ROWS_LAUNCH(8, 8);
        else if (key == 86) ROWS_LAUNCH(8, 6);
        else if (key == 84) ROWS_LAUNCH(8, 4);
        else if (key == 48) ROWS_LAUNCH(4, 8);
        else if (key == 44) ROWS_LAUNCH(4, 4);
        else pv.nmax = 0;                              // gemm_plan_rows makes no other: nothing launched, nothing to read
#undef ROWS_LAUNCH
        return pv;
    }
    switch (p.MB) {                                    // one or two row blocks
    case 1: SK_LAUNCH(k_gemm_sk<1>, 512); break;
    case 2: SK_LAUNCH(k_gemm_sk<2>, 512); break;
    default:                                           // plans are only ever made for 1, 2, 4 or 8 row blocks
        pv.nmax = 0;                                   // nothing launched, nothing for a consumer to read
        pv.cnt = nullptr;
        break;
    }
#undef SK_LAUNCH
#undef SK_ARGS
    return pv;
}
