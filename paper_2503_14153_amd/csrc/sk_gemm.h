// The weight-streaming GEMM of the verifying pass as a device function, shared by the stand-alone kernel
// (gemm.hip) and the persistent layer kernel (fused.hip). See gemm.hip for the design.
#pragma once
#include "sd_internal.h"

struct SkIter { int kb, ng, valid, last; };

// A workgroup's walk over its unit range [u, u1) in outer iterations of R steps, without any division
// after the first position: the next iteration starts at (ng, kb), covers min(R, rest of the segment)
// steps and is the segment's last if the segment ends within it.
struct SkWalk { int u, u1, ng, kb; };
// kb_magic = ceil(2^32 / KB): u / KB = high word of u * kb_magic for every u < 2^32 / KB (units number < 2^20)
static __device__ inline SkWalk sk_walk_init(int g, int upw, int rem, int KB, uint32_t kb_magic) {
    SkWalk w;
    w.u = g * upw + (g < rem ? g : rem);               // workgroup g takes upw units, the first `rem` one more
    w.u1 = w.u + upw + (g < rem ? 1 : 0);
    w.ng = KB == 1 ? w.u : (int)__umulhi((uint32_t)w.u, kb_magic);
    w.kb = w.u - w.ng * KB;
    return w;
}
template <int R>
static __device__ inline SkIter sk_walk_next(SkWalk& w, int KB) {
    SkIter r = {0, 0, 0, 0};
    if (w.u >= w.u1) return r;
    int send = (w.ng + 1) * KB;
    if (send > w.u1) send = w.u1;
    const int len = send - w.u;
    r.kb = w.kb;
    r.ng = w.ng;
    r.valid = len < R ? len : R;
    r.last = len <= R;
    w.u += r.valid;
    w.kb += r.valid;
    if (w.kb >= KB) { w.kb = 0; ++w.ng; }
    return r;
}

// LDS the GEMM needs: two activation chunks of 16 fragments, and (for a GEMM that applies the deferred RMS scale
// of its rows) the per-row factors and the scratch of their reduction
#define SK_LDS_UNITS (2 * 16 * 64)
#define SK_LDS_SCALE_FLOATS (256 + 512)

// One weight-streaming GEMM of workgroup g (512 threads), in pieces, so that a caller can request the first ring of
// weight fragments long before the activations exist (the persistent layer kernel does, across a grid barrier):
//     setup()      the workgroup's unit range and first iterations (no memory traffic but one table entry)
//     issue_ring() requests the first R weight fragments of this wave
//     issue_x()    requests the activation chunks of the first iteration (they must have been written by now)
//     run()        the main loop and the partial-tile stores; every thread of the workgroup calls it
// A workgroup (or a whole launch) without units: has_work() is false, the other calls do nothing.
template <int MT>
struct SkGemm {
    static_assert(MT == 1 || MT == 2 || MT == 8, "four row blocks: k_gemm_sk_rows only");
    // ring depth. Eight row blocks: the 128 accumulators leave two waves per SIMD room for a ring of
    // 4 steps (210 registers), and a step then holds 16 MFMAs, so 4 steps cover the same time as 16 do
    // with two row blocks (rings of 6 and 8 steps measured slower: 62.3 and 62.8 us against 59.8)
    static constexpr int R = MT == 8 ? 4 : 16;
    static constexpr int XK = 8 / MT;                // contraction blocks per chunk
    static constexpr int CPI = R / XK;               // chunks per outer iteration (2 or 4)
    static constexpr int XF = 16;                    // fragments per chunk = XK * MT * 2
    static constexpr int XP = XF * 64 / 512;         // 16-byte pieces per thread per chunk = 2
    static constexpr int PER_KB = MT * 2 * 64;       // 16-byte units of the row blocks per contraction block

    const bf16x8 *Xp, *Wp, *zl;
    float* out;
    int KB, NB, ldo, tid, wave, lane, slot0;
    const int32_t* slot0_at;
    size_t slot_stride, wstep;
    SkWalk walk;
    SkIter cur, nxt, nx2;
    bf16x8 w[R], xr[CPI][XP];

    __device__ __forceinline__ void setup(const bf16x8* __restrict__ Xp_, const bf16x8* __restrict__ Wp_,
                                          const bf16x8* __restrict__ zfrag, float* __restrict__ out_, int KB_, int NB_,
                                          int ldo_, size_t slot_stride_, int upw, int rem, uint32_t kb_magic,
                                          const int32_t* __restrict__ slot0_tab, int g, int G) {
        Xp = Xp_; Wp = Wp_; out = out_; KB = KB_; NB = NB_; ldo = ldo_; slot_stride = slot_stride_;
        tid = threadIdx.x; wave = tid >> 6; lane = tid & 63;
        wstep = (size_t)NB * 64;
        // Every load is unconditional and its result is used as loaded: a fragment past the end of a segment is
        // fetched from a 1 KiB page of zeros (zfrag) by selecting the ADDRESS. A branch around a load, or a select
        // on its result, makes the compiler wait for the whole ring (s_waitcnt vmcnt(0)) in every iteration;
        // straight-line loads are counted exactly.
        zl = zfrag + lane;
        cur = nxt = nx2 = SkIter{0, 0, 0, 0};
        slot0 = 0;
        slot0_at = slot0_tab + (g < G ? g : 0);        // read once the ring has been issued (issue_ring)
        if (g < G) {
            walk = sk_walk_init(g, upw, rem, KB, kb_magic);
            cur = sk_walk_next<R>(walk, KB);
            nxt = sk_walk_next<R>(walk, KB);
            nx2 = sk_walk_next<R>(walk, KB);
        }
    }
    __device__ __forceinline__ bool has_work() const { return cur.valid != 0; }
    __device__ __forceinline__ const bf16x8* wptr(const SkIter& I) const {
        int nb = I.ng * 8 + wave;
        if (nb >= NB) nb = NB - 1;
        return Wp + ((size_t)I.kb * NB + nb) * 64 + lane;
    }
    __device__ __forceinline__ void xload(bf16x8 (&dst)[XP], const SkIter& I, int c) const {
        int steps = I.valid - c * XK;
        steps = steps < 0 ? 0 : (steps > XK ? XK : steps);
        const int limit = steps * PER_KB;
        const bf16x8* base = Xp + (size_t)(I.kb + c * XK) * PER_KB;
#pragma unroll
        for (int p = 0; p < XP; ++p) {
            const int i = p * 512 + tid;
            dst[p] = *((i < limit) ? base + i : zl);
        }
    }
    __device__ __forceinline__ void issue_ring() {
        if (!has_work()) return;
        const bf16x8* wc = wptr(cur);
#pragma unroll
        for (int i = 0; i < R; ++i) w[i] = __builtin_nontemporal_load((i < cur.valid) ? wc + (size_t)i * wstep : zl);
        // The slot of this workgroup's first segment (later ones: 0), wanted only when that segment ends. Read here,
        // as a vector load behind the ring, so that nothing waits for it: read in setup it was a scalar load that the
        // next wait for a kernel argument also waited for, a memory round trip before the first weight was requested.
        int zero = 0;
        asm volatile("" : "+v"(zero));              // (a vector register: the load is a vector load)
        slot0 = slot0_at[zero];
    }
    __device__ __forceinline__ void issue_x() {
        if (!has_work()) return;
#pragma unroll
        for (int c = 0; c < CPI; ++c) xload(xr[c], cur, c);
    }

    // SCALE: apply the deferred row scale sc; lds_f: SK_LDS_SCALE_FLOATS floats of LDS, used only with a scale
    template <bool SCALE>
    __device__ __forceinline__ void run(bf16x8* __restrict__ xs_flat, const SkRowScale& sc, float* __restrict__ lds_f) {
        if (!has_work()) return;
        bf16x8(*xs)[XF * 64] = (bf16x8(*)[XF * 64])xs_flat;
        auto xstore = [&](const bf16x8(&src)[XP], int buf) {
#pragma unroll
            for (int p = 0; p < XP; ++p) xs[buf][p * 512 + tid] = src[p];
        };
        f32x16 acc[MT];
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

        if constexpr (SCALE) {
            // per-row factor 1 / sqrt(mean(x^2) + eps) from the partial sums of squares, summed in a fixed order:
            // thread (row m, slice s) adds its slice of the parts in ascending order, then the slices in order.
            // The parts lie four to a float4 ([part / 4][row][part % 4]); a thread's loads are issued in batches of
            // eight before any is used (a quad index past the slice re-reads its last quad and adds nothing).
            constexpr int Mp = MT * 32, SL = 512 / Mp;
            const int m = tid % Mp, sl = tid / Mp;
            const int n_q = (sc.n_parts + 3) >> 2, per = (n_q + SL - 1) / SL, q0 = sl * per, q1 = min(q0 + per, n_q);
            const float4* sq = (const float4*)sc.ssq + m;
            float t = 0.f;
            for (int b0 = q0; b0 < q1; b0 += 8) {
                float4 v[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) v[i] = sq[(size_t)min(b0 + i, q1 - 1) * Mp];
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (b0 + i < q1) t += (v[i].x + v[i].y) + (v[i].z + v[i].w);
            }
            lds_f[256 + sl * Mp + m] = t;
            __syncthreads();
            if (tid < Mp) {
                float tot = 0.f;
#pragma unroll
                for (int q = 0; q < SL; ++q) tot += lds_f[256 + q * Mp + tid];
                lds_f[tid] = rsqrtf(tot * sc.inv_d + sc.eps);
            }
            // (the barrier below, before the first MFMA, also publishes the factors)
        }

        int nseg = 0;
        xstore(xr[0], 0);
        xload(xr[0], nxt, 0);
        __syncthreads();

        for (;;) {
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
                // slot = ordinal of this workgroup among those whose ranges meet column group cur.ng: known
                // from the plan for the first segment; every later segment starts its column group
                const int slot = nseg == 0 ? slot0 : 0;
                ++nseg;
                const int nb = cur.ng * 8 + wave;
                if (nb < NB) {
                    float* o = out + (size_t)slot * slot_stride + (size_t)nb * 32 + (lane & 31);
                    // the row stride and the lane's row group are made opaque here so that the row offsets
                    // m * ldo are computed where they are used: hoisted out of the loop (which the compiler
                    // does otherwise) they occupy registers for the whole kernel, 64 of them here and some
                    // 150 in the 128-row kernel
                    int gq = lane >> 5, ldo_here = ldo;
                    asm volatile("" : "+v"(gq), "+s"(ldo_here));
#pragma unroll
                    // write-through stores: the tiles are consumed by other XCDs anyway, and lines left dirty
                    // in this XCD's L2 would only be written back at the end of the kernel, lengthening it
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            int m = mt * 32 + 8 * (v >> 2) + 4 * gq + (v & 3);
                            float val = acc[mt][v];
                            if constexpr (SCALE) val *= lds_f[m];
                            __hip_atomic_store(&o[(size_t)m * ldo_here], val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
            nx2 = sk_walk_next<R>(walk, KB);
        }
    }
};
