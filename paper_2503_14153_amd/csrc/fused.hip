// The persistent layer kernel: every stage of the verifying pass between two attention launches in ONE
// launch of one workgroup per compute unit.
//
// Launched one kernel per stage, a decoder layer costs ten launches, and every weight-streaming GEMM starts cold:
// some 5 us pass between its first instruction and the first weight fragment's arrival from HBM, during which
// HBM idles. Here the stages of half a layer before and half a layer after an attention launch
//     merge of the attention parts -> O projection -> residual + RMSNorm -> gate/up projection -> SwiGLU
//     -> down projection -> residual + RMSNorm (next layer) -> QKV projection -> rotary embedding + tree K/V write
// run as phases of one kernel, separated by barriers across the grid, and the first ring of weight fragments of
// every GEMM is requested before the barrier that precedes it. The phases share their code with the stand-alone
// kernels (sk_gemm.h, row_ops.h); the one arithmetic difference is that the two RMSNorms apply their 1 / rms factor
// after the following GEMM instead of before it (norm_tile in row_ops.h), so the two paths agree to rounding.
//
// Prefetch. A wave's loads return in order, so a wave with a ring in flight can neither poll a barrier nor load
// anything else before its ring has landed. Every wave therefore requests its ring after its share of the row-wise
// phase has left and before the barrier that precedes the GEMM: the polling thread's answer comes back behind its
// wave's ring, i.e. when the weights are there, and the GEMM starts at the streaming rate instead of waiting out
// the first HBM round trip after the barrier.
//
// How data passes from one phase to the next without a kernel boundary (measured on MI355X, where each of the
// eight XCDs has an L2 of its own that is not kept coherent with the others during a kernel):
//   * a producer writes what another workgroup will read with write-through stores (sc1) and waits until they are
//     acknowledged (s_waitcnt vmcnt(0)) before it arrives at the barrier; written as whole fragments (row_ops.h)
//     that wait is ~0.4 us;
//   * a consumer reads with plain loads. They cannot hit a stale line, because inside one launch every address
//     of an exchange buffer is written at most once and never read before that write (each GEMM of the launch
//     has partial-sum and operand buffers of its own; the launch boundary invalidates the L2s). Invalidating
//     the L2 instead (buffer_inv sc1) costs 10-14 us, and loads that bypass it would fetch the activations from
//     memory once per workgroup instead of once per XCD;
//   * the barrier is a counter per group of workgroups (ids equal mod 8, which the dispatcher deals to one XCD
//     each) whose last arriver bumps a global counter that all poll: 2.3 us, against 3.9 us for one flat counter.
//     Every wait is bounded: a workgroup that waits longer than the limit raises a flag that the host reports,
//     stops waiting for the rest of the launch, and the kernel still ends normally.
// All workgroups must be resident at once: the grid is 256 workgroups of 512 threads, one per compute unit, and
// the host only uses this kernel when the device can hold them (see api.hip).
#include <type_traits>
#include "sd_internal.h"
#include "sk_gemm.h"
#include "row_ops.h"

static __device__ __forceinline__ PartView part_view(const FusedGemm& g) {
    PartView pv;
    pv.base = g.out; pv.slot_stride = g.slot_stride; pv.ld = g.ldo; pv.cnt = g.cnt; pv.nmax = g.nmax;
    return pv;
}

// Barrier across the grid, with a bounded wait. epoch counts the barriers of this launch (the counters start at
// zero). What a wave wrote for other workgroups must have been acknowledged before it comes here (drain()).
// Returns false once a wait has given up; the caller then skips all later waits.
static __device__ __forceinline__ bool grid_barrier(const FusedSync& sy, unsigned epoch, unsigned G, int* lds_flag) {
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned grp = blockIdx.x & 7u, ngrp = G < 8u ? G : 8u;
        const unsigned per = (G - grp + 7u) >> 3;                   // workgroups with id = grp (mod 8)
        unsigned* gc = sy.counters + grp * 64;                      // 256 bytes apart
        unsigned* all = sy.counters + 8 * 64;
        const unsigned old = __hip_atomic_fetch_add(gc, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old + 1 == epoch * per) __hip_atomic_fetch_add(all, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int ok = 1;
        const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
        unsigned spins = 0;
        while (__hip_atomic_load(all, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < epoch * ngrp) {
            __builtin_amdgcn_s_sleep(1);
            if ((++spins & 15u) == 0 || sy.timeout_ticks == 0) {
                const bool late = __builtin_amdgcn_s_memrealtime() - t0 >= sy.timeout_ticks;
                if (late || __hip_atomic_load(sy.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
                    __hip_atomic_store(sy.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    ok = 0;
                    break;
                }
            }
        }
        *lds_flag = ok;
    }
    __syncthreads();
    return *lds_flag != 0;
}
// every vector memory operation of this wave has completed: its write-through stores have reached memory
static __device__ __forceinline__ void drain() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <int MT>
__global__ __launch_bounds__(512, MT == 8 ? 1 : 2) void k_layer(const FusedArgs a) {
    __shared__ bf16x8 xs[SK_LDS_UNITS];
    __shared__ float scale_lds[SK_LDS_SCALE_FLOATS];
    __shared__ int sync_flag;
    const unsigned G = gridDim.x, g = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const unsigned gw = g * 8 + wave, GW = G * 8;          // this wave's index among all waves of the grid
    unsigned epoch = 0;
    bool waiting = true;                                   // false once a wait has given up
    bool started = false;                                  // something of this launch has run already
    int stamp = 0;
    auto mark = [&]() {                                    // diagnostic time line, see sd_set_layer_timeline
        if (a.timeline && tid == 0 && stamp < 24) a.timeline[(size_t)stamp * G + g] = __builtin_amdgcn_s_memrealtime();
        ++stamp;
    };
    auto barrier = [&]() {
        if (waiting) waiting = grid_barrier(a.sync, ++epoch, G, &sync_flag);
    };
    const int M = a.M, MB = a.MB, d = a.d, Mp = MT * 32;
    SkGemm<MT> gm;

    // One row-wise phase followed by the GEMM that consumes its output. `rows`: the phase's work for one wave.
    auto pair = [&](const FusedGemm& fg, auto scaled, auto&& rows) {
        mark();                                            // [4p] the GEMM before (if any) has issued its last store
        if (started) {
            drain();                                       // this wave's partial tiles have left
            barrier();
        }
        started = true;
        mark();                                            // [4p+1] row-wise phase starts
        rows();
        drain();
        mark();                                            // [4p+2] ... and its results have left this workgroup
        gm.setup(fg.X, fg.W, a.zfrag, fg.out, fg.KB, fg.NB, fg.ldo, fg.slot_stride, fg.upw, fg.rem, fg.kb_magic, fg.slot0,
                 (int)g, fg.G);
        gm.issue_ring();                                   // the first ring sets out while the grid gathers
        barrier();
        mark();                                            // [4p+3] GEMM starts
        gm.issue_x();
        gm.template run<decltype(scaled)::value>(xs, fg.sc, scale_lds);
    };

    if (a.phases & FUSED_GEMM_O) {                         // attention parts -> O projection
        pair(a.g_o, std::false_type{}, [&]() {
            const unsigned nk = (unsigned)a.hd >> 4, TB = (unsigned)a.Tp >> 5, total = (unsigned)a.B * a.nh * TB * nk;
            for (unsigned item = gw; item < total; item += GW) {
                const unsigned kbh = item % nk, r1 = item / nk, tblk = r1 % TB, r2 = r1 / TB;
                const unsigned h = r2 % (unsigned)a.nh, b = r2 / (unsigned)a.nh;
                attn_merge_item<true>(a.opart, a.mlpart, a.att, a.nh, a.hd, a.Tp, a.nparts, MB, b, h,
                                      tblk * 32 + (lane & 31), kbh * 2 + (lane >> 5));
            }
        });
    }
    if (a.phases & FUSED_GEMM_GU) {                        // x += O partials, norm -> gate/up projection
        const PartView pv = part_view(a.g_o);
        pair(a.g_gu, std::true_type{}, [&]() {
            const unsigned nkb = (unsigned)d >> 4, total = ((unsigned)M >> 5) * nkb;
            for (unsigned item = gw; item < total; item += GW)
                norm_tile<true>(a.x, pv, a.gain_f, a.xn_f, a.ssq_f, d, MB, Mp, item / nkb, item % nkb, lane);
        });
    }
    if (a.phases & FUSED_GEMM_DN) {                        // SwiGLU -> down projection
        const PartView pv = part_view(a.g_gu);
        pair(a.g_dn, std::false_type{}, [&]() {
            const unsigned nkb = (unsigned)a.F >> 4, total = ((unsigned)M >> 5) * nkb;
            for (unsigned item = gw; item < total; item += GW)
                swiglu_item<true>(pv, a.F, a.Fpad, a.act, MB, (item / nkb) * 32 + (lane & 31), (item % nkb) * 2 + (lane >> 5));
        });
    }
    if (a.phases & FUSED_GEMM_Q) {                         // x += down partials (or what the caller says), norm -> QKV / LM head
        PartView pv = part_view(a.g_dn);
        if (!(a.phases & FUSED_GEMM_DN)) pv = a.prev;
        pair(a.g_q, std::true_type{}, [&]() {
            const unsigned nkb = (unsigned)d >> 4, total = ((unsigned)M >> 5) * nkb;
            for (unsigned item = gw; item < total; item += GW)
                norm_tile<true>(a.x, pv, a.gain_a, a.xn_a, a.ssq_a, d, MB, Mp, item / nkb, item % nkb, lane);
        });
    }
    if (a.phases & FUSED_ROPE) {                           // rotary embedding, tree K/V rows: all eight waves
        mark();
        drain();
        barrier();
        mark();
        const PartView pv = part_view(a.g_q);
        const unsigned na = (unsigned)a.hd >> 4, han = (unsigned)a.nh * na, total = 3u * (unsigned)M * han;
        for (unsigned item = g * 512u + tid; item < total; item += G * 512u) {
            const unsigned ha = item % han, r1 = item / han, m = r1 % (unsigned)M, which = r1 / (unsigned)M;
            const unsigned b = m / (unsigned)a.Tp, t = m % (unsigned)a.Tp;
            rope_kv_item<true>(pv, a.rt, a.q, a.kt, a.vt, a.Tp, a.nh, a.hd, which, ha / na, ha % na, t, b);
        }
    }
    mark();
}

int fused_max_resident(int device) {
    // workgroups of the persistent kernel the device can hold at once (all row-block variants are checked)
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return 0;
    int worst = 1 << 30;
    const void* fns[3] = {(const void*)k_layer<1>, (const void*)k_layer<2>, (const void*)k_layer<8>};
    for (const void* fn : fns) {
        int per_cu = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, 512, 0) != hipSuccess) return 0;
        worst = per_cu * cus < worst ? per_cu * cus : worst;
    }
    return worst;
}

void launch_layer(const FusedArgs& a, int G, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1) {
#define LAYER_LAUNCH(MT_)                                                                            \
    do {                                                                                             \
        if (ev0 || ev1) hipExtLaunchKernelGGL(k_layer<MT_>, dim3(G), dim3(512), 0, s, ev0, ev1, 0, a); \
        else hipLaunchKernelGGL(k_layer<MT_>, dim3(G), dim3(512), 0, s, a);                          \
    } while (0)
    switch (a.MB) {
    case 1: LAYER_LAUNCH(1); break;
    case 2: LAYER_LAUNCH(2); break;
    case 8: LAYER_LAUNCH(8); break;
    default: break;                                        // the caller only comes here with 1, 2 or 8 row blocks
    }
#undef LAYER_LAUNCH
}
