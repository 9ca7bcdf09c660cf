// Tree-masked attention over the KV cache (the verifying pass of one speculative step).
//
// Every tree node attends all committed cache rows plus its own ancestors in the tree. The
// cache part is a pure stream: K and V of each head are read once from HBM and reused by all
// T queries of that head, so the kernel is HBM-bound and is organised around that stream:
//   * keys and values are stored as ready-made MFMA fragments (see sd_internal.h), so a
//     32-row block is sixteen contiguous 1 KiB pieces that go from memory to registers to the
//     matrix core without a transpose or a pass through LDS;
//   * S^T = K Q^T puts query t in lane t%32, and the value rows inside a block are permuted
//     so that exp(S) -- still in the accumulator registers -- already is the B operand of
//     O^T = V^T P^T: no cross-lane traffic between the two products;
//   * K and V are bf16 (the cache's storage type) but queries and probabilities are not: both
//     enter their MFMAs as two-term bf16 expansions (hi + lo), paid for with matrix-core time
//     that an HBM-bound kernel has to spare;
//   * the cache range is split over workgroups (split-KV) and over the four waves of each;
//     the waves merge through LDS, the workgroups' partial (max, sum, O) triples are merged
//     by a second small kernel, which also emits the packed bf16 operand of the O-projection.
#include "sd_internal.h"
#include "row_ops.h"

#define NEG_INF (-__builtin_inff())

// grid: x = part, y = head * TG + tg (query-block group), z = sequence. Cache part p owns the
// cache blocks [p*per, (p+1)*per) of the head. The tree blocks go to a part of their own (short
// contexts: one more workgroup per head, running beside the others) or to the last cache part
// (long contexts, where every workgroup slot of the chip is wanted for the stream).
// One workgroup = 4 waves, one per SIMD; each wave takes a contiguous quarter of the part's
// blocks, so it reads two plain sequential streams (its K blocks and its V blocks), the access
// pattern that streams fastest from HBM.
//
// Every wave keeps a ring of two blocks of K and V in registers (the fragments are MFMA operands
// as loaded): block j+2 is requested as soon as block j's registers have been multiplied, so
// between one and two blocks (16-32 KiB) are in flight per wave while it works; the loads are
// plain and unconditional, so the compiler counts them exactly (one vmcnt step per fragment).
// The first two blocks of every wave are requested before the sequence length is known (the
// host's bound fixes the geometry; a block past the end is fetched, in bounds, and ignored).
// The queries of the head sit in LDS, shared by the four waves; they get there by direct
// global-to-LDS loads issued from inline assembly, which the compiler does not count: each wave
// waits for vmcnt(0) once, before the barrier that publishes the queries.
//
// The running maximum is only raised when a block's maximum exceeds it by more than 2^8: the
// softmax is invariant to the reference point, exp2 of at most 8 cannot overflow anything, and
// the accumulators are then rescaled a few times per stream instead of once per block.
#define SD_LAZY_MAX 8.0f

static __device__ __forceinline__ void lds_dma16(const void* src_lane, uint32_t lds_byte_addr) {
    // lane i's 16 bytes land at lds_byte_addr + 16 * i; M0 (the LDS base of the load) is put back
    uint32_t saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0) : "s"(lds_byte_addr), "v"(src_lane) : "memory");
}
// x *= alpha for an accumulator that lives in an AGPR (keeps the compiler from moving the whole
// accumulator set to VGPRs and back around the rarely taken rescaling branch)
static __device__ __forceinline__ void acc_scale(float& x, float alpha) {
    float t;
    asm volatile("v_accvgpr_read_b32 %1, %0\n\tv_mul_f32 %1, %1, %2\n\tv_accvgpr_write_b32 %0, %1"
                 : "+a"(x), "=&v"(t) : "v"(alpha));
}
template <int N> static __device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }

// AW = ancestor words a query row needs: 4 for trees of up to 128 nodes, 8 beyond
// FR ("from the projection"): there is no rotary-embedding launch before this one. The workgroup builds the queries
// of its head itself, from the QKV projection's partial sums (slot sums, rotation, two-term expansion, straight into
// the LDS area the loop reads them from), and the workgroup that reads the tree blocks first builds the tree's keys
// and values the same way, writes them to the tree scratch (the commit stage needs them there) and reads them back
// as blocks. One query group only (Tp = 32 * TBW). NS: the projection's slot count if the same everywhere, else 0.
template <int HD, int TBW, int AW, int FR = 0, int NS = 0>
__global__ __launch_bounds__(256) void k_tree_attn(const bf16x8* __restrict__ Qp, const bf16x8* Kc, const bf16x8* Vc,
                                                   const bf16x8* Kt, const bf16x8* Vt, const int32_t* __restrict__ kv_len,
                                                   const uint32_t* __restrict__ anc, float* __restrict__ opart,
                                                   float2* __restrict__ mlpart, int nh, int Tp, int cap_blocks,
                                                   int ncparts, int per, int tree_sep, float scale_log2,
                                                   int xcd_stride, int nseq, PartView pv, RowTable rt) {
    constexpr int KK = HD / 16;        // contraction steps of QK^T = K fragments per block
    constexpr int EB = HD / 32;        // 32-wide output blocks of PV
    constexpr int NV = 2 * EB;         // V fragments per block
    constexpr int BLK = HD * 4;        // bf16x8 units per 32-row block
    constexpr int QF = TBW * KK * 2;   // query fragments held in LDS
    constexpr int QW = QF / 4;         // of which every wave fetches this many
    constexpr int NT = TBW * EB;       // 32x32 output tiles of one wave
    constexpr int WAVE_UNITS = NT * 4 * 64;          // 16-byte units of one wave's O in the merge buffer
    static_assert(4 * TBW * 2 * 64 * 4 <= QF * 1024, "merge scalars must fit the query area");
    __shared__ __attribute__((aligned(1024))) bf16x8 lds[QF * 64 + 4 * WAVE_UNITS];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, tl = lane & 31;
    const int TB = Tp / 32, TG = TB / TBW;
    const int nparts = ncparts + tree_sep;             // tree_sep: parts that hold tree blocks only (0, 1, or one per block)
    int part, h, tg, b;
    if (xcd_stride == 0) {                             // grid (part, head x query group, sequence)
        part = blockIdx.x;
        h = blockIdx.y / TG;
        tg = blockIdx.y % TG;
        b = blockIdx.z;
    } else if (xcd_stride < 0) {
        // One query group, a multiple of eight heads: grid (head, part, sequence). Workgroups are dealt to the eight
        // XCDs round-robin, so the parts of a head share an L2: what every part of a head fetches alike (the queries;
        // under FR the projection's partial sums they are built from, the same bytes for every part) comes from
        // memory once per head instead of once per part.
        h = blockIdx.x;
        tg = 0;
        part = blockIdx.y;
        b = blockIdx.z;
    } else {
        // Several query groups: one-dimensional grid in which the query groups of one (sequence, head, part)
        // lie xcd_stride workgroups apart. Workgroups are dealt to the eight XCDs round-robin and the stride
        // is a multiple of eight, so the groups that read the same K/V blocks share an L2 and those blocks
        // come from HBM once. Workgroups of the padding leave at once.
        tg = blockIdx.x / xcd_stride;
        const int combo = blockIdx.x - tg * xcd_stride;
        if (combo >= nparts * nh * nseq) return;
        part = combo % nparts;
        const int hb = combo / nparts;
        h = hb % nh;
        b = hb / nh;
    }
    bf16x8* qs = lds;
    const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) bf16x8*)lds);
    const uint32_t myq_addr = __builtin_amdgcn_readfirstlane(lds_addr + wave * QW * 1024);
    const bool has_cache = part < ncparts;
    // Tree blocks of this part: all of them up to the query group's own (later ones hold no ancestors) in the last
    // part, or, when every tree block has a part of its own (tree_sep >= 2, one query group), block part - ncparts.
    const bool split_tree = tree_sep >= 2;
    const int tb0 = (split_tree && part >= ncparts) ? part - ncparts : 0;
    const int ntree = split_tree ? (part >= ncparts ? 1 : 0) : ((part == nparts - 1) ? tg * TBW + TBW : 0);

    // ancestor words of this lane's query rows: only the part with the tree blocks masks by them
    static_assert(SD_ANC_WORDS == 8 && (AW == 4 || AW == 8), "one or two 16-byte loads per row");
    uint4 ancq[TBW][AW / 4];
#pragma unroll
    for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
        for (int q = 0; q < AW / 4; ++q) ancq[tb][q] = make_uint4(0u, 0u, 0u, 0u);
    if (ntree) {
#pragma unroll
        for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
            for (int q = 0; q < AW / 4; ++q)
                ancq[tb][q] = *(const uint4*)(anc + ((size_t)b * Tp + (tg * TBW + tb) * 32 + tl) * SD_ANC_WORDS + 4 * q);
    }

    // The part's items: its tree blocks first, then its cache blocks; wave w owns items
    // [w*share, (w+1)*share). Which of them exist depends on the sequence length, known later.
    const int c0 = part * per;
    const int total = ntree + (has_cache ? per : 0);
    const int share = (total + 3) >> 2;
    const int jw = __builtin_amdgcn_readfirstlane(wave * share);
    const bf16x8* kcb = Kc + ((size_t)b * nh + h) * cap_blocks * BLK + lane;
    const bf16x8* vcb = Vc + ((size_t)b * nh + h) * cap_blocks * BLK + lane;
    const bf16x8* ktb = Kt + ((size_t)b * nh + h) * TB * BLK + lane;
    const bf16x8* vtb = Vt + ((size_t)b * nh + h) * TB * BLK + lane;
    // item -> block address, always inside the tree scratch or the cache allocation
    auto kaddr = [&](int j) -> const bf16x8* {
        j = min(j, total - 1);
        return (j < ntree) ? ktb + (size_t)(tb0 + j) * BLK : kcb + (size_t)min(c0 + j - ntree, cap_blocks - 1) * BLK;
    };
    auto vaddr = [&](int j) -> const bf16x8* {
        j = min(j, total - 1);
        return (j < ntree) ? vtb + (size_t)(tb0 + j) * BLK : vcb + (size_t)min(c0 + j - ntree, cap_blocks - 1) * BLK;
    };
    // FR: a workgroup whose items are tree blocks only (the tree has a part of its own) keeps the blocks it builds in
    // LDS too (in the area the final merge uses, which is idle until the loop is over) and reads its operands from
    // there: no wait for the stores to the scratch, no round trip to read them back.
    bf16x8* const tkv = lds + QF * 64;                 // K blocks of the tree, then its V blocks
    const bool tree_only = FR && ntree && !has_cache;  // (workgroup-uniform)
    if constexpr (FR) {
        static_assert(2 * TBW * BLK <= 4 * WAVE_UNITS, "the tree blocks fit the merge area");
        if (ntree) {                                   // (workgroup-uniform) the tree's keys and values of this head
            constexpr int NA = HD / 16;                // pieces of 8 dims + their rotary partners per row
            uint16_t* ktw = (uint16_t*)const_cast<bf16x8*>(Kt);
            uint16_t* vtw = (uint16_t*)const_cast<bf16x8*>(Vt);
            uint16_t* kcp = tree_only ? (uint16_t*)tkv : nullptr;
            uint16_t* vcp = tree_only ? (uint16_t*)(tkv + TBW * BLK) : nullptr;
            constexpr int TPC = TBW * 32;              // = Tp here; compile-time trip counts: no guard between the items' loads
            static_assert((2 * 32 * NA) % 256 == 0, "whole rounds");
            if (split_tree) {                          // the 32 rows of this part's block
#pragma unroll
                for (int u = 0; u < 2 * 32 * NA / 256; ++u) {
                    const int it = u * 256 + tid;
                    const int which = 1 + it / (32 * NA), rem_ = it % (32 * NA);
                    rope_kv_item<true, NS>(pv, rt, nullptr, ktw, vtw, TPC, nh, HD, which, h, rem_ % NA, tb0 * 32 + rem_ / NA, b, 0, kcp, vcp);
                }
            } else {
#pragma unroll
                for (int u = 0; u < 2 * TPC * NA / 256; ++u) {
                    const int it = u * 256 + tid;
                    const int which = 1 + it / (TPC * NA), rem_ = it % (TPC * NA);
                    rope_kv_item<true, NS>(pv, rt, nullptr, ktw, vtw, TPC, nh, HD, which, h, rem_ % NA, rem_ / NA, b, 0, kcp, vcp);
                }
            }
            if (!tree_only) {
                wait_vm<0>();                          // the stores have reached L2 ...
                __syncthreads();                       // ... of every wave, before any wave reads the blocks back
            }
        }
    }
    bf16x8 kr[2][KK], vr[2][NV];
    auto request_k = [&](bf16x8(&kd)[KK], int j) {
        const bf16x8* kp = kaddr(j);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kd[kk] = __builtin_nontemporal_load(kp + kk * 64);
    };
    auto request_v = [&](bf16x8(&vd)[NV], int j) {
        const bf16x8* vp = vaddr(j);
#pragma unroll
        for (int i = 0; i < NV; ++i) vd[i] = __builtin_nontemporal_load(vp + i * 64);
    };
    auto lds_k = [&](bf16x8(&kd)[KK], int j) {
        const bf16x8* kp = tkv + (size_t)(tb0 + min(j, total - 1)) * BLK + lane;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kd[kk] = kp[kk * 64];
    };
    auto lds_v = [&](bf16x8(&vd)[NV], int j) {
        const bf16x8* vp = tkv + (size_t)(TBW + tb0 + min(j, total - 1)) * BLK + lane;
#pragma unroll
        for (int i = 0; i < NV; ++i) vd[i] = vp[i * 64];
    };
    if (!tree_only) { request_k(kr[0], jw); request_v(vr[0], jw); request_k(kr[1], jw + 1); request_v(vr[1], jw + 1); }
    if constexpr (FR) {                                // queries of this head, built here, -> LDS
        constexpr int NA = HD / 16;
        const size_t q_unit0 = ((size_t)b * nh + h) * TB * (KK * 2 * 64);
        constexpr int TPC = TBW * 32;
        static_assert((TPC * NA) % 256 == 0 || TPC * NA < 256, "whole rounds, or a part of one");
#pragma unroll
        for (int u = 0; u < (TPC * NA + 255) / 256; ++u) {
            const int it = u * 256 + tid;
            if (TPC * NA >= 256 || it < TPC * NA)
                rope_kv_item<true, NS>(pv, rt, (bf16x8*)lds, nullptr, nullptr, TPC, nh, HD, 0, h, it % NA, it / NA, b, q_unit0);
        }
    } else {   // queries of this (sequence, head, query group) -> LDS, a quarter per wave
        const bf16x8* qsrc = Qp + (((size_t)b * nh + h) * TB + tg * TBW) * (KK * 2 * 64) + lane;
#pragma unroll
        for (int i = 0; i < QW; ++i) lds_dma16(qsrc + (wave * QW + i) * 64, myq_addr + i * 1024);
    }

    const int n = kv_len[b];
    const int nblk = (n + 31) >> 5;
    const int ncache = has_cache ? max(0, min(per, nblk - c0)) : 0;
    const int nit = __builtin_amdgcn_readfirstlane(max(0, min(share, ntree + ncache - jw)));       // this wave's items [jw, jw + nit)

    f32x16 O[TBW][EB];
    float mrun[TBW], lrun[TBW];
#pragma unroll
    for (int tb = 0; tb < TBW; ++tb) {
        mrun[tb] = NEG_INF;
        lrun[tb] = 0.f;
#pragma unroll
        for (int eb = 0; eb < EB; ++eb)
#pragma unroll
            for (int v = 0; v < 16; ++v) O[tb][eb][v] = 0.f;
    }

    // QK^T of one block. The query operands come from LDS in stages of one contraction step (the
    // 2*TBW query fragments that meet one K fragment); two stages are requested ahead of the one
    // being multiplied, and the scheduler is fenced so that it keeps them that far ahead.
    auto qk = [&](const bf16x8(&ks)[KK], f32x16(&S)[TBW]) {
        int ql = lane;
        asm volatile("" : "+v"(ql));       // keep the query reads in the loop: hoisted, they cost 128 registers
        bf16x8 st[3][1 + 2 * TBW];
        auto stage = [&](int si, int kk) {
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
#pragma unroll
                for (int tb = 0; tb < TBW; ++tb) st[si][1 + pt * TBW + tb] = qs[((tb * KK + kk) * 2 + pt) * 64 + ql];
        };
        stage(0, 0);
        stage(1, 1);
#pragma unroll
        for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
            for (int v = 0; v < 16; ++v) S[tb][v] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            if (kk + 2 < KK) stage((kk + 2) % 3, kk + 2);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
#pragma unroll
                for (int tb = 0; tb < TBW; ++tb)
                    S[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ks[kk], st[kk % 3][1 + pt * TBW + tb], S[tb], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // softmax of the block's scores for both query blocks, then PV
    auto softmax_pv = [&](const bf16x8(&vf)[NV], f32x16(&S)[TBW], int it) {
        const int j = jw + it;
        const bool tr = j < ntree;
        const int blk = tr ? tb0 + j : c0 + j - ntree;
        const int left = n - blk * 32;
        const bool need_mask = tr || left < 32;                 // wave-uniform
        bf16x8 pf[TBW][2], pl[TBW][2];     // probabilities, two-term expansion
#pragma unroll
        for (int tb = 0; tb < TBW; ++tb) {
            if (need_mask) {
                uint32_t vis;
                if (tr) {
                    uint4 aq = ancq[tb][0];
                    if constexpr (AW == 8) {
                        const bool up = (blk & 4) != 0;
                        aq.x = up ? ancq[tb][1].x : aq.x; aq.y = up ? ancq[tb][1].y : aq.y;
                        aq.z = up ? ancq[tb][1].z : aq.z; aq.w = up ? ancq[tb][1].w : aq.w;
                    }
                    const uint64_t lo64 = aq.x | ((uint64_t)aq.y << 32), hi64 = aq.z | ((uint64_t)aq.w << 32);
                    vis = (uint32_t)(((blk & 2) ? hi64 : lo64) >> ((blk & 1) * 32));     // word blk of the row's ancestor set
                }
                else vis = (1u << left) - 1u;
                vis >>= 4 * g;          // lane (t = tl, g) holds rows 8*(v/4) + 4*g + v%4 of the block
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    S[tb][v] = (vis & (1u << (8 * (v >> 2) + (v & 3)))) ? S[tb][v] : NEG_INF;
            }
            float mx = S[tb][0];
#pragma unroll
            for (int v = 1; v < 16; ++v) mx = fmaxf(mx, S[tb][v]);
            mx = fmaxf(mx, __shfl_xor(mx, 32)) * scale_log2;
            const bool upd = mx > mrun[tb] + SD_LAZY_MAX;
            if (__any(upd)) {
                const float alpha = upd ? __builtin_amdgcn_exp2f(mrun[tb] - mx) : 1.f;
                mrun[tb] = upd ? mx : mrun[tb];
                lrun[tb] *= alpha;
                asm volatile("s_nop 7\n\ts_nop 7");          // the last PV product has long left the pipe; be explicit
#pragma unroll
                for (int eb = 0; eb < EB; ++eb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) { float x = O[tb][eb][v]; acc_scale(x, alpha); O[tb][eb][v] = x; }
                asm volatile("s_nop 7");
            }
            const float muse = (mrun[tb] == NEG_INF) ? 0.f : mrun[tb];
            float psum = 0.f;
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(S[tb][8 * p + s], scale_log2, -muse));
                    psum += pv;
                    const __bf16 hi = (__bf16)pv;
                    pf[tb][p][s] = hi;
                    pl[tb][p][s] = (__bf16)(pv - (float)hi);
                }
            lrun[tb] += psum;
        }
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int eb = 0; eb < EB; ++eb) {
#pragma unroll
                for (int tb = 0; tb < TBW; ++tb)
                    O[tb][eb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[p * EB + eb], pf[tb][p], O[tb][eb], 0, 0, 0);
#pragma unroll
                for (int tb = 0; tb < TBW; ++tb)
                    O[tb][eb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[p * EB + eb], pl[tb][p], O[tb][eb], 0, 0, 0);
            }
    };

    // Everything this wave has requested so far has landed, its quarter of the queries included. (No
    // smaller count is safe: the ring's loads are the compiler's to place, so how many of them follow
    // the query loads in the instruction stream is not known here.)
    wait_vm<0>();
    __syncthreads();                                   // queries are in LDS
    // the loop in two copies, so that each has loads of one kind in a straight line (a branch around a load makes the
    // compiler wait for everything in flight)
    auto run_items = [&](auto&& req_k, auto&& req_v) {
        for (int it = 0; it < nit; it += 2) {
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const bool live = it + r < nit;
                f32x16 S[TBW];
                if (live) qk(kr[r], S);
                req_k(kr[r], jw + min(it + r + 2, nit - 1));   // past the wave's last item: that item again
                if (live) softmax_pv(vr[r], S, it + r);
                req_v(vr[r], jw + min(it + r + 2, nit - 1));
            }
        }
    };
    if (FR && tree_only) {
        lds_k(kr[0], jw); lds_v(vr[0], jw); lds_k(kr[1], jw + 1); lds_v(vr[1], jw + 1);
        if (nit > 0) run_items(lds_k, lds_v);
    } else if (nit > 0) {
        run_items(request_k, request_v);
    }

    // ---- merge the four waves. Every wave parks its O tiles in its own part of LDS and its (max, sum)
    //      pairs in the query area; then the NT output tiles are shared out over the waves, each
    //      combining the four contributions to its tiles and writing them straight to the partials.
    float4* mo_all = (float4*)(lds + QF * 64);         // [wave][tile][i = 0..3][lane] as float4
    float* mml = (float*)lds;                          // [wave][tb][2][64]
    constexpr int WAVE_F4 = WAVE_UNITS;                // one float4 per 16-byte unit
    __syncthreads();                                   // all waves are done with the queries
#pragma unroll
    for (int tb = 0; tb < TBW; ++tb) {
#pragma unroll
        for (int eb = 0; eb < EB; ++eb)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                mo_all[wave * WAVE_F4 + ((tb * EB + eb) * 4 + i) * 64 + lane] =
                    make_float4(O[tb][eb][4 * i], O[tb][eb][4 * i + 1], O[tb][eb][4 * i + 2], O[tb][eb][4 * i + 3]);
        mml[((wave * TBW + tb) * 2 + 0) * 64 + lane] = mrun[tb];
        mml[((wave * TBW + tb) * 2 + 1) * 64 + lane] = lrun[tb];
    }
    __syncthreads();
    for (int ti = wave; ti < NT; ti += 4) {
        const int tb = ti / EB, eb = ti % EB;
        float mw[4], lw[4], M = NEG_INF;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            mw[w] = mml[((w * TBW + tb) * 2 + 0) * 64 + lane];
            lw[w] = mml[((w * TBW + tb) * 2 + 1) * 64 + lane];
            M = fmaxf(M, mw[w]);
        }
        const float Muse = (M == NEG_INF) ? 0.f : M;
        float L = 0.f, sc[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            sc[w] = exp2f(mw[w] - Muse);               // exp2(-inf) = 0 for a wave that saw nothing
            L += sc[w] * lw[w];
        }
        const int t = (tg * TBW + tb) * 32 + tl;
        const size_t row = (((size_t)b * nh + h) * nparts + part) * Tp + t;
        if (eb == 0) {
            const float ltot = L + __shfl_xor(L, 32);
            if (g == 0) mlpart[row] = make_float2(M, ltot);
        }
        float* o = opart + row * HD;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float4 x = mo_all[w * WAVE_F4 + (ti * 4 + i) * 64 + lane];
                acc.x += sc[w] * x.x; acc.y += sc[w] * x.y; acc.z += sc[w] * x.z; acc.w += sc[w] * x.w;
            }
            *(float4*)(o + eb * 32 + 8 * i + 4 * g) = acc;
        }
    }
}

// qkv: NULL (the queries and the tree's keys / values were made by launch_rope_kv), or the QKV projection's partial
// sums: then this launch makes them itself (one query group only: Tp <= 64), and `rt` gives the rotation table
void launch_tree_attn(const void* q_packed, const void* kc, const void* vc, const void* kt, const void* vt,
                      const int32_t* kv_len, const uint32_t* anc, float* opart, float2* mlpart, int B, int nh,
                      int hd, int Tp, int cap_blocks, int ncparts, int per, int tree_sep, hipStream_t s, hipEvent_t ev0,
                      hipEvent_t ev1, const PartView* qkv, const RowTable* rt) {
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)hd);
    const int TB = Tp / 32;
    const int TBW = (TB % 2 == 0) ? 2 : 1;
    const int nparts = ncparts + tree_sep, TG = TB / TBW;     // tree_sep: number of parts with tree blocks only
    dim3 grid(nparts, nh * TG, B);
    int xcd_stride = 0;
    if (TG > 1) {                                      // query groups of one head on one XCD (see the kernel)
        xcd_stride = (nparts * nh * B + 7) / 8 * 8;
        grid = dim3(xcd_stride * TG, 1, 1);
    } else if (nh % 8 == 0 && nparts > 1) {            // parts of one head on one XCD
        xcd_stride = -1;
        grid = dim3(nh, nparts, B);
    }
#define ATT_ARGS (const bf16x8*)q_packed, (const bf16x8*)kc, (const bf16x8*)vc, (const bf16x8*)kt, (const bf16x8*)vt, \
                 kv_len, anc, opart, mlpart, nh, Tp, cap_blocks, ncparts, per, tree_sep, scale_log2, xcd_stride, B, pv_arg, rt_arg
#define ATT(HD_, TBW_, AW_, ...)                                                                                     \
    do {                                                                                                        \
        if (ev0 || ev1)                                                                                         \
            hipExtLaunchKernelGGL((k_tree_attn<HD_, TBW_, AW_, ##__VA_ARGS__>), grid, dim3(256), 0, s, ev0, ev1, 0, ATT_ARGS); \
        else                                                                                                    \
            hipLaunchKernelGGL((k_tree_attn<HD_, TBW_, AW_, ##__VA_ARGS__>), grid, dim3(256), 0, s, ATT_ARGS);  \
    } while (0)
#define ATT2(HD_, TBW_) do { if (Tp > 128) ATT(HD_, TBW_, 8); else ATT(HD_, TBW_, 4); } while (0)
    PartView pv_arg = {nullptr, 0, 0, nullptr, 0};
    RowTable rt_arg = {nullptr, nullptr, nullptr, nullptr};
    if (qkv && rt && TG == 1) {
        pv_arg = *qkv;
        rt_arg = *rt;
        const bool four = qkv->cnt == nullptr && qkv->nmax == 4;     // the aligned QKV plan of the 7B and 13B shapes
#define ATT_FR(HD_, TBW_) do { if (four) ATT(HD_, TBW_, 4, 1, 4); else ATT(HD_, TBW_, 4, 1, 0); } while (0)
        if (hd == 128) { if (TBW == 2) ATT_FR(128, 2); else ATT_FR(128, 1); }
        else           { if (TBW == 2) ATT_FR(64, 2);  else ATT_FR(64, 1); }
#undef ATT_FR
    }
    else if (hd == 128) { if (TBW == 2) ATT2(128, 2); else ATT2(128, 1); }
    else                { if (TBW == 2) ATT2(64, 2);  else ATT2(64, 1); }
#undef ATT2
#undef ATT
#undef ATT_ARGS
}

// ------------------------------------------------------------------------------------------
// Merge the split-KV partials and emit the packed bf16 operand of the O-projection (body: row_ops.h).
// one thread per (seq, head, query t, 8 consecutive output dims), grid (chunks of t x dims, head, seq)
__global__ void k_attn_merge(const float* __restrict__ opart, const float2* __restrict__ mlpart,
                             bf16x8* __restrict__ xp, int nh, int hd, int e8_shift, int Tp, int nparts, int MB) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;      // hd / 8 = 1 << e8_shift pieces per query row
    const int e8 = idx & ((1 << e8_shift) - 1), t = idx >> e8_shift;
    if (t >= Tp) return;
    attn_merge_item<false>(opart, mlpart, xp, nh, hd, Tp, nparts, MB, /*b=*/blockIdx.z, /*h=*/blockIdx.y, t, e8);
}

void launch_attn_merge(const float* opart, const float2* mlpart, void* x_packed, int B, int nh, int hd, int Tp,
                       int nparts, int MB, hipStream_t s) {
    const int e8_shift = hd == 128 ? 4 : 3;            // head_dim is 128 or 64
    hipLaunchKernelGGL(k_attn_merge, dim3((Tp * (hd / 8) + 255) / 256, nh, B), dim3(256), 0, s, opart, mlpart,
                       (bf16x8*)x_packed, nh, hd, e8_shift, Tp, nparts, MB);
}
