// Bodies of the row-wise stages between the weight-streaming GEMMs (RMSNorm with the residual add, rotary
// embedding with the tree K/V write, SwiGLU, merge of the split-KV attention parts), as device functions of
// one work item each. The stand-alone kernels (rows.hip, attn.hip) and the persistent layer kernel (fused.hip)
// call the same functions, so both paths do the same arithmetic in the same order.
//
// WT ("write-through"): the stores of results that another workgroup of the SAME launch reads are issued with the
// write-through bit (sc1: agent scope), so that the data has left this XCD's L2 once the stores are acknowledged.
// Four-byte stores get it from an agent-scope relaxed atomic store; for 16 bytes no builtin gives it (a
// nontemporal store does NOT make the data visible to the other XCDs, measured), so those are inline assembly.
// The stand-alone kernels pass WT = false.
//
// Work items are WAVE TILES of 32 rows x 16 columns: lane l works on row (l % 32) and the 8 columns (l / 32) * 8 ..
// of its tile, which is exactly the lane order of a 1 KiB operand fragment, so a wave writes whole fragments
// (eight full 128-byte lines per store instruction). Written through as single 16-byte pieces scattered over
// as many lines, the same bytes took ten times as long to be acknowledged.
#pragma once
#include "sd_internal.h"

#define NEG_INF_F (-__builtin_inff())

static __device__ inline float bf16_bits_to_float(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

template <bool WT>
static __device__ __forceinline__ void store_frag16(bf16x8* p, const bf16x8& v) {
    if constexpr (WT) {
        // the compiler does not see this store: the s_nop covers the wait states a VALU write of the data registers
        // needs after a store of more than 8 bytes; the store is counted in vmcnt like any other, after the
        // compiler's own, so its waits can only get longer, never too short
        asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" :: "v"(p), "v"(v) : "memory");
    } else {
        *p = v;
    }
}

// Sum of the `n` partial-sum slots of eight consecutive columns at p0 (slot s lies s * stride floats further on),
// added to t[] in slot order. The loads of a batch of SLOT_BATCH slots are all issued before any is used: the
// slots sit in other XCDs' memory, a dependent chain of them costs a memory round trip each. A slot index past
// the end re-reads the last slot and adds nothing. (BATCH = false: a plain loop; as kernels of their own the
// row-wise stages measured faster that way.)
#define SLOT_BATCH 8
template <bool BATCH>
static __device__ __forceinline__ void add_slots8(float (&t)[8], const float* __restrict__ p0, size_t stride, int n) {
    if constexpr (!BATCH) {                                // one slot after the other (same sums, same order)
#pragma unroll 4
        for (int sp = 0; sp < n; ++sp) {
            const float* p = p0 + (size_t)sp * stride;
            float4 pa = *(const float4*)p, pc = *(const float4*)(p + 4);
            t[0] += pa.x; t[1] += pa.y; t[2] += pa.z; t[3] += pa.w;
            t[4] += pc.x; t[5] += pc.y; t[6] += pc.z; t[7] += pc.w;
        }
        return;
    }
    for (int s0 = 0; s0 < n; s0 += SLOT_BATCH) {
        float4 a[SLOT_BATCH], c[SLOT_BATCH];
#pragma unroll
        for (int i = 0; i < SLOT_BATCH; ++i) {
            const float* p = p0 + (size_t)min(s0 + i, n - 1) * stride;
            a[i] = *(const float4*)p;
            c[i] = *(const float4*)(p + 4);
        }
#pragma unroll
        for (int i = 0; i < SLOT_BATCH; ++i) {
            if (s0 + i < n) {
                t[0] += a[i].x; t[1] += a[i].y; t[2] += a[i].z; t[3] += a[i].w;
                t[4] += c[i].x; t[5] += c[i].y; t[6] += c[i].z; t[7] += c[i].w;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// x += sum of split partials (residual add of the previous projection), then
// xn = x * rsqrt(mean(x^2) + eps) * gain, written as bf16 in fragment order. The whole workgroup of
// NP_THREADS threads works on one row (source row `src` of x and of the partials, written as row `m` of the
// packed operand); a thread owns groups of 8 consecutive columns. `red`: NP_THREADS / 64 floats of LDS.
#define NP_THREADS 512
#define NP_MAXG 2   // d <= 8 * NP_THREADS * NP_MAXG = 8192
template <bool WT>
static __device__ __forceinline__ void norm_pack_row(float* __restrict__ x, const PartView& pv,
                                                     const uint16_t* __restrict__ gain, float eps,
                                                     bf16x8* __restrict__ xn, float* __restrict__ hf, int d, int MB,
                                                     int src, int m, float* red) {
    float* xr = x + (size_t)src * d;
    const int ngroups = d >> 3;
    float v[NP_MAXG][8];
    float ss = 0.f;
#pragma unroll
    for (int gi = 0; gi < NP_MAXG; ++gi) {
        int grp = gi * NP_THREADS + threadIdx.x;
        if (grp < ngroups) {
            float4 a = *(const float4*)(xr + grp * 8), c = *(const float4*)(xr + grp * 8 + 4);
            float t[8] = {a.x, a.y, a.z, a.w, c.x, c.y, c.z, c.w};
            const int nsplit = pv.nmax > 0 ? part_count(pv, grp * 8) : 0;
            if (nsplit > 0) add_slots8<WT>(t, pv.base + (size_t)src * pv.ld + grp * 8, pv.slot_stride, nsplit);
            if (nsplit > 0) {
                *(float4*)(xr + grp * 8) = make_float4(t[0], t[1], t[2], t[3]);
                *(float4*)(xr + grp * 8 + 4) = make_float4(t[4], t[5], t[6], t[7]);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) { v[gi][i] = t[i]; ss += t[i] * t[i]; }
        }
    }
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    ss = 0.f;
#pragma unroll
    for (int w = 0; w < NP_THREADS / 64; ++w) ss += red[w];
    const float r = rsqrtf(ss / (float)d + eps);
#pragma unroll
    for (int gi = 0; gi < NP_MAXG; ++gi) {
        int grp = gi * NP_THREADS + threadIdx.x;
        if (grp < ngroups) {
            bf16x8 hi, lo;
            float f[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) f[i] = v[gi][i] * r * bf16_bits_to_float(gain[grp * 8 + i]);
            split_hilo(f, hi, lo);
            const size_t u = xpack_index(m, grp * 8, MB) >> 3;
            store_frag16<WT>(xn + u, hi);
            store_frag16<WT>(xn + u + XPART / 8, lo);
            if (hf) {
                *(float4*)(hf + (size_t)m * d + grp * 8) = make_float4(f[0], f[1], f[2], f[3]);
                *(float4*)(hf + (size_t)m * d + grp * 8 + 4) = make_float4(f[4], f[5], f[6], f[7]);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// RMSNorm with the scale deferred, one wave tile (32 rows x 16 columns: row block mb, contraction block kb):
// x += sum of split partials (residual add), operand = bf16 two-term expansion of x * gain WITHOUT the row's
// 1 / rms factor, and part kb of ssq_part = the tile's share of sum(x^2) of row m. The GEMM that consumes the operand
// multiplies its outputs by the factor (a GEMM is linear in its rows), see SkRowScale. No reduction across the row
// is needed here, so the rows spread over the whole chip and every store is a whole fragment.
template <bool WT>
static __device__ __forceinline__ void norm_tile(float* __restrict__ x, const PartView& pv,
                                                 const uint16_t* __restrict__ gain, bf16x8* __restrict__ xn,
                                                 float* __restrict__ ssq_part, int d, int MB, int Mp, int mb, int kb,
                                                 int lane) {
    const int r = lane & 31, g = lane >> 5, m = mb * 32 + r, c0 = kb * 16 + g * 8;
    float* xr = x + (size_t)m * d + c0;
    float4 a = *(const float4*)xr, c = *(const float4*)(xr + 4);
    float t[8] = {a.x, a.y, a.z, a.w, c.x, c.y, c.z, c.w};
    const int nsplit = pv.nmax > 0 ? part_count(pv, c0) : 0;
    if (nsplit > 0) {
        add_slots8<WT>(t, pv.base + (size_t)m * pv.ld + c0, pv.slot_stride, nsplit);
        *(float4*)xr = make_float4(t[0], t[1], t[2], t[3]);
        *(float4*)(xr + 4) = make_float4(t[4], t[5], t[6], t[7]);
    }
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) ss += t[i] * t[i];
    ss += __shfl_xor(ss, 32);
    if (g == 0) {
        float* dst = ssq_part + ((size_t)(kb >> 2) * Mp + m) * 4 + (kb & 3);       // SkRowScale's layout
        if constexpr (WT) __hip_atomic_store(dst, ss, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else *dst = ss;
    }
    bf16x8 hi, lo;
    float f[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = t[i] * bf16_bits_to_float(gain[c0 + i]);
    split_hilo(f, hi, lo);
    bf16x8* dst = xn + ((size_t)(kb * MB + mb) * 2) * 64 + lane;
    store_frag16<WT>(dst, hi);
    store_frag16<WT>(dst + 64, lo);
}

// ------------------------------------------------------------------------------------------
// Sum the QKV partials, rotate q and k to the row's position, and write q (fragment order, two-term
// expansion), k and v (tree scratch, block layouts, bf16). One item = (row t of sequence b, head h, piece a,
// which): dims [8a, 8a+8) and their rotary partners [hd/2 + 8a, +8) of q (which = 0), k (1) or v (2).
// Nothing written here is read again within the launch (the attention kernel is the consumer).
// NS > 0: every column group of the QKV projection has NS slots (its plan says so): all loads in a straight line.
// q_unit0: subtracted from the 16-byte unit index of the query fragments (a caller that keeps one head's queries in a
// buffer of its own, e.g. in LDS, passes that head's offset). k_copy / v_copy: if not NULL, this head's key / value
// blocks are written there as well (block layouts, offsets within the head).
template <bool BATCH, int NS = 0>
static __device__ __forceinline__ void rope_kv_item(const PartView& pv, const RowTable& rt, bf16x8* __restrict__ qp,
                                                    uint16_t* __restrict__ kt, uint16_t* __restrict__ vt, int Tp, int nh,
                                                    int hd, int which, int h, int a, int t, int b, size_t q_unit0 = 0,
                                                    uint16_t* k_copy = nullptr, uint16_t* v_copy = nullptr) {
    const int m = b * Tp + t;
    const int d = nh * hd, half = hd / 2;
    const int col0 = which * d + h * hd + a * 8;
    const float* p0 = pv.base + (size_t)m * pv.ld + col0;
    const int nsplit = NS > 0 ? NS : part_count(pv, col0);           // a head's columns share one 256-column group
    float lo[8] = {0, 0, 0, 0, 0, 0, 0, 0}, hi[8] = {0, 0, 0, 0, 0, 0, 0, 0};     // dims 8a..8a+7, half+8a..+7
    if constexpr (NS > 0) {
        float4 x0[NS], x1[NS], x2[NS], x3[NS];
#pragma unroll
        for (int sp = 0; sp < NS; ++sp) {
            const float* p = p0 + (size_t)sp * pv.slot_stride;
            x0[sp] = *(const float4*)p; x1[sp] = *(const float4*)(p + 4);
            x2[sp] = *(const float4*)(p + half); x3[sp] = *(const float4*)(p + half + 4);
        }
#pragma unroll
        for (int sp = 0; sp < NS; ++sp) {
            lo[0] += x0[sp].x; lo[1] += x0[sp].y; lo[2] += x0[sp].z; lo[3] += x0[sp].w;
            lo[4] += x1[sp].x; lo[5] += x1[sp].y; lo[6] += x1[sp].z; lo[7] += x1[sp].w;
            hi[0] += x2[sp].x; hi[1] += x2[sp].y; hi[2] += x2[sp].z; hi[3] += x2[sp].w;
            hi[4] += x3[sp].x; hi[5] += x3[sp].y; hi[6] += x3[sp].z; hi[7] += x3[sp].w;
        }
    } else if constexpr (BATCH) {
        add_slots8<true>(lo, p0, pv.slot_stride, nsplit);
        add_slots8<true>(hi, p0 + half, pv.slot_stride, nsplit);
    } else {
        for (int sp = 0; sp < nsplit; ++sp) {
            const float* p = p0 + (size_t)sp * pv.slot_stride;
            float4 x0 = *(const float4*)p, x1 = *(const float4*)(p + 4);
            float4 x2 = *(const float4*)(p + half), x3 = *(const float4*)(p + half + 4);
            lo[0] += x0.x; lo[1] += x0.y; lo[2] += x0.z; lo[3] += x0.w;
            lo[4] += x1.x; lo[5] += x1.y; lo[6] += x1.z; lo[7] += x1.w;
            hi[0] += x2.x; hi[1] += x2.y; hi[2] += x2.z; hi[3] += x2.w;
            hi[4] += x3.x; hi[5] += x3.y; hi[6] += x3.z; hi[7] += x3.w;
        }
    }
    const int TB = Tp / 32;
    const size_t head_off = ((size_t)b * nh + h) * TB * (32 * hd);
    if (which == 2) {                                   // values: not rotated, scattered bf16
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __bf16 w1 = (__bf16)lo[i], w2 = (__bf16)hi[i];
            vt[head_off + vblk_index(t, a * 8 + i, hd)] = __builtin_bit_cast(uint16_t, w1);
            vt[head_off + vblk_index(t, half + a * 8 + i, hd)] = __builtin_bit_cast(uint16_t, w2);
            if (v_copy) {
                v_copy[vblk_index(t, a * 8 + i, hd)] = __builtin_bit_cast(uint16_t, w1);
                v_copy[vblk_index(t, half + a * 8 + i, hd)] = __builtin_bit_cast(uint16_t, w2);
            }
        }
        return;
    }
    float r1[8], r2[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float2 cs = rt.cs[(size_t)m * half + a * 8 + i];
        r1[i] = lo[i] * cs.x - hi[i] * cs.y;
        r2[i] = hi[i] * cs.x + lo[i] * cs.y;
    }
    if (which == 0) {                                   // queries: two-term expansion
        bf16x8 h1, l1, h2, l2;
        split_hilo(r1, h1, l1);
        split_hilo(r2, h2, l2);
        size_t q1i = 2 * head_off + qblk_index(t, a * 8, hd), q2i = 2 * head_off + qblk_index(t, half + a * 8, hd);
        qp[(q1i >> 3) - q_unit0] = h1;
        qp[(q1i >> 3) - q_unit0 + 64] = l1;
        qp[(q2i >> 3) - q_unit0] = h2;
        qp[(q2i >> 3) - q_unit0 + 64] = l2;
    } else {                                            // keys: bf16, the cache's storage type
        bf16x8 k1, k2;
#pragma unroll
        for (int i = 0; i < 8; ++i) { k1[i] = (__bf16)r1[i]; k2[i] = (__bf16)r2[i]; }
        ((bf16x8*)kt)[(head_off + kblk_index(t, a * 8, hd)) >> 3] = k1;
        ((bf16x8*)kt)[(head_off + kblk_index(t, half + a * 8, hd)) >> 3] = k2;
        if (k_copy) {
            ((bf16x8*)k_copy)[kblk_index(t, a * 8, hd) >> 3] = k1;
            ((bf16x8*)k_copy)[kblk_index(t, half + a * 8, hd) >> 3] = k2;
        }
    }
}

// ------------------------------------------------------------------------------------------
// act = silu(gate) * up from the gate/up partials (gate in columns [0,F), up in [Fpad, Fpad+F)).
// One item = (row m, group of 8 columns grp < F / 8).
template <bool WT>
static __device__ __forceinline__ void swiglu_item(const PartView& pv, int F, int Fpad, bf16x8* __restrict__ act, int MB,
                                                   int m, int grp) {
    float gsum[8] = {0, 0, 0, 0, 0, 0, 0, 0}, usum[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const int ng_ = part_count(pv, grp * 8), nu_ = part_count(pv, Fpad + grp * 8);
    add_slots8<WT>(gsum, pv.base + (size_t)m * pv.ld + grp * 8, pv.slot_stride, ng_);
    add_slots8<WT>(usum, pv.base + (size_t)m * pv.ld + Fpad + grp * 8, pv.slot_stride, nu_);
    bf16x8 hi, lo;
    float f[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = gsum[i] / (1.f + __expf(-gsum[i])) * usum[i];
    split_hilo(f, hi, lo);
    const size_t u = xpack_index(m, grp * 8, MB) >> 3;
    store_frag16<WT>(act + u, hi);
    store_frag16<WT>(act + u + XPART / 8, lo);
}

// ------------------------------------------------------------------------------------------
// Merge the split-KV partials of one (sequence b, head h, query t, 8 consecutive output dims e8) and emit
// the packed bf16 operand of the O-projection. The parts are read in batches of eight whose loads are all
// issued before any is used (a part index past the end re-reads the last part with weight zero, so no load
// sits behind a branch).
template <bool WT>
static __device__ __forceinline__ void attn_merge_item(const float* __restrict__ opart, const float2* __restrict__ mlpart,
                                                       bf16x8* __restrict__ xp, int nh, int hd, int Tp, int nparts, int MB,
                                                       int b, int h, int t, int e8) {
    constexpr int PB = 8;
    size_t base = ((size_t)b * nh + h) * nparts;
    float M = NEG_INF_F, den = 0.f, o[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int p0 = 0; p0 < nparts; p0 += PB) {
        float2 ml[PB];
        float4 a[PB], c[PB];
#pragma unroll
        for (int i = 0; i < PB; ++i) {
            const int p = min(p0 + i, nparts - 1);
            ml[i] = mlpart[(base + p) * Tp + t];
            const float4* src = (const float4*)(opart + ((base + p) * Tp + t) * hd + e8 * 8);
            a[i] = src[0];
            c[i] = src[1];
        }
        float Mb = M;
#pragma unroll
        for (int i = 0; i < PB; ++i)
            if (p0 + i < nparts && ml[i].y != 0.f) Mb = fmaxf(Mb, ml[i].x);       // an empty part has sum 0
        if (Mb == NEG_INF_F) continue;
        const float sold = exp2f(M - Mb);              // 0 when nothing was merged yet
        den *= sold;
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] *= sold;
#pragma unroll
        for (int i = 0; i < PB; ++i) {
            const float w = (p0 + i < nparts && ml[i].y != 0.f) ? exp2f(ml[i].x - Mb) : 0.f;
            den += w * ml[i].y;
            o[0] += w * a[i].x; o[1] += w * a[i].y; o[2] += w * a[i].z; o[3] += w * a[i].w;
            o[4] += w * c[i].x; o[5] += w * c[i].y; o[6] += w * c[i].z; o[7] += w * c[i].w;
        }
        M = Mb;
    }
    float inv = den > 0.f ? 1.f / den : 0.f;
    bf16x8 hi, lo;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] *= inv;
    split_hilo(o, hi, lo);
    int m = b * Tp + t, k = h * hd + e8 * 8;
    const size_t u = xpack_index(m, k, MB) >> 3;
    store_frag16<WT>(xp + u, hi);
    store_frag16<WT>(xp + u + XPART / 8, lo);
}
