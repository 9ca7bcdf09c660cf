// Tree-masked attention over the KV cache (the verifying pass of one speculative step).
//
// Every tree node attends all committed cache rows plus its own ancestors in the tree. The
// cache part is a pure stream: K and V of each head are read once from HBM and reused by all
// T queries of that head, so the kernel is HBM-bound and is organised around that stream:
//   * keys and values are stored as ready-made MFMA fragments (see sd_internal.h), so a wave
//     fetches a 32-row block with sixteen fully coalesced 1 KiB loads and no LDS transpose;
//   * S^T = K Q^T puts query t in lane t%32, and the value rows inside a block are permuted
//     so that exp(S) -- still in the accumulator registers -- already is the B operand of
//     O^T = V^T P^T: no cross-lane traffic between the two products;
//   * K and V are bf16 (the cache's storage type) but queries and probabilities are not: both
//     enter their MFMAs as two-term bf16 expansions (hi + lo), paid for with matrix-core time
//     that an HBM-bound kernel has to spare;
//   * the cache range is split over workgroups (split-KV); partial (max, sum, O) triples are
//     merged by a second small kernel, which also emits the packed bf16 operand of the
//     O-projection.
#include "sd_internal.h"

#define NEG_INF (-__builtin_inff())

// grid: x = part (0..nchunks-1 cache chunks, nchunks = the tree rows), y = head * TG + tg, z = seq
// one wave per workgroup; TBW = query blocks (32 rows) per wave
template <int HD, int TBW>
__global__ __launch_bounds__(64) void k_tree_attn(const bf16x8* __restrict__ Qp, const bf16x8* __restrict__ Kc,
                                                  const bf16x8* __restrict__ Vc, const bf16x8* __restrict__ Kt,
                                                  const bf16x8* __restrict__ Vt, const int32_t* __restrict__ kv_len,
                                                  const uint32_t* __restrict__ anc, float* __restrict__ opart,
                                                  float2* __restrict__ mlpart, int nh, int Tp, int cap_blocks,
                                                  int nchunks, int blocks_per_chunk, float scale_log2) {
    constexpr int KK = HD / 16;        // contraction steps of QK^T
    constexpr int EB = HD / 32;        // 32-wide output blocks of PV
    constexpr int BLK = HD * 4;        // bf16x8 units per 32-row block
    const int lane = threadIdx.x, g = lane >> 5, tl = lane & 31;
    const int part = blockIdx.x;
    const int TB = Tp / 32, TG = TB / TBW;
    const int h = blockIdx.y / TG, tg = blockIdx.y % TG;
    const int b = blockIdx.z;
    const int n = kv_len[b];
    const bool tree_part = part == nchunks;

    bf16x8 q[TBW][KK][2];              // two-term bf16 expansion of every query
#pragma unroll
    for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
                q[tb][kk][pt] = Qp[(((((size_t)b * nh + h) * TB + tg * TBW + tb) * KK + kk) * 2 + pt) * 64 + lane];

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

    int blk0, blk1;
    const bf16x8 *kbase, *vbase;
    uint32_t ancw[TBW][SD_ANC_WORDS];
    if (tree_part) {
        blk0 = 0;
        blk1 = tg * TBW + TBW;                       // later tree blocks hold no ancestors
        kbase = Kt + ((size_t)b * nh + h) * TB * BLK;
        vbase = Vt + ((size_t)b * nh + h) * TB * BLK;
#pragma unroll
        for (int tb = 0; tb < TBW; ++tb)
#pragma unroll
            for (int w = 0; w < SD_ANC_WORDS; ++w)
                ancw[tb][w] = anc[((size_t)b * Tp + (tg * TBW + tb) * 32 + tl) * SD_ANC_WORDS + w];
    } else {
        const int nblk = (n + 31) >> 5;
        blk0 = part * blocks_per_chunk;
        blk1 = blk0 + blocks_per_chunk;
        if (blk1 > nblk) blk1 = nblk;
        kbase = Kc + ((size_t)b * nh + h) * cap_blocks * BLK;
        vbase = Vc + ((size_t)b * nh + h) * cap_blocks * BLK;
    }

    for (int blk = blk0; blk < blk1; ++blk) {
        bf16x8 kf[KK], vf[2][EB];
        const bf16x8* kp = kbase + (size_t)blk * BLK + lane;
        const bf16x8* vp = vbase + (size_t)blk * BLK + lane;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kf[kk] = kp[kk * 64];
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int eb = 0; eb < EB; ++eb) vf[p][eb] = vp[(p * EB + eb) * 64];

#pragma unroll
        for (int tb = 0; tb < TBW; ++tb) {
            f32x16 S;
#pragma unroll
            for (int v = 0; v < 16; ++v) S[v] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], q[tb][kk][0], S, 0, 0, 0);
                S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], q[tb][kk][1], S, 0, 0, 0);
            }
            // lane (t = tl, g) holds rows c = 8*(v/4) + 4*g + v%4 of this block
            uint32_t vis;
            if (tree_part) {
                vis = ancw[tb][0];
#pragma unroll
                for (int w = 1; w < SD_ANC_WORDS; ++w) vis = (blk == w) ? ancw[tb][w] : vis;
            } else {
                int left = n - blk * 32;
                vis = left >= 32 ? 0xffffffffu : ((1u << left) - 1u);
            }
            float mx = NEG_INF;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int c = 8 * (v >> 2) + 4 * g + (v & 3);
                float sv = ((vis >> c) & 1u) ? S[v] * scale_log2 : NEG_INF;
                S[v] = sv;
                mx = fmaxf(mx, sv);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            float mnew = fmaxf(mrun[tb], mx);
            float muse = (mnew == NEG_INF) ? 0.f : mnew;
            float alpha = exp2f(mrun[tb] - muse);
            float psum = 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float p = exp2f(S[v] - muse);
                S[v] = p;
                psum += p;
            }
            lrun[tb] = lrun[tb] * alpha + psum;
            mrun[tb] = mnew;
            bf16x8 pf[2], pl[2];               // probabilities, two-term expansion
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    __bf16 hi = (__bf16)S[8 * p + s];
                    pf[p][s] = hi;
                    pl[p][s] = (__bf16)(S[8 * p + s] - (float)hi);
                }
#pragma unroll
            for (int eb = 0; eb < EB; ++eb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) O[tb][eb][v] *= alpha;
#pragma unroll
                for (int p = 0; p < 2; ++p) {
                    O[tb][eb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[p][eb], pf[p], O[tb][eb], 0, 0, 0);
                    O[tb][eb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[p][eb], pl[p], O[tb][eb], 0, 0, 0);
                }
            }
        }
    }

    const int nparts = nchunks + 1;
#pragma unroll
    for (int tb = 0; tb < TBW; ++tb) {
        int t = (tg * TBW + tb) * 32 + tl;
        size_t row = (((size_t)b * nh + h) * nparts + part) * Tp + t;
        float ltot = lrun[tb] + __shfl_xor(lrun[tb], 32);
        if (g == 0) mlpart[row] = make_float2(mrun[tb], ltot);
        float* o = opart + row * HD;
#pragma unroll
        for (int eb = 0; eb < EB; ++eb)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int e = eb * 32 + 8 * i + 4 * g;
                *(float4*)(o + e) = make_float4(O[tb][eb][4 * i], O[tb][eb][4 * i + 1], O[tb][eb][4 * i + 2],
                                                O[tb][eb][4 * i + 3]);
            }
    }
}

void launch_tree_attn(const void* q_packed, const void* kc, const void* vc, const void* kt, const void* vt,
                      const int32_t* kv_len, const uint32_t* anc, float* opart, float2* mlpart, int B, int nh,
                      int hd, int Tp, int cap_blocks, int nchunks, int blocks_per_chunk, hipStream_t s) {
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)hd);
    const int TB = Tp / 32;
    const int TBW = (TB % 2 == 0) ? 2 : 1;
    dim3 grid(nchunks + 1, nh * (TB / TBW), B);
#define ATT(HD_, TBW_)                                                                                          \
    hipLaunchKernelGGL((k_tree_attn<HD_, TBW_>), grid, dim3(64), 0, s, (const bf16x8*)q_packed,                \
                       (const bf16x8*)kc, (const bf16x8*)vc, (const bf16x8*)kt, (const bf16x8*)vt, kv_len, anc, \
                       opart, mlpart, nh, Tp, cap_blocks, nchunks, blocks_per_chunk, scale_log2)
    if (hd == 128) { if (TBW == 2) ATT(128, 2); else ATT(128, 1); }
    else           { if (TBW == 2) ATT(64, 2);  else ATT(64, 1); }
#undef ATT
}

// ------------------------------------------------------------------------------------------
// Merge the split-KV partials and emit the packed bf16 operand of the O-projection.
// one thread per (seq, head, query t, 8 consecutive output dims)
__global__ void k_attn_merge(const float* __restrict__ opart, const float2* __restrict__ mlpart,
                             bf16x8* __restrict__ xp, int B, int nh, int hd, int Tp, int nparts, int MB) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    int e8n = hd / 8;
    int total = B * nh * Tp * e8n;
    if (idx >= total) return;
    int e8 = idx % e8n;
    int t = (idx / e8n) % Tp;
    int h = (idx / (e8n * Tp)) % nh;
    int b = idx / (e8n * Tp * nh);
    size_t base = ((size_t)b * nh + h) * nparts;
    float M = NEG_INF;
    for (int p = 0; p < nparts; ++p) M = fmaxf(M, mlpart[(base + p) * Tp + t].x);
    float den = 0.f, o[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int p = 0; p < nparts; ++p) {
        float2 ml = mlpart[(base + p) * Tp + t];
        if (ml.y == 0.f) continue;                      // empty part
        float w = exp2f(ml.x - M);
        den += w * ml.y;
        const float4* src = (const float4*)(opart + ((base + p) * Tp + t) * hd + e8 * 8);
        float4 a = src[0], c = src[1];
        o[0] += w * a.x; o[1] += w * a.y; o[2] += w * a.z; o[3] += w * a.w;
        o[4] += w * c.x; o[5] += w * c.y; o[6] += w * c.z; o[7] += w * c.w;
    }
    float inv = den > 0.f ? 1.f / den : 0.f;
    bf16x8 hi, lo;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] *= inv;
    split_hilo(o, hi, lo);
    int m = b * Tp + t, k = h * hd + e8 * 8;
    const size_t u = xpack_index(m, k, MB) >> 3;
    xp[u] = hi;
    xp[u + XPART / 8] = lo;
}

void launch_attn_merge(const float* opart, const float2* mlpart, void* x_packed, int B, int nh, int hd, int Tp,
                       int nparts, int MB, hipStream_t s) {
    int total = B * nh * Tp * (hd / 8);
    hipLaunchKernelGGL(k_attn_merge, dim3((total + 255) / 256), dim3(256), 0, s, opart, mlpart, (bf16x8*)x_packed,
                       B, nh, hd, Tp, nparts, MB);
}
