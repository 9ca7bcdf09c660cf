// Row-wise kernels of the verifying pass: tree assembly + embedding, RMSNorm, rotary embedding
// with the tree K/V write, SwiGLU, and the draft-head activation. They sit between the
// weight-streaming GEMMs, reduce the GEMMs' split partial sums, and emit the next GEMM's
// operand directly in MFMA fragment order (bf16), so no separate conversion pass exists.
#include "sd_internal.h"

static __device__ inline float bf16_bits_to_float(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// ------------------------------------------------------------------------------------------
// Rotary angle table entry, in float64 so that positions up to ~17k lose nothing.
static __device__ inline float2 rope_cs(int pos, int i, int hd, float theta) {
    double inv = pow((double)theta, -2.0 * (double)i / (double)hd);
    double s, c;
    sincos((double)pos * inv, &s, &c);
    return make_float2((float)c, (float)s);
}

static __device__ inline void embed_row(const uint16_t* __restrict__ embed, int tok, int d, float* __restrict__ xrow,
                                        bool valid) {
    const uint16_t* e = embed + (size_t)tok * d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) xrow[i] = valid ? bf16_bits_to_float(e[i]) : 0.f;
}

// Tree assembly (paper Section III-B): node 0 = the base model's token, node j >= 1 = the
// candidate number rank[j] of head depth[j]-1; position = committed length + depth; a node
// attends its ancestors and itself.  One workgroup per row.
__global__ void k_build_rows_tree(RowTable rt, const int32_t* __restrict__ parent, const int32_t* __restrict__ depth,
                                  const int32_t* __restrict__ rank, const int32_t* __restrict__ root_tok,
                                  const int32_t* __restrict__ cand, const int32_t* __restrict__ kv_len, int T, int Tp,
                                  int H, int topk, int hd, float theta, const uint16_t* __restrict__ embed, int d,
                                  int V, float* __restrict__ x) {
    const int m = blockIdx.x, b = m / Tp, j = m % Tp;
    const bool valid = j < T;
    int tok = 0, pos = kv_len[b];
    uint32_t a[SD_ANC_WORDS] = {};
    if (valid) {
        int dj = depth[j];
        tok = (j == 0) ? root_tok[b] : cand[((size_t)b * H + (dj - 1)) * topk + rank[j]];
        tok = min(max(tok, 0), V - 1);               // a bad candidate id must not become a bad address
        pos += dj;
        for (int i = j, guard = 0; i >= 0 && guard <= H; i = parent[i], ++guard) a[i >> 5] |= 1u << (i & 31);
    } else {
        a[j >> 5] |= 1u << (j & 31);
    }
    if (threadIdx.x == 0) {
        rt.tok[m] = tok;
        rt.pos[m] = pos;
        for (int w = 0; w < SD_ANC_WORDS; ++w) rt.anc[(size_t)m * SD_ANC_WORDS + w] = a[w];
    }
    for (int i = threadIdx.x; i < hd / 2; i += blockDim.x) rt.cs[(size_t)m * (hd / 2) + i] = rope_cs(pos, i, hd, theta);
    embed_row(embed, tok, d, x + (size_t)m * d, valid);
}

void launch_build_rows_tree(RowTable rt, const int32_t* parent, const int32_t* depth, const int32_t* rank,
                            const int32_t* root_tok, const int32_t* cand, const int32_t* kv_len, int B, int T, int Tp,
                            int H, int topk, int hd, float theta, const void* embed, int d, int V, float* x, hipStream_t s) {
    hipLaunchKernelGGL(k_build_rows_tree, dim3(B * Tp), dim3(256), 0, s, rt, parent, depth, rank, root_tok, cand,
                       kv_len, T, Tp, H, topk, hd, theta, (const uint16_t*)embed, d, V, x);
}

// Prompt chunk as a chain: row j of sequence b is prompt token off[b] + j at position
// committed length + j and attends rows 0..j of the chunk.
__global__ void k_build_rows_chain(RowTable rt, const int32_t* __restrict__ tokens, ChainArgs ca,
                                   const int32_t* __restrict__ kv_len, int Tp, int hd, float theta,
                                   const uint16_t* __restrict__ embed, int d, int V, float* __restrict__ x) {
    const int m = blockIdx.x, b = m / Tp, j = m % Tp;
    const bool valid = j < ca.len[b];
    int tok = valid ? min(max(tokens[ca.off[b] + j], 0), V - 1) : 0;
    int pos = kv_len[b] + (valid ? j : 0);
    uint32_t a[SD_ANC_WORDS] = {};
    if (valid) {
        for (int w = 0; w < SD_ANC_WORDS; ++w) {
            int hi = j - 32 * w;
            a[w] = hi >= 31 ? 0xffffffffu : (hi < 0 ? 0u : ((2u << hi) - 1u));
        }
    } else {
        a[j >> 5] |= 1u << (j & 31);
    }
    if (threadIdx.x == 0) {
        rt.tok[m] = tok;
        rt.pos[m] = pos;
        for (int w = 0; w < SD_ANC_WORDS; ++w) rt.anc[(size_t)m * SD_ANC_WORDS + w] = a[w];
    }
    for (int i = threadIdx.x; i < hd / 2; i += blockDim.x) rt.cs[(size_t)m * (hd / 2) + i] = rope_cs(pos, i, hd, theta);
    embed_row(embed, tok, d, x + (size_t)m * d, valid);
}

void launch_build_rows_chain(RowTable rt, const int32_t* tokens, const ChainArgs& ca, const int32_t* kv_len, int B,
                             int Tp, int hd, float theta, const void* embed, int d, int V, float* x, hipStream_t s) {
    hipLaunchKernelGGL(k_build_rows_chain, dim3(B * Tp), dim3(256), 0, s, rt, tokens, ca, kv_len, Tp, hd, theta,
                       (const uint16_t*)embed, d, V, x);
}

// ------------------------------------------------------------------------------------------
// x += sum of split partials (residual add of the previous projection), then
// xn = x * rsqrt(mean(x^2) + eps) * gain, written as bf16 in fragment order.
// One workgroup per row; a thread owns groups of 8 consecutive columns.
#define NP_THREADS 512
#define NP_MAXG 2   // d <= 8 * NP_THREADS * NP_MAXG = 8192
__global__ __launch_bounds__(NP_THREADS) void k_norm_pack(float* __restrict__ x, PartView pv,
                                                          const uint16_t* __restrict__ gain, float eps,
                                                          bf16x8* __restrict__ xn, float* __restrict__ hf, int d,
                                                          int MB, const int32_t* __restrict__ gather) {
    const int m = blockIdx.x;
    const int src = gather ? gather[m] : m;
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
#pragma unroll 4
            for (int sp = 0; sp < nsplit; ++sp) {
                const float* p = pv.base + (size_t)sp * pv.slot_stride + (size_t)src * pv.ld + grp * 8;
                float4 pa = *(const float4*)p, pc = *(const float4*)(p + 4);
                t[0] += pa.x; t[1] += pa.y; t[2] += pa.z; t[3] += pa.w;
                t[4] += pc.x; t[5] += pc.y; t[6] += pc.z; t[7] += pc.w;
            }
            if (nsplit > 0) {
                *(float4*)(xr + grp * 8) = make_float4(t[0], t[1], t[2], t[3]);
                *(float4*)(xr + grp * 8 + 4) = make_float4(t[4], t[5], t[6], t[7]);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) { v[gi][i] = t[i]; ss += t[i] * t[i]; }
        }
    }
    __shared__ float red[NP_THREADS / 64];
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
            xn[u] = hi;
            xn[u + XPART / 8] = lo;
            if (hf) {
                *(float4*)(hf + (size_t)m * d + grp * 8) = make_float4(f[0], f[1], f[2], f[3]);
                *(float4*)(hf + (size_t)m * d + grp * 8 + 4) = make_float4(f[4], f[5], f[6], f[7]);
            }
        }
    }
}

void launch_norm_pack(float* x, PartView pv, const void* gain, float eps, void* xn_packed, float* hf_out, int M, int d,
                      int MB, const int32_t* gather, hipStream_t s) {
    hipLaunchKernelGGL(k_norm_pack, dim3(M), dim3(NP_THREADS), 0, s, x, pv,
                       (const uint16_t*)gain, eps, (bf16x8*)xn_packed, hf_out, d, MB, gather);
}

// ------------------------------------------------------------------------------------------
// Sum the QKV partials, rotate q and k to the row's position, and write q (fragment order,
// two-term expansion), k and v (tree scratch, block layouts, bf16). Thread (m, h, a, which)
// owns dims [8a, 8a+8) and their rotary partners [hd/2 + 8a, +8) of q (which=0), k (1) or v (2).
// grid (chunks of (h, a) x which, t, b): no index needs a division.
__global__ void k_rope_kv(PartView pv, RowTable rt, bf16x8* __restrict__ qp, uint16_t* __restrict__ kt, uint16_t* __restrict__ vt, int Tp,
                          int nh, int hd, int na_shift) {
    const int which = blockIdx.x % 3;                   // a constant divisor: a multiplication
    const int ha = (blockIdx.x / 3) * blockDim.x + threadIdx.x;
    const int a = ha & ((1 << na_shift) - 1), h = ha >> na_shift;      // hd / 16 = 1 << na_shift
    if (h >= nh) return;
    const int t = blockIdx.y, b = blockIdx.z, m = b * Tp + t;
    const int d = nh * hd, half = hd / 2;
    float4 s0 = make_float4(0, 0, 0, 0), s1 = s0, s2 = s0, s3 = s0;       // dims 8a..8a+7, half+8a..+7
    const int col0 = which * d + h * hd + a * 8;
    const float* p0 = pv.base + (size_t)m * pv.ld + col0;
    const int nsplit = part_count(pv, col0);           // a head's columns share one 256-column group
    for (int sp = 0; sp < nsplit; ++sp) {
        const float* p = p0 + (size_t)sp * pv.slot_stride;
        float4 x0 = *(const float4*)p, x1 = *(const float4*)(p + 4);
        float4 x2 = *(const float4*)(p + half), x3 = *(const float4*)(p + half + 4);
        s0.x += x0.x; s0.y += x0.y; s0.z += x0.z; s0.w += x0.w;
        s1.x += x1.x; s1.y += x1.y; s1.z += x1.z; s1.w += x1.w;
        s2.x += x2.x; s2.y += x2.y; s2.z += x2.z; s2.w += x2.w;
        s3.x += x3.x; s3.y += x3.y; s3.z += x3.z; s3.w += x3.w;
    }
    float lo[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
    float hi[8] = {s2.x, s2.y, s2.z, s2.w, s3.x, s3.y, s3.z, s3.w};
    const int TB = Tp / 32;
    const size_t head_off = ((size_t)b * nh + h) * TB * (32 * hd);
    if (which == 2) {                                   // values: not rotated, scattered bf16
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __bf16 w1 = (__bf16)lo[i], w2 = (__bf16)hi[i];
            vt[head_off + vblk_index(t, a * 8 + i, hd)] = __builtin_bit_cast(uint16_t, w1);
            vt[head_off + vblk_index(t, half + a * 8 + i, hd)] = __builtin_bit_cast(uint16_t, w2);
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
        qp[q1i >> 3] = h1;
        qp[(q1i >> 3) + 64] = l1;
        qp[q2i >> 3] = h2;
        qp[(q2i >> 3) + 64] = l2;
    } else {                                            // keys: bf16, the cache's storage type
        bf16x8 k1, k2;
#pragma unroll
        for (int i = 0; i < 8; ++i) { k1[i] = (__bf16)r1[i]; k2[i] = (__bf16)r2[i]; }
        ((bf16x8*)kt)[(head_off + kblk_index(t, a * 8, hd)) >> 3] = k1;
        ((bf16x8*)kt)[(head_off + kblk_index(t, half + a * 8, hd)) >> 3] = k2;
    }
}

void launch_rope_kv(PartView pv, RowTable rt, void* q_packed, void* kt, void* vt, int B, int Tp, int nh, int hd,
                    hipStream_t s) {
    const int na_shift = hd == 128 ? 3 : 2;            // head_dim is 128 or 64
    hipLaunchKernelGGL(k_rope_kv, dim3(((nh << na_shift) + 255) / 256 * 3, Tp, B), dim3(256), 0, s, pv, rt,
                       (bf16x8*)q_packed, (uint16_t*)kt, (uint16_t*)vt, Tp, nh, hd, na_shift);
}

// ------------------------------------------------------------------------------------------
// act = silu(gate) * up from the gate/up partials (gate in columns [0,F), up in [Fpad, Fpad+F)).
// grid (chunks of 8-column groups, row)
__global__ void k_swiglu_pack(PartView pv, int F, int Fpad, bf16x8* __restrict__ act, int MB) {
    const int grp = blockIdx.x * blockDim.x + threadIdx.x, m = blockIdx.y;
    if (grp >= F / 8) return;
    float gsum[8] = {0, 0, 0, 0, 0, 0, 0, 0}, usum[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const int ng_ = part_count(pv, grp * 8), nu_ = part_count(pv, Fpad + grp * 8);
    for (int sp = 0; sp < ng_; ++sp) {
        const float* p = pv.base + (size_t)sp * pv.slot_stride + (size_t)m * pv.ld + grp * 8;
        float4 a = *(const float4*)p, c = *(const float4*)(p + 4);
        gsum[0] += a.x; gsum[1] += a.y; gsum[2] += a.z; gsum[3] += a.w;
        gsum[4] += c.x; gsum[5] += c.y; gsum[6] += c.z; gsum[7] += c.w;
    }
    for (int sp = 0; sp < nu_; ++sp) {
        const float* p = pv.base + (size_t)sp * pv.slot_stride + (size_t)m * pv.ld + Fpad + grp * 8;
        float4 ua = *(const float4*)p, uc = *(const float4*)(p + 4);
        usum[0] += ua.x; usum[1] += ua.y; usum[2] += ua.z; usum[3] += ua.w;
        usum[4] += uc.x; usum[5] += uc.y; usum[6] += uc.z; usum[7] += uc.w;
    }
    bf16x8 hi, lo;
    float f[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = gsum[i] / (1.f + __expf(-gsum[i])) * usum[i];
    split_hilo(f, hi, lo);
    const size_t u = xpack_index(m, grp * 8, MB) >> 3;
    act[u] = hi;
    act[u + XPART / 8] = lo;
}

void launch_swiglu_pack(PartView pv, int F, int Fpad, void* act_packed, int M, int MB, hipStream_t s) {
    hipLaunchKernelGGL(k_swiglu_pack, dim3((F / 8 + 255) / 256, M), dim3(256), 0, s, pv, F, Fpad, (bf16x8*)act_packed,
                       MB);
}

// ------------------------------------------------------------------------------------------
// Draft heads, activation stage: row (i, b) = h_b + silu(W_i h_b + bias_i), packed as the
// operand of the shared LM-head GEMM. part columns [i*d, (i+1)*d) hold W_i h_b for row b.
// The i*B + b output rows are laid out in chunks of `chunk_rows` rows (a power of two >= 32, or
// >= H*B for a single operand): chunk c is a packed activation of its own, `chunk_rows * d * 2`
// elements after the previous one, with MB row blocks (MBlast in the last chunk).
__global__ void k_medusa_act(PartView pv, const float* __restrict__ h_rows, MedusaBias bias, int B, int H, int d,
                             bf16x8* __restrict__ xp, int chunk_rows, int MB, int MBlast) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    int ng = d / 8;
    if (idx >= H * B * ng) return;
    int grp = idx % ng, b = (idx / ng) % B, i = idx / (ng * B);
    float z[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    const int nsplit = part_count(pv, i * d + grp * 8);
    for (int sp = 0; sp < nsplit; ++sp) {
        const float* p = pv.base + (size_t)sp * pv.slot_stride + (size_t)b * pv.ld + (size_t)i * d + grp * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] += p[e];
    }
    const uint16_t* bi = bias.p[i];
    bf16x8 hi, lo;
    float f[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float zz = z[e] + (bi ? bf16_bits_to_float(bi[grp * 8 + e]) : 0.f);
        f[e] = h_rows[(size_t)b * d + grp * 8 + e] + zz / (1.f + __expf(-zz));
    }
    split_hilo(f, hi, lo);
    const int row = i * B + b, chunk = row / chunk_rows, last = (H * B - 1) / chunk_rows;
    const size_t u = ((size_t)chunk * chunk_rows * d * 2 + xpack_index(row - chunk * chunk_rows, grp * 8,
                                                                       chunk == last ? MBlast : MB)) >> 3;
    xp[u] = hi;
    xp[u + XPART / 8] = lo;
}

void launch_medusa_act(PartView pv, const float* h_rows, const MedusaBias& bias, int B, int H, int d, void* x_packed,
                       int chunk_rows, int MB, int MBlast, hipStream_t s) {
    int total = H * B * (d / 8);
    hipLaunchKernelGGL(k_medusa_act, dim3((total + 255) / 256), dim3(256), 0, s, pv, h_rows, bias, B, H, d,
                       (bf16x8*)x_packed, chunk_rows, MB, MBlast);
}
