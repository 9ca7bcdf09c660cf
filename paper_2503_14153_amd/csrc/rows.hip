// Row-wise kernels of the verifying pass: tree assembly + embedding, RMSNorm, rotary embedding
// with the tree K/V write, SwiGLU, and the draft-head activation. They sit between the
// weight-streaming GEMMs, reduce the GEMMs' split partial sums, and emit the next GEMM's
// operand directly in MFMA fragment order (bf16), so no separate conversion pass exists.
#include "sd_internal.h"
#include "row_ops.h"

// ------------------------------------------------------------------------------------------
// Rotary angle table entry, in float64 so that positions up to ~17k lose nothing.
static __device__ inline float2 rope_cs(int pos, int i, int hd, float theta) {
    double inv = pow((double)theta, -2.0 * (double)i / (double)hd);
    double s, c;
    sincos((double)pos * inv, &s, &c);
    return make_float2((float)c, (float)s);
}

// (embed_f32: the table holds float32 instead of bfloat16)
static __device__ inline void embed_row(const void* __restrict__ embed, int embed_f32, int tok, int d,
                                        float* __restrict__ xrow, bool valid) {
    if (embed_f32) {
        const float* e = (const float*)embed + (size_t)tok * d;
        for (int i = threadIdx.x; i < d; i += blockDim.x) xrow[i] = valid ? e[i] : 0.f;
        return;
    }
    const uint16_t* e = (const uint16_t*)embed + (size_t)tok * d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) xrow[i] = valid ? bf16_bits_to_float(e[i]) : 0.f;
}

// Tree assembly (paper Section III-B): node 0 = the base model's token, node j >= 1 = the
// candidate number rank[j] of head depth[j]-1; position = committed length + depth; a node
// attends its ancestors and itself.  One workgroup per row.
__global__ void k_build_rows_tree(RowTable rt, const int32_t* __restrict__ parent, const int32_t* __restrict__ depth,
                                  const int32_t* __restrict__ rank, const int32_t* __restrict__ root_tok,
                                  const int32_t* __restrict__ cand, const int32_t* __restrict__ kv_len, int T, int Tp,
                                  int H, int topk, int hd, float theta, const void* __restrict__ embed, int embed_f32,
                                  int d, int V, float* __restrict__ x) {
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
    embed_row(embed, embed_f32, tok, d, x + (size_t)m * d, valid);
}

void launch_build_rows_tree(RowTable rt, const int32_t* parent, const int32_t* depth, const int32_t* rank,
                            const int32_t* root_tok, const int32_t* cand, const int32_t* kv_len, int B, int T, int Tp,
                            int H, int topk, int hd, float theta, const void* embed, int embed_f32, int d, int V, float* x,
                            hipStream_t s) {
    hipLaunchKernelGGL(k_build_rows_tree, dim3(B * Tp), dim3(256), 0, s, rt, parent, depth, rank, root_tok, cand,
                       kv_len, T, Tp, H, topk, hd, theta, embed, embed_f32, d, V, x);
}

// Prompt chunk as a chain: row j of sequence b is prompt token off[b] + j at position
// committed length + j and attends rows 0..j of the chunk.
__global__ void k_build_rows_chain(RowTable rt, const int32_t* __restrict__ tokens, ChainArgs ca,
                                   const int32_t* __restrict__ kv_len, int Tp, int hd, float theta,
                                   const void* __restrict__ embed, int embed_f32, int d, int V,
                                   float* __restrict__ x) {
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
    embed_row(embed, embed_f32, tok, d, x + (size_t)m * d, valid);
}

void launch_build_rows_chain(RowTable rt, const int32_t* tokens, const ChainArgs& ca, const int32_t* kv_len, int B,
                             int Tp, int hd, float theta, const void* embed, int embed_f32, int d, int V, float* x,
                             hipStream_t s) {
    hipLaunchKernelGGL(k_build_rows_chain, dim3(B * Tp), dim3(256), 0, s, rt, tokens, ca, kv_len, Tp, hd, theta,
                       embed, embed_f32, d, V, x);
}

// ------------------------------------------------------------------------------------------
// RMSNorm with the residual add of the previous projection's partial sums (body: row_ops.h). One workgroup per row.
__global__ __launch_bounds__(NP_THREADS) void k_norm_pack(float* __restrict__ x, PartView pv,
                                                          const uint16_t* __restrict__ gain, float eps,
                                                          bf16x8* __restrict__ xn, float* __restrict__ hf, int d,
                                                          int MB, const int32_t* __restrict__ gather) {
    __shared__ float red[NP_THREADS / 64];
    // Eight neighbouring rows share every 128-byte line of the packed operand (a row's 16-byte piece per lane), and
    // workgroups go to the eight XCDs round-robin: workgroups b, b + 8, b + 16, .. take neighbouring rows, so that
    // a line is put together in ONE L2 and leaves it whole instead of as eight masked pieces from eight L2s.
    int m = blockIdx.x;
    if ((gridDim.x & 63) == 0) m = (m & ~63) + (m & 7) * 8 + ((m & 63) >> 3);
    else if ((gridDim.x & 31) == 0) m = (m & ~31) + (m & 7) * 4 + ((m & 31) >> 3);      // one row block: half lines
    norm_pack_row<false>(x, pv, gain, eps, xn, hf, d, MB, gather ? gather[m] : m, m, red);
}

void launch_norm_pack(float* x, PartView pv, const void* gain, float eps, void* xn_packed, float* hf_out, int M, int d,
                      int MB, const int32_t* gather, hipStream_t s) {
    hipLaunchKernelGGL(k_norm_pack, dim3(M), dim3(NP_THREADS), 0, s, x, pv,
                       (const uint16_t*)gain, eps, (bf16x8*)xn_packed, hf_out, d, MB, gather);
}

// ------------------------------------------------------------------------------------------
// Rotary embedding and the tree K/V write from the QKV partial sums (body: row_ops.h).
// grid (head x which, row block, sequence); a workgroup is one head's 32 rows of q, k or v: wave w takes the pieces
// a = 2w and 2w + 1, lane = row + 32 * (a & 1), so that what a wave stores of q and k are whole 1 KiB fragments (the
// query and key layouts put row r, dim group g of contraction step w at lane r + 32 g) and what it reads of a row and
// slot are 64 contiguous bytes twice. (One thread per (h, a) of ONE row wrote the same bytes as 16-byte pieces 0.5-2
// KiB apart; the values' layout is transposed, their 2-byte stores stay scattered either way.)
__global__ void k_rope_kv(PartView pv, RowTable rt, bf16x8* __restrict__ qp, uint16_t* __restrict__ kt, uint16_t* __restrict__ vt, int Tp,
                          int nh, int hd, int na) {
    const int which = blockIdx.x % 3, h = blockIdx.x / 3;     // a constant divisor: a multiplication
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int t = blockIdx.y * 32 + (lane & 31);
    for (int a = 2 * wave + (lane >> 5); a < na; a += 8)      // hd / 16 pieces: 8 (one round) or 4 (waves 0 and 1)
        rope_kv_item<false>(pv, rt, qp, kt, vt, Tp, nh, hd, which, h, a, t, blockIdx.z);
}

void launch_rope_kv(PartView pv, RowTable rt, void* q_packed, void* kt, void* vt, int B, int Tp, int nh, int hd,
                    hipStream_t s) {
    hipLaunchKernelGGL(k_rope_kv, dim3(nh * 3, Tp / 32, B), dim3(256), 0, s, pv, rt, (bf16x8*)q_packed, (uint16_t*)kt,
                       (uint16_t*)vt, Tp, nh, hd, hd / 16);
}

// ------------------------------------------------------------------------------------------
// SwiGLU from the gate/up partial sums (body: row_ops.h). grid (chunks of four contraction blocks, row blocks):
// a wave takes the 32 rows of a row block and the 16 columns of one contraction block of the packed result, lane =
// row + 32 * (column group), so that its two stores are the two whole 1 KiB fragments (hi, lo) and the four waves of
// a workgroup read 256 contiguous bytes of every row and slot.
__global__ void k_swiglu_pack(PartView pv, int F, int Fpad, bf16x8* __restrict__ act, int MB, int M) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m = blockIdx.y * 32 + (lane & 31), grp = (blockIdx.x * 4 + wave) * 2 + (lane >> 5);
    if (grp >= F / 8 || m >= M) return;
    swiglu_item<false>(pv, F, Fpad, act, MB, m, grp);
}

void launch_swiglu_pack(PartView pv, int F, int Fpad, void* act_packed, int M, int MB, hipStream_t s) {
    hipLaunchKernelGGL(k_swiglu_pack, dim3((F / 16 + 3) / 4, (M + 31) / 32), dim3(256), 0, s, pv, F, Fpad,
                       (bf16x8*)act_packed, MB, M);
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
