// The float32 device path: the same speculative step with weights, activations and the KV cache held as
// float32 and every product accumulated in float32 on the vector ALUs. It exists for configurations that are
// specified in float32 (the small correctness configuration): shapes of that size are bound by launches, not by
// arithmetic, so these kernels are plain (one thread per output, LDS tiles, natural row-major layouts) and make no
// attempt at the matrix cores. The integer stages (tree assembly, arg-max, top-k, acceptance, fragment cut) and the
// sampling statistics are the same kernels as on the bf16 path: they only ever see float32 logits.
//
// Layouts: weights [out][in]; activations [row][col]; tree scratch [layer][row][d]; cache [layer][K|V][seq][cap][d].
#include "sd_internal.h"

// ------------------------------------------------------------------------------------------
// y[m] = x[src] * rsqrt(mean(x[src]^2) + eps) * gain; one workgroup of 256 threads per row.
__global__ __launch_bounds__(256) void k_f32_rmsnorm(const float* __restrict__ x, const float* __restrict__ gain, float eps,
                                                     float* __restrict__ y, int d, const int32_t* __restrict__ gather) {
    const int m = blockIdx.x, src = gather ? gather[m] : m;
    const float* xr = x + (size_t)src * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) ss += xr[i] * xr[i];
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    __shared__ float red[4];
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float r = rsqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += 256) y[(size_t)m * d + i] = xr[i] * r * gain[i];
}
void launch_f32_rmsnorm(const float* x, const float* gain, float eps, float* y, int M, int d, const int32_t* gather,
                        hipStream_t s) {
    hipLaunchKernelGGL(k_f32_rmsnorm, dim3(M), dim3(256), 0, s, x, gain, eps, y, d, gather);
}

// ------------------------------------------------------------------------------------------
// out[m][n] (+)= sum_k X[m][k] * W[n][k] (+ bias[n]). 32 x 32 outputs per workgroup of 256 threads, contraction in
// steps of 32 through LDS; thread (tx, ty) owns column tx of rows ty, ty+8, ty+16, ty+24 of the tile.
// accumulate = 1: the result is added to what `out` holds (the residual stream).
__global__ __launch_bounds__(256) void k_f32_linear(const float* __restrict__ X, const float* __restrict__ W,
                                                    const float* __restrict__ bias, float* __restrict__ out, int M, int N,
                                                    int K, int ldx, int ldo, int accumulate) {
    __shared__ float xs[32][33], ws[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < K; k0 += 32) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = ty + 8 * r, k = k0 + tx;
            xs[row][tx] = (m0 + row < M && k < K) ? X[(size_t)(m0 + row) * ldx + k] : 0.f;
            ws[row][tx] = (n0 + row < N && k < K) ? W[(size_t)(n0 + row) * K + k] : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int kk = 0; kk < 32; ++kk) {
            const float w = ws[tx][kk];
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] = fmaf(xs[ty + 8 * r][kk], w, acc[r]);
        }
        __syncthreads();
    }
    const int n = n0 + tx;
    if (n >= N) return;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int m = m0 + ty + 8 * r;
        if (m < M) {
            float v = acc[r] + (bias ? bias[n] : 0.f);
            float* o = out + (size_t)m * ldo + n;
            *o = accumulate ? *o + v : v;
        }
    }
}
void launch_f32_linear(const float* X, const float* W, const float* bias, float* out, int M, int N, int K, int ldx, int ldo,
                       int accumulate, hipStream_t s) {
    hipLaunchKernelGGL(k_f32_linear, dim3((N + 31) / 32, (M + 31) / 32), dim3(256), 0, s, X, W, bias, out, M, N, K, ldx,
                       ldo, accumulate);
}

// ------------------------------------------------------------------------------------------
// Rotary embedding of q and k at the row's position (half-split pairs), tree K/V rows to the scratch.
// qkv [M][3d]; q [M][d]; kt, vt [M][d]; one thread per (row, head, pair index i < hd/2).
__global__ void k_f32_rope_kv(const float* __restrict__ qkv, RowTable rt, float* __restrict__ q, float* __restrict__ kt,
                              float* __restrict__ vt, int M, int nh, int hd) {
    const int half = hd / 2, d = nh * hd;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)M * nh * half) return;
    const int i = (int)(idx % half), h = (int)((idx / half) % nh), m = (int)(idx / ((size_t)half * nh));
    const float2 cs = rt.cs[(size_t)m * half + i];
    const float* row = qkv + (size_t)m * 3 * d;
    const int c = h * hd + i;
    const float q1 = row[c], q2 = row[c + half], k1 = row[d + c], k2 = row[d + c + half];
    q[(size_t)m * d + c] = q1 * cs.x - q2 * cs.y;
    q[(size_t)m * d + c + half] = q2 * cs.x + q1 * cs.y;
    kt[(size_t)m * d + c] = k1 * cs.x - k2 * cs.y;
    kt[(size_t)m * d + c + half] = k2 * cs.x + k1 * cs.y;
    vt[(size_t)m * d + c] = row[2 * d + c];
    vt[(size_t)m * d + c + half] = row[2 * d + c + half];
}
void launch_f32_rope_kv(const float* qkv, RowTable rt, float* q, float* kt, float* vt, int M, int nh, int hd, hipStream_t s) {
    const size_t total = (size_t)M * nh * (hd / 2);
    hipLaunchKernelGGL(k_f32_rope_kv, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, qkv, rt, q, kt, vt, M, nh, hd);
}

// ------------------------------------------------------------------------------------------
// Tree-masked attention of one (sequence, head, tree row): softmax over the committed rows 0..n-1 and the tree rows
// in the row's ancestor set, in chunks of 256 keys with a running maximum. 128 threads: each computes the scores of
// two keys of a chunk, then thread e accumulates output dim e.
#define F32A_CHUNK 256
__global__ __launch_bounds__(128) void k_f32_attn(const float* __restrict__ q, const float* __restrict__ kc,
                                                  const float* __restrict__ vc, const float* __restrict__ kt,
                                                  const float* __restrict__ vt, const int32_t* __restrict__ kv_len,
                                                  const uint32_t* __restrict__ anc, float* __restrict__ out, int nh,
                                                  int hd, int Tp, int cap, float scale) {
    const int t = blockIdx.x, h = blockIdx.y, b = blockIdx.z, m = b * Tp + t, d = nh * hd, tid = threadIdx.x;
    const int n = kv_len[b], total = n + Tp;
    const float* qr = q + (size_t)m * d + h * hd;
    const float* kcb = kc + (size_t)b * cap * d + h * hd;
    const float* vcb = vc + (size_t)b * cap * d + h * hd;
    const float* ktb = kt + (size_t)b * Tp * d + h * hd;
    const float* vtb = vt + (size_t)b * Tp * d + h * hd;
    const uint32_t* am = anc + (size_t)m * SD_ANC_WORDS;
    __shared__ float p[F32A_CHUNK], qs[128], red[2];
    if (tid < hd) qs[tid] = qr[tid];
    __syncthreads();
    float mrun = -__builtin_inff(), lrun = 0.f, o = 0.f;
    for (int c0 = 0; c0 < total; c0 += F32A_CHUNK) {
        float sc[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int i = c0 + tid + 128 * u;
            bool vis = i < n;
            const float* kr = kcb + (size_t)i * d;
            if (i >= n && i < total) {
                const int j = i - n;
                vis = (am[j >> 5] >> (j & 31)) & 1u;
                kr = ktb + (size_t)j * d;
            }
            float s = -__builtin_inff();
            if (vis) {
                s = 0.f;
                for (int e = 0; e < hd; ++e) s = fmaf(qs[e], kr[e], s);
                s *= scale;
            }
            sc[u] = s;
        }
        float mx = fmaxf(sc[0], sc[1]);
        for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
        if ((tid & 63) == 0) red[tid >> 6] = mx;
        __syncthreads();
        mx = fmaxf(red[0], red[1]);
        const float mnew = fmaxf(mrun, mx);
        __syncthreads();                                   // red is reused below
        if (mnew == -__builtin_inff()) continue;           // nothing visible so far (uniform over the workgroup)
        const float alpha = mrun == -__builtin_inff() ? 0.f : __expf(mrun - mnew);
        float ps = 0.f;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const float e = sc[u] == -__builtin_inff() ? 0.f : __expf(sc[u] - mnew);
            p[tid + 128 * u] = e;
            ps += e;
        }
        for (int off = 32; off > 0; off >>= 1) ps += __shfl_xor(ps, off);
        if ((tid & 63) == 0) red[tid >> 6] = ps;
        __syncthreads();
        lrun = lrun * alpha + red[0] + red[1];
        o *= alpha;
        if (tid < hd) {
            const int lim = min(F32A_CHUNK, total - c0);
            for (int jj = 0; jj < lim; ++jj) {
                const float w = p[jj];
                if (w != 0.f) {
                    const int i = c0 + jj;
                    const float* vr = i < n ? vcb + (size_t)i * d : vtb + (size_t)(i - n) * d;
                    o = fmaf(w, vr[tid], o);
                }
            }
        }
        mrun = mnew;
        __syncthreads();                                   // p and red are rewritten by the next chunk
    }
    if (tid < hd) out[(size_t)m * d + h * hd + tid] = lrun > 0.f ? o / lrun : 0.f;
}
void launch_f32_attn(const float* q, const float* kc, const float* vc, const float* kt, const float* vt,
                     const int32_t* kv_len, const uint32_t* anc, float* out, int B, int nh, int hd, int Tp, int cap,
                     hipStream_t s) {
    hipLaunchKernelGGL(k_f32_attn, dim3(Tp, nh, B), dim3(128), 0, s, q, kc, vc, kt, vt, kv_len, anc, out, nh, hd, Tp, cap,
                       1.f / sqrtf((float)hd));
}

// ------------------------------------------------------------------------------------------
// act[m][f] = silu(gu[m][f]) * gu[m][F + f]
__global__ void k_f32_swiglu(const float* __restrict__ gu, float* __restrict__ act, int M, int F) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)M * F) return;
    const int f = (int)(idx % F), m = (int)(idx / F);
    const float g = gu[(size_t)m * 2 * F + f], u = gu[(size_t)m * 2 * F + F + f];
    act[idx] = g / (1.f + __expf(-g)) * u;
}
void launch_f32_swiglu(const float* gu, float* act, int M, int F, hipStream_t s) {
    const size_t total = (size_t)M * F;
    hipLaunchKernelGGL(k_f32_swiglu, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, gu, act, M, F);
}

// ------------------------------------------------------------------------------------------
// Draft heads: row (i, b) = h_b + silu(z[b][i*d ..]) (z already holds W_i h_b + bias_i)
__global__ void k_f32_medusa_act(const float* __restrict__ z, const float* __restrict__ h, float* __restrict__ out, int B,
                                 int H, int d) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)H * B * d) return;
    const int c = (int)(idx % d), b = (int)((idx / d) % B), i = (int)(idx / ((size_t)d * B));
    const float zz = z[(size_t)b * H * d + (size_t)i * d + c];
    out[idx] = h[(size_t)b * d + c] + zz / (1.f + __expf(-zz));
}
void launch_f32_medusa_act(const float* z, const float* h, float* out, int B, int H, int d, hipStream_t s) {
    const size_t total = (size_t)H * B * d;
    hipLaunchKernelGGL(k_f32_medusa_act, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, z, h, out, B, H, d);
}

// ------------------------------------------------------------------------------------------
// Commit: tree row src_slots[b][j] -> cache row n_old[b] + j for j < n_accept[b], every layer, K and V.
// grid (row j, layer * B + b), 256 threads over the d columns.
__global__ void k_f32_kv_commit(const float* __restrict__ kt, const float* __restrict__ vt, float* __restrict__ kc,
                                float* __restrict__ vc, const int32_t* __restrict__ src_slots,
                                const int32_t* __restrict__ n_accept, const int32_t* __restrict__ n_old, int B, int d,
                                int Tp, int cap, int W, size_t layer_stride_t, size_t layer_stride_c) {
    const int j = blockIdx.x, l = blockIdx.y / B, b = blockIdx.y % B;
    if (j >= min(n_accept[b], W)) return;
    const int src = min(max(src_slots[(size_t)b * W + j], 0), Tp - 1), dst = n_old[b] + j;
    const size_t so = l * layer_stride_t + ((size_t)b * Tp + src) * d, dofs = l * layer_stride_c + ((size_t)b * cap + dst) * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
        kc[dofs + c] = kt[so + c];
        vc[dofs + c] = vt[so + c];
    }
}
void launch_f32_kv_commit(const float* kt, const float* vt, float* kc, float* vc, const int32_t* src_slots,
                          const int32_t* n_accept, const int32_t* n_old, int L, int B, int d, int Tp, int cap, int W,
                          hipStream_t s) {
    hipLaunchKernelGGL(k_f32_kv_commit, dim3(W, L * B), dim3(256), 0, s, kt, vt, kc, vc, src_slots, n_accept, n_old, B, d, Tp,
                       cap, W, (size_t)B * Tp * d, (size_t)B * cap * d);
}

// natural-layout rows [nrows][d] <-> cache rows of one sequence and layer
__global__ void k_f32_kv_rows(float* __restrict__ kc, float* __restrict__ vc, float* __restrict__ k_rows,
                              float* __restrict__ v_rows, int row0, int d, int to_cache) {
    const int r = blockIdx.x;
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
        const size_t ci = (size_t)(row0 + r) * d + c, ni = (size_t)r * d + c;
        if (to_cache) { kc[ci] = k_rows[ni]; vc[ci] = v_rows[ni]; }
        else { k_rows[ni] = kc[ci]; v_rows[ni] = vc[ci]; }
    }
}
void launch_f32_kv_rows(float* kc, float* vc, float* k_rows, float* v_rows, int row0, int nrows, int d, int to_cache,
                        hipStream_t s) {
    hipLaunchKernelGGL(k_f32_kv_rows, dim3(nrows), dim3(256), 0, s, kc, vc, k_rows, v_rows, row0, d, to_cache);
}
