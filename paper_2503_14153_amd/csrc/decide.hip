// Integer stages of the step: arg-max / top-k over the vocabulary, greedy acceptance with
// the fragment cut (paper Section III-B), and the commit of the accepted K/V rows.
#include "sd_internal.h"

#define NEG_INF (-__builtin_inff())

// "better" = larger value, ties to the lower index
static __device__ inline bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

static __device__ inline void wave_best(float& v, int& i) {
    for (int o = 32; o > 0; o >>= 1) {
        float ov = __shfl_xor(v, o);
        int oi = __shfl_xor(i, o);
        if (better(ov, oi, v, i)) { v = ov; i = oi; }
    }
}

// ------------------------------------------------------------------------------------------
// Row-wise arg-max over V columns (lowest id on ties). One workgroup of 1024 threads per row;
// the loop is unrolled so that several 16-byte loads per thread are in flight.
#define ARGMAX_THREADS 1024
__global__ __launch_bounds__(ARGMAX_THREADS) void k_argmax(const float* __restrict__ logits, int ld, int V,
                                                           int32_t* __restrict__ am, int T, int Tp) {
    const int b = blockIdx.x / T, j = blockIdx.x % T;
    const int m = b * Tp + j;
    const float* row = logits + (size_t)m * ld;
    float bv = NEG_INF;
    int bi = 0x7fffffff;
#pragma unroll 4
    for (int i = threadIdx.x * 4; i < V; i += ARGMAX_THREADS * 4) {
        float4 f = *(const float4*)(row + i);         // rows are padded to a multiple of 4 columns
        float vals[4] = {f.x, f.y, f.z, f.w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (i + e < V && better(vals[e], i + e, bv, bi)) { bv = vals[e]; bi = i + e; }
    }
    wave_best(bv, bi);
    __shared__ float sv[ARGMAX_THREADS / 64];
    __shared__ int si[ARGMAX_THREADS / 64];
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
    __syncthreads();
    if (threadIdx.x < 64) {
        bv = threadIdx.x < ARGMAX_THREADS / 64 ? sv[threadIdx.x] : NEG_INF;
        bi = threadIdx.x < ARGMAX_THREADS / 64 ? si[threadIdx.x] : 0x7fffffff;
        wave_best(bv, bi);
        if (threadIdx.x == 0) am[m] = bi;
    }
}

void launch_argmax(const float* logits, int ld, int V, int32_t* am, int B, int T, int Tp, hipStream_t s) {
    hipLaunchKernelGGL(k_argmax, dim3(B * T), dim3(ARGMAX_THREADS), 0, s, logits, ld, V, am, T, Tp);
}

// ------------------------------------------------------------------------------------------
// The same arg-max straight from the LM-head GEMM's partial sums: a thread sums the slots of its columns (in slot
// order, as k_reduce_slots does, so the logits are the same numbers), keeps the best, and writes the logits out
// only when somebody wants them (WRITE: the caller asked for logits, or sampling decoding reads them). Saves a
// launch and, without WRITE, the 8 MB write and re-read of the logits of a 64-row step.
template <bool WRITE>
__global__ __launch_bounds__(ARGMAX_THREADS) void k_reduce_argmax(PartView pv, float* __restrict__ logits, int V,
                                                                  int32_t* __restrict__ am, int T, int Tp) {
    const int b = blockIdx.x / T, j = blockIdx.x % T;
    const int m = b * Tp + j;
    float bv = NEG_INF;
    int bi = 0x7fffffff;
    for (int i = threadIdx.x * 4; i < pv.ld; i += ARGMAX_THREADS * 4) {
        const int n = part_count(pv, i);
        float4 a = make_float4(0, 0, 0, 0);
        const float* p = pv.base + (size_t)m * pv.ld + i;
#pragma unroll 4
        for (int sp = 0; sp < n; ++sp) {
            float4 v = *(const float4*)(p + (size_t)sp * pv.slot_stride);
            a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
        }
        if (WRITE) *(float4*)(logits + (size_t)m * pv.ld + i) = a;
        float vals[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (i + e < V && better(vals[e], i + e, bv, bi)) { bv = vals[e]; bi = i + e; }
    }
    wave_best(bv, bi);
    __shared__ float sv[ARGMAX_THREADS / 64];
    __shared__ int si[ARGMAX_THREADS / 64];
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
    __syncthreads();
    if (threadIdx.x < 64) {
        bv = threadIdx.x < ARGMAX_THREADS / 64 ? sv[threadIdx.x] : NEG_INF;
        bi = threadIdx.x < ARGMAX_THREADS / 64 ? si[threadIdx.x] : 0x7fffffff;
        wave_best(bv, bi);
        if (threadIdx.x == 0) am[m] = bi;
    }
}

void launch_reduce_argmax(PartView pv, float* logits_or_null, int V, int32_t* am, int B, int T, int Tp, hipStream_t s) {
    if (logits_or_null)
        hipLaunchKernelGGL(k_reduce_argmax<true>, dim3(B * T), dim3(ARGMAX_THREADS), 0, s, pv, logits_or_null, V, am, T, Tp);
    else
        hipLaunchKernelGGL(k_reduce_argmax<false>, dim3(B * T), dim3(ARGMAX_THREADS), 0, s, pv, logits_or_null, V, am, T, Tp);
}

// ------------------------------------------------------------------------------------------
// Per-row top-k (descending logit, ties to the lower id). One workgroup of 1024 threads per
// row keeps the whole row in registers (thread t owns ids t, t+1024, ...); each of the k
// rounds is a thread-local scan plus one block-wide (value, id) reduction, after which the
// owner retires the selected element.
#define TOPK_THREADS 1024
template <int NPT>
__global__ __launch_bounds__(TOPK_THREADS) void k_topk(const float* __restrict__ logits, int ld, int V, int k,
                                                       int32_t* __restrict__ out, int B, int H, uint32_t seq_mask) {
    const int r = blockIdx.x;                 // row r = head i * B + sequence b
    const int i = r / B, b = r % B;
    if (!((seq_mask >> b) & 1u)) return;
    const float* row = logits + (size_t)r * ld;
    const int tid = threadIdx.x;
    float v[NPT];
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
        int c = j * TOPK_THREADS + tid;
        v[j] = c < V ? row[c] : NEG_INF;
    }
    __shared__ float sv[TOPK_THREADS / 64];
    __shared__ int si[TOPK_THREADS / 64];
    __shared__ int chosen;
    // thread-local best of the elements not yet retired; only the owner of a retired element rescans
    float lbv = NEG_INF;
    int lbi = 0x7fffffff;
#pragma unroll
    for (int j = 0; j < NPT; ++j) {           // ascending ids: strict > keeps the lowest id
        int c = j * TOPK_THREADS + tid;
        if (c < V && v[j] > lbv) { lbv = v[j]; lbi = c; }
    }
    for (int round = 0; round < k; ++round) {
        float bv = lbv;
        int bi = lbi;
        wave_best(bv, bi);
        if ((tid & 63) == 0) { sv[tid >> 6] = bv; si[tid >> 6] = bi; }
        __syncthreads();
        if (tid < 64) {
            float wv = tid < TOPK_THREADS / 64 ? sv[tid] : NEG_INF;
            int wi = tid < TOPK_THREADS / 64 ? si[tid] : 0x7fffffff;
            wave_best(wv, wi);
            if (tid == 0) {
                chosen = wi;
                out[((size_t)b * H + i) * k + round] = wi;
            }
        }
        __syncthreads();
        const int ch = chosen;
        if ((ch % TOPK_THREADS) == tid) {
            lbv = NEG_INF;
            lbi = 0x7fffffff;
#pragma unroll
            for (int j = 0; j < NPT; ++j) {
                if (j == ch / TOPK_THREADS) v[j] = NEG_INF;
                int c = j * TOPK_THREADS + tid;
                if (c < V && v[j] > lbv) { lbv = v[j]; lbi = c; }
            }
        }
    }
}

void launch_topk(const float* logits, int ld, int V, int k, int32_t* out, int B, int H, uint32_t seq_mask,
                 hipStream_t s) {
    const int npt = (V + TOPK_THREADS - 1) / TOPK_THREADS;
#define TOPK(N) hipLaunchKernelGGL((k_topk<N>), dim3(B * H), dim3(TOPK_THREADS), 0, s, logits, ld, V, k, out, B, H, seq_mask)
    if (npt <= 1) TOPK(1);
    else if (npt <= 4) TOPK(4);
    else if (npt <= 16) TOPK(16);
    else if (npt <= 32) TOPK(32);
    else if (npt <= 64) TOPK(64);
    else TOPK(160);          // vocabularies up to 163840 ids (validated at model creation)
#undef TOPK
}

// ------------------------------------------------------------------------------------------
// Sampling decoding, statistics of the base distribution of every tree row at a temperature:
// with x_v = (logit_v - max) / temperature, Z = sum exp(x_v), E = sum exp(x_v) x_v, the entropy
// of softmax is H = log Z - E / Z and the typical-acceptance threshold is min(eps, delta exp(-H)).
// A token passes iff exp(x_tok) / Z > threshold, i.e. x_tok > c with
// c = min(log eps, log delta - H) + log Z. One workgroup of 1024 threads per row, the row kept
// in registers between the two reductions; thread sums in fp32, cross-thread sums in fp64.
#define RS_THREADS 1024
static __device__ inline double block_sum_f64(double v, double* sh) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    __syncthreads();                                   // sh may still be read from the previous call
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < RS_THREADS / 64; ++w) t += sh[w];
    return t;
}
template <int NPT>
__global__ __launch_bounds__(RS_THREADS) void k_row_stats(const float* __restrict__ logits, int ld, int V,
                                                          float4* __restrict__ stats, int T, int Tp,
                                                          float inv_temperature, float log_eps, float log_delta) {
    const int j = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const size_t r = (size_t)b * Tp + j;
    const float* row = logits + r * ld;
    float v[NPT];
    float mx = NEG_INF;
#pragma unroll
    for (int i = 0; i < NPT; ++i) {
        const int c = i * RS_THREADS + tid;
        v[i] = c < V ? row[c] : NEG_INF;
        mx = fmaxf(mx, v[i]);
    }
    __shared__ float smax[RS_THREADS / 64];
    __shared__ double ssum[RS_THREADS / 64];
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if ((tid & 63) == 0) smax[tid >> 6] = mx;
    __syncthreads();
    mx = smax[0];
    for (int w = 1; w < RS_THREADS / 64; ++w) mx = fmaxf(mx, smax[w]);
    float z = 0.f, e = 0.f;
#pragma unroll
    for (int i = 0; i < NPT; ++i) {
        const int c = i * RS_THREADS + tid;
        if (c < V) {
            const float x = (v[i] - mx) * inv_temperature;
            const float ex = __expf(x);
            z += ex;
            e += ex * x;                               // exp(x) x -> 0 as x -> -inf
        }
    }
    const double Z = block_sum_f64((double)z, ssum);
    const double E = block_sum_f64((double)e, ssum);
    if (tid == 0) {
        const double H = log(Z) - E / Z;
        const double log_thr = fmin((double)log_eps, (double)log_delta - H);
        stats[r] = make_float4(mx, (float)Z, (float)H, (float)(log_thr + log(Z)));
    }
}

void launch_row_stats(const float* logits, int ld, int V, float4* stats, int B, int T, int Tp, float inv_temperature,
                      float epsilon, float delta, hipStream_t s) {
    const float log_eps = epsilon > 0.f ? logf(epsilon) : NEG_INF, log_delta = delta > 0.f ? logf(delta) : NEG_INF;
    const int npt = (V + RS_THREADS - 1) / RS_THREADS;
#define RS(N) hipLaunchKernelGGL((k_row_stats<N>), dim3(T, B), dim3(RS_THREADS), 0, s, logits, ld, V, stats, T, Tp, \
                                 inv_temperature, log_eps, log_delta)
    if (npt <= 1) RS(1);
    else if (npt <= 4) RS(4);
    else if (npt <= 16) RS(16);
    else if (npt <= 32) RS(32);
    else if (npt <= 64) RS(64);
    else RS(160);
#undef RS
}

// ------------------------------------------------------------------------------------------
// Sampling decoding, the next root: the smallest token id whose cumulative probability under
// softmax(logits[last_row] / temperature) exceeds u. One workgroup of 16 waves per sequence.
// Wave w owns the contiguous ids [w*S, (w+1)*S) and sums their weights exp((l - max)/temp) with
// coalesced loads; the wave whose segment holds the target u * total then walks it 64 ids at a
// time with a wave-wide inclusive scan. Sums are in fp64, so the draw only differs from an
// exact one when u lies within fp32 rounding of the weights of a boundary of the CDF.
static __device__ inline double wave_incl_scan_f64(double v, int lane) {
    for (int o = 1; o < 64; o <<= 1) {
        double t = __shfl_up(v, o);
        if (lane >= o) v += t;
    }
    return v;
}
__global__ __launch_bounds__(RS_THREADS) void k_sample_root(const float* __restrict__ logits, int ld, int V,
                                                            const int32_t* __restrict__ last_row,
                                                            const float* __restrict__ u, float inv_temperature,
                                                            int32_t* __restrict__ root_tok, int n_rows) {
    constexpr int NW = RS_THREADS / 64;
    const int b = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int r = last_row[b];
    if (r < 0 || r >= n_rows) {                        // uniform over the workgroup
        if (tid == 0) root_tok[b] = -1;
        return;
    }
    const float* row = logits + (size_t)r * ld;
    __shared__ float smax[NW];
    __shared__ double wsum[NW];
    float mx = NEG_INF;
#pragma unroll 4
    for (int c = tid; c < V; c += RS_THREADS) mx = fmaxf(mx, row[c]);
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if (lane == 0) smax[wave] = mx;
    __syncthreads();
    mx = smax[0];
    for (int w = 1; w < NW; ++w) mx = fmaxf(mx, smax[w]);
    const int S = ((V + NW - 1) / NW + 63) & ~63;      // segment length, a multiple of the wave size
    const int s0 = min(wave * S, V), s1 = min(s0 + S, V);
    double part = 0.0;
#pragma unroll 4
    for (int c = s0 + lane; c < s1; c += 64) part += (double)__expf((row[c] - mx) * inv_temperature);
    for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o);
    if (lane == 0) wsum[wave] = part;
    __syncthreads();
    double total = 0.0;
    for (int w = 0; w < NW; ++w) total += wsum[w];
    const double target = (double)u[b] * total;
    // the segment that holds the target; if rounding leaves none, the last one that has any mass, walked to its end
    int seg = -1, last_mass = 0;
    double base = 0.0, acc = 0.0;
    for (int w = 0; w < NW; ++w) {
        if (wsum[w] > 0.0) last_mass = w;
        if (seg < 0 && acc + wsum[w] > target) { seg = w; base = acc; }
        acc += wsum[w];
    }
    const bool to_end = seg < 0;
    if (to_end) seg = last_mass;
    if (wave != seg) return;
    int pick = -1, last_pos = s0;
    for (int c0 = s0; c0 < s1 && pick < 0; c0 += 64) {
        const int c = c0 + lane;
        const double e = c < s1 ? (double)__expf((row[c] - mx) * inv_temperature) : 0.0;
        const double cum = base + wave_incl_scan_f64(e, lane);
        const unsigned long long pos = __ballot(e > 0.0);
        if (pos) last_pos = c0 + 63 - __builtin_clzll(pos);
        const unsigned long long hit = __ballot(!to_end && cum > target);
        if (hit) pick = c0 + __builtin_ctzll(hit);
        base = __shfl(cum, 63);
    }
    if (lane == 0) root_tok[b] = pick >= 0 ? pick : last_pos;
}

void launch_sample_root(const float* logits, int ld, int V, const int32_t* last_row, const float* u,
                        float inv_temperature, int32_t* root_tok, int B, int n_rows, hipStream_t s) {
    hipLaunchKernelGGL(k_sample_root, dim3(B), dim3(RS_THREADS), 0, s, logits, ld, V, last_row, u, inv_temperature,
                       root_tok, n_rows);
}

// ------------------------------------------------------------------------------------------
// Greedy acceptance + fragment cut. One workgroup of 64*NW >= T threads per sequence, thread
// j = tree node j (NW = 2 for trees of up to 128 nodes, 4 beyond).
//   match[j]  = tok[j] == am[parent[j]]                     (root: true); under sampling decoding
//               instead: p(tok[j] | parent) > min(eps, delta * exp(-entropy)), from k_row_stats
//   ok[j]     = match holds on every node of j's root path  (prefix-closed acceptance): with
//               the per-wave ballots of `match` gathered into a T-bit mask, ok[j] is one
//               AND of j's ancestor bitset with the complement of that mask
//   best      = deepest ok node (lowest index on equal depth), by wavefront reduction
//   chain     = best's ancestor bitset; node j of the chain sits at chain index depth[j]
//   cut       = 1 + largest chain index whose token is in the stop set; without any stop
//               token: whole chain (keep_all) or 1 (keep_one)
template <int NW>
__global__ __launch_bounds__(64 * NW) void k_verify(VerifyArgs a) {
    const int b = blockIdx.x, j = threadIdx.x, T = a.T, H = a.H;
    const bool valid = j < T;
    const int32_t* tok = a.tok + (size_t)b * a.src_stride;
    const int32_t* am = a.am + (size_t)b * a.src_stride;
    __shared__ unsigned long long matchw[NW], bestanc[NW];
    __shared__ int wkey[NW], stopmax[NW];
    int dj = 0, tj = 0, pj = -1;
    unsigned long long anc[NW] = {};
    bool match = false;
    if (valid) {
        dj = a.depth[j];
        pj = a.parent[j];
        tj = tok[j];
        if (j == 0) {
            match = true;
        } else if (a.row_stats) {
            // the base model's probability of this token at its parent exceeds the threshold of that
            // row, tested on the log side: (logit - max) / temperature > log(threshold * Z)
            const size_t r = (size_t)b * a.src_stride + pj;
            const float4 st = a.row_stats[r];
            match = false;
            if (tj >= 0 && tj < a.V) match = (a.logits[r * a.ld + tj] - st.x) * a.inv_temperature > st.w;
        } else {
            match = tj == am[pj];
        }
        for (int i = j, guard = 0; i >= 0 && guard <= H; i = a.parent[i], ++guard) anc[i >> 6] |= 1ull << (i & 63);
    }
    unsigned long long bal = __ballot(match);
    if ((j & 63) == 0) matchw[j >> 6] = bal;
    __syncthreads();
    unsigned long long miss = 0ull;
#pragma unroll
    for (int w = 0; w < NW; ++w) miss |= anc[w] & ~matchw[w];
    const bool ok = valid && miss == 0ull;
    // deepest accepted node, lowest index on ties: maximise depth * 256 + (255 - j)
    static_assert(SD_MAX_TREE <= 256, "the key holds the node index in 8 bits");
    int key = ok ? dj * 256 + (255 - j) : -1;
    for (int o = 32; o > 0; o >>= 1) key = max(key, __shfl_xor(key, o));
    if ((j & 63) == 0) wkey[j >> 6] = key;
    __syncthreads();
    key = wkey[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) key = max(key, wkey[w]);
    const int best = 255 - (key & 255);
    const int n_raw = (key >> 8) + 1;
    if (j == best) {
#pragma unroll
        for (int w = 0; w < NW; ++w) bestanc[w] = anc[w];
    }
    __syncthreads();
    const bool on_chain = valid && ((bestanc[j >> 6] >> (j & 63)) & 1ull);
    const bool is_stop = on_chain && tj >= 0 && tj < a.V && ((a.stop_mask[tj >> 5] >> (tj & 31)) & 1u);
    int sm = is_stop ? dj : -1;
    for (int o = 32; o > 0; o >>= 1) sm = max(sm, __shfl_xor(sm, o));
    if ((j & 63) == 0) stopmax[j >> 6] = sm;
    __syncthreads();
    sm = stopmax[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) sm = max(sm, stopmax[w]);
    const int n_acc = sm >= 0 ? sm + 1 : (a.fallback == SD_TRUNC_KEEP_ALL ? n_raw : 1);
    const int W = H + 1;
    if (on_chain && dj < n_acc) {
        a.tokens[(size_t)b * W + dj] = tj;
        a.src_slots[(size_t)b * W + dj] = j;
        if (dj == n_acc - 1) {
            if (a.root_tok) a.root_tok[b] = am[j];
            if (a.last_row) a.last_row[b] = b * a.Tp + j;
        }
    }
    if (j >= n_acc && j < W) {
        a.tokens[(size_t)b * W + j] = -1;
        a.src_slots[(size_t)b * W + j] = -1;
    }
    if (j == 0) {
        a.n_accept[b] = n_acc;
        if (a.n_accept_raw) a.n_accept_raw[b] = n_raw;
        if (a.kv_len) {
            int n = a.kv_len[b];
            a.n_old[b] = n;
            a.kv_len[b] = n + n_acc;
        }
    }
}

void launch_verify(const VerifyArgs& a, int B, hipStream_t s) {
    if (a.T <= 128) hipLaunchKernelGGL(k_verify<2>, dim3(B), dim3(128), 0, s, a);
    else hipLaunchKernelGGL(k_verify<4>, dim3(B), dim3(256), 0, s, a);
}

// ------------------------------------------------------------------------------------------
// Commit the kept nodes' K/V rows: tree-scratch row src_slots[j] -> cache row n_old + j, for
// every layer and head. A kept node at chain index j was rotated for position n_old + j
// already (depth = chain index), so this is a pure copy.
// grid: x = head, y = sequence, z = layer; eight waves that share a list of wave-sized tasks, every task a run of
// whole 16-byte pieces that lie side by side in the cache:
//   values: a 16-byte piece of the value layout holds one dim of EIGHT rows (a "group": of a 16-row half of a block,
//     the four rows of one quad and of the quad two further on), so a row cannot move as a piece, and a piece
//     written in parts (2-byte elements, or its 8-byte halves from two workgroups) leaves the memory partial lines.
//     One task = one half x 32 dims: a lane owns one piece, reads it unless all of its eight rows are replaced
//     (its other rows are committed rows, which must survive, or rows past the new length, which nobody reads), takes
//     the new rows' elements and writes the piece whole: 1 KiB per wave, in order (writing only the 8-byte half that
//     has new rows, where one does not, was measured and is slower, short lists included). The new rows' elements
//     come from a copy in LDS of the scratch groups that hold a kept row, fetched once as whole pieces: picked out
//     of global memory two bytes at a time they cost a cache lookup per element and lane, eight times the lookups
//     of everything else here (mirror_groups = 0: no room for that copy, the elements are gathered from global
//     memory).
//   keys: a row's 16-byte pieces move as they are; one task = 8 rows x 8 pieces, rows fastest (the same piece of
//     neighbouring rows is 16 bytes further on, so eight lanes write 128 contiguous bytes).
// Every piece has one owner, and only this workgroup touches this layer's blocks of its (sequence, head).
#define KVC_THREADS 512
static __device__ inline int vgroup_of(int c) { return (c >> 5) * 4 + ((c >> 4) & 1) * 2 + ((c >> 2) & 1); }
__global__ __launch_bounds__(KVC_THREADS) void k_kv_commit(
    const uint16_t* __restrict__ kt, const uint16_t* __restrict__ vt, uint16_t* __restrict__ kc,
    uint16_t* __restrict__ vc, const int32_t* __restrict__ src_slots, const int32_t* __restrict__ n_accept,
    const int32_t* __restrict__ n_old, int nh, int hd, int TB, int cap_blocks, int W, int mirror_groups,
    int L, int lpw, size_t layer_stride_t, size_t layer_stride_c) {
    extern __shared__ __align__(16) uint16_t kvc_mirror[];          // [kept group][hd / 32][32 dims][8 rows]
    __shared__ int s_slots[SD_MAX_TREE];
    __shared__ uint32_t s_need;
    const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int l0 = blockIdx.z * lpw, l1 = min(l0 + lpw, L);
    const int wave = tid >> 6, lane = tid & 63;
    const int a = min(n_accept[b], W);                              // <= SD_MAX_TREE < KVC_THREADS
    if (a <= 0) return;
    const int n = n_old[b];
    const int slot = tid < a ? min(max(src_slots[(size_t)b * W + tid], 0), TB * 32 - 1) : 0;
    if (tid == 0) s_need = 0;
    __syncthreads();
    if (tid < a) {
        s_slots[tid] = slot;
        if (mirror_groups) atomicOr(&s_need, 1u << vgroup_of(slot));
    }
    __syncthreads();
    const size_t toff0 = ((size_t)b * nh + h) * TB * (32 * hd);
    const size_t coff0 = ((size_t)b * nh + h) * cap_blocks * (32 * hd);
    const int EB = hd / 32, KP = hd / 64;                  // wave tasks per 16-row half (values), per 8 rows (keys)
    typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const uint32_t need = s_need;
    const int half0 = n >> 4, nV = (((n + a - 1) >> 4) - half0 + 1) * EB;
    const int NT = nV + ((a + 7) >> 3) * KP;
    // The counts, the slots and the set of groups are the same for every layer: a workgroup reads them once and
    // then goes through its layers (the same number of times for every wave: all of them reach the barriers).
    for (int l = l0; l < l1; ++l) {
        const size_t toff = l * layer_stride_t + toff0, coff = l * layer_stride_c + coff0;
        if (mirror_groups) {                               // (at most min(a, groups of the scratch) <= mirror_groups bits)
            if (l > l0) __syncthreads();                   // the previous layer's readers are done
            for (int i = tid; i < TB * 4 * EB * 32; i += KVC_THREADS) {
                const int grp = i / (EB * 32), eb = (i >> 5) % EB, er = i & 31;
                if ((need >> grp) & 1u) {
                    const int c = (grp >> 2) * 32 + ((grp >> 1) & 1) * 16 + (grp & 1) * 4;   // the group's first row
                    const int at = ((__popc(need & ((1u << grp) - 1u)) * EB + eb) * 32 + er) * 8;
                    *(u16x8*)(kvc_mirror + at) = *(const u16x8*)(vt + toff + vblk_index(c, eb * 32 + er, hd));
                }
            }
            __syncthreads();
        }
        for (int tl = wave; tl < NT; tl += KVC_THREADS / 64) {
            if (tl < nV) {
                const int eb = tl % EB, er = lane & 31, e = eb * 32 + er;
                const int row0 = (half0 + tl / EB) * 16 + (lane >> 5) * 4;   // the piece's rows: row0 + {0..3, 8..11}
                const int lo = n - row0, hi = n + a - row0;                   // new rows: offsets lo <= r < hi
                const bool any = (lo < 4 && hi > 0) || (lo < 12 && hi > 8);
                const bool full = lo <= 0 && hi >= 12;
                if (!any) continue;
                uint16_t* piece = vc + coff + vblk_index(row0, e, hd);
                u16x8 v = {0, 0, 0, 0, 0, 0, 0, 0}, g;
                if (!full) v = *(const u16x8*)piece;
#pragma unroll
                for (int q = 0; q < 8; ++q) {              // (any kept row's element where the piece's row stays)
                    const int c = s_slots[min(max((q >> 2) * 8 + (q & 3) - lo, 0), a - 1)];
                    if (mirror_groups) {
                        const int cs = __popc(need & ((1u << vgroup_of(c)) - 1u));
                        g[q] = kvc_mirror[((cs * EB + eb) * 32 + er) * 8 + ((c >> 3) & 1) * 4 + (c & 3)];
                    } else {
                        g[q] = vt[toff + vblk_index(c, e, hd)];
                    }
                }
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const int r = (q >> 2) * 8 + (q & 3);
                    if (r >= lo && r < hi) v[q] = g[q];
                }
                *(u16x8*)piece = v;
            } else {
                const int tk = tl - nV;
                const int j = (tk / KP) * 8 + (lane & 7), e = ((tk % KP) * 8 + (lane >> 3)) * 8;
                if (j < a)
                    *(u32x4*)(kc + coff + kblk_index(n + j, e, hd)) =
                        *(const u32x4*)(kt + toff + kblk_index(s_slots[j], e, hd));
            }
        }
    }
}

void launch_kv_commit(const void* kt_all, const void* vt_all, void* kc_all, void* vc_all, const int32_t* src_slots,
                      const int32_t* n_accept, const int32_t* n_old, int L, int B, int nh, int hd, int TB,
                      int cap_blocks, int rows, int W, hipStream_t s) {
    (void)rows;
    size_t lst = (size_t)B * nh * TB * 32 * hd, lsc = (size_t)B * nh * cap_blocks * 32 * hd;
    // LDS copy of the scratch groups (8 rows x hd) with a kept row: at most one per row, at most all of them
    int groups = W < TB * 4 ? W : TB * 4;
    size_t mirror = (size_t)groups * 8 * hd * 2;
    if (mirror > 60 * 1024) { groups = 0; mirror = 0; }  // (eight-block scratch at head_dim 128, 31 rows or more)
    int lpw = (int)((size_t)B * nh * L / 1024);            // layers per workgroup: one while the launch is small
    lpw = lpw < 1 ? 1 : lpw > L ? L : lpw;
    hipLaunchKernelGGL(k_kv_commit, dim3(nh, B, (L + lpw - 1) / lpw), dim3(KVC_THREADS), mirror, s,
                       (const uint16_t*)kt_all, (const uint16_t*)vt_all, (uint16_t*)kc_all, (uint16_t*)vc_all, src_slots,
                       n_accept, n_old, nh, hd, TB, cap_blocks, W, groups, L, lpw, lst, lsc);
}

// ------------------------------------------------------------------------------------------
// Natural-layout rows [nrows][nh][hd] <-> one sequence's cache blocks of one layer.
__global__ void k_kv_rows(uint16_t* __restrict__ kc, uint16_t* __restrict__ vc, uint16_t* __restrict__ k_rows,
                          uint16_t* __restrict__ v_rows, int row0, int nh, int hd, int cap_blocks, int to_cache) {
    const int r = blockIdx.x, h = blockIdx.y, e = threadIdx.x;
    const size_t nat = ((size_t)r * nh + h) * hd + e;
    const size_t hoff = (size_t)h * cap_blocks * (32 * hd);
    const size_t ki = hoff + kblk_index(row0 + r, e, hd), vi = hoff + vblk_index(row0 + r, e, hd);
    if (to_cache) {
        kc[ki] = k_rows[nat];
        vc[vi] = v_rows[nat];
    } else {
        k_rows[nat] = kc[ki];
        v_rows[nat] = vc[vi];
    }
}

void launch_kv_rows(void* kc, void* vc, void* k_rows, void* v_rows, int row0, int nrows, int nh, int hd,
                    int cap_blocks, int to_cache, hipStream_t s) {
    hipLaunchKernelGGL(k_kv_rows, dim3(nrows, nh), dim3(hd), 0, s, (uint16_t*)kc, (uint16_t*)vc, (uint16_t*)k_rows,
                       (uint16_t*)v_rows, row0, nh, hd, cap_blocks, to_cache);
}

// ------------------------------------------------------------------------------------------
// Small copies out of the padded internal buffers into the caller's dense outputs.
__global__ void k_copy_logits(const float* __restrict__ src, int ld, float* __restrict__ dst, int V, int T, int Tp) {
    const int b = blockIdx.y / T, j = blockIdx.y % T;
    const float* s = src + (size_t)(b * Tp + j) * ld;
    float* d = dst + (size_t)(b * T + j) * V;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < V; i += gridDim.x * blockDim.x) d[i] = s[i];
}
void launch_copy_logits(const float* src, int ld, float* dst, int V, int B, int T, int Tp, hipStream_t s) {
    hipLaunchKernelGGL(k_copy_logits, dim3(16, B * T), dim3(256), 0, s, src, ld, dst, V, T, Tp);
}

__global__ void k_copy_row_stats(const float4* __restrict__ src, float4* __restrict__ dst, int B, int T, int Tp) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < B * T) dst[i] = src[(i / T) * Tp + i % T];
}
void launch_copy_row_stats(const float4* src, float4* dst, int B, int T, int Tp, hipStream_t s) {
    hipLaunchKernelGGL(k_copy_row_stats, dim3((B * T + 255) / 256), dim3(256), 0, s, src, dst, B, T, Tp);
}

__global__ void k_copy_rows_i32(const int32_t* __restrict__ src, int32_t* __restrict__ dst, int B, int T, int Tp) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < B * T) dst[i] = src[(i / T) * Tp + i % T];
}
void launch_copy_rows_i32(const int32_t* src, int32_t* dst, int B, int T, int Tp, hipStream_t s) {
    hipLaunchKernelGGL(k_copy_rows_i32, dim3((B * T + 255) / 256), dim3(256), 0, s, src, dst, B, T, Tp);
}

// head logits: internal row (i*B + b) -> dst [b][i][V]
__global__ void k_copy_head_logits(const float* __restrict__ src, int ld, float* __restrict__ dst, int V, int B, int H) {
    const int r = blockIdx.y, i = r / B, b = r % B;
    const float* s = src + (size_t)r * ld;
    float* d = dst + ((size_t)b * H + i) * V;
    for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < V; c += gridDim.x * blockDim.x) d[c] = s[c];
}
void launch_copy_head_logits(const float* src, int ld, float* dst, int V, int B, int H, hipStream_t s) {
    hipLaunchKernelGGL(k_copy_head_logits, dim3(16, B * H), dim3(256), 0, s, src, ld, dst, V, B, H);
}

__global__ void k_fill_i32(int32_t* p, int32_t v, int n) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
void launch_fill_i32(int32_t* p, int32_t v, int n, hipStream_t s) {
    hipLaunchKernelGGL(k_fill_i32, dim3((n + 255) / 256), dim3(256), 0, s, p, v, n);
}

__global__ void k_copy_i32(const int32_t* __restrict__ src, int32_t* __restrict__ dst, int n) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}
void launch_copy_i32(const int32_t* src, int32_t* dst, int n, hipStream_t s) {
    hipLaunchKernelGGL(k_copy_i32, dim3((n + 255) / 256), dim3(256), 0, s, src, dst, n);
}

// Prompt chunks commit every row: slots are the identity, the count is the chunk length.
__global__ void k_prefill_commit_setup(ChainArgs ca, int B, int Tp, int32_t* __restrict__ src_slots,
                                       int32_t* __restrict__ n_accept, int32_t* __restrict__ n_old,
                                       int32_t* __restrict__ kv_len, int32_t* __restrict__ last_row) {
    const int b = blockIdx.x, j = threadIdx.x;
    if (j < Tp) src_slots[(size_t)b * Tp + j] = j;
    if (j == 0) {
        int n = kv_len[b];
        n_old[b] = n;
        n_accept[b] = ca.len[b];
        kv_len[b] = n + ca.len[b];
        if (ca.len[b] > 0) last_row[b] = b * Tp + ca.len[b] - 1;
    }
}
void launch_prefill_commit_setup(const ChainArgs& ca, int B, int Tp, int32_t* src_slots, int32_t* n_accept,
                                 int32_t* n_old, int32_t* kv_len, int32_t* last_row, hipStream_t s) {
    hipLaunchKernelGGL(k_prefill_commit_setup, dim3(B), dim3(SD_MAX_TREE), 0, s, ca, B, Tp, src_slots, n_accept, n_old,
                       kv_len, last_row);
}

// commit stage alone: the count of every sequence clamped to [0, width], old length noted, new length set
__global__ void k_commit_setup(const int32_t* __restrict__ n_rows, int width, int B, int32_t* __restrict__ n_accept,
                               int32_t* __restrict__ n_old, int32_t* __restrict__ kv_len) {
    const int b = threadIdx.x;
    if (b >= B) return;
    const int a = min(max(n_rows[b], 0), width), n = kv_len[b];
    n_accept[b] = a;
    n_old[b] = n;
    kv_len[b] = n + a;
}
void launch_commit_setup(const int32_t* n_rows, int width, int B, int32_t* n_accept, int32_t* n_old, int32_t* kv_len,
                         hipStream_t s) {
    hipLaunchKernelGGL(k_commit_setup, dim3(1), dim3(SD_MAX_BATCH), 0, s, n_rows, width, B, n_accept, n_old, kv_len);
}

// root_tok[b] = arg-max at the last prompt row, for the sequences whose prompt just ended
__global__ void k_pick_root(const int32_t* __restrict__ am, const int32_t* __restrict__ last_row,
                            int32_t* __restrict__ root_tok, int B, uint32_t seq_mask) {
    int b = threadIdx.x;
    if (b < B && ((seq_mask >> b) & 1u)) root_tok[b] = am[last_row[b]];
}
void launch_pick_root(const int32_t* am, const int32_t* last_row, int32_t* root_tok, int B, uint32_t seq_mask,
                      hipStream_t s) {
    hipLaunchKernelGGL(k_pick_root, dim3(1), dim3(SD_MAX_BATCH), 0, s, am, last_row, root_tok, B, seq_mask);
}
