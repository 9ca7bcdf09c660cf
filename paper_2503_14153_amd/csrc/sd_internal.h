// Internal declarations shared by the HIP translation units of libspecdec (gfx950 only).
//
// Memory layouts (all "fragment" layouts are chosen so that one wave64 load instruction of
// 16 bytes per lane fetches one contiguous 1 KiB MFMA operand of v_mfma_f32_32x32x16_bf16:
// lane l supplies row/column (l % 32) and the eight contraction elements g*8 .. g*8+7 with
// g = l / 32):
//
//   packed activation  X[kb][mb][part][lane][8]  element (row m, col k): kb = k/16, mb = m/32,
//                                            lane = m%32 + 32*((k/8)&1), slot = k%8;
//                                            part 0 = bf16(x), part 1 = bf16(x - part 0): the
//                                            activations enter the MFMAs as a two-term bf16
//                                            expansion (about 16 mantissa bits), see gemm.hip
//   packed weight      W[kb][nb][lane][8]    element (out n, in k):  nb = n/32, kb = k/16,
//                                            lane = n%32 + 32*((k/8)&1), slot = k%8
//   key block (32 rows of one head)          K[kk][lane][8]: row c, dim e: kk = e/16,
//                                            lane = c%32 + 32*((e/8)&1), slot = e%8
//   value block (32 rows of one head)        V[p][eb][lane][8]: row c, dim e: p = (c%32)/16,
//                                            eb = e/32, lane = e%32 + 32*((c/4)&1),
//                                            slot = 4*((c/8)&1) + c%4
//     (the value rows are permuted inside a block so that the softmax probabilities, as they
//      come out of the QK^T accumulator, are already the B operand of the PV product)
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/specdec.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

#ifdef __HIPCC__
// two-term bf16 expansion of eight floats: hi = bf16(f), lo = bf16(f - hi)
static __device__ inline void split_hilo(const float (&f)[8], bf16x8& hi, bf16x8& lo) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        __bf16 h = (__bf16)f[i];
        hi[i] = h;
        lo[i] = (__bf16)(f[i] - (float)h);
    }
}
#endif

#define SD_MAX_TREE 256
#define SD_ANC_WORDS 8

// element index of (row m, col k) in part 0 of a packed activation; part 1 is XPART further
#define XPART 512
static __host__ __device__ inline size_t xpack_index(int m, int k, int MB) {
    int kb = k >> 4, g = (k >> 3) & 1, s = k & 7, mb = m >> 5, r = m & 31;
    return ((((size_t)kb * MB + mb) * 2 * 64) + (size_t)(r + 32 * g)) * 8 + s;
}
// same for a query block: Q[kk][part][lane][8] per 32 queries of one head
static __host__ __device__ inline size_t qblk_index(int t, int e, int HD) {
    int blk = t >> 5, r = t & 31, kk = e >> 4, g = (e >> 3) & 1, s = e & 7;
    return (size_t)blk * (64 * HD) + ((size_t)(kk * 2 * 64 + r + 32 * g)) * 8 + s;
}
// offset (in elements) of (row c, dim e) inside a head's key blocks; HD = head_dim
static __host__ __device__ inline size_t kblk_index(int c, int e, int HD) {
    int blk = c >> 5, r = c & 31, kk = e >> 4, g = (e >> 3) & 1, s = e & 7;
    return (size_t)blk * (32 * HD) + ((size_t)(kk * 64 + r + 32 * g)) * 8 + s;
}
static __host__ __device__ inline size_t vblk_index(int c, int e, int HD) {
    int blk = c >> 5, cc = c & 31, p = cc >> 4, g = (cc >> 2) & 1, s = ((cc >> 3) & 1) * 4 + (cc & 3);
    int eb = e >> 5, er = e & 31;
    return (size_t)blk * (32 * HD) + ((size_t)((p * (HD / 32) + eb) * 64 + er + 32 * g)) * 8 + s;
}

// ---- per-call row table (device) -----------------------------------------------------------
struct RowTable {
    int32_t* tok;      // [M] token id of every row (0 for padding rows)
    int32_t* pos;      // [M] position
    uint32_t* anc;     // [M][SD_ANC_WORDS] bit i set: row may attend tree row i of its sequence
    float2* cs;        // [M][head_dim/2] (cos, sin) of the rotary angle
};

// Partial results of a GEMM whose contraction was divided over several workgroups: the
// consumer sums `count(col)` slots. cnt == NULL means every column has nmax slots.
struct PartView {
    const float* base;
    size_t slot_stride;      // floats between slots
    int ld;                  // floats between rows
    const int32_t* cnt;      // [ceil(ld / 256)] slots per 256-column group, or NULL
    int nmax;
};
#ifdef __HIPCC__
static __device__ inline int part_count(const PartView& p, int col) { return p.cnt ? p.cnt[col >> 8] : p.nmax; }
#endif

// Rows whose RMSNorm scale is applied AFTER the contraction (the operand holds x * gain, see row_ops.h):
// ssq [ceil(n_parts / 4)][Mp][4] partial sums of squares of every row (Mp = the GEMM's padded row count, part p of
// row m at ((p / 4) * Mp + m) * 4 + p % 4; parts beyond n_parts are zero); every output of row m is multiplied by
// 1 / sqrt(sum_p ssq[p][m] * inv_d + eps).
struct SkRowScale {
    const float* ssq;        // NULL: no scaling
    int n_parts;
    float inv_d, eps;
};

// How one GEMM shape is launched (made once per shape at model creation).
struct GemmPlan {
    int MB, KB, NB;
    int G, NG;               // workgroups, 256-column groups
    int upw, rem;            // units per workgroup; the first `rem` workgroups take one more
    int slots;               // slots the output buffer must hold
    int uniform;             // 1: every column group has exactly `slots` contributors
    int CG, S;               // four / eight row blocks as launched by launch_gemm: column groups of CG blocks, each
                             // split into S segments of the contraction (workgroup = group * S + segment, slot =
                             // segment); 0 for one and two row blocks. The fields above then describe the balanced
                             // split that the persistent layer kernel walks at eight row blocks.
    int slots_max;           // slots the output buffer must hold for either
    int32_t* cnt_dev;        // [NG] contributors per column group (device)
    int32_t* slot0_dev;      // [G] slot of every workgroup's first segment (device)
};

// ---- the persistent layer kernel (fused.hip) -----------------------------------------------
// One weight-streaming GEMM as a phase: its plan, operands and the buffer of its partial sums.
struct FusedGemm {
    const bf16x8* X;         // packed activations (written by an earlier phase of the same launch)
    const bf16x8* W;         // packed weights
    float* out;              // partial sums [slot][row][col]
    size_t slot_stride;
    int KB, NB, ldo, upw, rem, G, nmax;
    uint32_t kb_magic;
    const int32_t* slot0;    // [G]
    const int32_t* cnt;      // [NG] or NULL (nmax slots everywhere)
    SkRowScale sc;           // deferred RMS scale of the rows (the GEMMs that follow a norm), or ssq NULL
};
struct FusedSync {
    unsigned* counters;      // this launch's barrier counters: 9 words 256 bytes apart, zero at launch
    unsigned* abort_flag;    // set to 1 by a workgroup whose wait ran out
    unsigned long long timeout_ticks;   // of the 100 MHz real-time counter
};
// what a launch runs, in this order; each GEMM comes with the row-wise phase that produces its operand
enum {
    FUSED_GEMM_O = 1,        // merge of the attention parts, O projection
    FUSED_GEMM_GU = 2,       // residual + norm (feed-forward), gate/up projection
    FUSED_GEMM_DN = 4,       // SwiGLU, down projection
    FUSED_GEMM_Q = 8,        // residual + norm (attention, or the final one), QKV projection or LM head
    FUSED_ROPE = 16          // rotary embedding and the tree K/V write
};
#define FUSED_SYNC_WORDS 1024    // counters of one launch (9 used, spaced 64 words)
struct FusedArgs {
    uint32_t phases;         // FUSED_* bits
    int M, MB, B, Tp, d, nh, hd, F, Fpad, nparts;
    float eps;
    float* x;                // residual stream [M][d]
    const float* opart; const float2* mlpart;      // attention parts (merge)
    bf16x8* att;             // merged attention output, operand of g_o
    FusedGemm g_o, g_gu, g_dn, g_q;
    const uint16_t* gain_f; bf16x8* xn_f; float* ssq_f;   // norm before the feed-forward block -> operand of g_gu
    bf16x8* act;             // SwiGLU output, operand of g_dn
    const uint16_t* gain_a; bf16x8* xn_a; float* ssq_a;   // norm before attention (or the final norm) -> operand of g_q
    PartView prev;           // what NORM_A adds when the launch starts with it
    RowTable rt; bf16x8* q; uint16_t* kt; uint16_t* vt;   // rotary phase outputs
    const bf16x8* zfrag;
    FusedSync sync;
    unsigned long long* timeline;   // NULL, or [24][gridDim.x] time stamps (100 MHz): entry to each phase, end of launch
};

#define SD_MAX_BATCH 32
#define SD_MAX_MEDUSA 15
struct ChainArgs { int32_t off[SD_MAX_BATCH]; int32_t len[SD_MAX_BATCH]; };
struct MedusaBias { const uint16_t* p[SD_MAX_MEDUSA + 1]; };
struct VerifyArgs {
    const int32_t *parent, *depth;      // device tree tables [T]
    int T, H, fallback, src_stride, Tp, V;
    const int32_t *tok, *am;            // [B][src_stride]
    const uint32_t* stop_mask;
    int32_t *n_accept, *n_accept_raw, *tokens, *src_slots;   // outputs, [B] / [B][H+1]
    int32_t *kv_len, *n_old, *root_tok, *last_row;           // carried state, may be NULL
    // typical acceptance (sampling decoding) instead of greedy when row_stats != NULL
    const float* logits;                // [B*Tp][ld]
    int ld;
    const float4* row_stats;            // [B*Tp]: {max logit, Z, entropy, c = log(threshold * Z)} per row
    float inv_temperature;
};

// ---- launchers (defined in the kernel translation units) ----------------------------------
// All take a stream; all sizes have been validated by the caller.
void launch_pack_weight(const void* src, void* dst, int N, int K, int nb_offset, int NBdst, int KB, hipStream_t s);
// fills every field of the plan except cnt_dev; cnt_host receives the per-group counts
// cnt_host [>= ceil(NB/8)] and slot0_host [>= 256] receive the tables the device copies hold
void gemm_plan_make(GemmPlan* p, int MB, int KB, int NB, int32_t* cnt_host, int32_t* slot0_host);
// out must hold plan.slots * (MB*32) * (NB*32) floats; zfrag: 1 KiB of zeros (device);
// returns the view consumers read
// ev0 / ev1 (both or neither): events that receive the kernel's own start and end time stamps,
// for per-kernel timing without launch gaps
// sc: deferred RMS scale of the rows (ssq NULL: none; not available at four row blocks)
PartView launch_gemm(const GemmPlan& p, const void* Xp, const void* Wp, const void* zfrag, float* out, hipStream_t s,
                     hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
// persistent layer kernel: G workgroups (all must be resident at once), a.MB in {1, 2, 8}
void launch_layer(const FusedArgs& a, int G, hipStream_t s, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
// how many of its workgroups the device can hold at once (0 on error)
int fused_max_resident(int device);
void launch_reduce_slots(PartView pv, float* dst, int rows, hipStream_t s);
// dst row i*B + b = summed row (i*M + sel[b]) - row0 of pv when it lies in [0, rows); i < H, b < B
void launch_reduce_selected(PartView pv, float* dst, const int32_t* sel, int B, int H, int M, int row0, int rows,
                            hipStream_t s);

void launch_build_rows_tree(RowTable rt, const int32_t* parent, const int32_t* depth, const int32_t* rank,
                            const int32_t* root_tok, const int32_t* cand, const int32_t* kv_len,
                            int B, int T, int Tp, int H, int topk, int hd, float theta,
                            const void* embed, int embed_f32, int d, int V, float* x, hipStream_t s);
void launch_build_rows_chain(RowTable rt, const int32_t* tokens, const ChainArgs& ca, const int32_t* kv_len,
                             int B, int Tp, int hd, float theta, const void* embed, int embed_f32, int d, int V,
                             float* x, hipStream_t s);
// float32 device path (f32.hip): natural row-major layouts, vector-ALU arithmetic
void launch_f32_rmsnorm(const float* x, const float* gain, float eps, float* y, int M, int d, const int32_t* gather,
                        hipStream_t s);
void launch_f32_linear(const float* X, const float* W, const float* bias, float* out, int M, int N, int K, int ldx, int ldo,
                       int accumulate, hipStream_t s);
void launch_f32_rope_kv(const float* qkv, RowTable rt, float* q, float* kt, float* vt, int M, int nh, int hd, hipStream_t s);
void launch_f32_attn(const float* q, const float* kc, const float* vc, const float* kt, const float* vt,
                     const int32_t* kv_len, const uint32_t* anc, float* out, int B, int nh, int hd, int Tp, int cap,
                     hipStream_t s);
void launch_f32_swiglu(const float* gu, float* act, int M, int F, hipStream_t s);
void launch_f32_medusa_act(const float* z, const float* h, float* out, int B, int H, int d, hipStream_t s);
void launch_f32_kv_commit(const float* kt, const float* vt, float* kc, float* vc, const int32_t* src_slots,
                          const int32_t* n_accept, const int32_t* n_old, int L, int B, int d, int Tp, int cap, int W,
                          hipStream_t s);
void launch_f32_kv_rows(float* kc, float* vc, float* k_rows, float* v_rows, int row0, int nrows, int d, int to_cache,
                        hipStream_t s);
void launch_norm_pack(float* x, PartView pv, const void* gain, float eps, void* xn_packed, float* hf_out,
                      int M, int d, int MB, const int32_t* gather, hipStream_t s);
// RMSNorm with the scale deferred: operand = x * gain, ssq_part = partial sums of squares in SkRowScale's layout
void launch_rope_kv(PartView pv, RowTable rt, void* q_packed, void* kt, void* vt, int B, int Tp, int nh, int hd,
                    hipStream_t s);
void launch_tree_attn(const void* q_packed, const void* kc, const void* vc, const void* kt, const void* vt,
                      const int32_t* kv_len, const uint32_t* anc, float* opart, float2* mlpart,
                      int B, int nh, int hd, int Tp, int cap_blocks, int ncparts, int per, int tree_sep,
                      hipStream_t s, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr, const PartView* qkv = nullptr,
                      const RowTable* rt = nullptr);
void launch_attn_merge(const float* opart, const float2* mlpart, void* x_packed, int B, int nh, int hd,
                       int Tp, int nparts, int MB, hipStream_t s);
void launch_swiglu_pack(PartView pv, int F, int Fpad, void* act_packed, int M, int MB, hipStream_t s);
// output rows i*B + b in chunks of chunk_rows rows, each a packed activation of MB (last: MBlast) row blocks
void launch_medusa_act(PartView pv, const float* h_rows, const MedusaBias& bias, int B, int H, int d,
                       void* x_packed, int chunk_rows, int MB, int MBlast, hipStream_t s);
// arg-max of the first T rows of every sequence from the LM head's partial sums; logits_or_null: also write the
// summed logits of those rows ([row][pv.ld])
void launch_reduce_argmax(PartView pv, float* logits_or_null, int V, int32_t* am, int B, int T, int Tp, hipStream_t s);
void launch_argmax(const float* logits, int ld, int V, int32_t* am, int B, int T, int Tp, hipStream_t s);
void launch_topk(const float* logits, int ld, int V, int k, int32_t* out, int B, int H, uint32_t seq_mask,
                 hipStream_t s);
void launch_pick_root(const int32_t* am, const int32_t* last_row, int32_t* root_tok, int B, uint32_t seq_mask,
                      hipStream_t s);
void launch_verify(const VerifyArgs& a, int B, hipStream_t s);
// per tree row: softmax statistics at a temperature and the typical-acceptance threshold (see decide.hip)
void launch_row_stats(const float* logits, int ld, int V, float4* stats, int B, int T, int Tp, float inv_temperature,
                      float epsilon, float delta, hipStream_t s);
// root_tok[b] = inverse-CDF draw at u[b] from softmax(logits[last_row[b]] * inv_temperature);
// -1 for a row index outside [0, n_rows)
void launch_sample_root(const float* logits, int ld, int V, const int32_t* last_row, const float* u,
                        float inv_temperature, int32_t* root_tok, int B, int n_rows, hipStream_t s);
// syntax-enriched label matrix [B][H+1][S] from the base label rows [B][S] (labels.hip)
void launch_build_labels(const int32_t* l0, int B, int S, int H, int32_t frag, int32_t pad, int32_t ignore,
                         int keep_all, int32_t* labels, hipStream_t s);
void launch_copy_row_stats(const float4* src, float4* dst, int B, int T, int Tp, hipStream_t s);
void launch_kv_commit(const void* kt_all, const void* vt_all, void* kc_all, void* vc_all,
                      const int32_t* src_slots, const int32_t* n_accept, const int32_t* n_old,
                      int L, int B, int nh, int hd, int TB, int cap_blocks, int rows, int W, hipStream_t s);
void launch_commit_setup(const int32_t* n_rows, int width, int B, int32_t* n_accept, int32_t* n_old, int32_t* kv_len,
                         hipStream_t s);
void launch_kv_rows(void* kc, void* vc, void* k_rows, void* v_rows, int row0, int nrows, int nh, int hd,
                    int cap_blocks, int to_cache, hipStream_t s);
void launch_copy_logits(const float* src, int ld, float* dst, int V, int B, int T, int Tp, hipStream_t s);
void launch_copy_rows_i32(const int32_t* src, int32_t* dst, int B, int T, int Tp, hipStream_t s);
void launch_copy_head_logits(const float* src, int ld, float* dst, int V, int B, int H, hipStream_t s);
void launch_fill_i32(int32_t* p, int32_t v, int n, hipStream_t s);
void launch_copy_i32(const int32_t* src, int32_t* dst, int n, hipStream_t s);
void launch_prefill_commit_setup(const ChainArgs& ca, int B, int Tp, int32_t* src_slots, int32_t* n_accept,
                                 int32_t* n_old, int32_t* kv_len, int32_t* last_row, hipStream_t s);
