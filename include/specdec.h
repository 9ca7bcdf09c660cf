/*
 * libspecdec -- the syntax-aligned speculative-decoding step on one MI355X (gfx950).
 *
 * One step (paper Section III-B, "Model Architecture"): at position t the base model's
 * token for t+1 and the top-k tokens of every draft head (head i drafts t+i+1) form a fixed
 * token tree; the base decoder verifies the whole tree in one forward pass (tree-masked
 * attention over the KV cache); a drafted token is accepted only if it and every token
 * before it is accepted (greedy decoding: equals the base arg-max given the tokens before
 * it); the accepted run is cut back to the end of its last complete syntactic fragment (a
 * token of the stop set, the paper's [FRAG] boundary, Section III-C); the longest such
 * prefix is emitted and its key/value rows are committed to the cache.
 *
 * Conventions
 *   - Every function returns SD_OK (0) or a negative sd_status. On error nothing has been
 *     enqueued and no state has changed; sd_last_error() gives a message (thread-local).
 *   - "dev" pointers are device memory owned by the caller (PyTorch allocates it) and are
 *     only borrowed for the duration documented per call. "host" pointers are host memory.
 *   - `stream` is a hipStream_t passed as void*. Calls that take a stream are asynchronous
 *     on it; results are valid once the caller has synchronised the stream. A handle must
 *     be used from one thread and one stream at a time.
 *   - All weight matrices are row-major [out_features][in_features] (y = W x), in the element
 *     type sd_config.dtype names.
 *   - dtype = SD_DTYPE_BF16: weights and cache rows are bfloat16, products run on the matrix
 *     cores with float32 accumulation: the production path, the one every performance figure is for.
 *     dtype = SD_DTYPE_F32: weights, activations and cache rows are float32 and every product is
 *     accumulated in float32 on the vector ALUs, with plain kernels: for configurations that are
 *     specified in float32 (small ones: correctness, not speed). Same entry points, same integer
 *     stages; differences: sd_kv_write_rows / sd_kv_read_rows move float32 rows, the draft heads
 *     always run after acceptance (sd_set_draft_schedule is accepted and has no effect),
 *     sd_set_fused has no effect, and sd_profile_end reports no launches.
 *   - head_dim must be 64 or 128; d_model a multiple of 32, d_ffn of 16; n_medusa <= 15;
 *     topk <= 32; tree nodes <= 256.
 */
#ifndef SPECDEC_H
#define SPECDEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sd_status {
    SD_OK = 0,
    SD_ERR_NULL = -1,      /* a required pointer was NULL                                   */
    SD_ERR_SHAPE = -2,     /* configuration or sizes not supported / inconsistent           */
    SD_ERR_BAD_TREE = -3,  /* tree_spec is not a valid candidate tree                       */
    SD_ERR_KV_FULL = -4,   /* the step could overflow the cache; nothing was enqueued       */
    SD_ERR_HIP = -5,       /* a HIP runtime call failed (text in sd_last_error)             */
    SD_ERR_STATE = -6      /* call order violated (e.g. a step before any prefill)          */
} sd_status;

enum { SD_DTYPE_F32 = 0, SD_DTYPE_BF16 = 1 };
/* What to keep when the accepted run holds no stop token at all: the paper only describes
 * the case where a complete fragment exists inside the run (Section III-B).               */
enum { SD_TRUNC_KEEP_ALL = 0, SD_TRUNC_KEEP_ONE = 1 };

typedef struct sd_config {
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    int32_t n_medusa;        /* H: draft heads                                              */
    int32_t topk;            /* k: candidates kept per head                                 */
    int32_t dtype;           /* SD_DTYPE_*                                                  */
    int32_t trunc_fallback;  /* SD_TRUNC_*                                                  */
    float rope_theta, rms_eps;
} sd_config;

/* Device pointers to the caller's weights (bfloat16 or float32, as sd_config.dtype says). Per-layer arrays are host arrays of
 * n_layers (resp. n_medusa) device pointers. medusa_b may be NULL (no bias).
 * wqkv stacks q, k, v along the output axis: [3*d_model][d_model].                         */
typedef struct sd_weights {
    const void* embed;              /* dev [vocab][d_model]                                  */
    const void* lm_head;            /* dev [vocab][d_model]                                  */
    const void* final_norm;         /* dev [d_model]                                         */
    const void* const* attn_norm;   /* host[n_layers] -> dev [d_model]                       */
    const void* const* wqkv;        /* host[n_layers] -> dev [3*d_model][d_model]            */
    const void* const* wo;          /* host[n_layers] -> dev [d_model][d_model]              */
    const void* const* ffn_norm;    /* host[n_layers] -> dev [d_model]                       */
    const void* const* w_gate;      /* host[n_layers] -> dev [d_ffn][d_model]                */
    const void* const* w_up;        /* host[n_layers] -> dev [d_ffn][d_model]                */
    const void* const* w_down;      /* host[n_layers] -> dev [d_model][d_ffn]                */
    const void* const* medusa_w;    /* host[n_medusa] -> dev [d_model][d_model]              */
    const void* const* medusa_b;    /* host[n_medusa] -> dev [d_model], or NULL              */
} sd_weights;

typedef struct sd_model sd_model;
typedef struct sd_kv sd_kv;
typedef struct sd_tree sd_tree;

/* ---- model ------------------------------------------------------------------------------
 * sd_model_create copies every weight into a library-owned device arena (bfloat16 models: re-tiled so
 * that one wavefront load instruction fetches one contiguous 1 KiB MFMA operand fragment; float32
 * models: as they are). The
 * caller's weight buffers are read on `stream` during this call only; the call synchronises
 * the stream before returning, after which the caller may free them. `max_rows` is the
 * largest batch * round_up(tree_nodes, 32) any later call will use (workspace is sized for
 * it). Blocking; allocates device memory. */
int sd_model_create(const sd_config* cfg, const sd_weights* w, int32_t max_rows, void* stream,
                    sd_model** out);
int sd_model_destroy(sd_model* m);

/* ---- KV cache ---------------------------------------------------------------------------
 * The cache lives in ONE caller-allocated device buffer of sd_kv_bytes(...) bytes; its
 * internal tiling is private (bfloat16: keys and values are stored as ready-made MFMA fragments of
 * 32 cache rows), use sd_kv_write_rows / sd_kv_read_rows to move rows in natural layout.
 * `cap` = capacity in rows per sequence. A step needs kv_len + n_medusa + 1 <= cap (the
 * tree's own keys/values live in a library-owned scratch, not in the cache).               */
size_t sd_kv_bytes(const sd_config* cfg, int32_t batch, int32_t cap);
/* dev_buf: dev, at least sd_kv_bytes(...) bytes, 16-byte aligned, owned by the caller and borrowed until
 * sd_kv_destroy. Its first sd_kv_bytes(...) bytes are cleared by this call (whatever the buffer held before
 * cannot reach a result); the call blocks until the device is idle and allocates a small state block.   */
int sd_kv_create(const sd_model* m, int32_t batch, int32_t cap, void* dev_buf, size_t bytes,
                 sd_kv** out);
int sd_kv_destroy(sd_kv* kv);
/* Committed length per sequence -> host out_len[batch]. Synchronises `stream`.              */
int sd_kv_len(sd_kv* kv, int32_t* out_len, void* stream);
/* Set the committed length per sequence from host len[batch] (roll back after a step, or
 * declare rows written by sd_kv_write_rows as committed). Rows beyond len are ignored.     */
int sd_kv_set_len(sd_kv* kv, const int32_t* len, void* stream);
/* Copy `nrows` rows starting at cache row `row0` of sequence `seq`, layer `layer`, between
 * the cache and natural-layout device arrays k_rows / v_rows: [nrows][n_heads][head_dim] of the
 * model's element type (bfloat16 or float32).
 * Keys are stored as given (they must already be rotated to their positions).              */
int sd_kv_write_rows(sd_kv* kv, int32_t layer, int32_t seq, int32_t row0, int32_t nrows,
                     const void* k_rows, const void* v_rows, void* stream);
int sd_kv_read_rows(sd_kv* kv, int32_t layer, int32_t seq, int32_t row0, int32_t nrows,
                    void* k_rows, void* v_rows, void* stream);
/* Overwrite the carried draft state of every sequence: the base model's token for the next
 * position (dev root_tok[batch]) and the heads' candidates (dev cand[batch][n_medusa][topk]).
 * Used with synthetic caches, and to resynchronise a lock-step comparison.                 */
int sd_kv_set_draft(sd_kv* kv, const int32_t* root_tok, const int32_t* cand, void* stream);
/* Read the carried draft state back (same shapes, dev pointers).                           */
int sd_kv_get_draft(sd_kv* kv, int32_t* root_tok, int32_t* cand, void* stream);

/* ---- candidate tree ---------------------------------------------------------------------
 * Host arrays of T entries: parent[0] = -1, parent[j] < j, depth[j] = depth[parent[j]] + 1
 * <= n_medusa, rank[j] < topk, siblings have distinct ranks. Node j >= 1 carries head
 * (depth[j]-1)'s candidate number rank[j]; node 0 carries the base model's token.
 * The arrays are copied. Returns SD_ERR_BAD_TREE if any rule is broken.                    */
int sd_tree_create(int32_t T, const int32_t* parent, const int32_t* depth, const int32_t* rank,
                   int32_t n_medusa, int32_t topk, sd_tree** out);
int sd_tree_destroy(sd_tree* t);

/* ---- decoding ---------------------------------------------------------------------------*/
/* Run the prompts through the base model (causal), commit their keys/values after the rows
 * already committed, and draft from each prompt's last position. tokens: dev int32, the
 * prompts back to back; lens: host [batch], each >= 1. kv_len + len must be <= cap.         */
int sd_prefill(sd_model* m, sd_kv* kv, const int32_t* tokens, const int32_t* lens, void* stream);

typedef struct sd_step_io {
    int32_t* n_accept;         /* dev [batch]: tokens emitted by this step, 1..n_medusa+1     */
    int32_t* tokens;           /* dev [batch][n_medusa+1]: emitted tokens, rest -1            */
    int32_t* src_slots;        /* dev [batch][n_medusa+1]: tree node whose K/V row was
                                  committed at cache row old_len + j, rest -1                 */
    int32_t* n_accept_raw;     /* dev [batch] or NULL: accepted length before the cut         */
    float* logits;             /* dev [batch][T][vocab] or NULL: base logits of every node    */
    int32_t* argmax;           /* dev [batch][T] or NULL: base arg-max of every node          */
    float* head_logits;        /* dev [batch][n_medusa][vocab] or NULL: draft-head logits at
                                  the last kept node                                          */
    const int32_t* forced_cand;/* dev [batch][n_medusa][topk] or NULL: use these candidates
                                  instead of the carried ones (test / planted-draft hook)     */
} sd_step_io;

/* One speculative step for every sequence of `kv` (Section III-B). stop_mask: dev uint32
 * words, bit (id % 32) of word (id / 32) set for syntactically significant token ids,
 * ceil(vocab / 32) words. Needs a prior sd_prefill or sd_kv_set_draft.
 * SD_ERR_KV_FULL if some sequence might exceed `cap` (judged from the lengths the host
 * knows; call sd_kv_len to refresh them).                                                  */
int sd_spec_step(sd_model* m, sd_kv* kv, const sd_tree* tree, const uint32_t* stop_mask,
                 sd_step_io* io, void* stream);
/* Sampling decoding (Section III-B, Eq. 1; Section IV-A runs it at temperature 0.8). The step
 * is sd_spec_step with two changes. A drafted node is accepted iff its parent is and the base
 * model's probability of its token given the tokens up to its parent, under
 * softmax(logits / temperature), is greater than min(epsilon, delta * exp(-H)), H being the
 * entropy (natural log) of that same distribution; the root is always accepted, the longest
 * accepted path wins (lowest node index on equal depth) and the cut at the last stop token is
 * unchanged. The token that starts the next step is not the arg-max but the inverse-CDF draw
 * at u[b] from the base distribution at the last kept node: the smallest id whose cumulative
 * probability exceeds u[b]. The caller owns the random numbers, so a run is reproducible.    */
typedef struct sd_typical {
    float temperature;         /* > 0                                                         */
    float epsilon;             /* hard threshold, 0..1                                        */
    float delta;               /* entropy-dependent threshold factor, >= 0                    */
    const float* u;            /* dev [batch]: uniform numbers in [0, 1), read by this step   */
    float* row_stats;          /* dev [batch][T][4] or NULL: per node {max logit, Z, H, c} of
                                  its base distribution, Z = sum exp((logit - max) / temp) and
                                  c = log(threshold * Z): a child token v passes iff
                                  (logit_v - max) / temperature > c                           */
} sd_typical;
/* Arguments as sd_spec_step plus `ty` (host struct, read during the call). Probabilities are
 * formed in fp32 with fp64 sums across the vocabulary. Never runs as a captured graph.
 * SD_ERR_SHAPE for a temperature, epsilon or delta outside the ranges above.                */
int sd_spec_step_typical(sd_model* m, sd_kv* kv, const sd_tree* tree, const uint32_t* stop_mask,
                         sd_step_io* io, const sd_typical* ty, void* stream);
/* Plain next-token greedy decoding: a step whose tree is the root alone (the paper's NTP
 * baseline, Section IV-B). Fills n_accept (=1), tokens, src_slots (=0); logits is
 * [batch][1][vocab].                                                                       */
int sd_greedy_step(sd_model* m, sd_kv* kv, sd_step_io* io, void* stream);

/* ---- single stages, for per-kernel parity tests -------------------------------------------
 * Acceptance + fragment cut alone (no forward): am dev [batch][T] = base arg-max per node,
 * tok dev [batch][T] = node tokens. Writes n_accept, n_accept_raw, tokens, src_slots as in
 * sd_step_io (token ids outside [0, vocab) are never stop tokens). Touches no cache.                                                   */
int sd_verify_tree(const sd_tree* tree, int32_t batch, int32_t n_medusa, int32_t trunc_fallback,
                   int32_t vocab, const int32_t* tok, const int32_t* am, const uint32_t* stop_mask,
                   int32_t* n_accept, int32_t* n_accept_raw, int32_t* tokens, int32_t* src_slots,
                   void* stream);

/* Commit of key/value rows alone (the last stage of a step, Section III-B: the accepted tokens become part of the
 * sequence): for every sequence b of `kv`, rows src_slots[b][0 .. n_rows[b]) of the tree rows that the LAST step or
 * prefill chunk of this model over this cache's batch computed are appended to the cache, in that order, and the
 * committed length grows by n_rows[b] (clamped to 0 .. width). src_slots: dev [batch][width], tree row numbers
 * below the last pass's padded tree size (clamped); n_rows: dev [batch]. Keys are copied as they are (they were
 * rotated for the position depth(node) after the old length: only meaningful when row j has depth j). SD_ERR_STATE
 * without such a pass, SD_ERR_SHAPE for a bad width, SD_ERR_KV_FULL judged on width rows per sequence.              */
int sd_kv_commit_rows(sd_model* m, sd_kv* kv, const int32_t* src_slots, const int32_t* n_rows, int32_t width,
                      void* stream);

/* Typical acceptance + fragment cut alone (Section III-B, Eq. 1): logits dev
 * [batch][T][vocab] = base logits of every node, tok dev [batch][T]. Writes row_stats (dev
 * [batch][T][4], required, layout as in sd_typical) and then the four outputs as above.     */
int sd_verify_tree_typical(const sd_tree* tree, int32_t batch, int32_t n_medusa, int32_t trunc_fallback,
                           int32_t vocab, const int32_t* tok, const float* logits, float temperature,
                           float epsilon, float delta, const uint32_t* stop_mask, float* row_stats,
                           int32_t* n_accept, int32_t* n_accept_raw, int32_t* tokens, int32_t* src_slots,
                           void* stream);
/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): sd_verify_tree_typical without its row_stats argument. The per-node
 * statistics live in a static device array inside the library (64 KiB per GPU, held until the process
 * ends) instead of a buffer the caller brings; the call allocates nothing and calls no allocating routine.
 * Arguments and outputs as sd_verify_tree_typical. Limit: batch * tree nodes <= 4096, SD_ERR_SHAPE beyond
 * (nothing is enqueued). All calls on one GPU share that GPU's array: two calls whose kernels may overlap
 * in time there (different streams, or threads) race on it; calls on one stream are safe. The first call
 * on a device looks the array's address up; use it from one device context per thread as the other calls. */
int sd_verify_tree_typical_static(const sd_tree* tree, int32_t batch, int32_t n_medusa, int32_t trunc_fallback,
                                  int32_t vocab, const int32_t* tok, const float* logits, float temperature,
                                  float epsilon, float delta, const uint32_t* stop_mask,
                                  int32_t* n_accept, int32_t* n_accept_raw, int32_t* tokens, int32_t* src_slots,
                                  void* stream);
/* Inverse-CDF draws alone (the sampling half of Section IV-A's decoding setting): out[i] =
 * smallest id whose cumulative probability under softmax(logits[rows[i]] / temperature)
 * exceeds u[i]. logits dev [n_rows][ld] with ld >= vocab; rows, u, out dev [n], n <= 65535;
 * out[i] = -1 for a row index outside [0, n_rows).                                           */
int sd_sample_tokens(const float* logits, int32_t n_rows, int32_t ld, int32_t vocab, const int32_t* rows,
                     const float* u, int32_t n, float temperature, int32_t* out, void* stream);

/* ---- training-side data preparation ----------------------------------------------------------
 * Syntax-enriched labels (Section III-C, Fig. 3). l0: dev int32 [batch][seq], the base model's
 * label rows: token ids with frag_id at every fragment boundary, filled up with pad_id.
 * labels: dev int32 [batch][n_heads + 1][seq], written in full: row i of a sequence is its l0
 * row shifted left by i (entries past the end = pad_id); then, per position, every entry in a
 * row after the last row that holds frag_id becomes ignore_id. A position whose n_heads + 1
 * entries hold no frag_id keeps row 0 only (SD_LABELS_KEEP_BASE) or stays as it is
 * (SD_LABELS_KEEP_ALL). seq >= 0 (0 writes nothing), 0 <= n_heads <= SD_LABELS_MAX_HEADS,
 * 1 <= batch <= 65535; l0 and labels must not overlap. The caller owns both buffers.       */
#define SD_LABELS_MAX_HEADS 64
#define SD_LABELS_KEEP_BASE 0
#define SD_LABELS_KEEP_ALL  1
int sd_build_labels(const int32_t* l0, int32_t batch, int32_t seq, int32_t n_heads, int32_t frag_id,
                    int32_t pad_id, int32_t ignore_id, int32_t no_frag, int32_t* labels, void* stream);

/* Where in a step the draft heads run (Section III-B: every head predicts from the base model's
 * last hidden state at one position; which positions get evaluated is a schedule, not part of
 * the method, and both give the same candidates up to summation order).
 *   SD_DRAFT_AFTER_ACCEPT (default): after acceptance, on the one row of every sequence that
 *     was kept last: H head rows per sequence through the shared LM head, a second read of it.
 *   SD_DRAFT_ALL_NODES: inside the verifying pass, on all tree rows (the schedule of a
 *     single-pass multi-head decoder): H * T head rows per sequence go through the LM head, and
 *     the H rows of the last kept node are ranked afterwards. sd_greedy_step and sd_prefill
 *     always use the first schedule (they have one candidate row).
 * Returns SD_ERR_NULL / SD_ERR_SHAPE (unknown value); takes effect from the next step.          */
#define SD_DRAFT_AFTER_ACCEPT 0
#define SD_DRAFT_ALL_NODES     1
int sd_set_draft_schedule(sd_model* m, int32_t schedule);

/* Plain greedy decoding with or without the draft heads. sd_greedy_step runs them by default, so that
 * a speculative step can follow it at once. With on = 0 it leaves them out (the paper's next-token
 * baseline has none, Section IV-B) and the carried candidates stay as they were: a later speculative
 * step is still lossless, its drafts are merely stale. Returns SD_ERR_NULL for a NULL model.             */
int sd_set_greedy_drafts(sd_model* m, int32_t on);

/* The persistent layer kernel (on by default where the device can hold its 256 workgroups of 512 threads at once,
 * and for passes of 32, 64 or 256 rows): all stages of the verifying pass between two attention launches run as
 * phases of one launch, separated by barriers across the grid, instead of one launch per stage; results are
 * bit-identical either way. sd_set_fused(m, 0) selects one launch per stage.
 * Every wait of that kernel is bounded (default 50 ms; sd_set_sync_timeout: 0 .. 10 s, in microseconds). If a
 * wait runs out, the kernel still ends, the outputs enqueued since are invalid, and the next sd_kv_len on a cache
 * of this model returns SD_ERR_HIP once (after which decoding can go on, e.g. with sd_set_fused(m, 0)).           */
int sd_set_fused(sd_model* m, int32_t on);
int sd_set_sync_timeout(sd_model* m, int64_t microseconds);
/* Diagnostic: time stamps of the persistent layer kernel. dev_buf: dev, [launches][24][256] uint64, or NULL to
 * switch it off; launch l of a pass (0 .. n_layers) writes, for each of its 256 workgroups w, buf[l][i][w] = the
 * device's 100 MHz real-time counter when the workgroup finished the work of a phase (even i) and when it left the
 * barrier after it (odd i), in the order the phases run; entries of phases a launch does not run keep their old
 * contents. Launches beyond bytes / 49152 are not recorded. The caller owns the buffer and keeps it alive while set. */
int sd_set_layer_timeline(sd_model* m, void* dev_buf, size_t bytes);

/* Graph mode (off by default). When on, sd_spec_step / sd_greedy_step capture their kernel
 * sequence into a HIP graph the first time a given combination of (cache, tree, split-KV
 * geometry, stop mask, output and candidate pointers) is seen and replay it afterwards: one
 * launch per step instead of several hundred. The caller must then keep those pointers'
 * memory alive and, to benefit, reuse the same buffers from step to step (e.g. copy planted
 * candidates into one fixed buffer). Results are identical to the eager path. Graphs are
 * not used while sd_profile_begin is active.                                               */
int sd_set_graph_mode(sd_model* m, int32_t on);

/* ---- measurement ---------------------------------------------------------------------------
 * Between sd_profile_begin and sd_profile_end every launch of the two bandwidth-bound kernel
 * classes is bracketed by HIP events on the stream it is launched on (up to max_launches
 * launches; later ones are not recorded). sd_profile_end synchronises `stream` and returns,
 * per class (index 0 = weight-streaming GEMM, 1 = tree attention): the summed launch
 * durations in ms, the number of launches, and the summed algorithmic bytes (GEMM: one read
 * of the weight matrix; attention: one read of K and V of the committed rows, taken at the
 * host's upper bound of the length, plus the tree rows). Arrays of 2 entries, host.        */
int sd_profile_begin(sd_model* m, int32_t max_launches);
int sd_profile_end(sd_model* m, void* stream, double* ms_total, int64_t* launches, double* bytes_total);

const char* sd_last_error(void);
/* Library version string; also proves the shared object loads without a GPU.              */
const char* sd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPECDEC_H */
