// Host side of libspecdec: handle management, argument validation, and the sequencing of the
// kernels of one speculative step (paper Section III-B) on a caller-supplied HIP stream.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "sd_internal.h"

// ------------------------------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";

static int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
#define HIP_TRY(expr)                                                                              \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess) return fail(SD_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));     \
    } while (0)

extern "C" const char* sd_last_error(void) { return g_err; }
extern "C" const char* sd_version(void) { return "libspecdec 0.1 (gfx950)"; }

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline int pow2_blocks(int rows) {   // 32-row blocks, rounded up to 1, 2, 4 or 8
    int mb = ceil_div(rows, 32), p = 1;
    while (p < mb) p *= 2;
    return p;
}

// ------------------------------------------------------------------------------------------ handles
struct LayerW {
    const void *attn_norm, *ffn_norm;       // bf16 [d]
    const void *wqkv, *wo, *wgu, *wdown;    // packed fragments
};

// Optional per-launch timing of the two bandwidth-bound kernel classes with HIP events on the
// caller's stream (sd_profile_begin / sd_profile_end).
enum { PROF_GEMM = 0, PROF_ATTN = 1, PROF_CLASSES = 2 };
struct Profile {
    bool on = false;
    std::vector<hipEvent_t> ev;              // pairs (start, stop)
    std::vector<int> cls;                    // class of pair i
    std::vector<double> bytes;               // algorithmic bytes of pair i
    size_t used = 0;                         // pairs used
};

struct sd_model {
    sd_config cfg;
    Profile prof;
    int max_rows, MBmax;
    int KBd, KBf, Fpad, NBqkv, NBo, NBgu, NBv, Vpad, NBmed;
    char* arena = nullptr;                   // packed weights
    char* work = nullptr;                    // workspace
    const void *embed, *lm_head, *final_norm, *medusa_w;
    MedusaBias medusa_b;
    std::vector<LayerW> layers;
    // workspace
    float *x, *part, *logits, *hlogits, *hf, *h_rows, *opart;
    float2* mlpart;
    void *xn, *attn_x, *act, *q, *kt, *vt;
    void* xh;                                // draft-head rows of every tree row, in 256-row operand chunks
    int draft_schedule = SD_DRAFT_AFTER_ACCEPT;
    RowTable rt;
    int32_t *am, *g_parent, *g_depth, *g_rank;
    float4* row_stats;                     // [Mp]: per tree row, statistics for typical acceptance
    uint32_t* zero_stop;
    const void* zfrag;                       // 1 KiB of zeros
    size_t part_floats;
    int max_parts;
    // HIP-graph mode: one captured graph per distinct launch sequence of a step
    struct StepGraph { std::vector<uint64_t> key; hipGraphExec_t exec; };
    bool use_graphs = false;
    std::vector<StepGraph> graphs;
    hipStream_t cap_stream = nullptr;      // capture happens here: the caller's stream may be the null stream
    std::vector<GemmPlan> plans;             // one per (row blocks, K blocks, N blocks) in use
    int32_t* plan_cnt = nullptr;             // device: the plans' per-group slot counts
    // every shape a call can issue is planned at creation; the entry points check the plans they need
    // (have_plans) before they enqueue anything, so a miss here cannot happen after that check
    const GemmPlan* find_plan(int MB, int KB, int NB) const {
        for (const GemmPlan& p : plans)
            if (p.MB == MB && p.KB == KB && p.NB == NB) return &p;
        return nullptr;
    }
    // persistent layer kernel (fused.hip)
    bool fused_ok = false;                   // the device holds its 256 workgroups at once and the buffers exist
    bool use_fused = false;                  // sd_set_fused
    bool fused_dirty = false;                // launched since the host last looked at the give-up flag
    float *part_o = nullptr, *part_gu = nullptr, *part_dn = nullptr, *part_q = nullptr;   // one per GEMM of a launch
    void* xn2 = nullptr;                     // second packed operand (norm before the feed-forward block)
    float *ssq_a = nullptr, *ssq_f = nullptr;   // [d / 16][Mp] partial sums of squares of the two deferred norms
    unsigned* sync_ctr = nullptr;            // [(n_layers + 1)][FUSED_SYNC_WORDS] barrier counters, + the give-up flag
    unsigned* sync_abort = nullptr;
    unsigned long long sync_timeout_ticks = 5000000ull;     // 50 ms of the 100 MHz counter
    unsigned long long* timeline = nullptr;  // caller's buffer for the layer kernel's time stamps, or NULL
    size_t timeline_launches = 0;
    int scratch_B = 0, scratch_Tp = 0;       // geometry of the tree K/V scratch as the last pass left it
    bool plan_missing = false;               // set by run_gemm if it ever had to skip a launch
    bool greedy_drafts = true;               // sd_greedy_step also runs the draft heads
    // float32 path (dtype SD_DTYPE_F32; f32.hip): weights [out][in] as float, natural activation layouts
    bool f32 = false;
    struct F32Layer { const float *attn_norm, *wqkv, *wo, *ffn_norm, *wgu, *wdown; };
    struct F32 {
        const float *embed, *lm_head, *final_norm, *medusa_w, *medusa_b;
        std::vector<F32Layer> layers;
        float *xn, *qkv, *q, *attn, *gu, *act, *kt, *vt, *z, *xh;
    } f;
};

// Handles get a process-wide serial number: graph keys use it instead of the handle's address, which a
// later handle can be given again after this one is destroyed.
static uint64_t next_uid() {
    static uint64_t n = 0;
    return ++n;
}

struct sd_kv {
    uint64_t uid = next_uid();
    const sd_model* m;
    int B, cap, cap_blocks;
    uint16_t* buf;
    size_t layer_stride;                     // elements between layers, per K or V plane
    uint16_t *kc, *vc;                       // plane bases
    float *kc32 = nullptr, *vc32 = nullptr;  // float32 models: planes [layer][seq][cap][d], layer_stride = B * cap * d
    int32_t* state = nullptr;                // device: kv_len, n_old, root_tok, last_row, cand, io scratch
    int32_t *kv_len, *n_old, *root_tok, *last_row, *cand, *i_nacc, *i_tokens, *i_slots;
    std::vector<int32_t> len_hi;             // host upper bound of the committed lengths
    bool has_draft = false;
};

struct sd_tree {
    uint64_t uid = next_uid();
    int T, Tp, H, topk;
    int32_t* dev = nullptr;                  // parent | depth | rank
    const int32_t *parent, *depth, *rank;
};

// ------------------------------------------------------------------------------------------ model
static int check_config(const sd_config* c) {
    if (c->dtype != SD_DTYPE_BF16 && c->dtype != SD_DTYPE_F32) return fail(SD_ERR_SHAPE, "dtype must be SD_DTYPE_BF16 or SD_DTYPE_F32");
    if (c->head_dim != 64 && c->head_dim != 128) return fail(SD_ERR_SHAPE, "head_dim must be 64 or 128");
    if (c->n_layers < 1 || c->n_heads < 1 || c->vocab < 2 || c->vocab > 163840) return fail(SD_ERR_SHAPE, "bad sizes");
    if (c->d_model != c->n_heads * c->head_dim) return fail(SD_ERR_SHAPE, "d_model != n_heads * head_dim");
    if (c->d_model % 32 || c->d_model > 8192) return fail(SD_ERR_SHAPE, "d_model must be a multiple of 32, <= 8192");
    if (c->d_ffn % 16 || c->d_ffn < 16) return fail(SD_ERR_SHAPE, "d_ffn must be a multiple of 16");
    if (c->n_medusa < 1 || c->n_medusa > SD_MAX_MEDUSA) return fail(SD_ERR_SHAPE, "n_medusa must be in 1..15");
    if (c->topk < 1 || c->topk > 32 || c->topk > c->vocab) return fail(SD_ERR_SHAPE, "topk must be in 1..32");
    if (c->trunc_fallback != SD_TRUNC_KEEP_ALL && c->trunc_fallback != SD_TRUNC_KEEP_ONE)
        return fail(SD_ERR_SHAPE, "bad trunc_fallback");
    if (!(c->rope_theta > 0.f) || !(c->rms_eps >= 0.f)) return fail(SD_ERR_SHAPE, "bad rope_theta / rms_eps");
    return SD_OK;
}

// The float32 model: weights copied as they are ([out][in] float; gate and up stacked, the draft heads stacked, a
// zero bias where none is given) and a workspace in natural row-major layouts. No launch plans, no packing.
static int create_f32(const sd_config* cfg, const sd_weights* w, int max_rows, hipStream_t s, sd_model** out) {
    const int L = cfg->n_layers, d = cfg->d_model, F = cfg->d_ffn, V = cfg->vocab, H = cfg->n_medusa, hd = cfg->head_dim;
    sd_model* m = new (std::nothrow) sd_model();
    if (!m) return fail(SD_ERR_HIP, "out of host memory");
    m->cfg = *cfg;
    m->f32 = true;
    m->max_rows = max_rows;
    m->MBmax = pow2_blocks(max_rows);
    m->Vpad = ceil_div(V, 32) * 32;
    const int Mp = m->MBmax * 32;
    const int HBp = pow2_blocks(H * SD_MAX_BATCH > 256 ? 256 : H * SD_MAX_BATCH) * 32;
    size_t sz = 0;
    auto take = [&](size_t floats) { size_t o = sz; sz = align_up(sz + floats * 4, 256); return o; };
    const size_t o_embed = take((size_t)V * d), o_lm = take((size_t)V * d), o_fn = take(d);
    const size_t o_mw = take((size_t)H * d * d), o_mb = take((size_t)H * d);
    std::vector<size_t> o_an(L), o_qkv(L), o_o(L), o_ffn(L), o_gu(L), o_dn(L);
    for (int l = 0; l < L; ++l) {
        o_an[l] = take(d); o_qkv[l] = take((size_t)3 * d * d); o_o[l] = take((size_t)d * d);
        o_ffn[l] = take(d); o_gu[l] = take((size_t)2 * F * d); o_dn[l] = take((size_t)d * F);
    }
    hipError_t e = hipMalloc((void**)&m->arena, sz);
    if (e != hipSuccess) { delete m; return fail(SD_ERR_HIP, "hipMalloc(%zu) for weights: %s", sz, hipGetErrorString(e)); }
    char* A = m->arena;
    auto copy = [&](size_t off, const void* src, size_t floats) {
        if (e == hipSuccess) e = hipMemcpyAsync(A + off, src, floats * 4, hipMemcpyDeviceToDevice, s);
        return (const float*)(A + off);
    };
    e = hipMemsetAsync(A + o_mb, 0, (size_t)H * d * 4, s);
    m->f.embed = copy(o_embed, w->embed, (size_t)V * d);
    m->f.lm_head = copy(o_lm, w->lm_head, (size_t)V * d);
    m->f.final_norm = copy(o_fn, w->final_norm, d);
    for (int i = 0; i < H; ++i) {
        copy(o_mw + (size_t)i * d * d * 4, w->medusa_w[i], (size_t)d * d);
        if (w->medusa_b && w->medusa_b[i]) copy(o_mb + (size_t)i * d * 4, w->medusa_b[i], d);
    }
    m->f.medusa_w = (const float*)(A + o_mw);
    m->f.medusa_b = (const float*)(A + o_mb);
    m->f.layers.resize(L);
    for (int l = 0; l < L; ++l) {
        sd_model::F32Layer& lw = m->f.layers[l];
        lw.attn_norm = copy(o_an[l], w->attn_norm[l], d);
        lw.wqkv = copy(o_qkv[l], w->wqkv[l], (size_t)3 * d * d);
        lw.wo = copy(o_o[l], w->wo[l], (size_t)d * d);
        lw.ffn_norm = copy(o_ffn[l], w->ffn_norm[l], d);
        lw.wgu = copy(o_gu[l], w->w_gate[l], (size_t)F * d);
        copy(o_gu[l] + (size_t)F * d * 4, w->w_up[l], (size_t)F * d);
        lw.wdown = copy(o_dn[l], w->w_down[l], (size_t)d * F);
    }
    m->embed = m->f.embed;

    size_t wz = 0;
    auto wtake = [&](size_t bytes) { size_t o = wz; wz = align_up(wz + bytes, 256); return o; };
    const size_t w_x = wtake((size_t)Mp * d * 4), w_logits = wtake((size_t)Mp * m->Vpad * 4);
    const size_t w_hlog = wtake((size_t)HBp * m->Vpad * 4), w_hrows = wtake((size_t)SD_MAX_BATCH * d * 4);
    const size_t w_xn = wtake((size_t)Mp * d * 4), w_qkv = wtake((size_t)Mp * 3 * d * 4), w_q = wtake((size_t)Mp * d * 4);
    const size_t w_attn = wtake((size_t)Mp * d * 4), w_gu = wtake((size_t)Mp * 2 * F * 4), w_act = wtake((size_t)Mp * F * 4);
    const size_t w_kt = wtake((size_t)L * Mp * d * 4), w_vt = wtake((size_t)L * Mp * d * 4);
    const size_t w_z = wtake((size_t)SD_MAX_BATCH * H * d * 4), w_xh = wtake((size_t)HBp * d * 4);
    const size_t w_tok = wtake((size_t)Mp * 4), w_pos = wtake((size_t)Mp * 4), w_anc = wtake((size_t)Mp * SD_ANC_WORDS * 4);
    const size_t w_cs = wtake((size_t)Mp * (hd / 2) * 8), w_am = wtake((size_t)Mp * 4), w_g = wtake(3 * 4);
    const size_t w_rs = wtake((size_t)Mp * 16), w_zs = wtake((size_t)ceil_div(V, 32) * 4);
    if (e == hipSuccess) e = hipMalloc((void**)&m->work, wz);
    if (e == hipSuccess) e = hipMemsetAsync(m->work, 0, wz, s);
    if (e != hipSuccess) {
        hipStreamSynchronize(s);
        hipFree(m->arena);
        if (m->work) hipFree(m->work);
        delete m;
        return fail(SD_ERR_HIP, "float32 model: weights or workspace: %s", hipGetErrorString(e));
    }
    char* Wk = m->work;
    m->x = (float*)(Wk + w_x); m->logits = (float*)(Wk + w_logits); m->hlogits = (float*)(Wk + w_hlog);
    m->h_rows = (float*)(Wk + w_hrows);
    m->f.xn = (float*)(Wk + w_xn); m->f.qkv = (float*)(Wk + w_qkv); m->f.q = (float*)(Wk + w_q);
    m->f.attn = (float*)(Wk + w_attn); m->f.gu = (float*)(Wk + w_gu); m->f.act = (float*)(Wk + w_act);
    m->f.kt = (float*)(Wk + w_kt); m->f.vt = (float*)(Wk + w_vt); m->f.z = (float*)(Wk + w_z); m->f.xh = (float*)(Wk + w_xh);
    m->rt.tok = (int32_t*)(Wk + w_tok); m->rt.pos = (int32_t*)(Wk + w_pos); m->rt.anc = (uint32_t*)(Wk + w_anc);
    m->rt.cs = (float2*)(Wk + w_cs);
    m->am = (int32_t*)(Wk + w_am);
    m->row_stats = (float4*)(Wk + w_rs);
    m->g_parent = (int32_t*)(Wk + w_g); m->g_depth = m->g_parent + 1; m->g_rank = m->g_parent + 2;
    m->zero_stop = (uint32_t*)(Wk + w_zs);
    launch_fill_i32(m->g_parent, -1, 1, s);
    e = hipStreamSynchronize(s);
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) {
        hipFree(m->arena); hipFree(m->work); delete m;
        return fail(SD_ERR_HIP, "float32 model: set-up failed: %s", hipGetErrorString(e));
    }
    *out = m;
    return SD_OK;
}

extern "C" int sd_model_create(const sd_config* cfg, const sd_weights* w, int32_t max_rows, void* stream,
                               sd_model** out) {
    if (!cfg || !w || !out) return fail(SD_ERR_NULL, "sd_model_create: NULL argument");
    *out = nullptr;
    int rc = check_config(cfg);
    if (rc) return rc;
    if (max_rows < 1 || max_rows > 256) return fail(SD_ERR_SHAPE, "max_rows must be in 1..256");
    if (!w->embed || !w->lm_head || !w->final_norm || !w->attn_norm || !w->wqkv || !w->wo || !w->ffn_norm ||
        !w->w_gate || !w->w_up || !w->w_down || !w->medusa_w)
        return fail(SD_ERR_NULL, "sd_model_create: NULL weight pointer");
    const int L = cfg->n_layers, d = cfg->d_model, F = cfg->d_ffn, V = cfg->vocab, H = cfg->n_medusa;
    for (int l = 0; l < L; ++l)
        if (!w->attn_norm[l] || !w->wqkv[l] || !w->wo[l] || !w->ffn_norm[l] || !w->w_gate[l] || !w->w_up[l] ||
            !w->w_down[l])
            return fail(SD_ERR_NULL, "sd_model_create: NULL weight pointer in layer %d", l);
    for (int i = 0; i < H; ++i)
        if (!w->medusa_w[i]) return fail(SD_ERR_NULL, "sd_model_create: NULL draft-head weight %d", i);

    hipStream_t s = (hipStream_t)stream;
    if (cfg->dtype == SD_DTYPE_F32) return create_f32(cfg, w, max_rows, s, out);
    sd_model* m = new (std::nothrow) sd_model();
    if (!m) return fail(SD_ERR_HIP, "out of host memory");
    m->cfg = *cfg;
    m->max_rows = max_rows;
    m->MBmax = pow2_blocks(max_rows);
    m->KBd = d / 16;
    m->KBf = F / 16;
    m->Fpad = (int)align_up(F, 32);
    m->NBqkv = 3 * d / 32;
    m->NBo = d / 32;
    m->NBgu = 2 * m->Fpad / 32;
    m->NBv = ceil_div(V, 32);
    m->Vpad = m->NBv * 32;
    m->NBmed = H * d / 32;

    // ---- arena of packed weights
    const size_t frag = 1024;    // bytes per fragment
    size_t sz = 0;
    auto take = [&](size_t bytes) { size_t o = sz; sz = align_up(sz + bytes, 256); return o; };
    size_t o_embed = take((size_t)V * d * 2), o_lm = take((size_t)m->NBv * m->KBd * frag), o_fn = take((size_t)d * 2);
    size_t o_med = take((size_t)m->NBmed * m->KBd * frag);
    std::vector<size_t> o_mb(H), o_an(L), o_qkv(L), o_o(L), o_ffn(L), o_gu(L), o_dn(L);
    for (int i = 0; i < H; ++i) o_mb[i] = take((size_t)d * 2);
    for (int l = 0; l < L; ++l) {
        o_an[l] = take((size_t)d * 2);
        o_qkv[l] = take((size_t)m->NBqkv * m->KBd * frag);
        o_o[l] = take((size_t)m->NBo * m->KBd * frag);
        o_ffn[l] = take((size_t)d * 2);
        o_gu[l] = take((size_t)m->NBgu * m->KBd * frag);
        o_dn[l] = take((size_t)m->NBo * m->KBf * frag);
    }
    hipError_t e = hipMalloc((void**)&m->arena, sz);
    if (e != hipSuccess) { delete m; return fail(SD_ERR_HIP, "hipMalloc(%zu) for weights: %s", sz, hipGetErrorString(e)); }
    char* A = m->arena;
    auto copy = [&](size_t off, const void* src, size_t bytes) {
        return hipMemcpyAsync(A + off, src, bytes, hipMemcpyDeviceToDevice, s);
    };
    e = copy(o_embed, w->embed, (size_t)V * d * 2);
    if (e == hipSuccess) e = copy(o_fn, w->final_norm, (size_t)d * 2);
    if (e != hipSuccess) { hipFree(m->arena); delete m; return fail(SD_ERR_HIP, "weight copy: %s", hipGetErrorString(e)); }
    m->embed = A + o_embed;
    m->final_norm = A + o_fn;
    launch_pack_weight(w->lm_head, A + o_lm, V, d, 0, m->NBv, m->KBd, s);
    m->lm_head = A + o_lm;
    for (int i = 0; i < H; ++i) {
        launch_pack_weight(w->medusa_w[i], A + o_med, d, d, i * (d / 32), m->NBmed, m->KBd, s);
        if (w->medusa_b && w->medusa_b[i]) {
            if (e == hipSuccess) e = copy(o_mb[i], w->medusa_b[i], (size_t)d * 2);
            m->medusa_b.p[i] = (const uint16_t*)(A + o_mb[i]);
        } else {
            m->medusa_b.p[i] = nullptr;
        }
    }
    m->medusa_w = A + o_med;
    m->layers.resize(L);
    for (int l = 0; l < L; ++l) {
        LayerW& lw = m->layers[l];
        if (e == hipSuccess) e = copy(o_an[l], w->attn_norm[l], (size_t)d * 2);
        if (e == hipSuccess) e = copy(o_ffn[l], w->ffn_norm[l], (size_t)d * 2);
        launch_pack_weight(w->wqkv[l], A + o_qkv[l], 3 * d, d, 0, m->NBqkv, m->KBd, s);
        launch_pack_weight(w->wo[l], A + o_o[l], d, d, 0, m->NBo, m->KBd, s);
        launch_pack_weight(w->w_gate[l], A + o_gu[l], F, d, 0, m->NBgu, m->KBd, s);
        launch_pack_weight(w->w_up[l], A + o_gu[l], F, d, m->Fpad / 32, m->NBgu, m->KBd, s);
        launch_pack_weight(w->w_down[l], A + o_dn[l], d, F, 0, m->NBo, m->KBf, s);
        lw.attn_norm = A + o_an[l];
        lw.ffn_norm = A + o_ffn[l];
        lw.wqkv = A + o_qkv[l];
        lw.wo = A + o_o[l];
        lw.wgu = A + o_gu[l];
        lw.wdown = A + o_dn[l];
    }

    // ---- workspace
    const int Mp = m->MBmax * 32, nh = cfg->n_heads, hd = cfg->head_dim;
    const int ld_max = std::max(std::max(3 * d, 2 * m->Fpad), H * d);
    // launch plans for every GEMM shape this model can issue
    size_t pf = 0;
    std::vector<int32_t> cnt_all;
    std::vector<size_t> cnt_off;
    {
        const int shapes[6][2] = {{m->KBd, m->NBqkv}, {m->KBd, m->NBo}, {m->KBd, m->NBgu},
                                  {m->KBf, m->NBo},   {m->KBd, m->NBv}, {m->KBd, m->NBmed}};
        for (int mb = 1; mb <= 8; mb *= 2)
            for (int si = 0; si < 6; ++si) {
                const int* sh = shapes[si];
                // beyond MBmax only the LM head is used (draft-head rows); the draft-head
                // projection has one row block, or the step's when the heads run on every tree row
                if (mb > m->MBmax && si != 4) continue;
                bool dup = false;
                for (const GemmPlan& q : m->plans) dup |= q.MB == mb && q.KB == sh[0] && q.NB == sh[1];
                if (dup) continue;
                GemmPlan pl;
                std::vector<int32_t> cnt((sh[1] + 7) / 8 + 1, 0), slot0(256, 0);
                gemm_plan_make(&pl, mb, sh[0], sh[1], cnt.data(), slot0.data());
                cnt_off.push_back(cnt_all.size());
                cnt_all.insert(cnt_all.end(), cnt.begin(), cnt.end());
                cnt_all.insert(cnt_all.end(), slot0.begin(), slot0.end());
                m->plans.push_back(pl);
                pf = std::max(pf, (size_t)pl.slots_max * (mb * 32) * (size_t)sh[1] * 32);
            }
    }
    (void)ld_max;
    m->part_floats = pf;
    m->max_parts = 65;
    const int HBp = pow2_blocks(H * SD_MAX_BATCH > 256 ? 256 : H * SD_MAX_BATCH) * 32;
    size_t wz = 0;
    auto wtake = [&](size_t bytes) { size_t o = wz; wz = align_up(wz + bytes, 256); return o; };
    size_t w_x = wtake((size_t)Mp * d * 4), w_part = wtake(pf * 4), w_logits = wtake((size_t)Mp * m->Vpad * 4);
    size_t w_hlog = wtake((size_t)HBp * m->Vpad * 4), w_hf = wtake((size_t)Mp * d * 4);
    size_t w_hrows = wtake((size_t)SD_MAX_BATCH * d * 4);
    size_t w_opart = wtake((size_t)Mp * nh * m->max_parts * hd * 4), w_ml = wtake((size_t)Mp * nh * m->max_parts * 8);
    size_t w_xn = wtake((size_t)std::max(Mp, HBp) * d * 4), w_attn = wtake((size_t)Mp * d * 4);
    size_t w_act = wtake((size_t)Mp * F * 4), w_q = wtake((size_t)Mp * d * 4);
    size_t w_kt = wtake((size_t)L * Mp * d * 2), w_vt = wtake((size_t)L * Mp * d * 2);
    size_t w_tok = wtake((size_t)Mp * 4), w_pos = wtake((size_t)Mp * 4), w_anc = wtake((size_t)Mp * SD_ANC_WORDS * 4);
    size_t w_cs = wtake((size_t)Mp * (hd / 2) * 8), w_am = wtake((size_t)Mp * 4), w_g = wtake(3 * 4);
    size_t w_rs = wtake((size_t)Mp * 16);
    size_t w_xh = wtake(align_up((size_t)H * Mp, 256) * d * 4);
    size_t w_zs = wtake((size_t)ceil_div(V, 32) * 4), w_zf = wtake(1024);
    size_t w_ssqa = wtake((size_t)align_up(d / 16, 4) * Mp * 4), w_ssqf = wtake((size_t)align_up(d / 16, 4) * Mp * 4);
    size_t w_xn2 = wtake((size_t)Mp * d * 4);
    // the persistent layer kernel: partial sums of each of its four GEMMs in a buffer of their own, a second
    // packed operand, and the barrier counters of every launch of a pass
    int dev_now = 0;
    const bool fused_fits = hipGetDevice(&dev_now) == hipSuccess && fused_max_resident(dev_now) >= 256;
    size_t w_po = 0, w_pgu = 0, w_pdn = 0, w_pq = 0, w_sync = 0;
    if (fused_fits) {
        w_po = wtake(pf * 4); w_pgu = wtake(pf * 4); w_pdn = wtake(pf * 4); w_pq = wtake(pf * 4);
        w_sync = wtake(((size_t)(L + 1) * FUSED_SYNC_WORDS + 64) * 4);
    }
    if (e != hipSuccess) {                             // one of the per-layer / per-head weight copies was refused
        hipStreamSynchronize(s);
        hipFree(m->arena); delete m;
        return fail(SD_ERR_HIP, "weight copy: %s", hipGetErrorString(e));
    }
    e = hipMalloc((void**)&m->work, wz);
    if (e == hipSuccess) e = hipMalloc((void**)&m->plan_cnt, cnt_all.size() * 4);
    if (e == hipSuccess) e = hipMemcpy(m->plan_cnt, cnt_all.data(), cnt_all.size() * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        hipFree(m->arena);
        if (m->work) hipFree(m->work);
        if (m->plan_cnt) hipFree(m->plan_cnt);
        delete m;
        return fail(SD_ERR_HIP, "hipMalloc(%zu) for workspace: %s", wz, hipGetErrorString(e));
    }
    for (size_t i = 0; i < m->plans.size(); ++i) {
        m->plans[i].cnt_dev = m->plan_cnt + cnt_off[i];
        m->plans[i].slot0_dev = m->plans[i].cnt_dev + (m->plans[i].NB + 7) / 8 + 1;      // right behind the counts
    }
    e = hipMemsetAsync(m->work, 0, wz, s);
    if (e != hipSuccess) {
        hipStreamSynchronize(s);
        hipFree(m->arena); hipFree(m->work); hipFree(m->plan_cnt); delete m;
        return fail(SD_ERR_HIP, "workspace clear: %s", hipGetErrorString(e));
    }
    char* Wk = m->work;
    m->x = (float*)(Wk + w_x); m->part = (float*)(Wk + w_part); m->logits = (float*)(Wk + w_logits);
    m->hlogits = (float*)(Wk + w_hlog); m->hf = (float*)(Wk + w_hf); m->h_rows = (float*)(Wk + w_hrows);
    m->opart = (float*)(Wk + w_opart); m->mlpart = (float2*)(Wk + w_ml);
    m->xn = Wk + w_xn; m->attn_x = Wk + w_attn; m->act = Wk + w_act; m->q = Wk + w_q;
    m->kt = Wk + w_kt; m->vt = Wk + w_vt;
    m->xh = Wk + w_xh;
    m->rt.tok = (int32_t*)(Wk + w_tok); m->rt.pos = (int32_t*)(Wk + w_pos); m->rt.anc = (uint32_t*)(Wk + w_anc);
    m->rt.cs = (float2*)(Wk + w_cs);
    m->am = (int32_t*)(Wk + w_am);
    m->row_stats = (float4*)(Wk + w_rs);
    m->g_parent = (int32_t*)(Wk + w_g); m->g_depth = m->g_parent + 1; m->g_rank = m->g_parent + 2;
    m->zero_stop = (uint32_t*)(Wk + w_zs);
    m->zfrag = Wk + w_zf;
    m->ssq_a = (float*)(Wk + w_ssqa); m->ssq_f = (float*)(Wk + w_ssqf);
    m->xn2 = Wk + w_xn2;
    if (fused_fits) {
        m->part_o = (float*)(Wk + w_po); m->part_gu = (float*)(Wk + w_pgu); m->part_dn = (float*)(Wk + w_pdn);
        m->part_q = (float*)(Wk + w_pq);
        m->sync_ctr = (unsigned*)(Wk + w_sync);
        m->sync_abort = m->sync_ctr + (size_t)(L + 1) * FUSED_SYNC_WORDS;
        m->fused_ok = true;
    }
    launch_fill_i32(m->g_parent, -1, 1, s);
    e = hipStreamSynchronize(s);
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) {
        hipFree(m->arena); hipFree(m->work); hipFree(m->plan_cnt); delete m;
        return fail(SD_ERR_HIP, "weight packing failed: %s", hipGetErrorString(e));
    }
    *out = m;
    return SD_OK;
}

static void prof_free(sd_model* m) {
    for (hipEvent_t e : m->prof.ev) hipEventDestroy(e);
    m->prof = Profile();
}

extern "C" int sd_profile_begin(sd_model* m, int32_t max_launches) {
    if (!m) return fail(SD_ERR_NULL, "sd_profile_begin: NULL model");
    if (max_launches < 1 || max_launches > (1 << 20)) return fail(SD_ERR_SHAPE, "sd_profile_begin: bad max_launches");
    prof_free(m);
    m->prof.ev.resize((size_t)max_launches * 2);
    m->prof.cls.assign(max_launches, 0);
    m->prof.bytes.assign(max_launches, 0.0);
    for (size_t i = 0; i < m->prof.ev.size(); ++i) {
        hipError_t e = hipEventCreate(&m->prof.ev[i]);
        if (e != hipSuccess) {
            m->prof.ev.resize(i);
            prof_free(m);
            return fail(SD_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e));
        }
    }
    m->prof.on = true;
    return SD_OK;
}

extern "C" int sd_profile_end(sd_model* m, void* stream, double* ms_total, int64_t* launches, double* bytes_total) {
    if (!m || !ms_total || !launches || !bytes_total) return fail(SD_ERR_NULL, "sd_profile_end: NULL argument");
    if (!m->prof.on) return fail(SD_ERR_STATE, "sd_profile_end: profiling is not on");
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) { prof_free(m); return fail(SD_ERR_HIP, "sync: %s", hipGetErrorString(e)); }
    for (int c = 0; c < PROF_CLASSES; ++c) { ms_total[c] = 0.0; launches[c] = 0; bytes_total[c] = 0.0; }
    for (size_t i = 0; i < m->prof.used; ++i) {
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, m->prof.ev[2 * i], m->prof.ev[2 * i + 1]);
        if (e != hipSuccess) { prof_free(m); return fail(SD_ERR_HIP, "hipEventElapsedTime: %s", hipGetErrorString(e)); }
        int c = m->prof.cls[i];
        ms_total[c] += ms;
        launches[c] += 1;
        bytes_total[c] += m->prof.bytes[i];
    }
    prof_free(m);
    return SD_OK;
}

extern "C" int sd_build_labels(const int32_t* l0, int32_t batch, int32_t seq, int32_t n_heads, int32_t frag_id,
                               int32_t pad_id, int32_t ignore_id, int32_t no_frag, int32_t* labels, void* stream) {
    if (batch < 1 || batch > 65535 || seq < 0) return fail(SD_ERR_SHAPE, "sd_build_labels: bad batch or seq");
    if (n_heads < 0 || n_heads > SD_LABELS_MAX_HEADS)
        return fail(SD_ERR_SHAPE, "sd_build_labels: n_heads must be in 0..%d", SD_LABELS_MAX_HEADS);
    if (no_frag != SD_LABELS_KEEP_BASE && no_frag != SD_LABELS_KEEP_ALL)
        return fail(SD_ERR_SHAPE, "sd_build_labels: bad no_frag policy");
    if (seq == 0) return SD_OK;                        // nothing to write; the pointers are not looked at
    if (!l0 || !labels) return fail(SD_ERR_NULL, "sd_build_labels: NULL argument");
    launch_build_labels(l0, batch, seq, n_heads, frag_id, pad_id, ignore_id, no_frag == SD_LABELS_KEEP_ALL, labels,
                        (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return SD_OK;
}

extern "C" int sd_set_draft_schedule(sd_model* m, int32_t schedule) {
    if (!m) return fail(SD_ERR_NULL, "sd_set_draft_schedule: NULL model");
    if (schedule != SD_DRAFT_AFTER_ACCEPT && schedule != SD_DRAFT_ALL_NODES)
        return fail(SD_ERR_SHAPE, "sd_set_draft_schedule: unknown schedule %d", schedule);
    m->draft_schedule = schedule;
    return SD_OK;
}

extern "C" int sd_set_fused(sd_model* m, int32_t on) {
    if (!m) return fail(SD_ERR_NULL, "sd_set_fused: NULL model");
    m->use_fused = on != 0;
    return SD_OK;
}

extern "C" int sd_set_layer_timeline(sd_model* m, void* dev_buf, size_t bytes) {
    if (!m) return fail(SD_ERR_NULL, "sd_set_layer_timeline: NULL model");
    if (dev_buf && (((uintptr_t)dev_buf) & 7)) return fail(SD_ERR_SHAPE, "sd_set_layer_timeline: buffer must be 8-byte aligned");
    m->timeline = (unsigned long long*)dev_buf;
    m->timeline_launches = dev_buf ? bytes / ((size_t)24 * 256 * 8) : 0;
    return SD_OK;
}

extern "C" int sd_set_sync_timeout(sd_model* m, int64_t microseconds) {
    if (!m) return fail(SD_ERR_NULL, "sd_set_sync_timeout: NULL model");
    if (microseconds < 0 || microseconds > 10000000) return fail(SD_ERR_SHAPE, "sd_set_sync_timeout: 0 .. 10 s");
    m->sync_timeout_ticks = (unsigned long long)microseconds * 100ull;
    return SD_OK;
}

// Has a workgroup of the persistent kernel given up a wait since the last look? Called where the host has just
// synchronised the stream anyway. The flag is cleared, so one failure is reported once.
static int check_fused_abort(sd_model* m, const char* who) {
    if (!m->fused_dirty || !m->sync_abort) return SD_OK;
    unsigned flag = 0;
    HIP_TRY(hipMemcpy(&flag, m->sync_abort, 4, hipMemcpyDeviceToHost));
    m->fused_dirty = false;
    if (flag) {
        HIP_TRY(hipMemset(m->sync_abort, 0, 4));
        return fail(SD_ERR_HIP, "%s: a wait between workgroups inside the layer kernel ran out of time; the results "
                    "enqueued since the last successful check are invalid", who);
    }
    return SD_OK;
}

extern "C" int sd_set_greedy_drafts(sd_model* m, int32_t on) {
    if (!m) return fail(SD_ERR_NULL, "sd_set_greedy_drafts: NULL model");
    m->greedy_drafts = on != 0;
    return SD_OK;
}

extern "C" int sd_set_graph_mode(sd_model* m, int32_t on) {
    if (!m) return fail(SD_ERR_NULL, "sd_set_graph_mode: NULL model");
    m->use_graphs = on != 0;
    return SD_OK;
}

extern "C" int sd_model_destroy(sd_model* m) {
    if (!m) return SD_OK;
    for (sd_model::StepGraph& g : m->graphs) hipGraphExecDestroy(g.exec);
    m->graphs.clear();
    if (m->cap_stream) { hipStreamDestroy(m->cap_stream); m->cap_stream = nullptr; }
    prof_free(m);
    hipFree(m->arena);
    hipFree(m->work);
    hipFree(m->plan_cnt);
    delete m;
    return SD_OK;
}

// ------------------------------------------------------------------------------------------ KV cache
extern "C" size_t sd_kv_bytes(const sd_config* cfg, int32_t batch, int32_t cap) {
    if (!cfg || batch < 1 || cap < 1) return 0;
    if (cfg->dtype == SD_DTYPE_F32)
        return (size_t)cfg->n_layers * 2 * batch * cap * cfg->n_heads * cfg->head_dim * 4;
    size_t blocks = (size_t)ceil_div(cap, 32);
    return (size_t)cfg->n_layers * 2 * batch * cfg->n_heads * blocks * 32 * cfg->head_dim * 2;
}

extern "C" int sd_kv_create(const sd_model* m, int32_t batch, int32_t cap, void* dev_buf, size_t bytes, sd_kv** out) {
    if (!m || !dev_buf || !out) return fail(SD_ERR_NULL, "sd_kv_create: NULL argument");
    *out = nullptr;
    if (batch < 1 || batch > SD_MAX_BATCH) return fail(SD_ERR_SHAPE, "batch must be in 1..%d", SD_MAX_BATCH);
    if (batch * m->cfg.n_medusa > 256) return fail(SD_ERR_SHAPE, "batch * n_medusa must be <= 256");
    if (cap < m->cfg.n_medusa + 2) return fail(SD_ERR_SHAPE, "cap too small");
    if (bytes < sd_kv_bytes(&m->cfg, batch, cap)) return fail(SD_ERR_SHAPE, "KV buffer too small");
    if (((uintptr_t)dev_buf) & 15) return fail(SD_ERR_SHAPE, "KV buffer must be 16-byte aligned");
    sd_kv* kv = new (std::nothrow) sd_kv();
    if (!kv) return fail(SD_ERR_HIP, "out of host memory");
    kv->m = m;
    kv->B = batch;
    kv->cap = cap;
    kv->cap_blocks = ceil_div(cap, 32);
    kv->buf = (uint16_t*)dev_buf;
    kv->layer_stride = (size_t)batch * m->cfg.n_heads * kv->cap_blocks * 32 * m->cfg.head_dim;
    kv->kc = kv->buf;
    kv->vc = kv->buf + (size_t)m->cfg.n_layers * kv->layer_stride;
    if (m->f32) {
        kv->layer_stride = (size_t)batch * cap * m->cfg.d_model;
        kv->kc32 = (float*)dev_buf;
        kv->vc32 = kv->kc32 + (size_t)m->cfg.n_layers * kv->layer_stride;
    }
    const int H = m->cfg.n_medusa, k = m->cfg.topk;
    const int W = std::max(H + 1, SD_MAX_TREE);
    size_t n = (size_t)batch * (4 + H * k + 1 + 2 * W);
    hipError_t e = hipMalloc((void**)&kv->state, n * 4);
    if (e != hipSuccess) { delete kv; return fail(SD_ERR_HIP, "hipMalloc state: %s", hipGetErrorString(e)); }
    e = hipMemset(kv->state, 0, n * 4);
    // The cache itself starts as zeros: attention multiplies the value rows of a partly filled block by
    // probabilities that are exactly 0 for the rows past the committed length, and 0 * NaN is NaN, so no
    // row the kernels can touch may hold a non-finite bit pattern left behind by the buffer's last user.
    if (e == hipSuccess) e = hipMemset(dev_buf, 0, sd_kv_bytes(&m->cfg, batch, cap));
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) { hipFree(kv->state); delete kv; return fail(SD_ERR_HIP, "hipMemset: %s", hipGetErrorString(e)); }
    int32_t* p = kv->state;
    kv->kv_len = p; p += batch;
    kv->n_old = p; p += batch;
    kv->root_tok = p; p += batch;
    kv->last_row = p; p += batch;
    kv->cand = p; p += (size_t)batch * H * k;
    kv->i_nacc = p; p += batch;
    kv->i_tokens = p; p += (size_t)batch * W;
    kv->i_slots = p;
    kv->len_hi.assign(batch, 0);
    *out = kv;
    return SD_OK;
}

extern "C" int sd_kv_destroy(sd_kv* kv) {
    if (!kv) return SD_OK;
    hipFree(kv->state);
    delete kv;
    return SD_OK;
}

extern "C" int sd_kv_len(sd_kv* kv, int32_t* out_len, void* stream) {
    if (!kv || !out_len) return fail(SD_ERR_NULL, "sd_kv_len: NULL argument");
    HIP_TRY(hipMemcpyAsync(out_len, kv->kv_len, kv->B * 4, hipMemcpyDeviceToHost, (hipStream_t)stream));
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    for (int b = 0; b < kv->B; ++b) kv->len_hi[b] = out_len[b];
    if (int rc = check_fused_abort(const_cast<sd_model*>(kv->m), "sd_kv_len")) return rc;
    return SD_OK;
}

extern "C" int sd_kv_set_len(sd_kv* kv, const int32_t* len, void* stream) {
    if (!kv || !len) return fail(SD_ERR_NULL, "sd_kv_set_len: NULL argument");
    for (int b = 0; b < kv->B; ++b)
        if (len[b] < 0 || len[b] > kv->cap) return fail(SD_ERR_SHAPE, "sd_kv_set_len: length %d out of range", len[b]);
    HIP_TRY(hipMemcpyAsync(kv->kv_len, len, kv->B * 4, hipMemcpyHostToDevice, (hipStream_t)stream));
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));   // `len` may be a temporary of the caller
    for (int b = 0; b < kv->B; ++b) kv->len_hi[b] = len[b];
    return SD_OK;
}

static int kv_rows_common(sd_kv* kv, int layer, int seq, int row0, int nrows, void* k_rows, void* v_rows, int to_cache,
                          void* stream) {
    if (!kv || !k_rows || !v_rows) return fail(SD_ERR_NULL, "sd_kv_*_rows: NULL argument");
    const sd_config& c = kv->m->cfg;
    if (layer < 0 || layer >= c.n_layers || seq < 0 || seq >= kv->B || row0 < 0 || nrows < 0 || row0 + nrows > kv->cap)
        return fail(SD_ERR_SHAPE, "sd_kv_*_rows: index out of range");
    if (nrows == 0) return SD_OK;
    if (kv->m->f32) {
        const size_t o = layer * kv->layer_stride + (size_t)seq * kv->cap * c.d_model;
        launch_f32_kv_rows(kv->kc32 + o, kv->vc32 + o, (float*)k_rows, (float*)v_rows, row0, nrows, c.d_model, to_cache,
                           (hipStream_t)stream);
        HIP_TRY(hipGetLastError());
        return SD_OK;
    }
    size_t off = layer * kv->layer_stride + (size_t)seq * c.n_heads * kv->cap_blocks * 32 * c.head_dim;
    launch_kv_rows(kv->kc + off, kv->vc + off, k_rows, v_rows, row0, nrows, c.n_heads, c.head_dim, kv->cap_blocks,
                   to_cache, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return SD_OK;
}
extern "C" int sd_kv_write_rows(sd_kv* kv, int32_t layer, int32_t seq, int32_t row0, int32_t nrows, const void* k_rows,
                                const void* v_rows, void* stream) {
    return kv_rows_common(kv, layer, seq, row0, nrows, (void*)k_rows, (void*)v_rows, 1, stream);
}
extern "C" int sd_kv_read_rows(sd_kv* kv, int32_t layer, int32_t seq, int32_t row0, int32_t nrows, void* k_rows,
                               void* v_rows, void* stream) {
    return kv_rows_common(kv, layer, seq, row0, nrows, k_rows, v_rows, 0, stream);
}

extern "C" int sd_kv_set_draft(sd_kv* kv, const int32_t* root_tok, const int32_t* cand, void* stream) {
    if (!kv || !root_tok || !cand) return fail(SD_ERR_NULL, "sd_kv_set_draft: NULL argument");
    const sd_config& c = kv->m->cfg;
    launch_copy_i32(root_tok, kv->root_tok, kv->B, (hipStream_t)stream);
    launch_copy_i32(cand, kv->cand, kv->B * c.n_medusa * c.topk, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    kv->has_draft = true;
    return SD_OK;
}
extern "C" int sd_kv_get_draft(sd_kv* kv, int32_t* root_tok, int32_t* cand, void* stream) {
    if (!kv || !root_tok || !cand) return fail(SD_ERR_NULL, "sd_kv_get_draft: NULL argument");
    const sd_config& c = kv->m->cfg;
    launch_copy_i32(kv->root_tok, root_tok, kv->B, (hipStream_t)stream);
    launch_copy_i32(kv->cand, cand, kv->B * c.n_medusa * c.topk, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return SD_OK;
}

// ------------------------------------------------------------------------------------------ tree
static int validate_tree(int T, const int32_t* parent, const int32_t* depth, const int32_t* rank, int H, int k) {
    if (T < 1 || T > SD_MAX_TREE) return fail(SD_ERR_BAD_TREE, "tree must have 1..%d nodes", SD_MAX_TREE);
    if (parent[0] != -1 || depth[0] != 0) return fail(SD_ERR_BAD_TREE, "node 0 must be the root (parent -1, depth 0)");
    for (int j = 1; j < T; ++j) {
        if (parent[j] < 0 || parent[j] >= j) return fail(SD_ERR_BAD_TREE, "node %d: parent must precede it", j);
        if (depth[j] != depth[parent[j]] + 1) return fail(SD_ERR_BAD_TREE, "node %d: depth != parent's depth + 1", j);
        if (depth[j] > H) return fail(SD_ERR_BAD_TREE, "node %d: depth %d exceeds the number of draft heads", j, depth[j]);
        if (rank[j] < 0 || rank[j] >= k) return fail(SD_ERR_BAD_TREE, "node %d: rank out of range", j);
        for (int i = 1; i < j; ++i)
            if (parent[i] == parent[j] && rank[i] == rank[j])
                return fail(SD_ERR_BAD_TREE, "nodes %d and %d: siblings with equal rank", i, j);
    }
    return SD_OK;
}

extern "C" int sd_tree_create(int32_t T, const int32_t* parent, const int32_t* depth, const int32_t* rank,
                              int32_t n_medusa, int32_t topk, sd_tree** out) {
    if (!parent || !depth || !rank || !out) return fail(SD_ERR_NULL, "sd_tree_create: NULL argument");
    *out = nullptr;
    if (n_medusa < 0 || n_medusa > SD_MAX_MEDUSA || topk < 1) return fail(SD_ERR_SHAPE, "bad n_medusa / topk");
    int rc = validate_tree(T, parent, depth, rank, n_medusa, topk);
    if (rc) return rc;
    sd_tree* t = new (std::nothrow) sd_tree();
    if (!t) return fail(SD_ERR_HIP, "out of host memory");
    t->T = T;
    t->Tp = ceil_div(T, 32) * 32;
    t->H = n_medusa;
    t->topk = topk;
    hipError_t e = hipMalloc((void**)&t->dev, (size_t)3 * T * 4);
    if (e == hipSuccess) e = hipMemcpy(t->dev, parent, (size_t)T * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(t->dev + T, depth, (size_t)T * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(t->dev + 2 * T, rank, (size_t)T * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        if (t->dev) hipFree(t->dev);
        delete t;
        return fail(SD_ERR_HIP, "tree upload: %s", hipGetErrorString(e));
    }
    t->parent = t->dev;
    t->depth = t->dev + T;
    t->rank = t->dev + 2 * T;
    *out = t;
    return SD_OK;
}

extern "C" int sd_tree_destroy(sd_tree* t) {
    if (!t) return SD_OK;
    hipFree(t->dev);
    delete t;
    return SD_OK;
}

// ------------------------------------------------------------------------------------------ forward
// Layers 0..L-1 on the rows described by m->rt / m->x (B sequences of Tp rows each). Leaves the
// last down-projection's partial sums in m->part (added by the caller's next norm).
// Claims the next pair of profile events (or -1): the launcher hands them to the kernel launch, which
// stamps them with the kernel's own start and end, so launch gaps are not counted.
static int prof_claim(sd_model* m, int cls, double bytes) {
    Profile& p = m->prof;
    if (!p.on || p.used * 2 + 1 >= p.ev.size()) return -1;
    int i = (int)p.used++;
    p.cls[i] = cls;
    p.bytes[i] = bytes;
    return i;
}
static hipEvent_t prof_ev(sd_model* m, int i, int which) { return i >= 0 ? m->prof.ev[2 * i + which] : nullptr; }

// One weight-streaming GEMM; algorithmic bytes = one read of the (unpadded) weight matrix.
static SkRowScale row_scale(const sd_model* m, const float* ssq) {
    return SkRowScale{ssq, m->cfg.d_model / 16, 1.f / (float)m->cfg.d_model, m->cfg.rms_eps};
}
static const SkRowScale NO_SCALE = {nullptr, 0, 0.f, 0.f};

static PartView run_gemm(sd_model* m, const void* Xp, const void* Wp, float* out, int MB, int KB, int NB, int n_real,
                         hipStream_t s) {
    const GemmPlan* p = m->find_plan(MB, KB, NB);
    if (!p) {                                          // unreachable after have_plans(); never launch with another shape's plan
        m->plan_missing = true;
        return PartView{out, 0, NB * 32, nullptr, 0};  // no slots: the consumer adds nothing
    }
    const int pi = prof_claim(m, PROF_GEMM, (double)n_real * KB * 16 * 2);
    return launch_gemm(*p, Xp, Wp, m->zfrag, out, s, prof_ev(m, pi, 0), prof_ev(m, pi, 1));
}

// Every GEMM shape a pass over M rows issues (and, with heads = true, the draft heads after it, in the
// schedule given) has a launch plan: checked by the entry points before anything is enqueued.
static bool have_plans(const sd_model* m, int M, int B, bool heads, bool all_rows) {
    if (m->f32) return true;                           // the float32 kernels take any shape
    const int MB = pow2_blocks(M), H = m->cfg.n_medusa;
    bool ok = m->find_plan(MB, m->KBd, m->NBqkv) && m->find_plan(MB, m->KBd, m->NBo) && m->find_plan(MB, m->KBd, m->NBgu) &&
              m->find_plan(MB, m->KBf, m->NBo) && m->find_plan(MB, m->KBd, m->NBv);
    if (heads && !all_rows)
        ok = ok && m->find_plan(1, m->KBd, m->NBmed) && m->find_plan(pow2_blocks(H * B), m->KBd, m->NBv);
    if (heads && all_rows) {
        const int R = H * M, n_chunks = ceil_div(R, 256);
        ok = ok && m->find_plan(MB, m->KBd, m->NBmed) && m->find_plan(pow2_blocks(R - (n_chunks - 1) * 256), m->KBd, m->NBv) &&
             (n_chunks == 1 || m->find_plan(8, m->KBd, m->NBv));
    }
    return ok;
}

// How the attention of one step is cut into workgroups (one resident per compute unit: the kernel
// takes the whole LDS). A group is one (sequence, head, query-block group); it gets `ncparts` cache
// parts of `per` 32-row blocks each, sized from the host's bound on the sequence lengths, and the
// tree blocks go to a part of their own while the chip has room for it (short contexts) or to the
// last cache part (long contexts).
// tree_sep: parts that hold tree blocks only: 0 (the last cache part takes them), 1, or, when the attention launch
// builds the tree's keys and values itself (one query group of two blocks: split_ok), one per tree block, so that the
// building is shared by two workgroups.
struct AttnGeom { int ncparts, per, tree_sep, nparts; };
static AttnGeom attn_geometry(const sd_model* m, int B, int Tp, int n_hi, bool split_ok = false) {
    const int nblk = ceil_div(n_hi, 32);
    const int TB = Tp / 32, TG = (TB % 2 == 0) ? TB / 2 : TB;
    const int groups = B * m->cfg.n_heads * TG;
    int P = 256 / groups;                                  // parts per group that fit the chip at once
    if (P < 1) P = 1;
    if (P > m->max_parts) P = m->max_parts;
    AttnGeom g;
    if (nblk == 0) { g.ncparts = 0; g.per = 1; g.tree_sep = 1; g.nparts = 1; return g; }
    const int by_work = ceil_div(nblk, 4);                 // at least one block per wave
    const int ntp = (split_ok && TB == 2 && P >= 3) ? 2 : 1;
    // The tree keeps parts of its own while the cache parts are short: up to eight blocks per cache part, or, when a
    // single sequence has the chip (eight parts per head, of which the tree's one or two idle while the others stream),
    // up to forty: there the launch without the rotary stage before it wins up to ~8 k rows (64-node tree, step at
    // 1.5 / 3 / 6 k rows: 5.18 -> 5.06, 5.25 -> 5.20, 5.55 -> 5.47 ms; at 16 k rows 6.40 -> 6.45, so not there).
    const int short_mult = P >= 8 ? 40 : 8;
    if (P >= 2 && nblk <= short_mult * (P - ntp)) {        // short: the tree beside the cache parts
        // (two blocks per wave before another part is opened: every part repeats the queries' set-up and adds a term
        // to the merge; 7B shape, 64-node tree over 512-1800 rows: attention launch 18.4 -> 16.8 us, step -1 %)
        const int by_two = ceil_div(nblk, 8);
        g.tree_sep = ntp;
        g.ncparts = P - ntp < by_two ? P - ntp : by_two;
    } else {
        g.tree_sep = 0;
        g.ncparts = P < by_work ? P : by_work;
    }
    g.per = ceil_div(nblk, g.ncparts);
    g.ncparts = ceil_div(nblk, g.per);
    g.nparts = g.ncparts + g.tree_sep;
    return g;
}

static PartView run_layers(sd_model* m, sd_kv* kv, int B, int Tp, int n_hi, hipStream_t s) {
    const sd_config& c = m->cfg;
    const int M = B * Tp, MB = pow2_blocks(M), d = c.d_model, nh = c.n_heads, hd = c.head_dim, TB = Tp / 32;
    const AttnGeom ag = attn_geometry(m, B, Tp, n_hi, /*split_ok=*/Tp == 64);   // (one query group of two blocks)
    PartView prev = {nullptr, 0, d, nullptr, 0};
    const size_t t_stride = (size_t)B * nh * TB * 32 * hd;     // elements per layer of tree scratch
    for (int l = 0; l < c.n_layers; ++l) {
        const LayerW& lw = m->layers[l];
        launch_norm_pack(m->x, prev, lw.attn_norm, c.rms_eps, m->xn, nullptr, M, d, MB, nullptr, s);
        PartView pq = run_gemm(m, m->xn, lw.wqkv, m->part, MB, m->KBd, m->NBqkv, 3 * d, s);
        uint16_t* kt = (uint16_t*)m->kt + l * t_stride;
        uint16_t* vt = (uint16_t*)m->vt + l * t_stride;
        // With one query group per head (trees of up to 64 nodes, plain decoding, short prompt chunks) the attention
        // launch builds the queries and the tree's keys / values from the QKV partial sums itself: one launch less per
        // layer (7B shape: plain decoding +3 %, the 64-node step 4.95 -> 4.89 ms once each of its two tree blocks has a
        // workgroup of its own to build it). With several query groups every group would repeat that work, and at long
        // contexts, where the tree blocks go to the last of several cache parts, that part would become the straggler
        // (16 k rows: attention 55 -> 64 us): there the stage stays a launch of its own. Where every (sequence, head) has
        // ONE workgroup (a batch that fills the chip) all workgroups carry the same extra work, none is a straggler, and
        // the launch saved is worth more than it costs (batch of eight 32-node trees: attention 65.4 -> 72.8 us, the
        // 11.8 us launch gone, step -0.8 %).
        const bool fr = Tp <= 64 && (ag.tree_sep || ag.ncparts == 1);
        if (!fr) launch_rope_kv(pq, m->rt, m->q, kt, vt, B, Tp, nh, hd, s);
        // algorithmic bytes: one read of K and V of the committed rows (upper bound n_hi) + tree rows
        const int pa = prof_claim(m, PROF_ATTN, (double)B * (n_hi + Tp) * 2.0 * d * 2.0);
        launch_tree_attn(m->q, kv->kc + l * kv->layer_stride, kv->vc + l * kv->layer_stride, kt, vt, kv->kv_len,
                         m->rt.anc, m->opart, m->mlpart, B, nh, hd, Tp, kv->cap_blocks, ag.ncparts, ag.per, ag.tree_sep, s,
                         prof_ev(m, pa, 0), prof_ev(m, pa, 1), fr ? &pq : nullptr, fr ? &m->rt : nullptr);
        launch_attn_merge(m->opart, m->mlpart, m->attn_x, B, nh, hd, Tp, ag.nparts, MB, s);
        PartView po = run_gemm(m, m->attn_x, lw.wo, m->part, MB, m->KBd, m->NBo, d, s);
        launch_norm_pack(m->x, po, lw.ffn_norm, c.rms_eps, m->xn, nullptr, M, d, MB, nullptr, s);
        PartView pg = run_gemm(m, m->xn, lw.wgu, m->part, MB, m->KBd, m->NBgu, 2 * c.d_ffn, s);
        launch_swiglu_pack(pg, c.d_ffn, m->Fpad, m->act, M, MB, s);
        prev = run_gemm(m, m->act, lw.wdown, m->part, MB, m->KBf, m->NBo, d, s);
    }
    return prev;
}

// ---- the same pass through the persistent layer kernel: one launch per layer besides attention
static FusedGemm fused_gemm(const sd_model* m, int MB, int KB, int NB, const void* X, const void* W, float* out) {
    const GemmPlan* p = m->find_plan(MB, KB, NB);          // present: have_plans() ran before
    FusedGemm g;
    g.X = (const bf16x8*)X; g.W = (const bf16x8*)W; g.out = out;
    g.KB = KB; g.NB = NB; g.ldo = NB * 32;
    g.slot_stride = (size_t)MB * 32 * g.ldo;
    g.upw = p->upw; g.rem = p->rem; g.G = p->G; g.nmax = p->slots;
    g.kb_magic = (uint32_t)((0x100000000ull + (uint64_t)KB - 1) / (uint64_t)KB);
    g.slot0 = p->slot0_dev;
    g.cnt = p->uniform ? nullptr : p->cnt_dev;
    g.sc = NO_SCALE;
    return g;
}
static bool fused_eligible(const sd_model* m, int M) {
    if (m->f32) return false;
    const int MB = pow2_blocks(M);
    return m->use_fused && m->fused_ok && (MB == 1 || MB == 2 || MB == 8);
}
// Layers 0..L-1 and, with want_lm, the final norm and the LM-head GEMM, whose partial sums the returned view
// describes (without want_lm: the last down projection's, still to be added to m->x).
static PartView run_forward_fused(sd_model* m, sd_kv* kv, int B, int Tp, int n_hi, bool want_lm, hipStream_t s) {
    const sd_config& c = m->cfg;
    const int M = B * Tp, MB = pow2_blocks(M), d = c.d_model, nh = c.n_heads, hd = c.head_dim, TB = Tp / 32, L = c.n_layers;
    const AttnGeom ag = attn_geometry(m, B, Tp, n_hi);
    const size_t t_stride = (size_t)B * nh * TB * 32 * hd;
    launch_fill_i32((int32_t*)m->sync_ctr, 0, (L + 1) * FUSED_SYNC_WORDS, s);
    m->fused_dirty = true;
    FusedArgs a;
    memset(&a, 0, sizeof(a));
    a.M = M; a.MB = MB; a.B = B; a.Tp = Tp; a.d = d; a.nh = nh; a.hd = hd; a.F = c.d_ffn; a.Fpad = m->Fpad;
    a.nparts = ag.nparts; a.eps = c.rms_eps;
    a.x = m->x; a.opart = m->opart; a.mlpart = m->mlpart; a.att = (bf16x8*)m->attn_x;
    a.xn_f = (bf16x8*)m->xn2; a.act = (bf16x8*)m->act; a.xn_a = (bf16x8*)m->xn;
    a.ssq_f = m->ssq_f; a.ssq_a = m->ssq_a;
    a.rt = m->rt; a.q = (bf16x8*)m->q; a.zfrag = (const bf16x8*)m->zfrag;
    a.sync.abort_flag = m->sync_abort; a.sync.timeout_ticks = m->sync_timeout_ticks;
    const double w_attn_side = (double)(3 * d) * m->KBd * 32.0, w_ffn_side = ((double)d * m->KBd + 2.0 * c.d_ffn * m->KBd + (double)d * m->KBf) * 32.0;
    PartView last = {nullptr, 0, d, nullptr, 0};
    for (int l = 0; l <= L; ++l) {                         // launch l: the end of layer l-1 and the start of layer l
        double bytes = 0.0;
        a.phases = 0;
        a.sync.counters = m->sync_ctr + (size_t)l * FUSED_SYNC_WORDS;
        if (l > 0) {
            const LayerW& lw = m->layers[l - 1];
            a.phases |= FUSED_GEMM_O | FUSED_GEMM_GU | FUSED_GEMM_DN;
            a.g_o = fused_gemm(m, MB, m->KBd, m->NBo, m->attn_x, lw.wo, m->part_o);
            a.gain_f = (const uint16_t*)lw.ffn_norm;
            a.g_gu = fused_gemm(m, MB, m->KBd, m->NBgu, m->xn2, lw.wgu, m->part_gu);
            a.g_gu.sc = row_scale(m, m->ssq_f);
            a.g_dn = fused_gemm(m, MB, m->KBf, m->NBo, m->act, lw.wdown, m->part_dn);
            bytes += w_ffn_side;
            last = PartView{a.g_dn.out, a.g_dn.slot_stride, a.g_dn.ldo, a.g_dn.cnt, a.g_dn.nmax};
        }
        a.prev = PartView{nullptr, 0, d, nullptr, 0};
        if (l < L) {
            const LayerW& lw = m->layers[l];
            a.phases |= FUSED_GEMM_Q | FUSED_ROPE;
            a.gain_a = (const uint16_t*)lw.attn_norm;
            a.g_q = fused_gemm(m, MB, m->KBd, m->NBqkv, m->xn, lw.wqkv, m->part_q);
            a.g_q.sc = row_scale(m, m->ssq_a);
            a.kt = (uint16_t*)m->kt + l * t_stride;
            a.vt = (uint16_t*)m->vt + l * t_stride;
            bytes += w_attn_side;
        } else if (want_lm) {
            a.phases |= FUSED_GEMM_Q;
            a.gain_a = (const uint16_t*)m->final_norm;
            a.g_q = fused_gemm(m, MB, m->KBd, m->NBv, m->xn, m->lm_head, m->part_q);
            a.g_q.sc = row_scale(m, m->ssq_a);
            bytes += (double)c.vocab * m->KBd * 32.0;
            last = PartView{a.g_q.out, a.g_q.slot_stride, a.g_q.ldo, a.g_q.cnt, a.g_q.nmax};
        }
        a.timeline = (m->timeline && (size_t)l < m->timeline_launches) ? m->timeline + (size_t)l * 24 * 256 : nullptr;
        const int pi = prof_claim(m, PROF_GEMM, bytes);
        launch_layer(a, 256, s, prof_ev(m, pi, 0), prof_ev(m, pi, 1));
        if (l < L) {
            const int pa = prof_claim(m, PROF_ATTN, (double)B * (n_hi + Tp) * 2.0 * d * 2.0);
            launch_tree_attn(m->q, kv->kc + l * kv->layer_stride, kv->vc + l * kv->layer_stride, a.kt, a.vt, kv->kv_len,
                             m->rt.anc, m->opart, m->mlpart, B, nh, hd, Tp, kv->cap_blocks, ag.ncparts, ag.per, ag.tree_sep, s,
                             prof_ev(m, pa, 0), prof_ev(m, pa, 1));
        }
    }
    return last;
}

// final norm + LM head on all rows + arg-max of the first T rows of every sequence
// ------------------------------------------------------------------------------------------ float32 pass
static void commit_rows(sd_model* m, sd_kv* kv, const int32_t* slots, const int32_t* n_acc, int Tp, int W, hipStream_t s) {
    const sd_config& c = m->cfg;
    if (m->f32)
        launch_f32_kv_commit(m->f.kt, m->f.vt, kv->kc32, kv->vc32, slots, n_acc, kv->n_old, c.n_layers, kv->B, c.d_model, Tp,
                             kv->cap, W, s);
    else
        launch_kv_commit(m->kt, m->vt, kv->kc, kv->vc, slots, n_acc, kv->n_old, c.n_layers, kv->B, c.n_heads, c.head_dim,
                         Tp / 32, kv->cap_blocks, W, W, s);
}

static void run_forward_f32(sd_model* m, sd_kv* kv, int B, int T, int Tp, bool want_lm, hipStream_t s) {
    const sd_config& c = m->cfg;
    const int M = B * Tp, d = c.d_model, F = c.d_ffn;
    sd_model::F32& f = m->f;
    for (int l = 0; l < c.n_layers; ++l) {
        const sd_model::F32Layer& lw = f.layers[l];
        float* kt = f.kt + (size_t)l * M * d;
        float* vt = f.vt + (size_t)l * M * d;
        launch_f32_rmsnorm(m->x, lw.attn_norm, c.rms_eps, f.xn, M, d, nullptr, s);
        launch_f32_linear(f.xn, lw.wqkv, nullptr, f.qkv, M, 3 * d, d, d, 3 * d, 0, s);
        launch_f32_rope_kv(f.qkv, m->rt, f.q, kt, vt, M, c.n_heads, c.head_dim, s);
        launch_f32_attn(f.q, kv->kc32 + l * kv->layer_stride, kv->vc32 + l * kv->layer_stride, kt, vt, kv->kv_len, m->rt.anc,
                        f.attn, B, c.n_heads, c.head_dim, Tp, kv->cap, s);
        launch_f32_linear(f.attn, lw.wo, nullptr, m->x, M, d, d, d, d, 1, s);
        launch_f32_rmsnorm(m->x, lw.ffn_norm, c.rms_eps, f.xn, M, d, nullptr, s);
        launch_f32_linear(f.xn, lw.wgu, nullptr, f.gu, M, 2 * F, d, d, 2 * F, 0, s);
        launch_f32_swiglu(f.gu, f.act, M, F, s);
        launch_f32_linear(f.act, lw.wdown, nullptr, m->x, M, d, F, F, d, 1, s);
    }
    if (want_lm) {
        launch_f32_rmsnorm(m->x, f.final_norm, c.rms_eps, f.xn, M, d, nullptr, s);
        launch_f32_linear(f.xn, f.lm_head, nullptr, m->logits, M, c.vocab, d, d, m->Vpad, 0, s);
        launch_argmax(m->logits, m->Vpad, c.vocab, m->am, B, T, Tp, s);
    }
}

static void run_draft_heads_f32(sd_model* m, sd_kv* kv, int B, uint32_t seq_mask, float* head_logits_out, hipStream_t s) {
    const sd_config& c = m->cfg;
    const int d = c.d_model, H = c.n_medusa;
    sd_model::F32& f = m->f;
    launch_f32_rmsnorm(m->x, f.final_norm, c.rms_eps, m->h_rows, B, d, kv->last_row, s);
    launch_f32_linear(m->h_rows, f.medusa_w, f.medusa_b, f.z, B, H * d, d, d, H * d, 0, s);
    launch_f32_medusa_act(f.z, m->h_rows, f.xh, B, H, d, s);
    launch_f32_linear(f.xh, f.lm_head, nullptr, m->hlogits, H * B, c.vocab, d, d, m->Vpad, 0, s);
    launch_topk(m->hlogits, m->Vpad, c.vocab, c.topk, kv->cand, B, H, seq_mask, s);
    if (head_logits_out) launch_copy_head_logits(m->hlogits, m->Vpad, head_logits_out, c.vocab, B, H, s);
}

// (keep_h: also leaves the normalised rows in m->hf as fp32, for draft heads on every row)
// need_logits: somebody reads m->logits afterwards (the caller's copy, sampling decoding); else only the arg-max
static void run_lm_head(sd_model* m, PartView prev, int B, int T, int Tp, hipStream_t s, bool keep_h, bool need_logits) {
    const sd_config& c = m->cfg;
    const int M = B * Tp, MB = pow2_blocks(M);
    launch_norm_pack(m->x, prev, m->final_norm, c.rms_eps, m->xn, keep_h ? m->hf : nullptr, M, c.d_model, MB, nullptr, s);
    PartView pl = run_gemm(m, m->xn, m->lm_head, m->part, MB, m->KBd, m->NBv, c.vocab, s);
    launch_reduce_argmax(pl, need_logits ? m->logits : nullptr, c.vocab, m->am, B, T, Tp, s);
}

// The whole verifying pass: layers, and with want_lm the final norm, the LM head and the arg-max of the first T rows
// of every sequence (logits in m->logits, arg-max in m->am).
static void run_forward(sd_model* m, sd_kv* kv, int B, int T, int Tp, int n_hi, bool want_lm, bool keep_h, bool need_logits,
                        hipStream_t s) {
    m->scratch_B = B;
    m->scratch_Tp = Tp;
    if (m->f32) { run_forward_f32(m, kv, B, T, Tp, want_lm, s); return; }
    if (fused_eligible(m, B * Tp)) {
        // (when the final norm's rows themselves are wanted, the last stage runs as kernels of its own)
        PartView pl = run_forward_fused(m, kv, B, Tp, n_hi, want_lm && !keep_h, s);
        if (want_lm && keep_h) run_lm_head(m, pl, B, T, Tp, s, true, need_logits);
        else if (want_lm) launch_reduce_argmax(pl, need_logits ? m->logits : nullptr, m->cfg.vocab, m->am, B, T, Tp, s);
        return;
    }
    PartView prev = run_layers(m, kv, B, Tp, n_hi, s);
    if (want_lm) run_lm_head(m, prev, B, T, Tp, s, keep_h, need_logits);
}

// draft heads at row last_row[b] of every sequence -> cand (sequences in seq_mask only)
static void run_draft_heads(sd_model* m, sd_kv* kv, int B, uint32_t seq_mask, float* head_logits_out, hipStream_t s) {
    if (m->f32) { run_draft_heads_f32(m, kv, B, seq_mask, head_logits_out, s); return; }
    const sd_config& c = m->cfg;
    const int d = c.d_model, H = c.n_medusa;
    const PartView none = {nullptr, 0, d, nullptr, 0};
    launch_norm_pack(m->x, none, m->final_norm, c.rms_eps, m->xn, m->h_rows, B, d, 1, kv->last_row, s);
    PartView pm = run_gemm(m, m->xn, m->medusa_w, m->part, 1, m->KBd, m->NBmed, H * d, s);
    const int MBh = pow2_blocks(H * B);
    launch_medusa_act(pm, m->h_rows, m->medusa_b, B, H, d, m->xn, MBh * 32, MBh, MBh, s);
    PartView pl = run_gemm(m, m->xn, m->lm_head, m->part, MBh, m->KBd, m->NBv, c.vocab, s);
    // (a top-k that sums the slots itself was measured: 54 us against 5 + 22 us for these two, its few workgroups
    // pull the partial sums too slowly)
    launch_reduce_slots(pl, m->hlogits, H * B, s);
    launch_topk(m->hlogits, m->Vpad, c.vocab, c.topk, kv->cand, B, H, seq_mask, s);
    if (head_logits_out) launch_copy_head_logits(m->hlogits, m->Vpad, head_logits_out, c.vocab, B, H, s);
}

// The other schedule: the draft heads run on all B*Tp rows of the verifying pass (m->xn and m->hf
// still hold the final norm's output), the shared LM head on all H*B*Tp head rows in chunks of 256
// rows, and only the H rows of every sequence's last kept row (kv->last_row, set by the acceptance kernel) are
// summed out of the partial tiles and ranked.
static void run_draft_heads_all_rows(sd_model* m, sd_kv* kv, int B, int Tp, float* head_logits_out, hipStream_t s) {
    const sd_config& c = m->cfg;
    const int d = c.d_model, H = c.n_medusa, M = B * Tp, MB = pow2_blocks(M), R = H * M, CH = 256;
    PartView pm = run_gemm(m, m->xn, m->medusa_w, m->part, MB, m->KBd, m->NBmed, H * d, s);
    const int n_chunks = ceil_div(R, CH), MBlast = pow2_blocks(R - (n_chunks - 1) * CH);
    launch_medusa_act(pm, m->hf, m->medusa_b, M, H, d, m->xh, CH, CH / 32, MBlast, s);
    for (int ch = 0; ch < n_chunks; ++ch) {
        const int rows = std::min(CH, R - ch * CH);
        const char* xc = (const char*)m->xh + (size_t)ch * CH * d * 4;
        PartView pl = run_gemm(m, xc, m->lm_head, m->part, ch == n_chunks - 1 ? MBlast : CH / 32, m->KBd, m->NBv,
                               c.vocab, s);
        launch_reduce_selected(pl, m->hlogits, kv->last_row, B, H, M, ch * CH, rows, s);
    }
    launch_topk(m->hlogits, m->Vpad, c.vocab, c.topk, kv->cand, B, H, 0xffffffffu, s);
    if (head_logits_out) launch_copy_head_logits(m->hlogits, m->Vpad, head_logits_out, c.vocab, B, H, s);
}

// ------------------------------------------------------------------------------------------ prefill
extern "C" int sd_prefill(sd_model* m, sd_kv* kv, const int32_t* tokens, const int32_t* lens, void* stream) {
    if (!m || !kv || !tokens || !lens) return fail(SD_ERR_NULL, "sd_prefill: NULL argument");
    if (kv->m != m) return fail(SD_ERR_STATE, "sd_prefill: cache belongs to another model");
    const sd_config& c = m->cfg;
    const int B = kv->B;
    hipStream_t s = (hipStream_t)stream;
    int Tp = (m->max_rows / B) / 32 * 32;
    if (Tp > 256) Tp = 256;                            // prompt chunks of up to 256 rows (the widest GEMM)
    if (Tp < 32) return fail(SD_ERR_SHAPE, "sd_prefill: max_rows %d too small for batch %d", m->max_rows, B);
    int maxlen = 0;
    for (int b = 0; b < B; ++b) {
        if (lens[b] < 1) return fail(SD_ERR_SHAPE, "sd_prefill: every prompt needs at least one token");
        if (kv->len_hi[b] + lens[b] > kv->cap) return fail(SD_ERR_KV_FULL, "sd_prefill: sequence %d does not fit", b);
        maxlen = std::max(maxlen, lens[b]);
    }
    if (!have_plans(m, B * Tp, B, true, false))
        return fail(SD_ERR_STATE, "sd_prefill: no launch plan for %d rows (internal inconsistency)", B * Tp);
    std::vector<int> start(B), done(B, 0);
    for (int b = 0, o = 0; b < B; ++b) { start[b] = o; o += lens[b]; }
    for (int pos = 0; pos < maxlen; pos += Tp) {
        ChainArgs ca;
        memset(&ca, 0, sizeof(ca));
        uint32_t fin = 0;
        int n_hi = 0;
        for (int b = 0; b < B; ++b) {
            int left = lens[b] - pos;
            ca.len[b] = left <= 0 ? 0 : std::min(left, Tp);
            ca.off[b] = start[b] + pos;
            if (left > 0 && left <= Tp) fin |= 1u << b;
            n_hi = std::max(n_hi, kv->len_hi[b]);
        }
        launch_build_rows_chain(m->rt, tokens, ca, kv->kv_len, B, Tp, c.head_dim, c.rope_theta, m->embed, m->f32 ? 1 : 0,
                                c.d_model, c.vocab, m->x, s);
        run_forward(m, kv, B, Tp, Tp, n_hi, fin != 0, false, false, s);
        launch_prefill_commit_setup(ca, B, Tp, kv->i_slots, kv->i_nacc, kv->n_old, kv->kv_len, kv->last_row, s);
        commit_rows(m, kv, kv->i_slots, kv->i_nacc, Tp, Tp, s);
        for (int b = 0; b < B; ++b) kv->len_hi[b] += ca.len[b];
        if (fin) {
            launch_pick_root(m->am, kv->last_row, kv->root_tok, B, fin, s);
            run_draft_heads(m, kv, B, fin, nullptr, s);
        }
    }
    HIP_TRY(hipGetLastError());
    if (m->plan_missing) return fail(SD_ERR_STATE, "sd_prefill: a GEMM launch plan was missing");
    kv->has_draft = true;
    return SD_OK;
}

// ------------------------------------------------------------------------------------------ steps
static int step_common(sd_model* m, sd_kv* kv, uint64_t tree_uid, const int32_t* parent, const int32_t* depth,
                       const int32_t* rank, int T, int Tp, const uint32_t* stop_mask, sd_step_io* io, hipStream_t s,
                       const char* who, const sd_typical* ty = nullptr) {
    const sd_config& c = m->cfg;
    const int B = kv->B, H = c.n_medusa;
    if (kv->m != m) return fail(SD_ERR_STATE, "%s: cache belongs to another model", who);
    if (!kv->has_draft) return fail(SD_ERR_STATE, "%s: no draft state (call sd_prefill or sd_kv_set_draft first)", who);
    if (pow2_blocks(B * Tp) > m->MBmax)
        return fail(SD_ERR_SHAPE, "%s: %d rows exceed the model's max_rows", who, B * Tp);
    int n_hi = 0;
    for (int b = 0; b < B; ++b) {
        if (kv->len_hi[b] + H + 1 > kv->cap)
            return fail(SD_ERR_KV_FULL, "%s: sequence %d may exceed the cache (len <= %d, cap %d)", who, b,
                        kv->len_hi[b], kv->cap);
        n_hi = std::max(n_hi, kv->len_hi[b]);
    }
    const bool all_rows = m->draft_schedule == SD_DRAFT_ALL_NODES && T > 1 && !m->f32;   // (float32: one schedule only)
    const bool heads = T > 1 || m->greedy_drafts;      // plain greedy decoding may leave the draft heads out
    if (!have_plans(m, B * Tp, B, heads, all_rows))
        return fail(SD_ERR_STATE, "%s: no launch plan for %d rows (internal inconsistency)", who, B * Tp);
    int32_t* n_accept = io->n_accept ? io->n_accept : kv->i_nacc;
    int32_t* tokens = io->tokens ? io->tokens : kv->i_tokens;
    int32_t* slots = io->src_slots ? io->src_slots : kv->i_slots;
    const int32_t* cand = io->forced_cand ? io->forced_cand : kv->cand;

    // everything the launch sequence depends on besides device-resident state
    auto enqueue = [&](hipStream_t s) {
    launch_build_rows_tree(m->rt, parent, depth, rank, kv->root_tok, cand, kv->kv_len, B, T, Tp, H, c.topk, c.head_dim,
                           c.rope_theta, m->embed, m->f32 ? 1 : 0, c.d_model, c.vocab, m->x, s);
    run_forward(m, kv, B, T, Tp, n_hi, true, all_rows, io->logits != nullptr || ty != nullptr, s);
    if (io->logits) launch_copy_logits(m->logits, m->Vpad, io->logits, c.vocab, B, T, Tp, s);
    if (io->argmax) launch_copy_rows_i32(m->am, io->argmax, B, T, Tp, s);
    VerifyArgs va;
    va.parent = parent; va.depth = depth; va.T = T; va.H = H; va.fallback = c.trunc_fallback;
    va.src_stride = Tp; va.Tp = Tp; va.V = c.vocab;
    va.tok = m->rt.tok; va.am = m->am; va.stop_mask = stop_mask;
    va.n_accept = n_accept; va.n_accept_raw = io->n_accept_raw; va.tokens = tokens; va.src_slots = slots;
    va.kv_len = kv->kv_len; va.n_old = kv->n_old; va.root_tok = kv->root_tok; va.last_row = kv->last_row;
    va.logits = nullptr; va.ld = 0; va.row_stats = nullptr; va.inv_temperature = 1.f;
    if (ty) {
        va.inv_temperature = 1.f / ty->temperature;
        launch_row_stats(m->logits, m->Vpad, c.vocab, m->row_stats, B, T, Tp, va.inv_temperature, ty->epsilon,
                         ty->delta, s);
        if (ty->row_stats) launch_copy_row_stats(m->row_stats, (float4*)ty->row_stats, B, T, Tp, s);
        va.logits = m->logits; va.ld = m->Vpad; va.row_stats = m->row_stats;
    }
    launch_verify(va, B, s);
    if (ty)      // the next root is drawn from the base distribution at the last kept node
        launch_sample_root(m->logits, m->Vpad, c.vocab, kv->last_row, ty->u, va.inv_temperature, kv->root_tok, B,
                           B * Tp, s);
    commit_rows(m, kv, slots, n_accept, Tp, H + 1, s);
    if (all_rows) run_draft_heads_all_rows(m, kv, B, Tp, io->head_logits, s);
    else if (heads) run_draft_heads(m, kv, B, 0xffffffffu, io->head_logits, s);
    };

    if (m->use_graphs && !m->prof.on && !ty) {
        const AttnGeom ag = attn_geometry(m, B, Tp, n_hi, Tp == 64);
        std::vector<uint64_t> key = {kv->uid, tree_uid, (uint64_t)(uintptr_t)parent, (uint64_t)T, (uint64_t)Tp,
                                     (uint64_t)ag.ncparts, (uint64_t)(ag.per * 4 + ag.tree_sep), (uint64_t)(uintptr_t)stop_mask,
                                     (uint64_t)(uintptr_t)n_accept, (uint64_t)(uintptr_t)tokens,
                                     (uint64_t)(uintptr_t)slots, (uint64_t)(uintptr_t)io->n_accept_raw,
                                     (uint64_t)(uintptr_t)io->logits, (uint64_t)(uintptr_t)io->argmax,
                                     (uint64_t)(uintptr_t)io->head_logits, (uint64_t)(uintptr_t)cand,
                                     (uint64_t)m->draft_schedule, (uint64_t)heads,
                                     (uint64_t)(m->use_fused ? 1 : 0) | ((uint64_t)m->sync_timeout_ticks << 1)};
        hipGraphExec_t exec = nullptr;
        for (const sd_model::StepGraph& g : m->graphs)
            if (g.key == key) { exec = g.exec; break; }
        if (!exec) {
            if (m->graphs.size() >= 64) {              // bounded cache: start over
                for (sd_model::StepGraph& g : m->graphs) hipGraphExecDestroy(g.exec);
                m->graphs.clear();
            }
            hipGraph_t graph = nullptr;
            if (!m->cap_stream) HIP_TRY(hipStreamCreateWithFlags(&m->cap_stream, hipStreamNonBlocking));
            HIP_TRY(hipStreamBeginCapture(m->cap_stream, hipStreamCaptureModeThreadLocal));
            enqueue(m->cap_stream);
            hipError_t e = hipStreamEndCapture(m->cap_stream, &graph);
            if (e != hipSuccess) return fail(SD_ERR_HIP, "%s: graph capture failed: %s", who, hipGetErrorString(e));
            e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
            hipGraphDestroy(graph);
            if (e != hipSuccess) return fail(SD_ERR_HIP, "%s: hipGraphInstantiate: %s", who, hipGetErrorString(e));
            m->graphs.push_back({key, exec});
        }
        HIP_TRY(hipGraphLaunch(exec, s));
    } else {
        enqueue(s);
    }
    HIP_TRY(hipGetLastError());
    if (m->plan_missing) return fail(SD_ERR_STATE, "%s: a GEMM launch plan was missing", who);
    for (int b = 0; b < B; ++b) kv->len_hi[b] += (T == 1) ? 1 : H + 1;
    return SD_OK;
}

extern "C" int sd_spec_step(sd_model* m, sd_kv* kv, const sd_tree* tree, const uint32_t* stop_mask, sd_step_io* io,
                            void* stream) {
    if (!m || !kv || !tree || !stop_mask || !io) return fail(SD_ERR_NULL, "sd_spec_step: NULL argument");
    if (tree->H != m->cfg.n_medusa || tree->topk != m->cfg.topk)
        return fail(SD_ERR_BAD_TREE, "sd_spec_step: tree was built for %d heads / top-%d", tree->H, tree->topk);
    return step_common(m, kv, tree->uid, tree->parent, tree->depth, tree->rank, tree->T, tree->Tp, stop_mask, io,
                       (hipStream_t)stream, "sd_spec_step");
}

// Commit stage alone: rows of the tree scratch, as the last pass over this cache's batch left them, appended to
// every sequence.
extern "C" int sd_kv_commit_rows(sd_model* m, sd_kv* kv, const int32_t* src_slots, const int32_t* n_rows, int32_t width,
                                 void* stream) {
    if (!m || !kv || !src_slots || !n_rows) return fail(SD_ERR_NULL, "sd_kv_commit_rows: NULL argument");
    if (kv->m != m) return fail(SD_ERR_STATE, "sd_kv_commit_rows: cache belongs to another model");
    if (m->scratch_B != kv->B || m->scratch_Tp < 32)
        return fail(SD_ERR_STATE, "sd_kv_commit_rows: no pass over a batch of %d has left tree rows to commit", kv->B);
    if (width < 1 || width > m->scratch_Tp)
        return fail(SD_ERR_SHAPE, "sd_kv_commit_rows: width must be in 1..%d (the rows of the last pass)", m->scratch_Tp);
    for (int b = 0; b < kv->B; ++b)
        if (kv->len_hi[b] + width > kv->cap)
            return fail(SD_ERR_KV_FULL, "sd_kv_commit_rows: sequence %d may exceed the cache (len <= %d, cap %d)", b,
                        kv->len_hi[b], kv->cap);
    hipStream_t s = (hipStream_t)stream;
    launch_commit_setup(n_rows, width, kv->B, kv->i_nacc, kv->n_old, kv->kv_len, s);
    commit_rows(m, kv, src_slots, kv->i_nacc, m->scratch_Tp, width, s);
    HIP_TRY(hipGetLastError());
    for (int b = 0; b < kv->B; ++b) kv->len_hi[b] += width;
    return SD_OK;
}

static int check_typical(float temperature, float epsilon, float delta, const char* who) {
    if (!(temperature > 0.f) || !std::isfinite(temperature))
        return fail(SD_ERR_SHAPE, "%s: temperature must be positive and finite", who);
    if (!(epsilon >= 0.f && epsilon <= 1.f) || !(delta >= 0.f) || !std::isfinite(delta))
        return fail(SD_ERR_SHAPE, "%s: need 0 <= epsilon <= 1 and 0 <= delta < inf", who);
    return SD_OK;
}

extern "C" int sd_spec_step_typical(sd_model* m, sd_kv* kv, const sd_tree* tree, const uint32_t* stop_mask,
                                    sd_step_io* io, const sd_typical* ty, void* stream) {
    if (!m || !kv || !tree || !stop_mask || !io || !ty) return fail(SD_ERR_NULL, "sd_spec_step_typical: NULL argument");
    if (tree->H != m->cfg.n_medusa || tree->topk != m->cfg.topk)
        return fail(SD_ERR_BAD_TREE, "sd_spec_step_typical: tree was built for %d heads / top-%d", tree->H, tree->topk);
    if (!ty->u) return fail(SD_ERR_NULL, "sd_spec_step_typical: sd_typical.u is NULL");
    if (int rc = check_typical(ty->temperature, ty->epsilon, ty->delta, "sd_spec_step_typical")) return rc;
    return step_common(m, kv, tree->uid, tree->parent, tree->depth, tree->rank, tree->T, tree->Tp, stop_mask, io,
                       (hipStream_t)stream, "sd_spec_step_typical", ty);
}

extern "C" int sd_greedy_step(sd_model* m, sd_kv* kv, sd_step_io* io, void* stream) {
    if (!m || !kv || !io) return fail(SD_ERR_NULL, "sd_greedy_step: NULL argument");
    return step_common(m, kv, 0, m->g_parent, m->g_depth, m->g_rank, 1, 32, m->zero_stop, io, (hipStream_t)stream,
                       "sd_greedy_step");
}

extern "C" int sd_verify_tree(const sd_tree* tree, int32_t batch, int32_t n_medusa, int32_t trunc_fallback,
                              int32_t vocab, const int32_t* tok, const int32_t* am, const uint32_t* stop_mask,
                              int32_t* n_accept, int32_t* n_accept_raw, int32_t* tokens, int32_t* src_slots,
                              void* stream) {
    if (!tree || !tok || !am || !stop_mask || !n_accept || !tokens || !src_slots)
        return fail(SD_ERR_NULL, "sd_verify_tree: NULL argument");
    if (batch < 1 || batch > 65535) return fail(SD_ERR_SHAPE, "sd_verify_tree: bad batch");
    if (n_medusa != tree->H) return fail(SD_ERR_BAD_TREE, "sd_verify_tree: tree was built for %d heads", tree->H);
    if (trunc_fallback != SD_TRUNC_KEEP_ALL && trunc_fallback != SD_TRUNC_KEEP_ONE)
        return fail(SD_ERR_SHAPE, "sd_verify_tree: bad trunc_fallback");
    VerifyArgs va;
    memset(&va, 0, sizeof(va));
    va.parent = tree->parent; va.depth = tree->depth; va.T = tree->T; va.H = tree->H; va.fallback = trunc_fallback;
    va.src_stride = tree->T; va.Tp = tree->Tp; va.V = vocab;
    va.tok = tok; va.am = am; va.stop_mask = stop_mask;
    va.n_accept = n_accept; va.n_accept_raw = n_accept_raw; va.tokens = tokens; va.src_slots = src_slots;
    launch_verify(va, batch, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return SD_OK;
}

extern "C" int sd_verify_tree_typical(const sd_tree* tree, int32_t batch, int32_t n_medusa, int32_t trunc_fallback,
                                      int32_t vocab, const int32_t* tok, const float* logits, float temperature,
                                      float epsilon, float delta, const uint32_t* stop_mask, float* row_stats,
                                      int32_t* n_accept, int32_t* n_accept_raw, int32_t* tokens, int32_t* src_slots,
                                      void* stream) {
    if (!tree || !tok || !logits || !stop_mask || !row_stats || !n_accept || !tokens || !src_slots)
        return fail(SD_ERR_NULL, "sd_verify_tree_typical: NULL argument");
    if (batch < 1 || batch > 65535) return fail(SD_ERR_SHAPE, "sd_verify_tree_typical: bad batch");
    if (vocab < 1 || vocab > 163840) return fail(SD_ERR_SHAPE, "sd_verify_tree_typical: bad vocab");
    if (n_medusa != tree->H) return fail(SD_ERR_BAD_TREE, "sd_verify_tree_typical: tree was built for %d heads", tree->H);
    if (trunc_fallback != SD_TRUNC_KEEP_ALL && trunc_fallback != SD_TRUNC_KEEP_ONE)
        return fail(SD_ERR_SHAPE, "sd_verify_tree_typical: bad trunc_fallback");
    if (int rc = check_typical(temperature, epsilon, delta, "sd_verify_tree_typical")) return rc;
    hipStream_t s = (hipStream_t)stream;
    const int T = tree->T;
    launch_row_stats(logits, vocab, vocab, (float4*)row_stats, batch, T, T, 1.f / temperature, epsilon, delta, s);
    VerifyArgs va;
    memset(&va, 0, sizeof(va));
    va.parent = tree->parent; va.depth = tree->depth; va.T = T; va.H = tree->H; va.fallback = trunc_fallback;
    va.src_stride = T; va.Tp = tree->Tp; va.V = vocab;
    va.tok = tok; va.am = tok; va.stop_mask = stop_mask;      // am is not read under typical acceptance
    va.n_accept = n_accept; va.n_accept_raw = n_accept_raw; va.tokens = tokens; va.src_slots = src_slots;
    va.logits = logits; va.ld = vocab; va.row_stats = (const float4*)row_stats; va.inv_temperature = 1.f / temperature;
    launch_verify(va, batch, s);
    HIP_TRY(hipGetLastError());
    return SD_OK;
}

// ------------------------------------------------------------------------------------------ no allocation
// Per-node statistics of sd_verify_tree_typical_static: one copy per GPU, held until the process ends.
#define SD_STATIC_ROWS 4096
static __device__ __align__(256) float4 scratch[SD_STATIC_ROWS];
// Device address of `scratch` on every GPU this process has used it on. The array's name is only a host-side
// handle: the address a kernel can use comes from hipGetSymbolAddress, per device.
#define SD_MAX_DEVICES 64
static float4* g_scratch_dev[SD_MAX_DEVICES] = {};

static int static_scratch(float4** out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= SD_MAX_DEVICES) return fail(SD_ERR_SHAPE, "device ordinal %d not supported", dev);
    float4* p = __atomic_load_n(&g_scratch_dev[dev], __ATOMIC_ACQUIRE);
    if (!p) {                                          // first call on this device (two racing threads get the same answer)
        void* addr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch)));
        if (!addr) return fail(SD_ERR_HIP, "hipGetSymbolAddress returned no address");
        p = (float4*)addr;
        __atomic_store_n(&g_scratch_dev[dev], p, __ATOMIC_RELEASE);
    }
    *out = p;
    return SD_OK;
}

extern "C" int sd_verify_tree_typical_static(const sd_tree* tree, int32_t batch, int32_t n_medusa,
                                             int32_t trunc_fallback, int32_t vocab, const int32_t* tok,
                                             const float* logits, float temperature, float epsilon, float delta,
                                             const uint32_t* stop_mask, int32_t* n_accept, int32_t* n_accept_raw,
                                             int32_t* tokens, int32_t* src_slots, void* stream) {
    if (!tree || !tok || !logits || !stop_mask || !n_accept || !tokens || !src_slots)
        return fail(SD_ERR_NULL, "sd_verify_tree_typical_static: NULL argument");
    if (batch < 1 || batch > 65535) return fail(SD_ERR_SHAPE, "sd_verify_tree_typical_static: bad batch");
    if ((int64_t)batch * tree->T > SD_STATIC_ROWS)
        return fail(SD_ERR_SHAPE, "sd_verify_tree_typical_static: batch * tree nodes = %lld exceeds the %d rows of the "
                    "static statistics buffer (use sd_verify_tree_typical with a buffer of your own)",
                    (long long)batch * tree->T, SD_STATIC_ROWS);
    if (vocab < 1 || vocab > 163840) return fail(SD_ERR_SHAPE, "sd_verify_tree_typical_static: bad vocab");
    if (n_medusa != tree->H)
        return fail(SD_ERR_BAD_TREE, "sd_verify_tree_typical_static: tree was built for %d heads", tree->H);
    if (trunc_fallback != SD_TRUNC_KEEP_ALL && trunc_fallback != SD_TRUNC_KEEP_ONE)
        return fail(SD_ERR_SHAPE, "sd_verify_tree_typical_static: bad trunc_fallback");
    if (int rc = check_typical(temperature, epsilon, delta, "sd_verify_tree_typical_static")) return rc;
    float4* stats = nullptr;
    if (int rc = static_scratch(&stats)) return rc;
    hipStream_t s = (hipStream_t)stream;
    const int T = tree->T;
    // every row of the statistics that the acceptance kernel reads is written first by this launch, so nothing
    // of the previous call's contents needs clearing
    launch_row_stats(logits, vocab, vocab, stats, batch, T, T, 1.f / temperature, epsilon, delta, s);
    VerifyArgs va;
    memset(&va, 0, sizeof(va));
    va.parent = tree->parent; va.depth = tree->depth; va.T = T; va.H = tree->H; va.fallback = trunc_fallback;
    va.src_stride = T; va.Tp = tree->Tp; va.V = vocab;
    va.tok = tok; va.am = tok; va.stop_mask = stop_mask;      // am is not read under typical acceptance
    va.n_accept = n_accept; va.n_accept_raw = n_accept_raw; va.tokens = tokens; va.src_slots = src_slots;
    va.logits = logits; va.ld = vocab; va.row_stats = stats; va.inv_temperature = 1.f / temperature;
    launch_verify(va, batch, s);
    HIP_TRY(hipGetLastError());
    return SD_OK;
}

extern "C" int sd_sample_tokens(const float* logits, int32_t n_rows, int32_t ld, int32_t vocab, const int32_t* rows,
                                const float* u, int32_t n, float temperature, int32_t* out, void* stream) {
    if (!logits || !rows || !u || !out) return fail(SD_ERR_NULL, "sd_sample_tokens: NULL argument");
    if (n < 1 || n > 65535 || n_rows < 1) return fail(SD_ERR_SHAPE, "sd_sample_tokens: bad n");
    if (vocab < 1 || vocab > 163840 || ld < vocab) return fail(SD_ERR_SHAPE, "sd_sample_tokens: bad vocab / ld");
    if (!(temperature > 0.f) || !std::isfinite(temperature))
        return fail(SD_ERR_SHAPE, "sd_sample_tokens: temperature must be positive and finite");
    launch_sample_root(logits, ld, vocab, rows, u, 1.f / temperature, out, n, n_rows, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return SD_OK;
}
