// Host side of the C ABI declared in ps_draft.h: argument validation, workspace layout,
// the per-phase launch plan, and the launch sequence of one parallel draft step
// (Section 4.1 "Inference").  No arithmetic of the method happens here except the rotary
// table (cos/sin of position * base^(-2j/d)), computed once at init in double precision.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <new>
#include <vector>

#include "ps_internal.h"

static const PsInstance* find_instance(int dtype, int d) {
    const PsInstance* all[4] = {ps_instance_f32_d64(), ps_instance_f32_d128(), ps_instance_bf16_d64(),
                                ps_instance_bf16_d128()};
    for (int i = 0; i < 4; ++i)
        if (all[i]->dtype == dtype && all[i]->head_dim == d) return all[i];
    return nullptr;
}

#define PS_MAX_WG 512   // upper bound on workgroups per phase used to size the workspace

// With PS_DRAFT_DEBUG set, a failing HIP call is named on stderr before PS_ERR_DEVICE is returned.
static bool hip_ok(hipError_t e, const char* what) {
    if (e == hipSuccess) return true;
    if (getenv("PS_DRAFT_DEBUG")) fprintf(stderr, "ps_draft: %s failed: %s\n", what, hipGetErrorString(e));
    return false;
}

struct ps_draft_ctx {
    ps_draft_config cfg;
    ps_draft_weights w;
    const PsInstance* inst;
    int fused;                        // 1: whole step as one persistent kernel, 0: one kernel per phase
    int device;
    int n_cu;
    int lds_limit;                    // dynamic LDS a workgroup may use on this device
    // workspace carve-up (device pointers)
    float2* rope;
    float *q_buf, *o_buf, *y_buf, *u_buf, *y2_buf, *kvnew, *part, *ssq_part, *attn_acc, *attn_ml, *lm_part, *logits_ws;
    unsigned seq;                     // sequence number of the last enqueued step
    size_t exch_begin, exch_end;      // workspace range of the tagged exchange buffers (cleared at init)
    char* act_base;                   // two copies of the activation buffers, act_bytes each
    size_t act_bytes;
    size_t off_q, off_o, off_y, off_u, off_y2, off_kvnew;   // offsets inside one copy
    int last_shape[3];                // batch, n_new, k of the previous step
    char* wpack[PH_COUNT];
    int* counters;
    int n_counters;
    size_t frag_cap;                  // 1 KiB split-K fragments the workspace holds
    int plan_override[PH_COUNT][2];   // S, KW from PS_DRAFT_PLAN (0 = automatic)
    bool profile;
    unsigned long long* timeline;
    hipEvent_t events[PS_PROFILE_EVENTS];
};

// ------------------------------------------------------------------------------------------
// validation and sizes (no HIP calls)
// ------------------------------------------------------------------------------------------
static int validate_config(const ps_draft_config* c) {
    if (!c) return PS_ERR_NULL;
    if (c->dtype != PS_F32 && c->dtype != PS_BF16) return PS_ERR_CONFIG;
    if (c->hidden < 1 || c->n_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 1 || c->ffn < 1 || c->vocab < 1)
        return PS_ERR_CONFIG;
    if (c->k_max < 0 || c->max_batch < 1 || c->max_new < 1 || c->max_topk < 1 || c->max_positions < 1)
        return PS_ERR_CONFIG;
    if (c->n_heads % c->n_kv_heads != 0) return PS_ERR_CONFIG;
    if (c->head_dim % 2 != 0) return PS_ERR_CONFIG;
    if (!(c->rms_eps >= 0.f) || !(c->rope_base > 0.f)) return PS_ERR_CONFIG;
    if (c->max_positions < c->max_new + c->k_max) return PS_ERR_CONFIG;
    if (c->flags & ~PS_FLAG_FINAL_NORM) return PS_ERR_CONFIG;
    // what this build has kernels for
    const int kmul = c->dtype == PS_BF16 ? 32 : 16;
    const long long qd = (long long)c->n_heads * c->head_dim;
    if (c->head_dim != 64 && c->head_dim != 128) return PS_ERR_UNSUPPORTED;
    if (c->hidden % kmul || qd % kmul || c->ffn % kmul) return PS_ERR_UNSUPPORTED;
    if (c->hidden % 16 || c->ffn % 8) return PS_ERR_UNSUPPORTED;
    if ((long long)c->max_batch * (c->max_new + c->k_max) > PS_MAX_ROWS) return PS_ERR_UNSUPPORTED;
    if ((long long)(c->n_heads / c->n_kv_heads) * (c->max_new + c->k_max) > PS_MAX_ROWS) return PS_ERR_UNSUPPORTED;
    if (c->max_topk > 32) return PS_ERR_UNSUPPORTED;
    if (qd > (1 << 20) || c->hidden > (1 << 20) || c->ffn > (1 << 22) || c->vocab > (1 << 24)) return PS_ERR_UNSUPPORTED;
    return PS_OK;
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct WsLayout {
    size_t wpack[PH_COUNT];
    size_t rope, q_buf, o_buf, y_buf, u_buf, y2_buf, kvnew, part, ssq_part, attn_acc, attn_ml, counters, lm_part, logits_ws, total;
    size_t exch_begin, exch_end;
    size_t act_base, act_bytes, off_q, off_o, off_y, off_u, off_y2, off_kvnew;
    size_t frag_cap;
    int n_counters;
};

static int max_tiles(const ps_draft_config* c) {
    const int qkv = (c->n_heads + 2 * c->n_kv_heads) * (c->head_dim / 16);
    int t = qkv;
    if (c->hidden / 16 > t) t = c->hidden / 16;
    if (c->ffn / 8 > t) t = c->ffn / 8;
    return t;
}

// tiles (16 weight rows) and steps (64-byte pieces of a row) of the five GEMM phases
static void phase_dims(const ps_draft_config* c, int* T, int* Kt) {
    const int kstep = c->dtype == PS_BF16 ? 32 : 16;
    const int qd = c->n_heads * c->head_dim;
    T[PH_QKV] = (c->n_heads + 2 * c->n_kv_heads) * (c->head_dim / 16); Kt[PH_QKV] = c->hidden / kstep;
    T[PH_OPROJ] = c->hidden / 16; Kt[PH_OPROJ] = qd / kstep;
    T[PH_GATEUP] = c->ffn / 8; Kt[PH_GATEUP] = c->hidden / kstep;
    T[PH_DOWN] = c->hidden / 16; Kt[PH_DOWN] = c->ffn / kstep;
    T[PH_LMHEAD] = (c->vocab + 15) / 16; Kt[PH_LMHEAD] = c->hidden / kstep;
}

static WsLayout ws_layout(const ps_draft_config* c) {
    WsLayout L;
    const size_t rows = (size_t)c->max_batch * (c->max_new + c->k_max);
    const size_t qd = (size_t)c->n_heads * c->head_dim;
    const int grp = c->n_heads / c->n_kv_heads;
    const int ch = find_instance(c->dtype, c->head_dim)->attn_chunk;
    const size_t max_items = (size_t)c->max_batch * c->n_kv_heads * ((c->max_positions + ch - 1) / ch);
    const size_t ra = (size_t)grp * (c->max_new + c->k_max);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
    int T[PH_COUNT], Kt[PH_COUNT];
    phase_dims(c, T, Kt);
    // padding: the streaming loop always loads PS_U steps ahead, also at the end of the last tile
    for (int ph = 0; ph < PH_COUNT; ++ph) L.wpack[ph] = take((size_t)T[ph] * Kt[ph] * 1024 + PS_U_MAX * 1024);
    L.rope = take((size_t)c->max_positions * (c->head_dim / 2) * sizeof(float2));
    // activations between phases: fp32, two alternating copies (see PS_SENT in ps_device.h)
    {
        size_t a = 0;
        auto sub = [&](size_t bytes) { size_t o = a; a = align256(a + bytes); return o; };
        L.off_q = sub(rows * qd * 4);
        L.off_o = sub(rows * qd * 4);
        L.off_y = sub(rows * c->hidden * 4);
        L.off_u = sub(rows * c->ffn * 4);
        L.off_y2 = sub(rows * c->hidden * 4);
        L.off_kvnew = sub(rows * 2 * (size_t)c->n_kv_heads * c->head_dim * 4);
        L.act_bytes = a;
        L.act_base = take(2 * a);
    }
    L.q_buf = L.o_buf = L.y_buf = L.u_buf = L.y2_buf = L.kvnew = 0;   // set per step from the copy in use
    // tagged exchange buffers: 8 bytes per element (value + tag)
    L.exch_begin = off;
    // split-K fragments: S * T never exceeds the wavefronts of a phase (see make_plan); one fragment
    // is 64 lanes x 4 values per column tile
    size_t frag = (size_t)PS_MAX_WG * PS_WAVES;
    if ((size_t)max_tiles(c) * 2 > frag) frag = (size_t)max_tiles(c) * 2;
    L.frag_cap = frag * 4;
    L.part = take(L.frag_cap * 2048);
    L.ssq_part = take(L.frag_cap * PS_MAX_ROWS * 8);
    L.attn_acc = take(max_items * ra * c->head_dim * 8);
    L.attn_ml = take(max_items * ra * 2 * 8);
    L.lm_part = take((size_t)PS_MAX_WG * rows * (2 + 2 * c->max_topk) * 8 + 64);
    L.exch_end = off;
    L.n_counters = 0;
    L.counters = take(64);   // error flag
    L.logits_ws = take(rows * c->vocab * 4);
    L.total = off;
    return L;
}

extern "C" size_t ps_draft_workspace_bytes(const ps_draft_config* config) {
    if (validate_config(config) != PS_OK) return 0;
    return ws_layout(config).total;
}

extern "C" const char* ps_draft_strerror(int status) {
    switch (status) {
        case PS_OK: return "success";
        case PS_ERR_NULL: return "a required pointer is NULL";
        case PS_ERR_CONFIG: return "invalid configuration";
        case PS_ERR_SHAPE: return "step arguments outside the configured bounds";
        case PS_ERR_KV_CAPACITY: return "KV cache capacity or max_positions exceeded";
        case PS_ERR_OFFSETS: return "kv_offsets is not a non-decreasing array of non-negative positions";
        case PS_ERR_WORKSPACE: return "workspace too small or not 256-byte aligned";
        case PS_ERR_UNSUPPORTED: return "shape not supported by this build";
        case PS_ERR_DEVICE: return "HIP device error";
        default: return "unknown status";
    }
}

// PS_DRAFT_PLAN="qkv:4:1,oproj:16:1,gateup:2:1,down:16:1,lm:1:2" overrides (S, KW) per phase (tuning aid)
static void parse_plan_override(ps_draft_ctx* ctx) {
    memset(ctx->plan_override, 0, sizeof(ctx->plan_override));
    const char* e = getenv("PS_DRAFT_PLAN");
    if (!e) return;
    static const char* names[PH_COUNT] = {"qkv", "oproj", "gateup", "down", "lm"};
    for (int ph = 0; ph < PH_COUNT; ++ph) {
        const char* p = strstr(e, names[ph]);
        if (!p) continue;
        int s = 0, kw = 0;
        if (sscanf(p + strlen(names[ph]), ":%d:%d", &s, &kw) == 2) {
            ctx->plan_override[ph][0] = s;
            ctx->plan_override[ph][1] = kw;
        }
    }
}

extern "C" int ps_draft_init(ps_draft_ctx** out, const ps_draft_config* config, const ps_draft_weights* weights,
                             void* workspace, size_t workspace_bytes, void* stream) {
    if (!out || !config || !weights) return PS_ERR_NULL;
    int st = validate_config(config);
    if (st != PS_OK) return st;
    const ps_draft_weights* w = weights;
    if (!w->g_in || !w->wq || !w->wk || !w->wv || !w->wo || !w->g_post || !w->w_gate || !w->w_up || !w->w_down || !w->w_lm)
        return PS_ERR_NULL;
    if ((config->flags & PS_FLAG_FINAL_NORM) && !w->g_final) return PS_ERR_NULL;
    if (config->k_max > 0 && !w->mask_emb) return PS_ERR_NULL;
    if (!workspace) return PS_ERR_NULL;
    const WsLayout L = ws_layout(config);
    if (workspace_bytes < L.total || ((uintptr_t)workspace & 255)) return PS_ERR_WORKSPACE;

    // ---- first HIP call happens here
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev), "hipGetDevice")) return PS_ERR_DEVICE;
    hipDeviceProp_t prop;
    if (!hip_ok(hipGetDeviceProperties(&prop, dev), "hipGetDeviceProperties")) return PS_ERR_DEVICE;
    int lds_limit = 0;
    if (!hip_ok(hipDeviceGetAttribute(&lds_limit, hipDeviceAttributeMaxSharedMemoryPerBlock, dev), "hipDeviceGetAttribute")) return PS_ERR_DEVICE;
    if (getenv("PS_DRAFT_DEBUG")) fprintf(stderr, "ps_draft: %s, %d CUs, LDS per workgroup %d\n", prop.name, prop.multiProcessorCount, lds_limit);
    if (lds_limit > PS_LDS_BYTES) lds_limit = PS_LDS_BYTES;
    if (lds_limit < 64 * 1024) return PS_ERR_DEVICE;
    const PsInstance* inst = find_instance(config->dtype, config->head_dim);
    if (!inst) return PS_ERR_UNSUPPORTED;
    if (!hip_ok(inst->prepare(lds_limit), "hipFuncSetAttribute")) return PS_ERR_DEVICE;
    const int coop = 1;

    ps_draft_ctx* ctx = new (std::nothrow) ps_draft_ctx;
    if (!ctx) return PS_ERR_DEVICE;
    ctx->cfg = *config;
    ctx->w = *weights;
    ctx->device = dev;
    ctx->inst = inst;
    {
        const char* mode = getenv("PS_DRAFT_MODE");   // "multi": one kernel per phase (profiling, fallback)
        ctx->fused = coop && !(mode && strcmp(mode, "multi") == 0);
    }
    ctx->lds_limit = lds_limit;
    ctx->n_cu = prop.multiProcessorCount;
    if (ctx->n_cu < 1) ctx->n_cu = 1;
    if (ctx->n_cu > PS_MAX_WG) ctx->n_cu = PS_MAX_WG;
    char* base = (char*)workspace;
    for (int ph = 0; ph < PH_COUNT; ++ph) ctx->wpack[ph] = base + L.wpack[ph];
    ctx->rope = (float2*)(base + L.rope);
    ctx->act_base = base + L.act_base; ctx->act_bytes = L.act_bytes;
    ctx->off_q = L.off_q; ctx->off_o = L.off_o; ctx->off_y = L.off_y; ctx->off_u = L.off_u;
    ctx->off_y2 = L.off_y2; ctx->off_kvnew = L.off_kvnew;
    ctx->last_shape[0] = ctx->last_shape[1] = ctx->last_shape[2] = -1;
    ctx->part = (float*)(base + L.part);
    ctx->ssq_part = (float*)(base + L.ssq_part);
    ctx->attn_acc = (float*)(base + L.attn_acc);
    ctx->attn_ml = (float*)(base + L.attn_ml);
    ctx->seq = 0;
    ctx->exch_begin = L.exch_begin; ctx->exch_end = L.exch_end;
    ctx->counters = (int*)(base + L.counters);
    ctx->n_counters = L.n_counters;
    ctx->frag_cap = L.frag_cap;
    ctx->lm_part = (float*)(base + L.lm_part);
    ctx->logits_ws = (float*)(base + L.logits_ws);
    parse_plan_override(ctx);
    ctx->profile = false;
    ctx->timeline = nullptr;

    // rotary table: (cos, sin) of pos * base^(-2j/d), rotate-half pairing (j, j + d/2)
    const int half = config->head_dim / 2;
    std::vector<float2> tab((size_t)config->max_positions * half);
    for (int j = 0; j < half; ++j) {
        const double inv = pow((double)config->rope_base, -2.0 * j / config->head_dim);
        for (int p = 0; p < config->max_positions; ++p) {
            const double a = (double)p * inv;
            tab[(size_t)p * half + j] = make_float2((float)cos(a), (float)sin(a));
        }
    }
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipMemcpyAsync(ctx->rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice, s);
    // sequence numbers start at 1: cleared exchange buffers never look valid
    if (e == hipSuccess) e = hipMemsetAsync(base + L.exch_begin, 0, L.exch_end - L.exch_begin, s);
    if (e == hipSuccess) e = hipMemsetAsync(ctx->act_base, 0xFF, 2 * L.act_bytes, s);   // both copies: nothing written yet
    if (e == hipSuccess) e = hipMemsetAsync(ctx->counters, 0, 64, s);
    {   // copy the five weight matrices into streaming order
        StepParams P;
        memset(&P, 0, sizeof(P));
        P.H = config->hidden; P.nq = config->n_heads; P.nkv = config->n_kv_heads; P.d = config->head_dim;
        P.F = config->ffn; P.V = config->vocab; P.QD = config->n_heads * config->head_dim;
        P.wq = w->wq; P.wk = w->wk; P.wv = w->wv; P.wo = w->wo; P.w_gate = w->w_gate; P.w_up = w->w_up;
        P.w_down = w->w_down; P.w_lm = w->w_lm;
        int T[PH_COUNT], Kt[PH_COUNT];
        phase_dims(config, T, Kt);
        for (int ph = 0; ph < PH_COUNT && e == hipSuccess; ++ph)
            e = inst->pack(P, ph, T[ph], Kt[ph], ctx->wpack[ph], s);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (!hip_ok(e, "rotary table upload")) { delete ctx; return PS_ERR_DEVICE; }
    *out = ctx;
    return PS_OK;
}

extern "C" void ps_draft_free(ps_draft_ctx* ctx) { delete ctx; }

// Debugging aid, not declared in the public header: device buffer of 32 x 1024 uint64 receiving
// per-workgroup wall-clock stamps of the following steps (NULL = off).
extern "C" __attribute__((visibility("default"))) int ps_draft_debug_timeline(ps_draft_ctx* ctx, void* buf) {
    if (!ctx) return PS_ERR_NULL;
    ctx->timeline = (unsigned long long*)buf;
    return PS_OK;
}

extern "C" int ps_draft_set_profile_events(ps_draft_ctx* ctx, void* const* events) {
    if (!ctx) return PS_ERR_NULL;
    ctx->profile = events != nullptr;
    if (events)
        for (int i = 0; i < PS_PROFILE_EVENTS; ++i) {
            if (!events[i]) { ctx->profile = false; return PS_ERR_NULL; }
            ctx->events[i] = (hipEvent_t)events[i];
        }
    return PS_OK;
}

// ------------------------------------------------------------------------------------------
// launch plan
// ------------------------------------------------------------------------------------------
static int floor_pow2(int v) { int p = 1; while (p * 2 <= v) p *= 2; return p; }

int panel_row_stride_host(int panel_steps) {
    const int len = panel_steps * 64;
    return len + ((64 - (len & 255)) + 256) % 256;
}

// Cuts one GEMM phase: T tiles x Kt steps over nwg workgroups of 16 wavefronts.
static bool make_plan(PhasePlan* pl, int ph, int T, int Kt, int rows, int mt, bool bf, int nwg, int cnt_base,
                      const int* override_, int lds_limit) {
    const int waves = nwg * PS_WAVES;
    int split = floor_pow2(waves / T > 0 ? waves / T : 1);
    while (split > 1 && Kt / split < 4) split /= 2;   // keep at least 4 steps per piece
    // S (K-slices across workgroups) costs a fragment exchange with one memory round trip per four
    // slices, but divides the activation panel every workgroup has to fetch; KW (K-split across the
    // wavefronts of a workgroup) is free.  The LM head keeps whole logits in the workgroup (S = 1);
    // the QKV phase reads caller data that is cached, so its panel is cheap (S = 1).
    int S, KW;
    if (ph == PH_LMHEAD || ph == PH_QKV) { S = 1; KW = split > PS_WAVES ? PS_WAVES : split; }
    else { S = split > 4 ? 4 : split; KW = split / S; if (KW > PS_WAVES) KW = PS_WAVES; }
    if (override_ && override_[0] > 0 && override_[1] > 0) { S = override_[0]; KW = override_[1]; }
    if (ph == PH_LMHEAD) S = 1;
    if (S > nwg) S = floor_pow2(nwg);
    if (KW > PS_WAVES) KW = PS_WAVES;
    if (PS_WAVES % KW) KW = floor_pow2(KW);
    pl->T = T; pl->Kt = Kt; pl->S = S; pl->KW = KW; pl->nwg = nwg; pl->cnt_base = cnt_base;
    const int Gs = nwg / S, SL = PS_WAVES / KW;
    const int rounds = (T + Gs * SL - 1) / (Gs * SL);
    const int fixed = 512 + PS_WAVES * mt * 1024 + (ph == PH_LMHEAD ? rounds * SL * rows * 64 : 0);
    const int budget = lds_limit - fixed - 1024;
    if (budget <= 0) return false;
    const int slice_steps = (Kt + S - 1) / S;
    int steps = slice_steps;
    const int per_row_arrays = bf ? 2 : 1;
    while (steps > 1 && (long long)rows * per_row_arrays * panel_row_stride_host(steps) > budget) steps = (steps + 1) / 2;
    if ((long long)rows * per_row_arrays * panel_row_stride_host(steps) > budget) return false;
    pl->panel_steps = steps;
    pl->lds_bytes = fixed + rows * per_row_arrays * panel_row_stride_host(steps);
    return true;
}

extern "C" int ps_draft_step(ps_draft_ctx* ctx, const ps_draft_step_args* a, void* stream) {
    if (!ctx || !a) return PS_ERR_NULL;
    const ps_draft_config& c = ctx->cfg;
    if (a->batch < 1 || a->batch > c.max_batch || a->n_new < 1 || a->n_new > c.max_new || a->k < 0 || a->k > c.k_max)
        return PS_ERR_SHAPE;
    if (a->topk < 1 || a->topk > c.max_topk || a->topk > c.vocab) return PS_ERR_SHAPE;
    if (a->out_rows != 0 && a->out_rows != 1) return PS_ERR_SHAPE;
    if (!a->x || !a->k_cache || !a->v_cache || !a->kv_offsets || !a->kv_len || !a->top_ids || !a->top_p || !a->lse)
        return PS_ERR_NULL;
    const int M = a->n_new + a->k;
    for (int b = 0; b < a->batch; ++b) {
        if (a->kv_offsets[b] < 0 || a->kv_offsets[b + 1] < a->kv_offsets[b]) return PS_ERR_OFFSETS;
    }
    for (int b = 0; b < a->batch; ++b) {
        if (a->kv_len[b] < 0) return PS_ERR_SHAPE;
        if ((long long)a->kv_len[b] + M > a->kv_offsets[b + 1] - a->kv_offsets[b]) return PS_ERR_KV_CAPACITY;
        if ((long long)a->kv_len[b] + M > c.max_positions) return PS_ERR_KV_CAPACITY;
    }

    StepParams P;
    memset(&P, 0, sizeof(P));
    P.H = c.hidden; P.nq = c.n_heads; P.nkv = c.n_kv_heads; P.d = c.head_dim; P.F = c.ffn; P.V = c.vocab;
    P.QD = c.n_heads * c.head_dim; P.KVD = c.n_kv_heads * c.head_dim;
    P.B = a->batch; P.n_new = a->n_new; P.k = a->k; P.M = M; P.Mtot = a->batch * M;
    P.all_rows = a->out_rows; P.R = a->out_rows ? M : a->k + 1; P.Rtot = a->batch * P.R; P.topk = a->topk;
    P.final_norm = (c.flags & PS_FLAG_FINAL_NORM) ? 1 : 0; P.max_positions = c.max_positions;
    P.eps = c.rms_eps; P.inv_sqrt_d = (float)(1.0 / sqrt((double)c.head_dim));
    P.g_in = ctx->w.g_in; P.wq = ctx->w.wq; P.wk = ctx->w.wk; P.wv = ctx->w.wv; P.wo = ctx->w.wo;
    P.g_post = ctx->w.g_post; P.w_gate = ctx->w.w_gate; P.w_up = ctx->w.w_up; P.w_down = ctx->w.w_down;
    P.g_final = ctx->w.g_final; P.w_lm = ctx->w.w_lm; P.mask_emb = ctx->w.mask_emb;
    P.x = a->x; P.kc = a->k_cache; P.vc = a->v_cache;
    for (int ph = 0; ph < PH_COUNT; ++ph) P.wpack[ph] = ctx->wpack[ph];
    P.rope = ctx->rope; P.part = ctx->part; P.attn_acc = ctx->attn_acc; P.attn_ml = ctx->attn_ml;
    P.lm_part = ctx->lm_part; P.ssq_part = ctx->ssq_part;
    P.error_flag = ctx->counters;
    ctx->seq = ctx->seq >= 0x1FFFFFF0u ? 1u : ctx->seq + 1u;   // seq * 8 + phase must fit in 32 bits; 0 = cleared
    P.seq = ctx->seq;
    {   // the activation copy of this step; the other one is reset while this one is written
        const int par = (int)(P.seq & 1u);
        char* cur = ctx->act_base + (size_t)par * ctx->act_bytes;
        P.q_buf = (float*)(cur + ctx->off_q); P.o_buf = (float*)(cur + ctx->off_o); P.y_buf = (float*)(cur + ctx->off_y);
        P.u_buf = (float*)(cur + ctx->off_u); P.y2_buf = (float*)(cur + ctx->off_y2); P.kvnew = (float*)(cur + ctx->off_kvnew);
        P.alt_delta = par ? -(long long)ctx->act_bytes : (long long)ctx->act_bytes;
        // a step only resets the elements it writes: when the row layout changes, elements the previous
        // step did not touch could still look written, so this step's copy is cleared first
        if (ctx->last_shape[0] != a->batch || ctx->last_shape[1] != a->n_new || ctx->last_shape[2] != a->k) {
            if (ctx->last_shape[0] >= 0 &&
                !hip_ok(hipMemsetAsync(cur, 0xFF, ctx->act_bytes, (hipStream_t)stream), "hipMemsetAsync")) return PS_ERR_DEVICE;
            ctx->last_shape[0] = a->batch; ctx->last_shape[1] = a->n_new; ctx->last_shape[2] = a->k;
        }
    }
    P.logits_store = a->logits ? a->logits : (a->probs ? ctx->logits_ws : nullptr);
    P.top_ids = a->top_ids; P.top_p = a->top_p; P.lse = a->lse; P.probs = a->probs; P.hidden_out = a->hidden_out;
    const int ch = ctx->inst->attn_chunk;
    int items = 0;
    for (int b = 0; b < a->batch; ++b) {
        P.kv_off[b] = a->kv_offsets[b];
        P.kv_len[b] = a->kv_len[b];
        items += c.n_kv_heads * ((a->kv_len[b] + M + ch - 1) / ch);
    }
    P.attn_items = items; P.attn_chunk = ch;
    P.attn_nwg = items < ctx->n_cu ? items : ctx->n_cu;

    const bool bf = c.dtype == PS_BF16;
    const int nwg = ctx->n_cu;
    const int mtiles = max_tiles(&c);
    int T[PH_COUNT], Kt[PH_COUNT];
    phase_dims(&c, T, Kt);
    for (int ph = 0; ph < PH_COUNT; ++ph) {
        const int rows = ph == PH_LMHEAD ? P.Rtot : P.Mtot;
        // the persistent kernel runs every phase with the column tiles of the widest one
        const int mt = (ctx->fused ? P.Mtot + 15 : rows + 15) / 16;
        if (!make_plan(&P.plan[ph], ph, T[ph], Kt[ph], rows, mt, bf, nwg, 0, ctx->plan_override[ph], ctx->lds_limit))
            return PS_ERR_UNSUPPORTED;
        if (P.plan[ph].S > 1 && (size_t)P.plan[ph].S * T[ph] * ((rows + 15) / 16) > ctx->frag_cap) return PS_ERR_UNSUPPORTED;
    }
    P.timeline = ctx->timeline;

    // the persistent kernel needs the largest LDS footprint of its phases and one workgroup per CU
    int lds = ctx->inst->attn_lds;
    for (int ph = 0; ph < PH_COUNT; ++ph) {
        if (P.plan[ph].lds_bytes > lds) lds = P.plan[ph].lds_bytes;
    }
    if (lds < 256 + 8192 + 128) lds = 256 + 8192 + 128;   // end-of-step merge scratch
    if (lds < 84 * 1024 && ctx->lds_limit >= 84 * 1024) lds = 84 * 1024;   // more than half a CU's LDS: one workgroup per CU
    P.fused_nwg = nwg; P.fused_lds = lds;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t* ev = ctx->profile ? ctx->events : nullptr;
    if (ctx->fused && lds <= ctx->lds_limit) {
        if (ev && !hip_ok(hipEventRecord(ev[0], st), "hipEventRecord")) return PS_ERR_DEVICE;
        if (!hip_ok(ctx->inst->launch_fused(P, st), "kernel launch")) return PS_ERR_DEVICE;
        if (ev)
            for (int i = 1; i < PS_PROFILE_EVENTS; ++i)
                if (!hip_ok(hipEventRecord(ev[i], st), "hipEventRecord")) return PS_ERR_DEVICE;
    } else {
        if (!hip_ok(ctx->inst->launch_multi(P, st, ev), "kernel launch")) return PS_ERR_DEVICE;
    }
    if (P.probs && !hip_ok(ctx->inst->launch_probs(P, st), "kernel launch")) return PS_ERR_DEVICE;
    return PS_OK;
}
