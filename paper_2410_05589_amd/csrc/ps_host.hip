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
#include "ps_draft_debug.h"

static const PsInstance* find_instance(int dtype, int d) {
    const PsInstance* all[4] = {ps_instance_f32_d64(), ps_instance_f32_d128(), ps_instance_bf16_d64(),
                                ps_instance_bf16_d128()};
    for (int i = 0; i < 4; ++i)
        if (all[i]->dtype == dtype && all[i]->head_dim == d) return all[i];
    return nullptr;
}

#define PS_MAX_WG 512   // upper bound on workgroups per phase used to size the workspace
#define PS_S_MAX 8      // most K-slices across workgroups

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
    float *q_buf, *o_buf, *y_buf, *u_buf, *y2_buf, *kvnew, *attn_acc, *attn_ml, *lm_part, *logits_ws;
    size_t exch_begin, exch_end;      // workspace range of the tagged exchange buffers (cleared at init)
    char* act_base;                   // two copies of the activation buffers, act_bytes each
    size_t act_bytes;
    size_t off_q, off_o, off_y, off_u, off_y2, off_kvnew, off_x;   // offsets inside one copy
    int spin_limit;                   // polls before a kernel gives up a wait (PS_SPIN_LIMIT; tests of that path: less)
    char* wpack[PH_COUNT];
    int* counters;
    int n_counters;
    int plan_override[PH_COUNT][2];   // K-slices, wavefronts per tile from PS_DRAFT_PLAN (0 = automatic)
    int attn_sep_override;            // PS_DRAFT_ATTN_SEP=0/1: who takes this step's rows in the attention (-1 = automatic)
    int attn_nk_override;             // PS_DRAFT_ATTN_NK=1/2/4/8/16: groups of 16 keys per wavefront and block, bf16 storage (0 = automatic)
    size_t off_frag[PH_COUNT], off_ssqf[PH_COUNT];
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
    if (c->flags & ~(PS_FLAG_FINAL_NORM | PS_FLAG_INPUT_FC)) return PS_ERR_CONFIG;
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
    if (c->max_positions > (1 << 24)) return PS_ERR_UNSUPPORTED;
    return PS_OK;
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct WsLayout {
    size_t wpack[PH_COUNT];
    size_t rope, q_buf, o_buf, y_buf, u_buf, y2_buf, kvnew, attn_acc, attn_ml, counters, lm_part, logits_ws, total;
    size_t exch_begin, exch_end;
    size_t act_base, act_bytes, off_q, off_o, off_y, off_u, off_y2, off_kvnew, off_x, off_frag[PH_COUNT], off_ssqf[PH_COUNT];
    int n_counters;
    bool fits32;   // the kernels address every exchange buffer with 32-bit byte offsets
};

// tiles (16 weight rows), contraction lengths and steps (64-byte pieces of a row) of the five GEMM phases
static void phase_dims(const ps_draft_config* c, int* T, int* Kt, int* K = nullptr) {
    const int kstep = c->dtype == PS_BF16 ? 32 : 16;
    const int qd = c->n_heads * c->head_dim;
    T[PH_QKV] = (c->n_heads + 2 * c->n_kv_heads) * (c->head_dim / 16); Kt[PH_QKV] = c->hidden / kstep;
    T[PH_OPROJ] = c->hidden / 16; Kt[PH_OPROJ] = qd / kstep;
    T[PH_GATEUP] = c->ffn / 8; Kt[PH_GATEUP] = c->hidden / kstep;
    T[PH_DOWN] = c->hidden / 16; Kt[PH_DOWN] = c->ffn / kstep;
    T[PH_LMHEAD] = (c->vocab + 15) / 16; Kt[PH_LMHEAD] = c->hidden / kstep;
    // the input projection [H, 2H] exists only with PS_FLAG_INPUT_FC
    const bool fc = (c->flags & PS_FLAG_INPUT_FC) != 0;
    T[PH_FC] = fc ? c->hidden / 16 : 0; Kt[PH_FC] = fc ? 2 * c->hidden / kstep : 0;
    if (K) { K[PH_QKV] = K[PH_GATEUP] = K[PH_LMHEAD] = c->hidden; K[PH_OPROJ] = qd; K[PH_DOWN] = c->ffn; K[PH_FC] = 2 * c->hidden; }
}
// steps per tile in the packed matrices: whole groups of PS_U steps
static int padded_steps(int kt) { return (kt + PS_U - 1) / PS_U * PS_U; }

static WsLayout ws_layout(const ps_draft_config* c) {
    WsLayout L;
    const size_t rows = (size_t)c->max_batch * (c->max_new + c->k_max);
    const size_t qd = (size_t)c->n_heads * c->head_dim;
    const int grp = c->n_heads / c->n_kv_heads;
    const int ch = PS_ATTN_KEYS;   // the smaller key block: the most work items
    const size_t max_items = (size_t)c->max_batch * c->n_kv_heads * ((c->max_positions + ch - 1) / ch);
    const size_t ra = (size_t)grp * (c->max_new + c->k_max);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
    int T[PH_COUNT], Kt[PH_COUNT];
    phase_dims(c, T, Kt);
    // padding: the streaming loop always loads PS_U steps ahead, also at the end of the last tile
    for (int ph = 0; ph < PH_COUNT; ++ph) L.wpack[ph] = take((size_t)T[ph] * padded_steps(Kt[ph]) * 1024 + PS_U_MAX * 1024);
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
        L.off_x = sub((c->flags & PS_FLAG_INPUT_FC) ? rows * c->hidden * 4 : 0);
        // parts of the tiles from up to PS_S_MAX K-slices (1 KiB per slice, tile and 16 rows)
        const size_t mt_max = (rows + 15) / 16;
        for (int ph = 0; ph < PH_COUNT; ++ph) L.off_ssqf[ph] = sub((size_t)PS_S_MAX * PS_MAX_ROWS * 4);
        for (int ph = 0; ph < PH_COUNT; ++ph) {
            const bool sliced = ph != PH_LMHEAD;
            L.off_frag[ph] = sub(sliced ? (size_t)PS_S_MAX * T[ph] * mt_max * 1024 : 256);
        }
        L.act_bytes = a;
        L.act_base = take(2 * a);
    }
    L.q_buf = L.o_buf = L.y_buf = L.u_buf = L.y2_buf = L.kvnew = 0;   // set per step from the copy in use
    // tagged exchange buffers: 8 bytes per element (value + tag)
    L.exch_begin = off;
    L.attn_acc = take(max_items * ra * c->head_dim * 8);
    L.attn_ml = take(max_items * ra * 2 * 8);
    L.lm_part = take((size_t)PS_MAX_WG * rows * (4 + 2 * c->max_topk) * 8 + 64);
    L.exch_end = off;
    L.n_counters = 0;
    L.counters = take(256);  // PS_CTR_*: error flag, steps completed, tickets of the running kernel, footprints
    L.logits_ws = take(rows * c->vocab * 4);
    L.total = off;
    const size_t lim = 0xFFFFFFF0ull;
    L.fits32 = L.act_bytes <= lim && L.lm_part - L.attn_acc <= lim && L.exch_end - L.lm_part <= lim;
    return L;
}
static_assert(PS_CTR_WORDS * 4 <= 256, "counters");

// a valid configuration whose exchange buffers the kernels can address
static int check_config(const ps_draft_config* c) {
    const int st = validate_config(c);
    if (st != PS_OK) return st;
    return ws_layout(c).fits32 ? PS_OK : PS_ERR_UNSUPPORTED;
}

extern "C" size_t ps_draft_workspace_bytes(const ps_draft_config* config) {
    if (check_config(config) != PS_OK) return 0;
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
        case PS_ERR_TIMEOUT: return "a step gave up waiting for its own workgroups (other work held the GPU?)";
        default: return "unknown status";
    }
}

// PS_DRAFT_PLAN="qkv:1:8,oproj:8:1,gateup:8:1,down:8:1,lm:1:1" overrides, per phase, the K-slices across
// workgroups and the wavefronts that share a tile (tuning aid)
static void parse_plan_override(ps_draft_ctx* ctx) {
    memset(ctx->plan_override, 0, sizeof(ctx->plan_override));
    const char* e = getenv("PS_DRAFT_PLAN");
    if (!e) return;
    static const char* names[PH_COUNT] = {"qkv", "oproj", "gateup", "down", "lm", "fc"};
    for (int ph = 0; ph < PH_COUNT; ++ph) {
        const char* p = strstr(e, names[ph]);
        if (!p) continue;
        int sl = 0, kw = 0;
        if (sscanf(p + strlen(names[ph]), ":%d:%d", &sl, &kw) == 2) {
            ctx->plan_override[ph][0] = sl;
            ctx->plan_override[ph][1] = kw;
        }
    }
}

extern "C" int ps_draft_init(ps_draft_ctx** out, const ps_draft_config* config, const ps_draft_weights* weights,
                             void* workspace, size_t workspace_bytes, void* stream) {
    if (!out || !config || !weights) return PS_ERR_NULL;
    int st = check_config(config);
    if (st != PS_OK) return st;
    const ps_draft_weights* w = weights;
    if (!w->g_in || !w->wq || !w->wk || !w->wv || !w->wo || !w->g_post || !w->w_gate || !w->w_up || !w->w_down || !w->w_lm)
        return PS_ERR_NULL;
    if ((config->flags & PS_FLAG_FINAL_NORM) && !w->g_final) return PS_ERR_NULL;
    if (config->k_max > 0 && !w->mask_emb) return PS_ERR_NULL;
    if ((config->flags & PS_FLAG_INPUT_FC) && (!w->w_fc || !w->embed)) return PS_ERR_NULL;
    if (!workspace) return PS_ERR_NULL;
    // rows of the embedding table are addressed with 32-bit byte offsets
    if (w->embed && (unsigned long long)config->vocab * config->hidden * (config->dtype == PS_BF16 ? 2 : 4) > 0xFFFFFFF0ull)
        return PS_ERR_UNSUPPORTED;
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
        // the persistent kernel's workgroups wait for each other: a device that cannot hold one of them per
        // compute unit (as this build assumes) runs the step as one kernel per phase instead
        int per_cu = 0;
        if (ctx->fused && (inst->fused_resident(1, lds_limit < 84 * 1024 ? lds_limit : 84 * 1024, &per_cu) != hipSuccess || per_cu < 1))
            ctx->fused = 0;
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
    ctx->off_y2 = L.off_y2; ctx->off_kvnew = L.off_kvnew; ctx->off_x = L.off_x;
    for (int ph = 0; ph < PH_COUNT; ++ph) { ctx->off_frag[ph] = L.off_frag[ph]; ctx->off_ssqf[ph] = L.off_ssqf[ph]; }
    ctx->spin_limit = PS_SPIN_LIMIT;
    ctx->attn_acc = (float*)(base + L.attn_acc);
    ctx->attn_ml = (float*)(base + L.attn_ml);
    ctx->exch_begin = L.exch_begin; ctx->exch_end = L.exch_end;
    ctx->counters = (int*)(base + L.counters);
    ctx->n_counters = L.n_counters;
    ctx->lm_part = (float*)(base + L.lm_part);
    ctx->logits_ws = (float*)(base + L.logits_ws);
    parse_plan_override(ctx);
    {
        const char* e = getenv("PS_DRAFT_ATTN_SEP");
        ctx->attn_sep_override = (e && (e[0] == '0' || e[0] == '1')) ? e[0] - '0' : -1;
        const char* e2 = getenv("PS_DRAFT_ATTN_NK");
        const int nk_ov = e2 ? atoi(e2) : 0;
        ctx->attn_nk_override = (nk_ov >= 1 && nk_ov <= (1 << PS_ATTN2_NK_LOG_MAX) && (nk_ov & (nk_ov - 1)) == 0) ? nk_ov : 0;
    }
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
    if (e == hipSuccess) e = hipMemsetAsync(ctx->counters, 0, 256, s);
    {   // copy the five weight matrices into streaming order
        StepParams P;
        memset(&P, 0, sizeof(P));
        P.H = config->hidden; P.nq = config->n_heads; P.nkv = config->n_kv_heads; P.d = config->head_dim;
        P.F = config->ffn; P.V = config->vocab; P.QD = config->n_heads * config->head_dim;
        P.wq = w->wq; P.wk = w->wk; P.wv = w->wv; P.wo = w->wo; P.w_gate = w->w_gate; P.w_up = w->w_up;
        P.w_down = w->w_down; P.w_lm = w->w_lm; P.w_fc = w->w_fc;
        int T[PH_COUNT], Kt[PH_COUNT];
        phase_dims(config, T, Kt);
        for (int ph = 0; ph < PH_COUNT && e == hipSuccess; ++ph) {
            if (T[ph] == 0) continue;
            const int ktp = padded_steps(Kt[ph]);
            e = inst->pack(P, ph, T[ph], ktp, Kt[ph], ctx->wpack[ph], s);
            // the streaming loop reads up to PS_U KiB past the last tile: make that zeros, not stale memory
            if (e == hipSuccess) e = hipMemsetAsync(ctx->wpack[ph] + (size_t)T[ph] * ktp * 1024, 0, PS_U_MAX * 1024, s);
        }
    }
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (!hip_ok(e, "rotary table upload")) { delete ctx; return PS_ERR_DEVICE; }
    *out = ctx;
    return PS_OK;
}

extern "C" void ps_draft_free(ps_draft_ctx* ctx) { delete ctx; }

// see ps_draft_debug.h
extern "C" int ps_draft_debug_timeline(ps_draft_ctx* ctx, void* buf) {
    if (!ctx) return PS_ERR_NULL;
    ctx->timeline = (unsigned long long*)buf;
    return PS_OK;
}
extern "C" int ps_draft_debug_spin_limit(ps_draft_ctx* ctx, int spins) {
    if (!ctx) return PS_ERR_NULL;
    ctx->spin_limit = spins > 0 ? spins : PS_SPIN_LIMIT;
    return PS_OK;
}

// Waits for the stream and reports whether a step since the previous query gave up a wait.  After such a
// step the exchange buffers may hold anything: they, the flag and the footprints are put back into
// their initial state (the step counter keeps running, so old tags stay invalid).
extern "C" int ps_draft_last_status(ps_draft_ctx* ctx, void* stream) {
    if (!ctx) return PS_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    int flag = 0;
    if (!hip_ok(hipMemcpyAsync(&flag, ctx->counters + PS_CTR_ERROR, sizeof(int), hipMemcpyDeviceToHost, s), "hipMemcpyAsync")) return PS_ERR_DEVICE;
    if (!hip_ok(hipStreamSynchronize(s), "hipStreamSynchronize")) return PS_ERR_DEVICE;
    if (!flag) return PS_OK;
    hipError_t e = hipMemsetAsync(ctx->act_base, 0xFF, 2 * ctx->act_bytes, s);
    if (e == hipSuccess) e = hipMemsetAsync(ctx->counters + PS_CTR_ERROR, 0, sizeof(int), s);
    if (e == hipSuccess) e = hipMemsetAsync(ctx->counters + PS_CTR_DONE, 0, (PS_CTR_WORDS - PS_CTR_DONE) * sizeof(int), s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (!hip_ok(e, "resetting the exchange buffers")) return PS_ERR_DEVICE;
    return PS_ERR_TIMEOUT;
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
int panel_row_stride_host(int panel_steps) {
    const int len = panel_steps * 64;
    return len + ((64 - (len & 255)) + 256) % 256;
}
static int panel_offset_host(int mt) { return PS_LDS_BASE + 2304 + PS_WAVES * mt * 1024; }   // see PS_LDS_RED in ps_device.h

// Cuts one GEMM phase: T tiles x Kt steps (K elements) over nwg workgroups of PS_WAVES wavefronts.
//
// S K-slices across workgroups (every phase but the LM head).  Every workgroup has to fetch the
// activations of its K range from memory (exchanged data bypasses the L2), so without slices the
// whole grid pulls nwg copies of the full activation matrix, tens of MB per phase, through the
// fabric.  With S slices a workgroup fetches 1/S of it; workgroup wg is slice wg % S, and since
// workgroups are dealt round-robin to the 8 XCDs, S = 8 makes all workgroups of an XCD read the
// same eighth.  The price is one more exchange: the slices' parts of a tile meet in global memory.
//
// kw wavefronts of a workgroup share a tile (kw = 1, 2, 4 or 8; partial sums meet in LDS).  More
// sharing keeps more wavefronts streaming when tiles are few, but a workgroup then takes fewer
// tiles per round and every extra round costs a synchronisation and a reduction: the score is the
// fraction of wavefront slots at work minus a charge per extra round.
static bool make_desc(PhaseDesc* d, int ph, int T, int Kt, int K, int rows, int mt, bool bf, int nwg,
                      const int* override_, int lds_limit) {
    const int ktp = padded_steps(Kt), NG = ktp / PS_U;
    const int arrays = bf ? 2 : 1;
    memset(d, 0, sizeof(*d));
    // Slices pay for the two narrow projections (few tiles, long K: measured), and for any phase but
    // the LM head whose activation panel does not fit in LDS as a whole (many rows): a workgroup
    // that needs only 1/S of the panel stages it in far fewer pieces.
    int s_log = 0;
    const bool whole_fits = (long long)rows * arrays * panel_row_stride_host(ktp) <= lds_limit - panel_offset_host(mt) - 256;
    if (ph == PH_OPROJ || ph == PH_DOWN || ph == PH_FC || (ph != PH_LMHEAD && !whole_fits))
        while (s_log < 3 && (2 << s_log) <= NG && (2 << s_log) <= nwg) ++s_log;
    if (override_[0] > 0 && ph != PH_LMHEAD) {
        s_log = 0;
        while (s_log < 3 && (2 << s_log) <= override_[0] && (2 << s_log) <= NG && (2 << s_log) <= nwg) ++s_log;
    }
    for (; s_log >= 0; --s_log) {
        const int S = 1 << s_log, Gs = nwg >> s_log;
        const int min_slice = NG / S, max_slice = (NG + S - 1) / S;   // groups per slice
        int best_log = 0;
        double best = -1e9;
        for (int lg = 0; lg <= PS_WAVES_LOG; ++lg) {
            const int kw = 1 << lg;
            if (kw > min_slice) break;
            const int per_round = Gs * (PS_WAVES >> lg);
            const int rounds = (T + per_round - 1) / per_round;
            const double util = (double)T * kw * S / ((double)rounds * nwg * PS_WAVES);
            const double score = util - 0.15 * (rounds - 1);
            if (score > best + 1e-9) { best = score; best_log = lg; }
        }
        if (override_[1] > 0) {
            best_log = 0;
            while ((2 << best_log) <= override_[1] && best_log < PS_WAVES_LOG && (2 << best_log) <= min_slice) ++best_log;
        }
        for (; best_log >= 0; --best_log) {
            const int kw = 1 << best_log, SL = PS_WAVES >> best_log;
            const int per_round = Gs * SL;
            const int rounds = (T + per_round - 1) / per_round;
            const int fixed = panel_offset_host(mt) + (ph == PH_LMHEAD ? rounds * SL * rows * 64 : 0);
            const int budget = lds_limit - fixed - 256;
            if (budget <= 0) continue;
            // fewest pieces whose panel fits; every slice must have the same number of pieces, each of
            // at least kw groups (the streaming loop relies on it)
            int np = 1;
            while (np <= max_slice && (long long)rows * arrays * panel_row_stride_host((max_slice + np - 1) / np * PS_U) > budget) ++np;
            if (np > max_slice) continue;
            const int pg = (max_slice + np - 1) / np;
            const int npieces = (max_slice + pg - 1) / pg;
            if ((min_slice + pg - 1) / pg != npieces) continue;
            const int last = min_slice - (npieces - 1) * pg;   // smallest last piece over the slices
            if (pg < kw || last < kw) continue;
            d->T = T; d->Kt = ktp; d->K = K; d->rows = rows; d->kw_log = best_log; d->s_log = s_log; d->Gs = Gs;
            d->nwg = nwg; d->per_round = per_round; d->rounds = rounds; d->piece_groups = pg; d->npieces = npieces;
            d->rs = panel_row_stride_host(pg * PS_U);
            int g2 = 6;
            while ((1 << g2) < pg * PS_U * 4 && (1 << g2) < PS_WG_THREADS) ++g2;
            d->g2_log = g2;
            d->lds_bytes = fixed + rows * arrays * d->rs + 256;
            // The longer the wait for the activations (the more of them the previous phase has to
            // produce), the more weights fit into it: one 8-KiB piece per wavefront for up to ~110 KB of
            // fp32 activations, two beyond, unless there are several column tiles of rows (then the
            // workgroups' reads of the panels already keep the L2s busy).  Measured on c1 .. c4.
            d->pf = (mt == 1 && (long long)rows * K * 4 > 110 * 1024) ? 2 : 1;
            return true;
        }
    }
    return false;
}

// see ps_draft_debug.h
extern "C" int ps_draft_debug_plan(const ps_draft_config* c, int batch, int n_new, int k, int all_rows, int n_cu, int lds_limit,
                                   int* out) {
    if (!c || !out) return PS_ERR_NULL;
    const int st = check_config(c);
    if (st != PS_OK) return st;
    if (batch < 1 || batch > c->max_batch || n_new < 1 || n_new > c->max_new || k < 0 || k > c->k_max) return PS_ERR_SHAPE;
    if (n_cu < 1 || n_cu > 1024 || lds_limit < 64 * 1024 || lds_limit > PS_LDS_BYTES) return PS_ERR_SHAPE;
    const int M = n_new + k, Mtot = batch * M, Rtot = batch * (all_rows ? M : k + 1);
    const int none[2] = {0, 0};
    int T[PH_COUNT], Kt[PH_COUNT], K[PH_COUNT];
    phase_dims(c, T, Kt, K);
    for (int ph = 0; ph <= PH_LMHEAD; ++ph) {
        PhaseDesc d;
        const int rows = ph == PH_LMHEAD ? Rtot : Mtot;
        if (!make_desc(&d, ph, T[ph], Kt[ph], K[ph], rows, (Mtot + 15) / 16, c->dtype == PS_BF16, n_cu, none, lds_limit))
            return PS_ERR_UNSUPPORTED;
        const int v[PS_PLAN_FIELDS] = {d.T, d.Kt, d.K, d.rows, d.kw_log, d.s_log, d.Gs, d.per_round, d.rounds,
                                       d.piece_groups, d.npieces, d.lds_bytes};
        for (int i = 0; i < PS_PLAN_FIELDS; ++i) out[ph * PS_PLAN_FIELDS + i] = v[i];
    }
    return PS_OK;
}

// The bf16 attention's work (attn_phase2 in ps_device.h).  Work units = (sequence, kv head, block of 128 NK cache
// keys, pass of 16 query rows); the rows of this step ride on a sequence's last block.  NK (a power of two) is chosen
// by a small cost model in microseconds, measured on the benchmark's workloads: a unit costs about 2 + 1 per group of
// 16 keys a wavefront takes in turn (two at a time), the workgroups take ceil(units / compute units) rounds of them,
// and a sequence of several blocks costs one more exchange through memory (the merge items).
struct Attn2Plan { int ch_log, npass, items, merge_items; };
static Attn2Plan plan_attn2(const int32_t* kv_len, int batch, int n_kv_heads, int ra, int M, int n_cu, int nk_override) {
    const int npass = (ra + 15) / 16, rt = (ra + PS_WAVES - 1) / PS_WAVES;
    int best_log = 0;
    double best = 1e30;
    for (int lg = 0; lg <= PS_ATTN2_NK_LOG_MAX; ++lg) {
        if (nk_override > 0 && (1 << lg) != nk_override) continue;
        const int chl = PS_ATTN_KEYS_LOG + lg;
        long long units = 0;
        int groups = 1;
        bool merge = false;
        for (int b = 0; b < batch; ++b) {
            const int L = kv_len[b];
            int nch = (int)(((long long)L + (1 << chl) - 1) >> chl);
            if (nch < 1) nch = 1;
            units += (long long)n_kv_heads * nch * npass;
            merge = merge || nch > 1;
            const int g = ((L < (1 << chl) ? L : (1 << chl)) + 15) / 16 + (M + 15) / 16;
            if (g > groups) groups = g;
        }
        const long long rounds = (units + n_cu - 1) / n_cu;
        const double cost = (double)rounds * (2.0 + 1.0 * ((groups + PS_WAVES - 1) / PS_WAVES)) + (merge ? 5.0 : 0.0);
        if (cost < best - 1e-9) { best = cost; best_log = lg; }
    }
    Attn2Plan ap;
    ap.ch_log = PS_ATTN_KEYS_LOG + best_log; ap.npass = npass; ap.items = 0; ap.merge_items = 0;
    for (int b = 0; b < batch; ++b) {
        int nch = (int)(((long long)kv_len[b] + (1 << ap.ch_log) - 1) >> ap.ch_log);
        if (nch < 1) nch = 1;
        ap.items += n_kv_heads * nch;
        if (nch > 1) ap.merge_items += n_kv_heads * rt;
    }
    return ap;
}

// see ps_draft_debug.h
extern "C" int ps_draft_debug_attn_plan(const ps_draft_config* c, int batch, const int32_t* kv_len, int n_new, int k, int n_cu,
                                        int* out) {
    if (!c || !kv_len || !out) return PS_ERR_NULL;
    const int st = check_config(c);
    if (st != PS_OK) return st;
    if (batch < 1 || batch > c->max_batch || n_new < 1 || n_new > c->max_new || k < 0 || k > c->k_max) return PS_ERR_SHAPE;
    if (n_cu < 1 || n_cu > 1024) return PS_ERR_SHAPE;
    if (c->dtype != PS_BF16) return PS_ERR_UNSUPPORTED;
    for (int b = 0; b < batch; ++b)
        if (kv_len[b] < 0 || (long long)kv_len[b] + n_new + k > c->max_positions) return PS_ERR_KV_CAPACITY;
    const int M = n_new + k;
    const Attn2Plan ap = plan_attn2(kv_len, batch, c->n_kv_heads, (c->n_heads / c->n_kv_heads) * M, M, n_cu, 0);
    out[0] = 1 << (ap.ch_log - PS_ATTN_KEYS_LOG); out[1] = ap.items * ap.npass; out[2] = ap.items; out[3] = ap.merge_items;
    return PS_OK;
}

extern "C" int ps_draft_step(ps_draft_ctx* ctx, const ps_draft_step_args* a, void* stream) {
    if (!ctx || !a) return PS_ERR_NULL;
    const ps_draft_config& c = ctx->cfg;
    if (a->batch < 1 || a->batch > c.max_batch || a->n_new < 1 || a->n_new > c.max_new || a->k < 0 || a->k > c.k_max)
        return PS_ERR_SHAPE;
    if (a->topk < 1 || a->topk > c.max_topk || a->topk > c.vocab) return PS_ERR_SHAPE;
    if (a->out_rows != 0 && a->out_rows != 1) return PS_ERR_SHAPE;
    if (!a->k_cache || !a->v_cache || !a->kv_offsets || !a->kv_len || !a->top_ids || !a->top_p || !a->lse)
        return PS_ERR_NULL;
    // where the real rows come from: hidden states x, or token ids (with the embedding table given at init),
    // or token ids and features (with the input projection given at init)
    int in_mode = PS_IN_HIDDEN;
    if (a->token_ids) {
        if (a->x) return PS_ERR_SHAPE;                       // one or the other
        if (!ctx->w.embed) return PS_ERR_NULL;
        in_mode = PS_IN_TOKENS;
        if (a->features) {
            if (!(c.flags & PS_FLAG_INPUT_FC)) return PS_ERR_SHAPE;
            in_mode = PS_IN_FUSED;
        }
    } else {
        if (!a->x) return PS_ERR_NULL;
        if (a->features) return PS_ERR_SHAPE;                // features go with token ids
    }
    if (!(a->temperature >= 0.f) || a->temperature > 1e30f) return PS_ERR_SHAPE;   // 0 stands for 1
    if (a->sample_p && !a->sample_ids) return PS_ERR_NULL;
    const int M = a->n_new + a->k;
    for (int b = 0; b < a->batch; ++b) {
        if (a->kv_offsets[b] < 0 || a->kv_offsets[b + 1] < a->kv_offsets[b]) return PS_ERR_OFFSETS;
    }
    for (int b = 0; b < a->batch; ++b) {
        if (a->kv_len[b] < 0) return PS_ERR_SHAPE;
        // rows of sequence b: its accepted tokens (n_new, or fewer with n_new_seq) and the k [MASK] slots
        if (a->n_new_seq && (a->n_new_seq[b] < 1 || a->n_new_seq[b] > a->n_new)) return PS_ERR_SHAPE;
        const int Mb = (a->n_new_seq ? a->n_new_seq[b] : a->n_new) + a->k;
        if ((long long)a->kv_len[b] + Mb > a->kv_offsets[b + 1] - a->kv_offsets[b]) return PS_ERR_KV_CAPACITY;
        if ((long long)a->kv_len[b] + Mb > c.max_positions) return PS_ERR_KV_CAPACITY;
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
    P.inv_temp = a->temperature > 0.f ? 1.0f / a->temperature : 1.0f;
    P.seed_lo = (unsigned)(a->sample_seed & 0xFFFFFFFFull); P.seed_hi = (unsigned)(a->sample_seed >> 32);
    P.sample_ids = a->sample_ids; P.sample_p = a->sample_p; P.kv_len_dev = a->kv_len_dev;
    P.in_mode = in_mode; P.token_ids = a->token_ids; P.features = a->features;
    P.embed = ctx->w.embed; P.w_fc = ctx->w.w_fc; P.b_fc = ctx->w.b_fc;
    P.n_magic = 0xFFFFFFFFu / (unsigned)a->n_new + 1u;
    P.rope = ctx->rope; P.attn_acc = ctx->attn_acc; P.attn_ml = ctx->attn_ml;
    P.lm_part = ctx->lm_part;
    P.m_magic = 0xFFFFFFFFu / (unsigned)M + 1u;   // ceil(2^32 / M); M = 1 is handled on the device
    P.tph_log = c.head_dim == 128 ? 3 : 2;
    P.error_flag = ctx->counters + PS_CTR_ERROR;
    // The step's sequence number is kept on the device (ctx->counters[1], advanced by the kernels), so a
    // captured launch can be replayed.  The exchange buffers exist twice, step n uses copy n & 1; the
    // pointers here are those of copy 0.
    P.step_ctr = (unsigned*)ctx->counters + PS_CTR_STEP;
    P.done_ctr = (unsigned*)ctx->counters + PS_CTR_DONE;
    char* const act0 = ctx->act_base;
    P.act_bytes = (long long)ctx->act_bytes;
    P.q_buf = (float*)(act0 + ctx->off_q); P.o_buf = (float*)(act0 + ctx->off_o); P.y_buf = (float*)(act0 + ctx->off_y);
    P.u_buf = (float*)(act0 + ctx->off_u); P.y2_buf = (float*)(act0 + ctx->off_y2); P.kvnew = (float*)(act0 + ctx->off_kvnew);
    P.x_buf = (c.flags & PS_FLAG_INPUT_FC) ? (float*)(act0 + ctx->off_x) : nullptr;
    P.spin_limit = ctx->spin_limit;
    P.foot_mem = (unsigned*)ctx->counters + PS_CTR_FOOT;
    P.logits_store = a->logits ? a->logits : (a->probs ? ctx->logits_ws : nullptr);
    P.top_ids = a->top_ids; P.top_p = a->top_p; P.lse = a->lse; P.probs = a->probs; P.hidden_out = a->hidden_out;
    for (int b = 0; b < a->batch; ++b) {
        P.kv_off[b] = a->kv_offsets[b];
        P.kv_len[b] = a->kv_len[b];
        P.skip[b] = a->n_new_seq ? a->n_new - a->n_new_seq[b] : 0;
    }
    // attention work items: (sequence, kv head, block of ch keys)
    const int ra = (c.n_heads / c.n_kv_heads) * M;
    int ch = PS_ATTN_KEYS;
    // The M rows of this step normally belong to the last key block of their sequence.  When they alone
    // make up that block (or spill into one more) and leaving them out spares the workgroups a whole
    // round of work items, the merge items take them instead (at most 16 rows: they are kept in registers).
    int items = 0, items_wo = 0;
    for (int b = 0; b < a->batch; ++b) {
        items += c.n_kv_heads * ((a->kv_len[b] + M + ch - 1) / ch);
        items_wo += c.n_kv_heads * ((a->kv_len[b] + ch - 1) / ch);
    }
    bool sep = M <= 16 && (items_wo + ctx->n_cu - 1) / ctx->n_cu < (items + ctx->n_cu - 1) / ctx->n_cu;
    if (ctx->attn_sep_override >= 0 && M <= 16) sep = ctx->attn_sep_override != 0;
    if (sep) items = items_wo;
    const int tail = sep ? 0 : M;
    // Key blocks of twice the size (two groups of 16 keys per wavefront) when the workgroups still face
    // more than one round of work items and that way every one of them gets at most a single item
    int nk = 1;
    if (items > ctx->n_cu && ra <= 16 && ps_attn_lds_bytes(c.head_dim, 2) <= ctx->lds_limit) {
        int items2 = 0;
        for (int b = 0; b < a->batch; ++b) items2 += c.n_kv_heads * ((a->kv_len[b] + tail + 2 * ch - 1) / (2 * ch));
        if (items2 <= ctx->n_cu) { nk = 2; ch *= 2; items = items2; }
    }
    P.attn_items = items; P.attn_single = ra <= 16; P.attn_sep = sep ? 1 : 0; P.attn_tail = tail; P.attn_nk = nk;
    const bool attn2 = c.dtype == PS_BF16;   // bf16 storage: attn_phase2 (ps_device.h)
    {   // sequences that span several key blocks are put together by (sequence, kv head, 8 rows) work items
        const int rt = (ra + PS_WAVES - 1) / PS_WAVES;
        int mi = 0;
        for (int b = 0; b < a->batch; ++b)
            if (sep || (a->kv_len[b] + tail + ch - 1) / ch > 1) mi += c.n_kv_heads * rt;
        P.attn_merge_items = mi;
        const int want = items > mi ? items : mi;
        P.attn_nwg = want < ctx->n_cu ? want : ctx->n_cu;
    }
    if (attn2) {
        const Attn2Plan ap = plan_attn2(a->kv_len, a->batch, c.n_kv_heads, ra, M, ctx->n_cu, ctx->attn_nk_override);
        P.attn_ch_log = ap.ch_log; P.attn_npass = ap.npass; P.pass_magic = 0xFFFFFFFFu / (unsigned)ap.npass + 1u;
        P.attn_items = ap.items; P.attn_units = ap.items * ap.npass; P.attn_merge_items = ap.merge_items;
        P.attn_sep = 0; P.attn_tail = 0; P.attn_nk = 1;
        const int want = P.attn_units > ap.merge_items ? P.attn_units : ap.merge_items;
        P.attn_nwg = want < ctx->n_cu ? want : ctx->n_cu;
    }

    const bool bf = c.dtype == PS_BF16;
    const int nwg = ctx->n_cu;
    P.r_magic = 0xFFFFFFFFu / (unsigned)P.R + 1u;
    int T[PH_COUNT], Kt[PH_COUNT], K[PH_COUNT];
    phase_dims(&c, T, Kt, K);
    for (int ph = 0; ph < PH_COUNT; ++ph) {
        if (T[ph] == 0) continue;                            // (no input projection in this configuration)
        const int rows = ph == PH_LMHEAD ? P.Rtot : ph == PH_FC ? a->batch * a->n_new : P.Mtot;
        // the persistent kernel runs every phase with the column tiles of the widest one
        const int mt = ((ctx->fused && ph != PH_FC) ? P.Mtot + 15 : rows + 15) / 16;
        if (!make_desc(&P.ph[ph], ph, T[ph], Kt[ph], K[ph], rows, mt, bf, nwg, ctx->plan_override[ph], ctx->lds_limit))
            return PS_ERR_UNSUPPORTED;
        P.ph[ph].wpack = ctx->wpack[ph];
        P.ph[ph].frag = (float*)(ctx->act_base + ctx->off_frag[ph]);
        P.ph[ph].ssq_frag = (float*)(ctx->act_base + ctx->off_ssqf[ph]);
    }
    P.ph[PH_QKV].norm = 1; P.ph[PH_QKV].gain = P.g_in; P.ph[PH_QKV].src = nullptr; P.ph[PH_QKV].src_ld = P.H;
    P.ph[PH_OPROJ].src = P.o_buf; P.ph[PH_OPROJ].src_ld = P.QD;
    P.ph[PH_GATEUP].norm = 1; P.ph[PH_GATEUP].gain = P.g_post; P.ph[PH_GATEUP].src = P.y_buf; P.ph[PH_GATEUP].src_ld = P.H;
    P.ph[PH_DOWN].src = P.u_buf; P.ph[PH_DOWN].src_ld = P.F;
    P.ph[PH_LMHEAD].norm = P.final_norm; P.ph[PH_LMHEAD].gain = P.g_final; P.ph[PH_LMHEAD].src = P.y2_buf; P.ph[PH_LMHEAD].src_ld = P.H;
    P.timeline = ctx->timeline;
    // what this step leaves in the sentinel-coded buffers of its copy (see sx_reset_stale in ps_device.h)
    P.foot[0] = (unsigned)P.Mtot;
    for (int ph = 0; ph < PH_COUNT; ++ph) {
        const PhaseDesc& d = P.ph[ph];
        const bool sliced = ph != PH_LMHEAD && d.s_log > 0 && d.T > 0 && (ph != PH_FC || in_mode == PS_IN_FUSED);
        const int mt = ((ph == PH_FC ? d.rows : P.Mtot) + 15) / 16;
        P.foot[1 + ph] = sliced ? (unsigned)(1 << d.s_log) * (unsigned)d.T * (unsigned)mt * 64u : 0u;
        P.foot[1 + PH_COUNT + ph] = (sliced && d.norm) ? 1u << d.s_log : 0u;
    }

    // the persistent kernel needs the largest LDS footprint of its phases and one workgroup per CU
    int lds = attn2 ? ps_attn2_lds_bytes(c.head_dim) : ps_attn_lds_bytes(c.head_dim, nk);
    for (int ph = 0; ph < PH_COUNT; ++ph) {
        if (P.ph[ph].lds_bytes > lds) lds = P.ph[ph].lds_bytes;
    }
    if (lds < PS_LDS_BASE + 8192 + 128) lds = PS_LDS_BASE + 8192 + 128;   // end-of-step merge scratch
    if (lds < 84 * 1024 && ctx->lds_limit >= 84 * 1024) lds = 84 * 1024;   // more than half a CU's LDS: one workgroup per CU
#ifdef PS_TIMELINE
    lds = ctx->lds_limit;   // the stamps live in the top 512 bytes of LDS
#endif
    P.fused_nwg = nwg; P.fused_lds = lds;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t* ev = ctx->profile ? ctx->events : nullptr;
    if (in_mode == PS_IN_FUSED && !hip_ok(ctx->inst->launch_fc(P, st), "kernel launch")) return PS_ERR_DEVICE;
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
