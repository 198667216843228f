/*
 * ps_draft.h - C ABI of the ParallelSpec parallel draft step on AMD MI355X (gfx950).
 *
 * One call of ps_draft_step runs the drafter of Section 4.1 ("Parallel Drafting",
 * paragraph "Inference") once: the k special tokens [MASK]_1..[MASK]_k are appended after
 * the sequence, ONE forward pass of the drafter produces the representation of the last
 * real token (which decodes x_t) and of the k mask tokens (which decode x_{t+1..t+k}), and
 * the LM head turns those k+1 representations into k+1 token distributions
 * q(x | x_<n), q(x | x_<n, [MASK]_1), ..., q(x | x_<n, [MASK]_1..k)  (Algorithm 1, draft line).
 * The drafter is a single Llama-style Transformer layer shaped like a layer of the target
 * model (Section 5.1 "Models"); its LM head is the target's, shared and frozen
 * (Section 4.3, Medusa integration).  The prefix x_<n is represented by the drafter's KV
 * cache plus the hidden states of the n_new positions accepted since the previous step.
 * [MASK] rows of earlier steps are never visible (Section 4.1, "Group-wise Parallel
 * Training": the model must behave the same in training and evaluation): a step writes
 * n_new + k new K/V rows after the valid cache rows, and the caller commits only the
 * first n_new of them by advancing kv_len by n_new, so the next step overwrites the rest.
 *
 * All pointers named "device" are HIP device pointers of the current device, owned by
 * the caller; nothing is copied or retained beyond what is stated.  No function throws
 * or aborts; every function returns a ps_status (0 = success, negative = error).  On an
 * argument error nothing has been enqueued on the stream.
 */
#ifndef PS_DRAFT_H
#define PS_DRAFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The library is built with hidden visibility: exactly the functions declared PS_API are exported. */
#define PS_API __attribute__((visibility("default")))

typedef struct ps_draft_ctx ps_draft_ctx;

enum ps_dtype { PS_F32 = 0, PS_BF16 = 1 };

enum ps_status {
    PS_OK = 0,
    PS_ERR_NULL = -1,        /* a required pointer is NULL */
    PS_ERR_CONFIG = -2,      /* a configuration field is out of range or inconsistent */
    PS_ERR_SHAPE = -3,       /* a step argument (batch, n_new, k, topk) is outside the configured bounds */
    PS_ERR_KV_CAPACITY = -4, /* kv_len + n_new + k exceeds the sequence's cache rows or max_positions */
    PS_ERR_OFFSETS = -5,     /* kv_offsets is negative or not non-decreasing */
    PS_ERR_WORKSPACE = -6,   /* workspace too small or misaligned (256 bytes) */
    PS_ERR_UNSUPPORTED = -7, /* a legal shape this build has no kernel for (see ps_draft_config) */
    PS_ERR_DEVICE = -8,      /* a HIP call failed (no device, launch failure) */
    PS_ERR_TIMEOUT = -9      /* ps_draft_last_status: a step gave up waiting for some of its own workgroups */
};

#define PS_FLAG_FINAL_NORM 1u /* apply the RMSNorm with gain g_final before the LM head */
#define PS_FLAG_INPUT_FC 2u   /* the drafter has the input projection w_fc (feature-fusion input mode, see ps_draft_step_args) */

/*
 * Shape of the drafter layer and bounds of the step.  Supported by this build:
 *   head_dim 64 or 128; n_heads a multiple of n_kv_heads;
 *   hidden, n_heads*head_dim and ffn multiples of 32 (PS_BF16) or 16 (PS_F32); ffn a multiple of 8;
 *   hidden a multiple of 16; vocab >= 1 (any value);
 *   max_batch * (max_new + k_max) <= 64 rows per step;
 *   (n_heads / n_kv_heads) * (max_new + k_max) <= 64; 1 <= max_topk <= 32;
 *   max_positions <= 2^24, and no exchange buffer of the workspace (activations and K-slice
 *   partial sums of one step; attention partials: max_batch * n_kv_heads * max_positions / 128
 *   blocks x (n_heads / n_kv_heads) * (max_new + k_max) rows x head_dim x 8 bytes) of 4 GiB or more.
 * Anything else legal returns PS_ERR_UNSUPPORTED, anything illegal PS_ERR_CONFIG.
 */
typedef struct ps_draft_config {
    int32_t hidden;        /* H: model width */
    int32_t n_heads;       /* query heads */
    int32_t n_kv_heads;    /* key/value heads (grouped-query attention when < n_heads) */
    int32_t head_dim;      /* d */
    int32_t ffn;           /* F: SwiGLU inner width */
    int32_t vocab;         /* V: rows of the LM head */
    int32_t k_max;         /* rows of mask_emb = largest k a step may use (>= 0) */
    int32_t max_batch;     /* largest batch a step may use (>= 1) */
    int32_t max_new;       /* largest n_new a step may use (>= 1) */
    int32_t max_positions; /* largest kv_len + n_new + k of any sequence (rotary table rows) */
    int32_t max_topk;      /* largest topk a step may use */
    int32_t dtype;         /* ps_dtype of weights, mask_emb, x and the KV cache */
    float rms_eps;         /* epsilon inside every RMSNorm */
    float rope_base;       /* rotary base; pair (j, j + d/2) turns by position * base^(-2j/d) */
    uint32_t flags;        /* PS_FLAG_* */
} ps_draft_config;

/*
 * Drafter weights: device pointers, row-major [out_features, in_features], element type
 * config.dtype, no biases (Section 5.1: 4H^2 + 3HF parameters give the printed 202M / 317M).
 * Borrowed for the lifetime of the context; never written.
 */
typedef struct ps_draft_weights {
    const void* g_in;     /* [H]                 gain of the RMSNorm before attention */
    const void* wq;       /* [n_heads*d, H] */
    const void* wk;       /* [n_kv_heads*d, H] */
    const void* wv;       /* [n_kv_heads*d, H] */
    const void* wo;       /* [H, n_heads*d] */
    const void* g_post;   /* [H]                 gain of the RMSNorm before the MLP */
    const void* w_gate;   /* [F, H] */
    const void* w_up;     /* [F, H] */
    const void* w_down;   /* [H, F] */
    const void* g_final;  /* [H]                 gain of the final RMSNorm (may be NULL without PS_FLAG_FINAL_NORM) */
    const void* w_lm;     /* [V, H]              LM head shared with the target model */
    const void* mask_emb; /* [k_max, H]          embeddings of [MASK]_1..[MASK]_k_max (may be NULL if k_max == 0) */
    /* Input stage (Section 4.3).  The drafter shares the target's embedding layer, frozen, to which the k [MASK]
     * tokens were added (mask_emb above are those added rows).  In the feature-level variant (EAGLE integration)
     * a fully connected layer maps [f ; e] - the target's last-layer hidden state f of a position and the
     * embedding e of its token - to the drafter's input. */
    const void* embed;    /* [V, H]              shared embedding table (NULL: steps must pass hidden states x) */
    const void* w_fc;     /* [H, 2H]             input projection: columns 0..H-1 multiply f, H..2H-1 multiply e
                                                 (required with PS_FLAG_INPUT_FC, else ignored) */
    const void* b_fc;     /* [H]                 its bias, or NULL for none */
} ps_draft_weights;

/*
 * Bytes of device scratch ps_draft_init needs for this configuration: a copy of the five
 * weight matrices in the kernels' streaming order (as large as the matrices themselves),
 * activations, split-K partial sums, attention partials, completion counters, rotary table.
 * Returns 0 if the configuration is invalid or unsupported.  Host-only; touches no device.
 */
PS_API size_t ps_draft_workspace_bytes(const ps_draft_config* config);

/*
 * Creates a context.  config and weights are copied (the structs, not the tensors).
 * workspace: device memory of at least ps_draft_workspace_bytes(config) bytes, 256-byte
 * aligned, owned by the caller, used exclusively by this context until ps_draft_free.
 * stream: hipStream_t (may be NULL = default stream); the repacking of the weight matrices,
 * the rotary table upload and the clearing of the counters are enqueued on it and the call
 * waits for them.  The matrices are read only during this call; the gain vectors and
 * mask_emb are read by every step.
 * Validation happens before any HIP call, so configuration errors are reported on a
 * machine without a GPU as well.  *out is set only on success.
 */
PS_API int ps_draft_init(ps_draft_ctx** out, const ps_draft_config* config, const ps_draft_weights* weights,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * Arguments of one draft step.  Sequences are independent; all use the same n_new and k.
 * Per sequence the step processes M = n_new + k rows: the n_new real rows x[b, 0..n_new-1]
 * followed by mask_emb[0..k-1], at positions kv_len[b] .. kv_len[b] + M - 1.
 * Output rows per sequence ("rows" below): out_rows == 0 -> the k+1 decoding rows
 * (last real row, then the k mask rows); out_rows == 1 -> all M rows (testing).
 */
typedef struct ps_draft_step_args {
    int32_t batch;  /* 1..max_batch */
    int32_t n_new;  /* 1..max_new: real positions accepted since the previous step (Section 3: 1..gamma+1) */
    int32_t k;      /* 0..k_max: [MASK] slots appended (k = 0 is an ordinary decode step) */
    int32_t topk;   /* 1..min(max_topk, vocab): candidates per output row (token tree fan-out, Appendix A.3) */
    int32_t out_rows;
    const void* x;  /* device [batch, n_new, H], config.dtype: hidden states of the new real positions
                       (NULL when token_ids is given) */
    void* k_cache;  /* device [total_positions, n_kv_heads, d], config.dtype; keys stored after rotary embedding */
    void* v_cache;  /* device, same layout.  Rows off[b]+kv_len[b] .. +M-1 of both are overwritten. */
    const int64_t* kv_offsets; /* HOST [batch+1], in positions: sequence b owns cache rows [off[b], off[b+1]) */
    const int32_t* kv_len;     /* HOST [batch]: valid positions of sequence b before this step (>= 0) */
    int32_t* top_ids;  /* device [batch, rows, topk]: token ids by descending logit, equal logits by ascending id */
    float* top_p;      /* device [batch, rows, topk]: softmax probability of each top id */
    float* lse;        /* device [batch, rows]: log-sum-exp of the row's logits */
    float* logits;     /* device [batch, rows, V] or NULL */
    float* probs;      /* device [batch, rows, V] or NULL: softmax(logits) */
    float* hidden_out; /* device [batch, M, H] or NULL: layer output before the final norm */
    /* Input stage fused into the step (Section 4.3), instead of x:
     *   token_ids alone     the real rows are rows token_ids[b][i] of weights.embed (Medusa integration: the
     *                       drafter reads token embeddings; [MASK] rows are the added embedding rows mask_emb);
     *   token_ids, features the real rows are w_fc . [features[b][i] ; embed[token_ids[b][i]]] (+ b_fc), computed in
     *                       float32 and never rounded to config.dtype (EAGLE integration; needs PS_FLAG_INPUT_FC).
     *                       The caller pairs feature and token as its drafter was trained; [MASK] rows are mask_emb
     *                       as they are (a learned [MASK] input needs no projection). */
    const int32_t* token_ids; /* device [batch, n_new] in [0, V), or NULL */
    const void* features;     /* device [batch, n_new, H], config.dtype, or NULL */
    /* Sampling epilogue (Algorithm 1 draws the draft tokens from the draft distributions; the T = 1 rows of
     * Table 1).  The softmax of every output row is taken over logits / temperature: lse, top_p, probs and the
     * draw below are those of the tempered distribution; `logits` stays the untempered LM-head output.
     * With sample_ids, one token per output row is drawn from that distribution inside the step's kernel by the
     * Gumbel-max construction: argmax_i (logit_i / T + g_i), g_i = -log(-log(u_i)), where u_i for output row m
     * (0 <= m < batch * rows) and token i is ((h >> 9) + 0.5) 2^-23 with h = three rounds of MurmurHash3's 32-bit
     * finaliser fmix32: h = fmix32(fmix32(fmix32(seed_lo + 0x9E3779B9 (m + 1)) ^ seed_hi) ^ (i * 0x9E3779B1 +
     * 0x7F4A7C15)) modulo 2^32; equal values go to the lower id.  The same seed gives the same draws: pass a new
     * one every step. */
    float temperature;        /* > 0; 0 stands for 1 */
    uint64_t sample_seed;
    int32_t* sample_ids;      /* device [batch, rows] or NULL: the drawn token per output row */
    float* sample_p;          /* device [batch, rows] or NULL: its probability under the tempered distribution */
    /* The sequences' lengths in DEVICE memory ([batch] int32, or NULL): when given, the kernel takes every
     * length from there and kv_len (host) only states upper bounds, kv_len_dev[b] <= kv_len[b], which the
     * capacity checks and the launch plan use.  A step captured in a HIP graph can then be replayed while the
     * caller advances the lengths on the device (by n_new per step, up to the bound it was captured with). */
    const int32_t* kv_len_dev;
    /* Sequences of one batch that accepted different numbers of tokens (Section 3: a verification round yields
     * 1..gamma+1 tokens per sequence).  HOST [batch] or NULL: sequence b has n_new_seq[b] real rows, 1 <=
     * n_new_seq[b] <= n_new; they are the LAST n_new_seq[b] of its n_new slots in x / token_ids / features (the
     * slots in front of them are not read); its rows get positions kv_len[b] .. kv_len[b] + n_new_seq[b] + k - 1
     * and only those cache rows are written.  Output rows are laid out as for n_new (out_rows == 1: the rows of the
     * unused slots, and their rows of hidden_out, are unspecified).  NULL: every sequence has n_new real rows. */
    const int32_t* n_new_seq;
} ps_draft_step_args;

/*
 * Enqueues one draft step on stream (hipStream_t, NULL = default stream) and returns
 * without waiting.  Performs no allocation, no host synchronisation and reads no device
 * memory from the host; kv_offsets and kv_len are read before the call returns.
 * top_ids, top_p and lse are required; logits, probs and hidden_out are optional.
 * Exactly one of x and token_ids must be given (else PS_ERR_NULL / PS_ERR_SHAPE); token ids are not
 * range-checked (they are device data): an id outside [0, V) reads outside the embedding table.
 * Steps of one context must not overlap in time (they share the workspace).
 * All arguments are checked and the launch is planned before anything is enqueued or any
 * state of the context changes: a call that returns PS_ERR_NULL, PS_ERR_SHAPE, PS_ERR_OFFSETS,
 * PS_ERR_KV_CAPACITY (kv_len[b] + the sequence's rows exceed off[b+1] - off[b] or max_positions) or
 * PS_ERR_UNSUPPORTED has done nothing; PS_ERR_DEVICE means a launch itself failed.
 *
 * The step runs as ONE kernel with one workgroup per compute unit whose workgroups hand data to
 * each other, so all of them must be running at once: no other work may occupy the GPU while a
 * step runs (work queued before or after it on any stream is fine: the step starts when the
 * compute units are free).  If the GPU withholds compute units all the same, the waiting
 * workgroups give up after about a second, the kernel ends normally, the step's outputs are
 * marked (every top_ids entry -1, top_p 0, lse NaN) and ps_draft_last_status says so.
 */
PS_API int ps_draft_step(ps_draft_ctx* ctx, const ps_draft_step_args* args, void* stream);

/*
 * Waits for everything enqueued on stream (the stream the steps ran on) and returns PS_OK, or
 * PS_ERR_TIMEOUT if a step since the previous query (or since ps_draft_init) gave up a wait:
 * the outputs of that step and of every later one are marked as described at ps_draft_step,
 * and this call has put the context's exchange buffers back into their initial state, so the
 * following steps are good again.  No part of the method; callers that never share the GPU
 * need not call it.  Errors: PS_ERR_NULL, PS_ERR_DEVICE.
 */
PS_API int ps_draft_last_status(ps_draft_ctx* ctx, void* stream);

/*
 * Measurement aid (no part of the method): when events is non-NULL, every following
 * ps_draft_step records events[0] before its first kernel and events[i] after kernel i
 * (i = 1..7: QKV projection, attention, output projection, gate/up projection, down
 * projection, LM head, LM-head merge incl. optional probabilities) on the step's stream, so
 * the caller can time each kernel with hipEventElapsedTime.  events: HOST array of
 * PS_PROFILE_EVENTS hipEvent_t handles created by the caller with timing enabled; the
 * array is copied.  NULL switches recording off again.  Returns PS_ERR_NULL for a NULL ctx.
 */
#define PS_PROFILE_EVENTS 8
PS_API int ps_draft_set_profile_events(ps_draft_ctx* ctx, void* const* events);

/* Releases the host-side context; ps_draft_free(NULL) is a no-op.  The workspace stays the caller's. */
PS_API void ps_draft_free(ps_draft_ctx* ctx);

/* Static, NUL-terminated description of a ps_status value. */
PS_API const char* ps_draft_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* PS_DRAFT_H */
