/*
 * ps_train.h - C ABI of the attention of group-wise parallel training (same library, libps_draft.so, same
 * conventions as ps_draft.h: extern "C", plain pointers and sizes, int ps_status results, nothing is enqueued
 * on an argument error, no allocation, asynchronous on the given hipStream_t).
 *
 * Section 4.1, "Group-wise Parallel Training": a training sequence of T real tokens is laid out as T parallel
 * groups, each an input token followed by k [MASK] tokens,
 *     x_0 m_1 .. m_k | x_1 m_1 .. m_k | ... | x_{T-1} m_1 .. m_k            rows = T (k + 1),
 * and attention over this layout uses a customised causal mask under which every token ignores the [MASK]
 * tokens of previous groups (caption of Figure 3), with position indices adjusted so that training and
 * inference see the same thing (caption of Figure 2): row (group g, slot s) attends to the real tokens of
 * groups 0..g and to the [MASK] tokens 1..s of its own group, and stands at position g + s - what the same
 * token sees and where it stands in ps_draft_step when x_0..x_g are the prefix.
 */
#ifndef PS_TRAIN_H
#define PS_TRAIN_H
#include <stddef.h>
#include <stdint.h>
#include "ps_draft.h"
#ifdef __cplusplus
extern "C" {
#endif

/*
 * One forward pass of that attention for `seqs` independent sequences of the same length.
 *   q          DEVICE [seqs, rows, n_heads, head_dim], dtype, BEFORE the rotary embedding
 *   k, v       DEVICE [seqs, rows, n_kv_heads, head_dim], dtype (k before the rotary embedding)
 *   out        DEVICE [seqs, rows, n_heads, head_dim] float32, written: softmax(q k^T / sqrt(head_dim)) v per head
 *              under the mask above; query head h uses kv head h / (n_heads / n_kv_heads)
 *   workspace  DEVICE, at least ps_group_attention_workspace_bytes(args) bytes, 256-byte aligned, owned by the
 *              caller: the rotary table and the rotated k (dtype: keys are rounded to the storage type after
 *              the rotary embedding, as the inference path caches them; queries are rotated in float32 on chip)
 * The rotary embedding (pairs (j, j + head_dim / 2), angle position * rope_base^(-2j / head_dim), computed in
 * double precision) is applied inside.  Supported: head_dim 64 or 128; k + 1 <= 16; n_heads a multiple of
 * n_kv_heads; dtype PS_F32 or PS_BF16; tokens + k <= 2^20; (k + 1) * n_kv_heads * head_dim <= 2^25.  Errors: PS_ERR_NULL, PS_ERR_SHAPE (a size < 1,
 * k < 0), PS_ERR_UNSUPPORTED, PS_ERR_WORKSPACE, PS_ERR_DEVICE.
 */
typedef struct ps_group_attn_args {
    int32_t seqs;       /* >= 1 */
    int32_t tokens;     /* T >= 1 real tokens per sequence */
    int32_t k;          /* [MASK] tokens per parallel group, 0 <= k <= 15 (0: ordinary causal attention) */
    int32_t n_heads, n_kv_heads, head_dim;
    int32_t dtype;      /* ps_dtype of q, k, v */
    float rope_base;
    const void* q;
    const void* k_;
    const void* v;
    float* out;
    void* workspace;
    size_t workspace_bytes;
} ps_group_attn_args;

/* Bytes of workspace ps_group_attention needs (0 if the arguments are invalid or unsupported).  Host only. */
PS_API size_t ps_group_attention_workspace_bytes(const ps_group_attn_args* args);

PS_API int ps_group_attention(const ps_group_attn_args* args, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PS_TRAIN_H */
