/*
 * ps_verify.h - C ABI of the steps that follow the parallel draft step in Algorithm 1:
 * building the draft token tree from the drafter's top-k output, and the acceptance walk
 * over that tree against the target model's distributions.  Same library as ps_draft.h
 * (libps_draft.so), same conventions: extern "C", plain pointers and sizes, int status
 * (ps_status of ps_draft.h: 0 = OK, negative = error), nothing is enqueued on an error,
 * no allocation, no host synchronisation, asynchronous on the given hipStream_t.
 * Pointers marked DEVICE are device memory owned by the caller, HOST ones are read before
 * the call returns.
 */
#ifndef PS_VERIFY_H
#define PS_VERIFY_H
#include <stdint.h>
#include "ps_draft.h"
#ifdef __cplusplus
extern "C" {
#endif

#define PS_TREE_MAX_NODES 64

/*
 * The shape of a draft tree (Algorithm 1: the tree N; Section 4.2): node 0 is the root (the
 * last token of the prefix), parent[0] = -1, and 0 <= parent[s] < s for every other node, so
 * a node's children follow it and are tried in ascending index.  A node at depth t >= 1
 * carries a token proposed by draft row t-1, i.e. by q(. | x_<n, [MASK]_1..t-1); rank[s] says
 * which of that row's top-k tokens (0 = most probable; rank[0] is ignored).  Both arrays are
 * HOST memory of n_nodes entries, 1 <= n_nodes <= PS_TREE_MAX_NODES, and are copied.
 */
typedef struct ps_tree_shape {
    int32_t n_nodes;
    const int32_t* parent;
    const int32_t* rank;
} ps_tree_shape;

/*
 * Tree construction (Algorithm 1, "Draft future token tree N"): tokens[b][s] =
 * top_ids[b][depth(s) - 1][rank[s]] for s >= 1 and -1 for the root.
 *   top_ids  DEVICE [batch][rows][topk] int32: ps_draft_step's output (rows = k+1 draft rows)
 *   tokens   DEVICE [batch][n_nodes] int32, written
 * Errors: PS_ERR_NULL; PS_ERR_SHAPE (batch < 1, a malformed tree, a depth beyond rows, a rank
 * outside [0, topk)); PS_ERR_DEVICE.
 */
PS_API int ps_tree_tokens(const ps_tree_shape* tree, int32_t batch, int32_t rows, int32_t topk,
                   const int32_t* top_ids, int32_t* tokens, void* stream);

/*
 * The acceptance walk of Algorithm 1 (its inner loops and the final draw), once per sequence,
 * in float64 on the float32 inputs.  Starting at the root with P = p[0]: the children s of
 * the current node are tried in ascending index; child s with token x = tokens[s] at depth t is
 * accepted when r[s] < min(1, P(x) / q[t-1](x)) (a proposal with q(x) = 0 counts as ratio 1);
 * then the walk moves to s and P = p[s].  A rejected child leaves P = the positive part of
 * P - q[t-1], divided by its sum.  When the current node has no child left to try, the last
 * token is drawn from P by inversion with r[0]: the number of token ids whose cumulative sum
 * of P (in id order) is <= r[0] * sum(P), at most vocab-1.
 *   tokens      DEVICE [batch][n_nodes] int32 (entry 0 ignored); a token outside [0, vocab)
 *               is treated as rejected and leaves P unchanged.  May be NULL when top_ids is
 *               given: node s then carries top_ids[b][depth(s) - 1][rank[s]], what
 *               ps_tree_tokens would have written (tree->rank is needed then)
 *   top_ids     DEVICE [batch][rows][topk] int32 or NULL; read only when tokens is NULL
 *   q           DEVICE [batch][rows][vocab] float32: the drafter's distributions
 *               (ps_draft_step's probs); rows >= the tree's depth
 *   p           DEVICE [batch][n_nodes][vocab] float32: the target's next-token distribution
 *               after the path to each node (entry 0: after the prefix alone)
 *   r           DEVICE [batch][n_nodes] float32 uniform numbers in [0, 1)
 *   n_accepted  DEVICE [batch] int32, written: accepted draft tokens
 *   path        DEVICE [batch][rows] int32, written: the accepted nodes, then -1
 *   out_tokens  DEVICE [batch][rows + 1] int32, written: the accepted tokens, the last drawn
 *               token, then -1
 *   workspace   DEVICE, optional (NULL = none): exchange memory for large vocabularies, at least
 *               ps_verify_workspace_bytes(batch, vocab) bytes, 256-byte aligned, owned by the caller,
 *               set to zero once before its first use and then left to the library (it may be
 *               used with any batch up to the one it was sized for)
 * vocab may be at most 262144 (1048576 when vocab % 4 == 0 and q and p are 16-byte aligned).
 * For vocab > 32768 (vocab % 4 == 0, aligned rows, batch * workgroups per sequence <= compute units) several
 * workgroups share a sequence and exchange their partial sums through device memory: the workspace if one is
 * given (calls with different workspaces may overlap in time), else, for batch <= 64, about 1 MB that belongs to
 * the library: calls that use the library's memory on one device must not overlap in time (calls on one stream
 * never do).  Without either, one workgroup walks each sequence (slower, same results).  Should the exchange
 * ever time out (it cannot while every workgroup of the launch gets a compute unit), n_accepted[b] = -2 marks
 * the sequence and its other outputs are undefined.
 * Errors: PS_ERR_NULL; PS_ERR_SHAPE (batch < 1, vocab < 1, a malformed tree, a depth beyond
 * rows; without tokens: topk < 1 or a rank outside [0, topk)); PS_ERR_UNSUPPORTED (vocab too
 * large); PS_ERR_DEVICE.
 */
typedef struct ps_verify_args {
    int32_t batch, rows, vocab;
    const int32_t* tokens;
    const float* q;
    const float* p;
    const float* r;
    int32_t* n_accepted;
    int32_t* path;
    int32_t* out_tokens;
    const int32_t* top_ids;
    int32_t topk;
    void* workspace;
    size_t workspace_bytes;
} ps_verify_args;
PS_API int ps_verify_walk(const ps_tree_shape* tree, const ps_verify_args* args, void* stream);

/* Bytes of exchange memory ps_verify_walk can use for this batch and vocabulary (0: none needed).  Host only. */
PS_API size_t ps_verify_workspace_bytes(int32_t batch, int32_t vocab);

/*
 * ps_verify_walk for callers that cannot allocate device memory or hand any in: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same arguments (args->workspace is
 * ignored), same results, same kernels; it allocates nothing, on the host or on the device.  The exchange
 * memory that large vocabularies need is a fixed array inside the library, 1,065,472 bytes, of which every GPU
 * the library runs on holds its own copy until the process ends.  Limits (beyond them PS_ERR_UNSUPPORTED, never
 * a silent slower path): when vocab > 32768 with vocab % 4 == 0 and aligned rows, batch <= 64 and
 * batch * workgroups per sequence (ceil(vocab / 16384), at most 16) <= compute units.  All calls on one GPU
 * share that array, which keeps what the last call left (tagged with a per-sequence launch count that lives in
 * the array too, so old contents are never taken for data): calls of this function, and calls of ps_verify_walk
 * without a workspace, that overlap in time on one GPU race with each other; calls on one stream never overlap.
 * The first call on a device asks the runtime for the array's address: make it outside graph capture.
 */
PS_API int ps_verify_walk_static(const ps_tree_shape* tree, const ps_verify_args* args, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PS_VERIFY_H */
