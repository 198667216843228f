// Draft-tree construction and the acceptance walk of Algorithm 1 (see include/ps_verify.h).
//
// The walk is sequential by nature (each test depends on the outcome of the one before), so one
// workgroup of 1024 threads walks one sequence's tree; the sequences of a batch run side by side.
// Only what is a vector operation over the vocabulary is spread over the threads: the residual
// (P - q)+ with its sum, and the final draw by inversion (chunk sums, a scan over the chunks, a count).
// The tree's shape travels in the kernel arguments, so nothing is copied or allocated per call.
// All arithmetic is float64; P is kept as (unnormalised vector, its sum) and divided where it is read.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ps_draft.h"
#include "ps_verify.h"

namespace {

constexpr int WALK_THREADS = 1024, WALK_WAVES = WALK_THREADS / 64;

struct TreeDev {
    int n_nodes, max_depth;
    int parent[PS_TREE_MAX_NODES], depth[PS_TREE_MAX_NODES], rank[PS_TREE_MAX_NODES];
};
struct WalkParams {
    TreeDev t;
    int rows, vocab;
    const int32_t* tokens;
    const float *q, *p, *r;
    double* residual;
    int32_t *n_accepted, *path, *out_tokens;
};
struct TokensParams {
    TreeDev t;
    int rows, topk;
    const int32_t* top_ids;
    int32_t* tokens;
};

// sum over the workgroup, the same in every thread: lanes pairwise, then the wavefronts in order
__device__ __forceinline__ double block_sum(double v, double* s_red) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o);
    __syncthreads();   // s_red may still be read from the previous use
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < WALK_WAVES; ++w) t += s_red[w];
    return t;
}
// exclusive prefix sum over the threads in thread order; total = the sum over all of them
__device__ __forceinline__ double block_exclusive_scan(double v, double* s_red, double& total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    double inc = v;
    for (int o = 1; o < 64; o <<= 1) {
        const double t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    __syncthreads();
    if (lane == 63) s_red[w] = inc;
    __syncthreads();
    double base = 0.0;
    total = 0.0;
    for (int i = 0; i < WALK_WAVES; ++i) {
        if (i < w) base += s_red[i];
        total += s_red[i];
    }
    return base + inc - v;
}

__global__ void __launch_bounds__(WALK_THREADS) verify_walk_kernel(const WalkParams W) {
    __shared__ double s_red[WALK_WAVES];
    const int b = blockIdx.x, tid = threadIdx.x, V = W.vocab, N = W.t.n_nodes;
    const int32_t* tokens = W.tokens + (size_t)b * N;
    const float* q = W.q + (size_t)b * W.rows * V;
    const float* p = W.p + (size_t)b * N * V;
    const float* r = W.r + (size_t)b * N;
    double* res = W.residual + (size_t)b * V;

    // P = fresh ? p[u] : res / tot.  Every thread takes every decision itself, from the same values.
    int u = 0, n_acc = 0;
    bool fresh = true;
    double tot = 1.0;
    auto P_at = [&](int i) -> double { return fresh ? (double)p[(size_t)u * V + i] : res[i] / tot; };
    int s = 1;
    while (s < N) {   // the children of u lie behind it; they are met in ascending index
        if (W.t.parent[s] != u) { ++s; continue; }
        const int x = tokens[s];
        bool accept = false;
        if ((unsigned)x < (unsigned)V) {
            const float* qt = q + (size_t)(W.t.depth[s] - 1) * V;
            const double Px = P_at(x), qx = (double)qt[x];
            const double ratio = qx > 0.0 ? fmin(1.0, Px / qx) : 1.0;
            accept = (double)r[s] < ratio;
            if (!accept) {
                __syncthreads();   // everyone has read P(x) before P changes
                double local = 0.0;
                for (int i = tid; i < V; i += WALK_THREADS) {
                    const double v = fmax(P_at(i) - (double)qt[i], 0.0);
                    res[i] = v;
                    local += v;
                }
                const double t = block_sum(local, s_red);   // (its barriers also publish res)
                tot = t > 0.0 ? t : 1.0;
                fresh = false;
            }
        }
        if (accept) {
            if (tid == 0) {
                W.path[(size_t)b * W.rows + n_acc] = s;
                W.out_tokens[(size_t)b * (W.rows + 1) + n_acc] = x;
            }
            ++n_acc;
            u = s;
            fresh = true;
            tot = 1.0;
            s = u + 1;
        } else {
            ++s;
        }
    }

    // the last token: inversion of the cumulative sum in token-id order
    const int chunk = (V + WALK_THREADS - 1) / WALK_THREADS;
    const int c0 = min(V, tid * chunk), c1 = min(V, c0 + chunk);
    double local = 0.0;
    for (int i = c0; i < c1; ++i) local += P_at(i);
    double total;
    double run = block_exclusive_scan(local, s_red, total);
    const double target = (double)r[0] * total;
    double cnt = 0.0;
    for (int i = c0; i < c1; ++i) {
        run += P_at(i);
        if (run <= target) cnt += 1.0;
    }
    const int n = (int)block_sum(cnt, s_red);   // (a count below 2^53: exact)
    if (tid == 0) {
        W.out_tokens[(size_t)b * (W.rows + 1) + n_acc] = n < V - 1 ? n : V - 1;
        for (int i = n_acc + 1; i <= W.rows; ++i) W.out_tokens[(size_t)b * (W.rows + 1) + i] = -1;
        for (int i = n_acc; i < W.rows; ++i) W.path[(size_t)b * W.rows + i] = -1;
        W.n_accepted[b] = n_acc;
    }
}

__global__ void __launch_bounds__(PS_TREE_MAX_NODES) tree_tokens_kernel(const TokensParams T) {
    const int b = blockIdx.x, s = threadIdx.x;
    if (s >= T.t.n_nodes) return;
    int tok = -1;
    if (s > 0) tok = T.top_ids[((size_t)b * T.rows + (T.t.depth[s] - 1)) * T.topk + T.t.rank[s]];
    T.tokens[(size_t)b * T.t.n_nodes + s] = tok;
}

// copies and checks a tree; rank is checked against topk when topk > 0
int load_tree(const ps_tree_shape* tree, int rows, int topk, TreeDev* out) {
    if (!tree || !tree->parent) return PS_ERR_NULL;
    if (topk > 0 && !tree->rank) return PS_ERR_NULL;
    const int N = tree->n_nodes;
    if (N < 1 || N > PS_TREE_MAX_NODES || tree->parent[0] != -1) return PS_ERR_SHAPE;
    out->n_nodes = N;
    out->max_depth = 0;
    for (int s = 0; s < PS_TREE_MAX_NODES; ++s) { out->parent[s] = -1; out->depth[s] = 0; out->rank[s] = 0; }
    for (int s = 1; s < N; ++s) {
        const int pa = tree->parent[s];
        if (pa < 0 || pa >= s) return PS_ERR_SHAPE;
        out->parent[s] = pa;
        out->depth[s] = out->depth[pa] + 1;
        if (out->depth[s] > rows) return PS_ERR_SHAPE;
        if (out->depth[s] > out->max_depth) out->max_depth = out->depth[s];
        if (topk > 0) {
            if (tree->rank[s] < 0 || tree->rank[s] >= topk) return PS_ERR_SHAPE;
            out->rank[s] = tree->rank[s];
        }
    }
    return PS_OK;
}

}   // namespace

extern "C" int ps_tree_tokens(const ps_tree_shape* tree, int32_t batch, int32_t rows, int32_t topk,
                              const int32_t* top_ids, int32_t* tokens, void* stream) {
    if (!top_ids || !tokens) return PS_ERR_NULL;
    if (batch < 1 || rows < 1 || topk < 1) return PS_ERR_SHAPE;
    TokensParams T;
    const int st = load_tree(tree, rows, topk, &T.t);
    if (st != PS_OK) return st;
    T.rows = rows; T.topk = topk; T.top_ids = top_ids; T.tokens = tokens;
    hipLaunchKernelGGL(tree_tokens_kernel, dim3(batch), dim3(PS_TREE_MAX_NODES), 0, (hipStream_t)stream, T);
    return hipGetLastError() == hipSuccess ? PS_OK : PS_ERR_DEVICE;
}

extern "C" int ps_verify_walk(const ps_tree_shape* tree, const ps_verify_args* a, void* stream) {
    if (!a) return PS_ERR_NULL;
    if (!a->tokens || !a->q || !a->p || !a->r || !a->residual || !a->n_accepted || !a->path || !a->out_tokens)
        return PS_ERR_NULL;
    if (a->batch < 1 || a->rows < 1 || a->vocab < 1 || ((uintptr_t)a->residual & 7)) return PS_ERR_SHAPE;
    WalkParams W;
    const int st = load_tree(tree, a->rows, 0, &W.t);
    if (st != PS_OK) return st;
    W.rows = a->rows; W.vocab = a->vocab;
    W.tokens = a->tokens; W.q = a->q; W.p = a->p; W.r = a->r; W.residual = a->residual;
    W.n_accepted = a->n_accepted; W.path = a->path; W.out_tokens = a->out_tokens;
    hipLaunchKernelGGL(verify_walk_kernel, dim3(a->batch), dim3(WALK_THREADS), 0, (hipStream_t)stream, W);
    return hipGetLastError() == hipSuccess ? PS_OK : PS_ERR_DEVICE;
}
