// Draft-tree construction and the acceptance walk of Algorithm 1 (see include/ps_verify.h).
//
// The walk is sequential by nature (each test depends on the outcome of the one before), so one
// workgroup of 1024 threads walks one sequence's tree; the sequences of a batch run side by side.
// Only what is a vector operation over the vocabulary is spread over the threads: the residual
// (P - q)+ with its sum, and the final draw by inversion (totals per slab of the vocabulary, then a scan
// inside one slab).  The tree's shape travels in the kernel arguments, so nothing is copied or allocated
// per call, and no scratch memory is used.  All arithmetic is float64; P is kept unscaled with 1 / its sum
// beside it.  What a test needs while P is still the target's own row (the token, r, P(x), q(x)) is fetched
// for all nodes at once when the kernel starts, so a walk without rejections reads the vocabulary only for
// the final draw.  Two kernels: P in registers for vocabularies up to 32768 entries, P recomputed from the
// target's and the drafter's rows for larger ones.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "ps_draft.h"
#include "ps_verify.h"
#include "ps_draft_debug.h"

namespace {

constexpr int WALK_THREADS = 1024, WALK_WAVES = WALK_THREADS / 64;

struct TreeDev {
    int n_nodes, max_depth;
    int parent[PS_TREE_MAX_NODES], depth[PS_TREE_MAX_NODES], rank[PS_TREE_MAX_NODES];
    int first_child[PS_TREE_MAX_NODES], next_sibling[PS_TREE_MAX_NODES];   // children in ascending index; -1 = none
};
struct WalkParams {
    TreeDev t;
    int rows, vocab;
    const int32_t* tokens;   // or NULL: the tokens come from top_ids
    const int32_t* top_ids;
    int topk;
    const float *q, *p, *r;
    int32_t *n_accepted, *path, *out_tokens;
    unsigned long long* xch;   // several workgroups per sequence: per sequence [XCH_ROUNDS][XCH_WGS][2] exchange slots and a
                               // launch count (the caller's workspace or the library's own memory) ...
    int slabs_per_wg;     // ... slabs of the vocabulary each of them takes
    int spin_limit;       // ... polls before a wait for another workgroup's sum is given up
    int ghosts;           // ... workgroups waited for that do not exist (0; tests of the give-up path: 1)
};
struct TokensParams {
    TreeDev t;
    int rows, topk;
    const int32_t* top_ids;
    int32_t* tokens;
};

// Wavefront-wide sums of doubles with DPP lane exchanges (a row = 16 lanes); a lane without a source
// receives 0.0 and adds nothing.  The order of the additions is fixed.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_f64(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, ROW_MASK, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, ROW_MASK, 0xF, false);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double lane63(double v) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 63), __builtin_amdgcn_readlane(__double2loint(v), 63));
}
// the sum over the wavefront, in every lane
__device__ __forceinline__ double wave_sum_f64(double v) {
    v += dpp_f64<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
    v += dpp_f64<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
    v += dpp_f64<0x141, 0xF>(v);   // row_half_mirror
    v += dpp_f64<0x140, 0xF>(v);   // row_mirror: every lane holds its row's sum
    v += dpp_f64<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3
    v += dpp_f64<0x143, 0xC>(v);   // row_bcast:31 into rows 2 and 3: lane 63 holds the total
    return lane63(v);
}
// inclusive prefix sum over the lanes of the wavefront
__device__ __forceinline__ double wave_inclusive_scan_f64(double v) {
    v += dpp_f64<0x111, 0xF>(v);   // row_shr:1
    v += dpp_f64<0x112, 0xF>(v);   // row_shr:2
    v += dpp_f64<0x114, 0xF>(v);   // row_shr:4
    v += dpp_f64<0x118, 0xF>(v);   // row_shr:8: prefix sums inside every row
    v += dpp_f64<0x142, 0xA>(v);   // rows 1 and 3 add the total of the row before
    v += dpp_f64<0x143, 0xC>(v);   // rows 2 and 3 add the total of rows 0 and 1
    return v;
}

// sum over the workgroup, the same in every thread: inside the wavefronts, then the wavefronts in order
template <int NWAVES = WALK_WAVES>
__device__ __forceinline__ double block_sum(double v, double* s_red) {
    v = wave_sum_f64(v);
    __syncthreads();   // s_red may still be read from the previous use
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < NWAVES; ++w) t += s_red[w];
    return t;
}
// exclusive prefix sum over the threads in thread order; total = the sum over all of them
template <int NWAVES = WALK_WAVES>
__device__ __forceinline__ double block_exclusive_scan(double v, double* s_red, double& total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const double inc = wave_inclusive_scan_f64(v);
    __syncthreads();
    if (lane == 63) s_red[w] = inc;
    __syncthreads();
    double base = 0.0;
    total = 0.0;
    for (int i = 0; i < NWAVES; ++i) {
        if (i < w) base += s_red[i];
        total += s_red[i];
    }
    return base + inc - v;
}

// What the walk needs per node, fetched by one thread per node in one round of loads and left in LDS: the
// node's links (read one after the other from the kernel arguments they would cost a scalar-cache miss
// each), its token (-1 if outside the vocabulary), its uniform number, and what a test of the node reads
// while P is still the target's own row at its parent: P(x) and q(x).
struct NodeLds {
    int tok[PS_TREE_MAX_NODES], first[PS_TREE_MAX_NODES], next[PS_TREE_MAX_NODES], depth[PS_TREE_MAX_NODES];
    float r[PS_TREE_MAX_NODES], px[PS_TREE_MAX_NODES], qx[PS_TREE_MAX_NODES];
};
__device__ __forceinline__ void load_nodes(const WalkParams& Wp, int b, const float* q, const float* p, NodeLds& L) {
    const int tid = threadIdx.x, V = Wp.vocab, N = Wp.t.n_nodes;
    if (tid < N) {
        int x = -1;
        if (Wp.tokens) x = Wp.tokens[(size_t)b * N + tid];
        else if (tid > 0) x = Wp.top_ids[((size_t)b * Wp.rows + (Wp.t.depth[tid] - 1)) * Wp.topk + Wp.t.rank[tid]];
        const bool ok = tid > 0 && (unsigned)x < (unsigned)V;
        L.tok[tid] = ok ? x : -1;
        L.first[tid] = Wp.t.first_child[tid];
        L.next[tid] = Wp.t.next_sibling[tid];
        L.depth[tid] = Wp.t.depth[tid];
        L.r[tid] = Wp.r[(size_t)b * N + tid];
        L.px[tid] = ok ? p[(size_t)Wp.t.parent[tid] * V + x] : 0.f;
        L.qx[tid] = ok ? q[(size_t)(Wp.t.depth[tid] - 1) * V + x] : 0.f;
    }
    __syncthreads();
}

// W consecutive vocabulary entries as one load (W = 4 needs vocab % 4 == 0 and 16-byte aligned rows)
template <int W> struct Vec;
template <> struct Vec<1> { typedef float f; };
template <> struct Vec<4> { typedef float4 f; };
template <int W> __device__ __forceinline__ void widen(const typename Vec<W>::f& v, double (&o)[W]);
template <> __device__ __forceinline__ void widen<1>(const float& v, double (&o)[1]) { o[0] = (double)v; }
template <> __device__ __forceinline__ void widen<4>(const float4& v, double (&o)[4]) {
    o[0] = (double)v.x; o[1] = (double)v.y; o[2] = (double)v.z; o[3] = (double)v.w;
}

// The walk for any vocabulary: nothing of P is stored.  All children of a node are proposals of the same
// draft row q_t, so after J rejections at a node the residual is an elementwise function of the target's row
// p and q_t alone: R_0 = p, R_j = (R_{j-1} c_{j-1} - q_t)+ with c_0 = 1 and c_j = 1 / sum(R_j), and P = R_J c_J.
// A rejection therefore reads the two rows (8 bytes per entry), re-applies the J steps in registers and adds
// up (J steps per entry for the J-th rejection at a node: fine for the few children a draft tree's node has);
// P(x) for a test is the same recurrence on the two numbers fetched when the kernel started.  The final
// draw cuts the vocabulary into slabs of W * WALK_THREADS entries: totals per slab first, then the cumulative
// sum inside the slab in which it passes the target.
//
// MULTI: gridDim.x workgroups share a sequence (blockIdx.y); workgroup g takes slabs [g S, (g + 1) S) of the
// vocabulary for every sum and all of them take every decision.  A sum over the vocabulary is then the sum, in
// workgroup order, of the workgroups' parts, which they leave for each other in exchange memory (Wp.xch: one
// slot per sequence, round and workgroup; a slot is two 8-byte units {half of the double, tag}, written and
// read with agent-scope atomics).  The tag is the sequence slot's launch count + 1: it is kept in device memory
// (xch_epoch), read by every workgroup when it starts and advanced by the workgroup that finishes the sequence -
// by then all of them have read it - so a launch replayed from a graph gets new tags too, and whatever an
// earlier call left in the slots is never taken for data.  Every wait is bounded; a workgroup whose wait runs
// out marks the sequence as failed (n_accepted = -2) and leaves.  All workgroups of a launch must be resident at
// once (the host launches at most one per compute unit), and launches that share exchange memory must not
// overlap in time.
constexpr int WALK_MAX_SLABS = 256;
constexpr int XCH_SEQS = 64, XCH_ROUNDS = PS_TREE_MAX_NODES + 1, XCH_WGS = 16, XCH_SPINS = 1 << 20;
constexpr size_t XCH_SLOT_WORDS = (size_t)XCH_ROUNDS * XCH_WGS * 2;       // 8-byte words of slots per sequence
constexpr size_t XCH_SEQ_WORDS = XCH_SLOT_WORDS + 1;                      // ... and one for the launch count
// bytes for `batch` sequences (a sequence's block does not depend on the batch it is used with)
constexpr size_t xch_bytes(size_t batch) { return (batch * XCH_SEQ_WORDS * 8 + 255) / 256 * 256; }

// The library's own exchange memory, for XCH_SEQS sequences: used when the caller passes no workspace, and by
// ps_verify_walk_static.  Zero when the code object is loaded (launch counts start at 0); every GPU holds its
// own copy.  Host code must not use the array's name as an address: scratch_ptr() asks the runtime for the
// address of the current device's copy once and keeps it.
constexpr size_t SCRATCH_BYTES = xch_bytes(XCH_SEQS);
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

__device__ __forceinline__ unsigned long long* xch_slot(const WalkParams& Wp, int b, int rnd, int g) {
    return Wp.xch + (size_t)b * XCH_SEQ_WORDS + ((size_t)rnd * XCH_WGS + g) * 2;
}
__device__ __forceinline__ unsigned* xch_epoch(const WalkParams& Wp, int b) {
    return reinterpret_cast<unsigned*>(Wp.xch + (size_t)b * XCH_SEQ_WORDS + XCH_SLOT_WORDS);
}

// all workgroups of sequence b: the sum over g of their `mine`, the same in every thread; false if a wait ran out
__device__ __forceinline__ bool xch_sum(const WalkParams& Wp, double mine, int b, int rnd, unsigned tag, double* s_x, double& sum) {
    const int g = blockIdx.x, G = gridDim.x, tid = threadIdx.x;
    if (tid == 0) {
        const unsigned long long bits = (unsigned long long)__double_as_longlong(mine);
        unsigned long long* mine_slot = xch_slot(Wp, b, rnd, g);
        __hip_atomic_store(mine_slot, ((bits & 0xFFFFFFFFull) << 32) | tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(mine_slot + 1, ((bits >> 32) << 32) | tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (tid < G + Wp.ghosts) {
        unsigned long long lo = 0, hi = 0;
        const unsigned long long* theirs = xch_slot(Wp, b, rnd, tid);
        int spins = 0;
        for (;;) {
            lo = __hip_atomic_load(theirs, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            hi = __hip_atomic_load(theirs + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (((unsigned)lo == tag && (unsigned)hi == tag) || ++spins > Wp.spin_limit) break;
            __builtin_amdgcn_s_sleep(2);
        }
        const bool ok = (unsigned)lo == tag && (unsigned)hi == tag;
        if (tid < G) s_x[tid] = ok ? __longlong_as_double((long long)((lo >> 32) | ((hi >> 32) << 32))) : 0.0;
        if (!ok) s_x[XCH_WGS] = 1.0;
    }
    __syncthreads();
    sum = 0.0;
    for (int i = 0; i < G; ++i) sum += s_x[i];
    const bool good = s_x[XCH_WGS] == 0.0;
    __syncthreads();   // s_x is written again in the next round
    return good;
}

template <int W, bool MULTI>
__global__ void __launch_bounds__(WALK_THREADS) verify_walk_kernel(const WalkParams Wp) {
    typedef typename Vec<W>::f VF;
    __shared__ double s_red[WALK_WAVES];
    __shared__ double s_c[PS_TREE_MAX_NODES + 1];
    __shared__ double s_part[WALK_MAX_SLABS][WALK_WAVES];
    __shared__ double s_x[XCH_WGS + 1];
    __shared__ NodeLds L;
    const int b = MULTI ? blockIdx.y : blockIdx.x, g = MULTI ? blockIdx.x : 0;
    const int tid = threadIdx.x, V = Wp.vocab, N = Wp.t.n_nodes;
    const int lane = tid & 63, wave = tid >> 6;
    __shared__ unsigned s_tag;
    if (tid == 0) {                     // (both read after the barrier in load_nodes at the earliest)
        s_x[XCH_WGS] = 0.0;
        unsigned t = MULTI ? __hip_atomic_load(xch_epoch(Wp, b), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u : 1u;
        s_tag = t ? t : 1u;             // 0 is what slots never written hold
    }
    int rnd = 0;
    const float* q = Wp.q + (size_t)b * Wp.rows * V;
    const float* p = Wp.p + (size_t)b * N * V;
    load_nodes(Wp, b, q, p, L);
    s_c[0] = 1.0;   // (every thread writes the same value and reads it back itself: no barrier needed)
    const unsigned tag = s_tag;
    auto fail = [&]() {   // a wait ran out: the sequence is marked, its tag is used up
        if (tid == 0) {
            Wp.n_accepted[b] = -2;
            __hip_atomic_store(xch_epoch(Wp, b), tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };

    // R_J of one entry; every thread takes every decision itself, from the same values
    int J = 0;
    auto residual = [&](double v, double qe) -> double {
        for (int t = 0; t < J; ++t) v = fmax(v * s_c[t] - qe, 0.0);
        return v;
    };
    const int nvec_all = V / W;           // (W = 4: V % 4 == 0)
    const int n_slabs_all = (nvec_all + WALK_THREADS - 1) / WALK_THREADS;   // <= WALK_MAX_SLABS (host)
    // this workgroup's slabs [slab0, slab0 + n_slabs) and vectors [jlo, nvec); this thread's: jlo + tid + WALK_THREADS * k
    const int slab0 = MULTI ? g * Wp.slabs_per_wg : 0;
    const int n_slabs = MULTI ? min(Wp.slabs_per_wg, n_slabs_all - slab0) : n_slabs_all;
    const int jlo = slab0 * WALK_THREADS, nvec = min(nvec_all, jlo + n_slabs * WALK_THREADS);
    constexpr int UN = 4;                 // vectors of each row on their way at once (8: measured slower)
    int u = 0, n_acc = 0;
    int s = L.first[0];
    while (s >= 0) {   // the children of u in ascending index
        const int x = L.tok[s];
        bool accept = false;
        if (x >= 0) {
            const double qx = (double)L.qx[s];
            const double Px = residual((double)L.px[s], qx) * s_c[J];
            const double ratio = qx > 0.0 ? fmin(1.0, Px / qx) : 1.0;
            accept = (double)L.r[s] < ratio;
            if (!accept) {
                ++J;
                const VF* pu = reinterpret_cast<const VF*>(p + (size_t)u * V);
                const VF* qt = reinterpret_cast<const VF*>(q + (size_t)(L.depth[s] - 1) * V);
                double local = 0.0;
                for (int j0 = jlo + tid; j0 < nvec; j0 += WALK_THREADS * UN) {
                    VF pv[UN], qv[UN];
#pragma unroll
                    for (int k = 0; k < UN; ++k) {
                        const int j = j0 + k * WALK_THREADS;
                        if (j < nvec) { pv[k] = pu[j]; qv[k] = qt[j]; }
                    }
#pragma unroll
                    for (int k = 0; k < UN; ++k) {
                        if (j0 + k * WALK_THREADS < nvec) {
                            double a[W], c[W];
                            widen<W>(pv[k], a);
                            widen<W>(qv[k], c);
#pragma unroll
                            for (int e = 0; e < W; ++e) local += residual(a[e], c[e]);
                        }
                    }
                }
                double t = block_sum(local, s_red);
                if (MULTI && !xch_sum(Wp, t, b, rnd++, tag, s_x, t)) {
                    fail();
                    return;
                }
                s_c[J] = t > 0.0 ? 1.0 / t : 1.0;
            }
        }
        if (accept) {
            if (tid == 0 && g == 0) {
                Wp.path[(size_t)b * Wp.rows + n_acc] = s;
                Wp.out_tokens[(size_t)b * (Wp.rows + 1) + n_acc] = x;
            }
            ++n_acc;
            u = s;
            J = 0;
            s = L.first[u];
        } else {
            s = L.next[s];
        }
    }

    // The last token.  P = R_J c_J at node u; its children's draft row is row depth(u) of q (unused if J = 0).
    const VF* pu = reinterpret_cast<const VF*>(p + (size_t)u * V);
    const VF* qt = reinterpret_cast<const VF*>(q + (size_t)(J > 0 ? L.depth[u] : 0) * V);
    const double cJ = s_c[J];
    auto P_of = [&](int j, double (&o)[W]) {   // entries of vector j (j < nvec)
        double a[W], c[W];
        widen<W>(pu[j], a);
        if (J > 0) widen<W>(qt[j], c);
#pragma unroll
        for (int e = 0; e < W; ++e) o[e] = (J > 0 ? residual(a[e], c[e]) : a[e]) * cJ;
    };
    constexpr int UF = 8;                 // slabs whose rows are on their way at once
    for (int k0 = 0; k0 < n_slabs; k0 += UF) {
        VF pv[UF], qv[UF];
#pragma unroll
        for (int i = 0; i < UF; ++i) {
            const int j = jlo + tid + WALK_THREADS * (k0 + i);
            if (j < nvec) {
                pv[i] = pu[j];
                if (J > 0) qv[i] = qt[j];
            }
        }
#pragma unroll
        for (int i = 0; i < UF; ++i) {
            const int j = jlo + tid + WALK_THREADS * (k0 + i);
            double v = 0.0;
            if (j < nvec) {
                double a[W], c[W];
                widen<W>(pv[i], a);
                if (J > 0) widen<W>(qv[i], c);
#pragma unroll
                for (int e = 0; e < W; ++e) v += (J > 0 ? residual(a[e], c[e]) : a[e]) * cJ;
            }
            v = wave_sum_f64(v);
            if (lane == 0 && k0 + i < n_slabs) s_part[k0 + i][wave] = v;
        }
    }
    __syncthreads();
    double total = 0.0;
    for (int k = 0; k < n_slabs; ++k)
        for (int w = 0; w < WALK_WAVES; ++w) total += s_part[k][w];
    double before = 0.0;                  // the cumulative sum in front of this workgroup's slabs
    if (MULTI) {
        // the workgroups' totals: the draw falls to the first workgroup whose cumulative sum exceeds the
        // target (the last one if none does); the others are done
        const double mine_total = total;
        if (!xch_sum(Wp, mine_total, b, rnd++, tag, s_x, total)) {
            fail();
            return;
        }
        // (s_x was overwritten by nobody since: xch_sum ends with a barrier and this is the last round)
        const double tgt = (double)L.r[0] * total;
        int owner = (int)gridDim.x - 1;
        double cumg = 0.0;
        for (int i = 0; i < (int)gridDim.x; ++i) {
            if (cumg + s_x[i] > tgt || i == (int)gridDim.x - 1) { owner = i; break; }
            cumg += s_x[i];
        }
        if (g != owner) return;
        before = cumg;
    }
    const double target = (double)L.r[0] * total;
    int ks = n_slabs - 1;
    double base = before, cum = before;
    for (int k = 0; k < n_slabs; ++k) {
        double t = 0.0;
        for (int w = 0; w < WALK_WAVES; ++w) t += s_part[k][w];
        if (cum + t > target || k == n_slabs - 1) { ks = k; base = cum; break; }
        cum += t;
    }
    double mine[W];
#pragma unroll
    for (int e = 0; e < W; ++e) mine[e] = 0.0;
    const int jm = jlo + tid + WALK_THREADS * ks;
    if (jm < nvec) P_of(jm, mine);
    double mysum = 0.0;
#pragma unroll
    for (int e = 0; e < W; ++e) mysum += mine[e];
    double dummy;
    double run = base + block_exclusive_scan(mysum, s_red, dummy);
    double cnt = 0.0;
#pragma unroll
    for (int e = 0; e < W; ++e) {
        run += mine[e];
        if (jm < nvec && run <= target) cnt += 1.0;
    }
    const int n = W * WALK_THREADS * (slab0 + ks) + (int)block_sum(cnt, s_red);   // every id of the slabs before counts
    if (tid == 0) {
        Wp.out_tokens[(size_t)b * (Wp.rows + 1) + n_acc] = n < V - 1 ? n : V - 1;
        for (int i = n_acc + 1; i <= Wp.rows; ++i) Wp.out_tokens[(size_t)b * (Wp.rows + 1) + i] = -1;
        for (int i = n_acc; i < Wp.rows; ++i) Wp.path[(size_t)b * Wp.rows + i] = -1;
        Wp.n_accepted[b] = n_acc;
        if (MULTI) __hip_atomic_store(xch_epoch(Wp, b), tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// The same walk for vocabularies of at most REG_EPT * REG_THREADS entries (a multiple of 4, rows 16-byte
// aligned): P lives in registers, so a rejection only reads its row of q (and, the first time at a node, the
// target's row) and the scratch buffer is not touched.  The vocabulary is cut into slabs of 4 * REG_THREADS
// entries; thread t holds entries [4t, 4t + 4) of every slab, so all loads are contiguous across a wavefront.
// P(x) of a residual goes from the thread that holds it to the others through LDS.  The final draw finds
// the slab in which the cumulative sum passes the target from the slabs' totals, then scans that slab.
constexpr int REG_EPT = 32, REG_THREADS = 1024, REG_WAVES = REG_THREADS / 64, REG_SLABS = REG_EPT / 4;
__global__ void __launch_bounds__(REG_THREADS) verify_walk_reg_kernel(const WalkParams Wp) {
    __shared__ double s_red[REG_WAVES];
    __shared__ double s_part[REG_SLABS][REG_WAVES];
    __shared__ double s_bc;
    __shared__ NodeLds L;
    const int b = blockIdx.x, tid = threadIdx.x, V = Wp.vocab, N = Wp.t.n_nodes;
    const float* q = Wp.q + (size_t)b * Wp.rows * V;
    const float* p = Wp.p + (size_t)b * N * V;
    load_nodes(Wp, b, q, p, L);

    const int nvec = V / 4;                      // float4 units; this thread's: tid + REG_THREADS * k
    double Pr[REG_EPT];                          // P (to be scaled by inv_tot) once it is no longer a row of p:
                                                 // Pr[4k + e] = entry 4 (tid + REG_THREADS k) + e, 0 beyond V
    int u = 0, n_acc = 0;
    bool fresh = true;
    double inv_tot = 1.0;
    // Pr <- the target's row at u (P = that row: inv_tot = 1)
    auto load_row = [&]() {
        const float4* pu4 = reinterpret_cast<const float4*>(p + (size_t)u * V);
        float4 pv[REG_SLABS];
#pragma unroll
        for (int k = 0; k < REG_SLABS; ++k) {
            const int j = tid + REG_THREADS * k;
            pv[k] = j < nvec ? pu4[j] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int k = 0; k < REG_SLABS; ++k) {
            Pr[4 * k] = (double)pv[k].x; Pr[4 * k + 1] = (double)pv[k].y;
            Pr[4 * k + 2] = (double)pv[k].z; Pr[4 * k + 3] = (double)pv[k].w;
        }
    };
    // Pr <- (Pr * inv_tot - qt)+; returns this thread's part of the sum
    auto subtract = [&](const float* __restrict__ qt) -> double {
        const float4* q4 = reinterpret_cast<const float4*>(qt);
        float4 qv[REG_SLABS];
#pragma unroll
        for (int k = 0; k < REG_SLABS; ++k) {
            const int j = tid + REG_THREADS * k;
            qv[k] = j < nvec ? q4[j] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        double local = 0.0;
#pragma unroll
        for (int k = 0; k < REG_SLABS; ++k) {
            const float qe[4] = {qv[k].x, qv[k].y, qv[k].z, qv[k].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const double v = fmax(Pr[4 * k + e] * inv_tot - (double)qe[e], 0.0);
                Pr[4 * k + e] = v;
                local += v;
            }
        }
        return local;
    };

    int s = L.first[0];
    while (s >= 0) {   // the children of u in ascending index
        const int x = L.tok[s];
        bool accept = false;
        if (x >= 0) {
            double Px;
            if (fresh) {
                Px = (double)L.px[s];
            } else {
                const int j = x >> 2;   // unit j is slab j / REG_THREADS of thread j % REG_THREADS
                if (tid == (j & (REG_THREADS - 1))) {
                    const int idx = 4 * (j / REG_THREADS) + (x & 3);
                    double v = 0.0;
#pragma unroll
                    for (int e = 0; e < REG_EPT; ++e)
                        if (e == idx) v = Pr[e];
                    s_bc = v * inv_tot;
                }
                __syncthreads();   // (the next write of s_bc lies behind the barriers of a block_sum)
                Px = s_bc;
            }
            const double qx = (double)L.qx[s];
            const double ratio = qx > 0.0 ? fmin(1.0, Px / qx) : 1.0;
            accept = (double)L.r[s] < ratio;
            if (!accept) {
                if (fresh) load_row();
                fresh = false;
                const double t = block_sum<REG_WAVES>(subtract(q + (size_t)(L.depth[s] - 1) * V), s_red);
                inv_tot = t > 0.0 ? 1.0 / t : 1.0;
            }
        }
        if (accept) {
            if (tid == 0) {
                Wp.path[(size_t)b * Wp.rows + n_acc] = s;
                Wp.out_tokens[(size_t)b * (Wp.rows + 1) + n_acc] = x;
            }
            ++n_acc;
            u = s;
            fresh = true;
            inv_tot = 1.0;
            s = L.first[u];
        } else {
            s = L.next[s];
        }
    }

    // The last token.  Totals of the slabs (each wavefront adds up its part of every slab, the wavefronts'
    // parts meet in LDS), the slab ks in which the cumulative sum first exceeds the target, then the
    // cumulative sum inside that slab in id order.
    if (fresh) load_row();
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int k = 0; k < REG_SLABS; ++k) {
        double v = 0.0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            Pr[4 * k + e] *= inv_tot;   // (1 for a row of p: exact)
            v += Pr[4 * k + e];
        }
        v = wave_sum_f64(v);
        if (lane == 0) s_part[k][wave] = v;
    }
    __syncthreads();
    double slab_tot[REG_SLABS], total = 0.0;
#pragma unroll
    for (int k = 0; k < REG_SLABS; ++k) {
        double t = 0.0;
        for (int w = 0; w < REG_WAVES; ++w) t += s_part[k][w];
        slab_tot[k] = t;
        total += t;
    }
    const double target = (double)L.r[0] * total;
    const int n_slabs = (nvec + REG_THREADS - 1) / REG_THREADS;
    int ks = n_slabs - 1;
    double base = 0.0, cum = 0.0;
    bool found = false;
#pragma unroll
    for (int k = 0; k < REG_SLABS; ++k) {
        if (k < n_slabs && !found) {
            if (cum + slab_tot[k] > target || k == n_slabs - 1) { ks = k; base = cum; found = true; }
            cum += slab_tot[k];
        }
    }
    double mine[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int k = 0; k < REG_SLABS; ++k)
        if (k == ks) { mine[0] = Pr[4 * k]; mine[1] = Pr[4 * k + 1]; mine[2] = Pr[4 * k + 2]; mine[3] = Pr[4 * k + 3]; }
    double dummy;
    double run = base + block_exclusive_scan<REG_WAVES>(mine[0] + mine[1] + mine[2] + mine[3], s_red, dummy);
    const int id0 = 4 * (tid + REG_THREADS * ks);
    double cnt = 0.0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        run += mine[e];
        if (id0 + e < V && run <= target) cnt += 1.0;
    }
    const int n = 4 * REG_THREADS * ks + (int)block_sum<REG_WAVES>(cnt, s_red);   // every id of the slabs before ks counts
    if (tid == 0) {
        Wp.out_tokens[(size_t)b * (Wp.rows + 1) + n_acc] = n < V - 1 ? n : V - 1;
        for (int i = n_acc + 1; i <= Wp.rows; ++i) Wp.out_tokens[(size_t)b * (Wp.rows + 1) + i] = -1;
        for (int i = n_acc; i < Wp.rows; ++i) Wp.path[(size_t)b * Wp.rows + i] = -1;
        Wp.n_accepted[b] = n_acc;
    }
}

__global__ void __launch_bounds__(PS_TREE_MAX_NODES) tree_tokens_kernel(const TokensParams T) {
    const int b = blockIdx.x, s = threadIdx.x;
    if (s >= T.t.n_nodes) return;
    int tok = -1;
    if (s > 0) tok = T.top_ids[((size_t)b * T.rows + (T.t.depth[s] - 1)) * T.topk + T.t.rank[s]];
    T.tokens[(size_t)b * T.t.n_nodes + s] = tok;
}

// compute units of the current device (0 if it cannot be asked): asked once per process and device
int compute_units() {
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    int n = cached[dev].load();
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n = -1;
        cached[dev].store(n);
    }
    return n > 0 ? n : 0;
}

// copies and checks a tree; rank is checked against topk when topk > 0
int load_tree(const ps_tree_shape* tree, int rows, int topk, TreeDev* out) {
    if (!tree || !tree->parent) return PS_ERR_NULL;
    if (topk > 0 && !tree->rank) return PS_ERR_NULL;
    const int N = tree->n_nodes;
    if (N < 1 || N > PS_TREE_MAX_NODES || tree->parent[0] != -1) return PS_ERR_SHAPE;
    out->n_nodes = N;
    out->max_depth = 0;
    for (int s = 0; s < PS_TREE_MAX_NODES; ++s) {
        out->parent[s] = -1; out->depth[s] = 0; out->rank[s] = 0; out->first_child[s] = -1; out->next_sibling[s] = -1;
    }
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
    for (int s = N - 1; s >= 1; --s) {   // prepending in descending order leaves every list ascending
        out->next_sibling[s] = out->first_child[out->parent[s]];
        out->first_child[out->parent[s]] = s;
    }
    return PS_OK;
}

// test hook (see ps_verify_debug_exchange)
std::atomic<int> g_spin_limit{XCH_SPINS}, g_ghosts{0};

}   // namespace

// see ps_draft_debug.h
extern "C" void ps_verify_debug_exchange(int spins, int ghosts) {
    g_spin_limit = spins > 0 ? spins : XCH_SPINS;
    g_ghosts = ghosts == 1 ? 1 : 0;
}

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

namespace {

// Address of the current device's copy of `scratch`: asked from the runtime on the first call on that device
// (with that device current) and kept; every GPU holds its own copy at its own address.
int scratch_ptr(unsigned char** out) {
    static std::atomic<unsigned char*> ptrs[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return PS_ERR_DEVICE;
    unsigned char* p = ptrs[dev].load();
    if (!p) {
        void* q = nullptr;
        if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) return PS_ERR_DEVICE;
        p = static_cast<unsigned char*>(q);
        ptrs[dev].store(p);
    }
    *out = p;
    return PS_OK;
}

// vocabularies that take the exchange between workgroups: whole vectors of four entries, more than the
// register kernel holds; slabs of the vocabulary per workgroup and workgroups per sequence
bool wants_exchange(int vocab, bool aligned, int* per, int* G) {
    if (vocab % 4 != 0 || !aligned || vocab <= REG_EPT * REG_THREADS) return false;
    const long long slabs = ((long long)vocab / 4 + WALK_THREADS - 1) / WALK_THREADS;
    int p = 4;
    while ((slabs + p - 1) / p > XCH_WGS) ++p;
    *per = p;
    *G = (int)((slabs + p - 1) / p);
    return *G > 1;
}

// static_only: the entry point that allocates nothing and takes no workspace (see ps_verify_walk_static)
int walk_impl(const ps_tree_shape* tree, const ps_verify_args* a, void* stream, bool static_only) {
    if (!a) return PS_ERR_NULL;
    if ((!a->tokens && !a->top_ids) || !a->q || !a->p || !a->r || !a->n_accepted || !a->path || !a->out_tokens)
        return PS_ERR_NULL;
    if (a->batch < 1 || a->rows < 1 || a->vocab < 1 || (!a->tokens && a->topk < 1)) return PS_ERR_SHAPE;
    WalkParams W;
    const int st = load_tree(tree, a->rows, a->tokens ? 0 : a->topk, &W.t);   // (ranks are needed without tokens)
    if (st != PS_OK) return st;
    W.rows = a->rows; W.vocab = a->vocab;
    W.tokens = a->tokens; W.top_ids = a->tokens ? nullptr : a->top_ids; W.topk = a->topk; W.q = a->q; W.p = a->p; W.r = a->r;
    W.n_accepted = a->n_accepted; W.path = a->path; W.out_tokens = a->out_tokens;
    W.xch = nullptr;
    // whole vectors of four entries when every row of q and p starts on a 16-byte boundary
    const bool aligned = (((uintptr_t)a->q | (uintptr_t)a->p) & 15) == 0;
    const bool vec = a->vocab % 4 == 0 && aligned;
    const long long slabs = ((long long)a->vocab / (vec ? 4 : 1) + WALK_THREADS - 1) / WALK_THREADS;
    if (slabs > WALK_MAX_SLABS) return PS_ERR_UNSUPPORTED;
    W.slabs_per_wg = (int)slabs;
    W.spin_limit = g_spin_limit;
    W.ghosts = 0;
    int per = 0, G = 1;
    const bool exchange = wants_exchange(a->vocab, aligned, &per, &G);
    if (static_only) {
        // this entry point never falls back silently: beyond what the library's own memory holds it says so
        if (exchange && (a->batch > XCH_SEQS || (long long)a->batch * G > compute_units())) return PS_ERR_UNSUPPORTED;
    }
    if (vec && a->vocab <= REG_EPT * REG_THREADS) {
        hipLaunchKernelGGL(verify_walk_reg_kernel, dim3(a->batch), dim3(REG_THREADS), 0, (hipStream_t)stream, W);
    } else if (vec) {
        // several workgroups per sequence (4 slabs each, at most XCH_WGS) when all of them get a compute unit
        // and there is exchange memory: the caller's workspace, else the library's own for up to XCH_SEQS sequences
        unsigned char* mem = nullptr;
        if (exchange && (long long)a->batch * G <= compute_units()) {
            if (!static_only && a->workspace && a->workspace_bytes >= xch_bytes(a->batch) && ((uintptr_t)a->workspace & 255) == 0)
                mem = static_cast<unsigned char*>(a->workspace);
            else if (a->batch <= XCH_SEQS && scratch_ptr(&mem) != PS_OK) {
                if (static_only) return PS_ERR_DEVICE;
                mem = nullptr;
            }
        }
        if (mem) {
            W.xch = reinterpret_cast<unsigned long long*>(mem);
            W.slabs_per_wg = per;
            W.ghosts = G < XCH_WGS ? (int)g_ghosts : 0;
            hipLaunchKernelGGL((verify_walk_kernel<4, true>), dim3(G, a->batch), dim3(WALK_THREADS), 0, (hipStream_t)stream, W);
        } else {
            hipLaunchKernelGGL((verify_walk_kernel<4, false>), dim3(a->batch), dim3(WALK_THREADS), 0, (hipStream_t)stream, W);
        }
    } else {
        hipLaunchKernelGGL((verify_walk_kernel<1, false>), dim3(a->batch), dim3(WALK_THREADS), 0, (hipStream_t)stream, W);
    }
    return hipGetLastError() == hipSuccess ? PS_OK : PS_ERR_DEVICE;
}

}   // namespace

extern "C" size_t ps_verify_workspace_bytes(int32_t batch, int32_t vocab) {
    int per = 0, G = 1;
    if (batch < 1 || vocab < 1 || !wants_exchange(vocab, true, &per, &G)) return 0;
    return xch_bytes((size_t)batch);
}

extern "C" int ps_verify_walk(const ps_tree_shape* tree, const ps_verify_args* a, void* stream) {
    return walk_impl(tree, a, stream, false);
}

extern "C" int ps_verify_walk_static(const ps_tree_shape* tree, const ps_verify_args* a, void* stream) {
    return walk_impl(tree, a, stream, true);
}
