// Internal declarations shared by the host dispatcher and the HIP kernels of the
// parallel draft step (not part of the public C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "ps_draft.h"

#define PS_MAX_ROWS 64     // activation rows per step (MFMA column tiles: up to 4 x 16)
// One workgroup per compute unit.  512 threads = 8 wavefronts of 64 lanes, two per SIMD: each lane
// may use 256 VGPRs, which pays for the weight loads in flight per lane and large staging batches
// without spills (1024 threads would cap lanes at 128 VGPRs).
#ifndef PS_WG_THREADS
#define PS_WG_THREADS 512
#endif
#define PS_WAVES (PS_WG_THREADS / 64)
#define PS_WAVES_LOG 3
#ifndef PS_U
#define PS_U 8             // 16-byte weight loads in flight per lane (PS_U KiB per wavefront)
#endif
#ifndef PS_PF
#define PS_PF 2            // at most this many 8-KiB pieces of its first weight stream a wavefront pulls into the L2 while it waits
#endif
#define PS_U_MAX 32        // packed weight buffers are padded by this many KiB (streaming reads ahead)
#define PS_LDS_BYTES (160 * 1024)
// The first PS_LDS_BASE bytes of dynamic LDS are the same in every phase's layout: what a workgroup reads once
// when the kernel starts and keeps for the whole step (see ps_device.h): the step's sequence number, the
// sequences' cache lengths and unused slots.
#define PS_LDS_BASE 1024
#define PS_LDS_SEQ 16        // the step's sequence number (see ps_seq)
#define PS_LDS_KVLEN 256     // int[PS_MAX_ROWS]: valid cache positions per sequence
#define PS_LDS_SKIP 512      // int[PS_MAX_ROWS]: unused leading slots of real rows per sequence (see StepParams::skip)
static_assert((1 << PS_WAVES_LOG) == PS_WAVES, "PS_WAVES_LOG");
static_assert((PS_U & (PS_U - 1)) == 0 && PS_U <= PS_U_MAX, "PS_U");

// Attention work items cover PS_ATTN_KEYS * nk keys of one (sequence, kv head): every wavefront
// takes nk = 1 or 2 groups of 16 keys.  LDS an item needs (see AttnCfg in ps_device.h):
#define PS_ATTN_KEYS (16 * PS_WAVES)
#define PS_ATTN_KEYS_LOG (4 + PS_WAVES_LOG)
constexpr int ps_attn_lds_bytes(int d, int nk) {
    return PS_LDS_BASE + 2 * PS_WAVES * 16 * 4 + PS_WAVES * nk * 16 * 16 * 4 + PS_WAVES * 16 * d * 4 + 16 * d * 4;
}

// bf16 storage (attn_phase2 in ps_device.h; Attn2Cfg): query operands, staged value rows, rescale factors, (max, sum), outputs
constexpr int ps_attn2_lds_bytes(int d) {
    return PS_LDS_BASE + 16 * d * 4 + PS_WAVES * 2 * 8 * (d + 8) * 4 + PS_WAVES * 16 * 4 + PS_WAVES * 16 * 2 * 4 + PS_WAVES * 16 * (d + 4) * 4;
}
#define PS_ATTN2_NK_LOG_MAX 4   // at most 16 groups of 16 keys per wavefront and block: blocks of up to 2048 cache keys

// The five GEMM phases of the step, and the input projection of the feature-fusion input mode (a kernel of
// its own in front of the step, built from the same engine)
enum { PH_QKV = 0, PH_OPROJ = 1, PH_GATEUP = 2, PH_DOWN = 3, PH_LMHEAD = 4, PH_FC = 5, PH_COUNT = 6 };
enum { PS_IN_HIDDEN = 0, PS_IN_TOKENS = 1, PS_IN_FUSED = 2 };   // where the real rows of Z come from
// Footprint of a step in the sentinel-coded exchange buffers: [0] activation rows, [1 + ph] 16-byte units of
// phase ph's K-slice fragments, [1 + PH_COUNT + ph] K-slices that left sums of squares (0 = none)
#define PS_FOOT_INTS (1 + 2 * PH_COUNT)
// Device counters of a context (32-bit words): error flag, steps completed, tickets, then the footprints
#define PS_CTR_ERROR 0
#define PS_CTR_STEP 1
#define PS_CTR_DONE 2
#define PS_CTR_FOOT 4
#define PS_CTR_WORDS (PS_CTR_FOOT + 2 * PS_FOOT_INTS)
#define PS_SPIN_LIMIT (1 << 20)

// How one weight-streaming GEMM phase is cut up.  A "tile" is 16 weight rows; a "step" is the
// 64-byte piece of a weight row one MFMA group consumes (32 bf16 or 16 f32 elements); a "group"
// is PS_U consecutive steps, the unit in which wavefronts share the contraction dimension.
// Everything a workgroup needs to find its work is precomputed here on the host, so the device
// code walks through a phase with a few scalar multiplications and no division.
struct PhaseDesc {
    int T;             // tiles
    int Kt;            // steps per tile in the packed matrix: a multiple of PS_U (zero weights beyond K)
    int K;             // contraction length in elements
    int rows;          // activation rows
    int norm;          // RMSNorm folded into the phase
    int kw_log;        // log2 of the wavefronts that share one tile (their partial sums meet in LDS)
    int s_log;         // log2 of the K-slices across workgroups (their partial sums meet in global memory)
    int Gs;            // workgroup columns: nwg >> s_log; workgroup wg is slice wg % S of column wg / S
    int nwg;           // workgroups of the grid
    int per_round;     // tiles the grid takes per round: Gs * (PS_WAVES >> kw_log)
    int rounds;
    int piece_groups;  // groups of the activation panel held in LDS at a time
    int npieces;
    int rs;            // bytes between panel rows in LDS
    int g2_log;        // staging: log2 of the threads laid along the contraction dimension
    int src_ld;        // elements between rows of src
    int lds_bytes;     // dynamic LDS the phase needs
    int pf;            // 8-KiB pieces of the first stream to pull into the L2 during the wait for the panel (<= PS_PF)
    const void* gain;  // RMSNorm gain (config dtype)
    const float* src;  // exchanged fp32 activations the phase reads (QKV reads x / mask_emb instead)
    const char* wpack; // the phase's matrices, prepacked at init in streaming order
    float* frag;       // [S][T][MT][64 lanes][4]: the K-slices' parts of every tile (coded like the activations)
    float* ssq_frag;   // [S][PS_MAX_ROWS]: the K-slices' sums of squares of the activation rows
};

struct StepParams {
    // shape
    int H, nq, nkv, d, F, V, QD, KVD;
    int B, n_new, k, M, Mtot, R, Rtot, all_rows, topk;
    int spin_limit;    // polls after which a wait for exchanged data is given up (see spin_again)
    int final_norm, max_positions;
    float eps, inv_sqrt_d;
    // sampling epilogue: logits are divided by the temperature before softmax, top-k probabilities and the
    // draw; sample_ids != NULL asks for one Gumbel-max draw per output row with the counter-based generator
    // (see gumbel_of in ps_device.h)
    float inv_temp;
    unsigned seed_lo, seed_hi;
    int32_t* sample_ids;
    float* sample_p;
    const int32_t* kv_len_dev;   // the sequences' lengths in device memory (then kv_len[] below holds upper bounds), or NULL
    // weights and step inputs (config dtype)
    const void *g_in, *wq, *wk, *wv, *wo, *g_post, *w_gate, *w_up, *w_down, *g_final, *w_lm, *mask_emb, *w_fc;
    const void* x;
    // input stage (Section 4.3): in_mode PS_IN_TOKENS: real row (b, i) is row token_ids[b][i] of the shared
    // embedding table; PS_IN_FUSED: it is w_fc . [features[b][i] ; that embedding row] (+ b_fc), worked out by the
    // input-projection kernel into x_buf (fp32, coded like the other activations); [MASK] rows always come from mask_emb
    int in_mode;
    unsigned n_magic;            // ceil(2^32 / n_new)
    const int32_t* token_ids;
    const void *features, *embed, *b_fc;
    float* x_buf;                // [Mtot][H]
    void *kc, *vc;
    // workspace
    const float2* rope; // [max_positions][d/2] (cos, sin)
    // Activations between phases: plain fp32, 0xFFFFFFFF = not written yet.  Two copies alternate; the
    // pointers are those of copy 0, step n uses copy n & 1.
    float *q_buf, *o_buf, *y_buf, *u_buf, *y2_buf;   // [Mtot][QD], [Mtot][QD], [Mtot][H], [Mtot][F], [Mtot][H]
    float* kvnew;      // [Mtot][2][KVD] this step's K and V rows as stored in the cache
    long long act_bytes;   // distance between the two copies
    unsigned *step_ctr, *done_ctr;   // steps completed so far; tickets of the running kernel (see step_begin)
    // What a step leaves behind in the sentinel-coded buffers of its copy (see sx_reset_stale): foot is this
    // step's footprint, foot_mem the device-side record [2][PS_FOOT_INTS] of the two latest steps' footprints.
    unsigned foot[PS_FOOT_INTS];
    unsigned* foot_mem;
    // Buffers below hold 8-byte units {value, tag}: element counts.
    float* attn_acc;   // [items][g*M][d] unnormalised partial outputs
    float* attn_ml;    // [items][g*M][2] (running max, sum of exponentials)
    int* error_flag;   // set if a wait for exchanged data timed out
    float* lm_part;    // [workgroups][Rtot][2 + 2*topk]: max, sum exp, top-k keys (low, high word)
    float* logits_store; // where logits go (caller's buffer, internal scratch, or NULL)
    // outputs
    int32_t* top_ids;
    float *top_p, *lse, *probs, *hidden_out;
    // attention work list
    int attn_items, attn_nwg;   // work items; workgroups of the attention kernel (multi mode)
    int attn_single;        // the g*M query rows of a kv head fit in one pass of 16
    int attn_nk;            // groups of 16 keys per wavefront and work item (1 or 2)
    // The rows written in this step are either the tail of the sequence's last key block (attn_tail = M,
    // attn_sep = 0), or no block's business: then the work items that put the blocks together also do
    // the attention over these rows (attn_tail = 0, attn_sep = 1; see ps_draft_step for when)
    int attn_tail, attn_sep;
    int attn_merge_items;   // (sequence, kv head, 8 query rows) of the sequences that span several key blocks
    // bf16 storage (attn_phase2): blocks of 2^attn_ch_log cache keys, passes of 16 query rows per kv head,
    // work units = blocks x passes
    int attn_ch_log, attn_npass, attn_units;
    unsigned pass_magic;    // ceil(2^32 / attn_npass)
    int fused_nwg, fused_lds;
    long long kv_off[PS_MAX_ROWS];
    int kv_len[PS_MAX_ROWS];
    // Sequences that accepted fewer than n_new tokens: sequence b uses the last n_new - skip[b] of its n_new slots
    // of real rows.  The rows of the unused slots run through the step as zero rows that nobody sees: they are
    // no keys, get no cache rows, and the positions of the sequence's rows start at kv_len[b] behind them.
    int skip[PS_MAX_ROWS];
    unsigned m_magic, r_magic;   // ceil(2^32 / M), ceil(2^32 / R): row -> sequence without a division
    int tph_log;                 // log2(head_dim / 16): QKV tile -> head
    PhaseDesc ph[PH_COUNT];
    unsigned long long* timeline; // debugging aid: per-workgroup time stamps, or NULL
};

// One compiled instantiation of the device code (storage type x head_dim) and its launchers.
struct PsInstance {
    int dtype, head_dim;
    hipError_t (*prepare)(int lds_limit);   // raises the dynamic-LDS limit of every kernel
    hipError_t (*launch_multi)(const StepParams& P, hipStream_t stream, hipEvent_t* events);
    hipError_t (*launch_fused)(const StepParams& P, hipStream_t stream);
    hipError_t (*launch_probs)(const StepParams& P, hipStream_t stream);
    hipError_t (*launch_fc)(const StepParams& P, hipStream_t stream);
    // workgroups of the persistent kernel (mt column tiles, lds bytes of dynamic LDS) a compute unit can hold
    hipError_t (*fused_resident)(int mt, int lds, int* per_cu);
    // copies one phase's weight matrix (T tiles x Kt steps, of which the first Kreal hold weights
    // and the rest zeros) into streaming order at dst (T*Kt KiB)
    hipError_t (*pack)(const StepParams& P, int ph, int T, int Kt, int Kreal, char* dst, hipStream_t stream);
};
const PsInstance* ps_instance_f32_d64();
const PsInstance* ps_instance_f32_d128();
const PsInstance* ps_instance_bf16_d64();
const PsInstance* ps_instance_bf16_d128();
