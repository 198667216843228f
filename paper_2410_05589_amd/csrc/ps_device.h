// Device code of the parallel draft step for CDNA4 (gfx950, 64-lane wavefronts).  Included by
// ps_inst.hip, which is compiled once per (storage type, head_dim).
//
// The step (Section 4.1 "Inference": one drafter forward over the n_new real rows plus k [MASK]
// rows; Section 5.1: the drafter is one Llama-style layer; Section 4.3: shared LM head) is five
// weight-streaming small-M GEMM phases plus attention:
//
//   QKV     RMSNorm(Z; g_in) . [Wq;Wk;Wv]^T   -> rotary -> q_buf, K/V cache rows
//   ATTN    per (sequence, kv head, key chunk) partial softmax.V, merged by the last chunk
//   OPROJ   Y  = Z + O . Wo^T
//   GATEUP  U  = silu(RMSNorm(Y; g_post) . Wg^T) * (RMSNorm(Y; g_post) . Wu^T)
//   DOWN    Y2 = Y + U . Wd^T
//   LMHEAD  logits = RMSNorm(Y2[rows]; g_final) . Wlm^T -> per-workgroup (max, sum exp, top-k)
//   MERGE   per row: log-sum-exp, top-k ids and probabilities
//
// They run either as one persistent kernel (one 512-thread workgroup per compute unit, no grid
// barriers, the next phase's first weight loads already in flight while a workgroup waits for its
// activations) or as one kernel per phase (profiling).
//
// GEMM engine.  Weights are the 16-row MFMA operand.  At init they are repacked so that one
// step (64 bytes of each of a tile's 16 rows) is one contiguous KiB in lane order; a wavefront
// streams its tiles with 16-byte non-temporal loads, PS_U in flight per lane, waiting only for
// the oldest.  The few activation rows are the 16-column operand, staged once per workgroup in LDS.
// bf16 weights use v_mfma_f32_16x16x32_bf16 twice per step: the fp32 activations are split into
// a bf16 high and a bf16 low part (x = hi + lo to ~2^-17), so products with the exactly-bf16
// weights keep fp32-class accuracy at no extra weight traffic.  f32 weights use
// v_mfma_f32_16x16x4_f32.  Accumulation is fp32.  RMSNorm is folded in: the panel holds
// x (.) gain, the per-row factor 1/rms multiplies the accumulator in the epilogue.
// The contraction dimension of a tile is shared by 1, 2, 4 or 8 wavefronts of one workgroup;
// their partial sums meet in LDS and are added in a fixed order.
//
// Data that one workgroup writes and another reads inside the same step (activations between
// phases, attention partials, LM-head statistics) is exchanged WITHOUT barriers, counters or
// fences, with agent-scope (sc1) buffer accesses that write through / bypass the per-XCD L2:
// activations are plain fp32 where the bit pattern 0xFFFFFFFF means "not written yet"; the other
// buffers hold 8-byte units {value, sequence number of the step}.  A consumer simply re-reads
// until the data is there.  The persistent kernel therefore has no grid-wide synchronisation:
// each workgroup walks through the phases at its own pace and waits only for the data it needs.
#pragma once
#include "ps_internal.h"
#include <type_traits>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned long long u64;

struct bf16_t { uint16_t v; };   // tag type for bf16 storage

template <typename WT> struct Traits;
template <> struct Traits<float> {
    static constexpr bool BF = false;
    static constexpr int KSTEP = 16; // elements per 64-byte step
    static constexpr int GE = 4;     // elements per 16-byte group
    static constexpr int ESZ = 4;
};
template <> struct Traits<bf16_t> {
    static constexpr bool BF = true;
    static constexpr int KSTEP = 32;
    static constexpr int GE = 8;
    static constexpr int ESZ = 2;
};

// ------------------------------------------------------------------------------------------
// small helpers
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {   // round to nearest even, finite inputs
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint4 ldg_stream16(const void* p) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ uint4 ld16(const void* p) { return *reinterpret_cast<const uint4*>(p); }

// GE stored elements (16 bytes) -> floats
template <typename WT> __device__ __forceinline__ void unpack_group(uint4 v, float* out);
template <> __device__ __forceinline__ void unpack_group<float>(uint4 v, float* out) {
    out[0] = __uint_as_float(v.x); out[1] = __uint_as_float(v.y);
    out[2] = __uint_as_float(v.z); out[3] = __uint_as_float(v.w);
}
template <> __device__ __forceinline__ void unpack_group<bf16_t>(uint4 v, float* out) {
    out[0] = bf16_to_f32(v.x & 0xFFFFu); out[1] = bf16_to_f32(v.x >> 16);
    out[2] = bf16_to_f32(v.y & 0xFFFFu); out[3] = bf16_to_f32(v.y >> 16);
    out[4] = bf16_to_f32(v.z & 0xFFFFu); out[5] = bf16_to_f32(v.z >> 16);
    out[6] = bf16_to_f32(v.w & 0xFFFFu); out[7] = bf16_to_f32(v.w >> 16);
}
template <typename WT> __device__ __forceinline__ void load_group(const void* p, float* out) {
    unpack_group<WT>(ld16(p), out);
}
// 4 stored elements -> floats
template <typename WT> __device__ __forceinline__ f32x4 load4(const void* p);
template <> __device__ __forceinline__ f32x4 load4<float>(const void* p) {
    return *reinterpret_cast<const f32x4*>(p);
}
template <> __device__ __forceinline__ f32x4 load4<bf16_t>(const void* p) {
    uint2 v = *reinterpret_cast<const uint2*>(p);
    f32x4 r = {bf16_to_f32(v.x & 0xFFFFu), bf16_to_f32(v.x >> 16), bf16_to_f32(v.y & 0xFFFFu), bf16_to_f32(v.y >> 16)};
    return r;
}

// ---- agent-scope ("coherent") access.  Wide accesses go through buffer instructions with the
// sc1 bit; the descriptor's base must be wavefront-uniform, offsets are 32-bit byte offsets.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0xFFFFFFFFu, 0x00020000);
}
#define PS_SC1 16
__device__ __forceinline__ u32x4 coh_ld16(rsrc_t r, unsigned off) { return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, PS_SC1); }
__device__ __forceinline__ u32x2 coh_ld8(rsrc_t r, unsigned off) { return __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, PS_SC1); }
__device__ __forceinline__ unsigned coh_ld4(rsrc_t r, unsigned off) { return __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, PS_SC1); }
__device__ __forceinline__ void coh_st16(rsrc_t r, unsigned off, u32x4 v) { __builtin_amdgcn_raw_buffer_store_b128(v, r, off, 0, PS_SC1); }
__device__ __forceinline__ void coh_st8(rsrc_t r, unsigned off, u32x2 v) { __builtin_amdgcn_raw_buffer_store_b64(v, r, off, 0, PS_SC1); }
__device__ __forceinline__ void coh_st4(rsrc_t r, unsigned off, unsigned v) { __builtin_amdgcn_raw_buffer_store_b32(v, r, off, 0, PS_SC1); }
__device__ __forceinline__ f32x4 coh_ld_f4(rsrc_t r, unsigned off) { return __builtin_bit_cast(f32x4, coh_ld16(r, off)); }
__device__ __forceinline__ void coh_st_f4(rsrc_t r, unsigned off, f32x4 v) { coh_st16(r, off, __builtin_bit_cast(u32x4, v)); }
__device__ __forceinline__ float coh_ld_f(rsrc_t r, unsigned off) { return __uint_as_float(coh_ld4(r, off)); }
__device__ __forceinline__ void coh_st_f(rsrc_t r, unsigned off, float v) { coh_st4(r, off, __float_as_uint(v)); }

// per-lane 64-bit addresses (KV-cache rows): relaxed agent-scope atomics, dword granularity
__device__ __forceinline__ void st_agent_u32(void* p, unsigned v) {
    __hip_atomic_store((unsigned*)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned ld_agent_u32(const void* p) {
    return __hip_atomic_load((const unsigned*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// ---- sequence-tagged exchange: element i of such a buffer is the 8-byte unit {value, seq} at
// byte offset 8 i.  Four consecutive elements are moved as two 16-byte accesses.
struct LL4 { u32x4 a, b; };
__device__ __forceinline__ void ll_st4(rsrc_t r, unsigned i, f32x4 v, unsigned seq) {
    const u32x4 a = {__float_as_uint(v[0]), seq, __float_as_uint(v[1]), seq};
    const u32x4 b = {__float_as_uint(v[2]), seq, __float_as_uint(v[3]), seq};
    coh_st16(r, i * 8, a);
    coh_st16(r, i * 8 + 16, b);
}
__device__ __forceinline__ void ll_st1(rsrc_t r, unsigned i, float v, unsigned seq) {
    const u32x2 a = {__float_as_uint(v), seq};
    coh_st8(r, i * 8, a);
}
__device__ __forceinline__ LL4 ll_ld4(rsrc_t r, unsigned i) {
    LL4 x;
    x.a = coh_ld16(r, i * 8);
    x.b = coh_ld16(r, i * 8 + 16);
    return x;
}
__device__ __forceinline__ bool ll_ok(const LL4& x, unsigned seq) {
    return x.a[1] == seq && x.a[3] == seq && x.b[1] == seq && x.b[3] == seq;
}
__device__ __forceinline__ f32x4 ll_val(const LL4& x) {
    const f32x4 v = {__uint_as_float(x.a[0]), __uint_as_float(x.a[2]), __uint_as_float(x.b[0]), __uint_as_float(x.b[2])};
    return v;
}
// Bounded wait: a consumer that never sees its data (a workgroup of the grid that got no compute unit
// because other work holds it, or a fault elsewhere) raises the context's error flag and goes on, so the
// kernel always terminates; the merge of the output rows then marks the step's outputs (lm_merge_row).
__device__ __forceinline__ bool spin_again(const StepParams& P, int& spins) {
    __builtin_amdgcn_s_sleep(2);
    if (++spins > P.spin_limit) {
        __hip_atomic_store(P.error_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");   // the flag is out before anything this thread publishes later
        return false;
    }
    return true;
}
// ---- sentinel-coded exchange for the activation buffers (the bulk of the exchanged bytes, read
// by every workgroup): plain fp32 values, "not written yet" is the bit pattern 0xFFFFFFFF (a NaN no
// computation on finite inputs produces).  Each buffer exists twice; step n uses copy n & 1, and
// whoever writes element i of the current copy also resets element i of the other copy, so the
// copy the next step uses is clean again without a separate clearing pass.
#define PS_SENT 0xFFFFFFFFu
struct SxBuf { rsrc_t cur, alt; };
// The step's sequence number.  It lives in device memory (the kernel arguments of a replayed
// graph launch never change): thread 0 of every workgroup reads the counter when the kernel
// starts and leaves number = counter + 1 in LDS (step_begin); the last workgroup to do so
// advances the counter for the next launch (step_end).
typedef __attribute__((address_space(3))) unsigned lds_u32;
__device__ __forceinline__ unsigned ps_seq() {
    return __builtin_amdgcn_readfirstlane(*(const lds_u32*)(unsigned)PS_LDS_SEQ);
}
// The sequences' cache lengths: every workgroup copies them into LDS when the kernel starts (kv_fill), from
// the kernel arguments or, if the caller keeps them in device memory (so that a replayed graph can move on),
// from there.  Readers come after at least one barrier.
typedef __attribute__((address_space(3))) int lds_i32;
__device__ __forceinline__ void kv_fill(const StepParams& P) {
    if (threadIdx.x >= 64) return;
    const int lane = threadIdx.x;
    int v = 0;
    if (P.kv_len_dev) {
        if (lane < P.B) v = __builtin_nontemporal_load(P.kv_len_dev + lane);
    } else {
        for (int b = 0; b < P.B; ++b) v = lane == b ? P.kv_len[b] : v;   // (uniform index: the arguments stay scalar data)
    }
    int sk = 0;
    for (int b = 0; b < P.B; ++b) sk = lane == b ? P.skip[b] : sk;
    if (lane < P.B) { ((lds_i32*)(unsigned)PS_LDS_KVLEN)[lane] = v; ((lds_i32*)(unsigned)PS_LDS_SKIP)[lane] = sk; }
}
__device__ __forceinline__ int kvlen(int b) { return ((const lds_i32*)(unsigned)PS_LDS_KVLEN)[b]; }
// unused leading slots of sequence b's real rows (see StepParams::skip); readers come after a barrier
__device__ __forceinline__ int skipof(int b) { return ((const lds_i32*)(unsigned)PS_LDS_SKIP)[b]; }
__device__ __forceinline__ int skipof_u(int b) { return __builtin_amdgcn_readfirstlane(skipof(b)); }
__device__ __forceinline__ int kvlen_u(int b) { return __builtin_amdgcn_readfirstlane(kvlen(b)); }   // wavefront-uniform b

// Exchange buffers exist twice; P holds the addresses in copy 0, step n uses copy n & 1
__device__ __forceinline__ const char* act_ptr(const StepParams& P, const void* copy0) {
    return reinterpret_cast<const char*>(copy0) + (ps_seq() & 1u) * P.act_bytes;
}
__device__ __forceinline__ SxBuf sx_buf(const StepParams& P, const void* copy0) {
    const unsigned par = ps_seq() & 1u;
    const char* base = reinterpret_cast<const char*>(copy0);
    SxBuf b;
    b.cur = make_rsrc(base + par * P.act_bytes);
    b.alt = make_rsrc(base + (1u - par) * P.act_bytes);
    return b;
}
__device__ __forceinline__ void sx_st4(const SxBuf& b, unsigned i, f32x4 v) {
    coh_st16(b.cur, i * 4, __builtin_bit_cast(u32x4, v));
    const u32x4 sent = {PS_SENT, PS_SENT, PS_SENT, PS_SENT};
    coh_st16(b.alt, i * 4, sent);
}
__device__ __forceinline__ void sx_st1(const SxBuf& b, unsigned i, float v) {
    coh_st4(b.cur, i * 4, __float_as_uint(v));
    coh_st4(b.alt, i * 4, PS_SENT);
}
// Keeping the copies clean without the host.  A step writes its footprint - its Mtot activation rows, a
// prefix of every sliced phase's fragment buffer, the slices' sums of squares - into its own copy and resets
// exactly that in the other copy.  The other copy was last written by the previous step; whatever of that
// step's footprint exceeds this one's (more rows, more column tiles, more K-slices) is reset here, at the end
// of the kernel where most workgroups have nothing left to do, so the next step finds its whole copy clean
// whatever shapes came before.  The footprints of the two latest steps live in device memory (foot_mem[n & 1]
// is written when step n ends and read by step n + 1), so a launch replayed from a graph works among steps
// of other shapes.
__device__ __forceinline__ void sx_reset_stale(const StepParams& P, int wg, int nwg) {
    const unsigned seq = ps_seq(), par = seq & 1u;
    const unsigned* prev = P.foot_mem + ((seq - 1u) & 1u) * PS_FOOT_INTS;
    const u32x4 sent = {PS_SENT, PS_SENT, PS_SENT, PS_SENT};
    const unsigned rows_prev = __builtin_amdgcn_readfirstlane(ld_agent_u32(prev));
    if (rows_prev > (unsigned)P.Mtot) {
        const float* bufs[7] = {P.q_buf, P.kvnew, P.o_buf, P.y_buf, P.u_buf, P.y2_buf, P.x_buf};
        const int lds[7] = {P.QD, 2 * P.KVD, P.QD, P.H, P.F, P.H, P.H};   // elements per row: multiples of 4
#pragma unroll
        for (int i = 0; i < 7; ++i) {
            if (!bufs[i]) continue;
            const rsrc_t alt = make_rsrc(reinterpret_cast<const char*>(bufs[i]) + (1u - par) * P.act_bytes);
            const unsigned lo = (unsigned)P.Mtot * lds[i], hi = rows_prev * lds[i];
            for (unsigned e = lo + 4u * (wg * PS_WG_THREADS + threadIdx.x); e < hi; e += 4u * nwg * PS_WG_THREADS)
                coh_st16(alt, e * 4, sent);
        }
    }
    for (int ph = 0; ph < PH_COUNT; ++ph) {
        if (!P.ph[ph].frag) continue;
        const unsigned fp = __builtin_amdgcn_readfirstlane(ld_agent_u32(prev + 1 + ph)), fc = P.foot[1 + ph];
        if (fp > fc) {   // 16-byte units [fc, fp) of the fragments
            const rsrc_t alt = make_rsrc(reinterpret_cast<const char*>(P.ph[ph].frag) + (1u - par) * P.act_bytes);
            for (unsigned u = fc + wg * PS_WG_THREADS + threadIdx.x; u < fp; u += nwg * PS_WG_THREADS) coh_st16(alt, u * 16, sent);
        }
        const unsigned sp = __builtin_amdgcn_readfirstlane(ld_agent_u32(prev + 1 + PH_COUNT + ph)), sc = P.foot[1 + PH_COUNT + ph];
        if (wg == 0 && sp > 0 && (sp > sc || rows_prev > (unsigned)P.Mtot)) {   // [slice][PS_MAX_ROWS] sums of squares
            const rsrc_t alt = make_rsrc(reinterpret_cast<const char*>(P.ph[ph].ssq_frag) + (1u - par) * P.act_bytes);
            for (unsigned x = threadIdx.x; x < sp * PS_MAX_ROWS; x += PS_WG_THREADS) {
                const unsigned sl = x / PS_MAX_ROWS, r = x % PS_MAX_ROWS;
                if (r < rows_prev && !(sl < sc && r < (unsigned)P.Mtot)) coh_st4(alt, x * 4, PS_SENT);
            }
        }
    }
}
__device__ __forceinline__ bool sx_ok(u32x4 x) {
    return x[0] != PS_SENT && x[1] != PS_SENT && x[2] != PS_SENT && x[3] != PS_SENT;
}
__device__ __forceinline__ f32x4 sx_wait4(const StepParams& P, rsrc_t r, unsigned i) {
    int spins = 0;
    for (;;) {
        const u32x4 x = coh_ld16(r, i * 4);
        if (__all(sx_ok(x)) || !spin_again(P, spins)) return __builtin_bit_cast(f32x4, x);
    }
}

// 4 values -> the cache's storage type: stores them, returns them as stored (widened again)
// (do_store false: only the rounding)
template <typename WT> __device__ __forceinline__ f32x4 store4(void* p, f32x4 v, bool do_store = true);
template <> __device__ __forceinline__ f32x4 store4<float>(void* p, f32x4 v, bool do_store) {
    if (do_store) *reinterpret_cast<f32x4*>(p) = v;
    return v;
}
template <> __device__ __forceinline__ f32x4 store4<bf16_t>(void* p, f32x4 v, bool do_store) {
    const unsigned b0 = f32_to_bf16(v[0]), b1 = f32_to_bf16(v[1]), b2 = f32_to_bf16(v[2]), b3 = f32_to_bf16(v[3]);
    uint2 o;
    o.x = b0 | (b1 << 16);
    o.y = b2 | (b3 << 16);
    if (do_store) *reinterpret_cast<uint2*>(p) = o;
    const f32x4 r = {bf16_to_f32(b0), bf16_to_f32(b1), bf16_to_f32(b2), bf16_to_f32(b3)};
    return r;
}

// ---- wavefront reductions with DPP (row = 16 lanes); the result is returned to every lane.
// Order of the combination is fixed, so float sums are reproducible.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ unsigned dpp_u32(unsigned self, unsigned v) {
    return (unsigned)__builtin_amdgcn_update_dpp((int)self, (int)v, CTRL, ROW_MASK, 0xF, false);
}
#define PS_DPP_STEPS(COMBINE)                                                        \
    COMBINE(0xB1, 0xF)  /* quad_perm [1,0,3,2] */                                    \
    COMBINE(0x4E, 0xF)  /* quad_perm [2,3,0,1] */                                    \
    COMBINE(0x141, 0xF) /* row_half_mirror */                                        \
    COMBINE(0x140, 0xF) /* row_mirror */                                             \
    COMBINE(0x142, 0xA) /* row_bcast:15 into rows 1 and 3 */                         \
    COMBINE(0x143, 0xC) /* row_bcast:31 into rows 2 and 3 */
__device__ __forceinline__ float wave_sum(float v) {
#define PS_C(CTRL, RM) { const float o = __uint_as_float(dpp_u32<CTRL, RM>(0u, __float_as_uint(v))); v += o; }
    // lanes outside the row mask receive 0 (old value) and add 0
    PS_DPP_STEPS(PS_C)
#undef PS_C
    return __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(v), 63));
}
__device__ __forceinline__ unsigned wave_max_u32(unsigned v) {
#define PS_C(CTRL, RM) { const unsigned o = dpp_u32<CTRL, RM>(0u, v); v = o > v ? o : v; }
    PS_DPP_STEPS(PS_C)
#undef PS_C
    return __builtin_amdgcn_readlane(v, 63);
}
// float maximum through the order-preserving map to unsigned (finite values and infinities): the
// unsigned reduction folds each lane exchange into its max instruction, the float one does not
__device__ __forceinline__ float wave_max(float v) {
    const unsigned u = __float_as_uint(v);
    const unsigned m = wave_max_u32(u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u));
    return __uint_as_float(m ^ ((m >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}
// maximum of 64-bit keys as two 32-bit reductions: the high words first, then the low words of
// the lanes that hold the winning high word
__device__ __forceinline__ u64 wave_max_u64(u64 v) {
    const unsigned hi = wave_max_u32((unsigned)(v >> 32));
    const unsigned lo = wave_max_u32((unsigned)(v >> 32) == hi ? (unsigned)v : 0u);
    return ((u64)hi << 32) | lo;
}

// The same reductions over a DPP row (16 lanes): four exchanges, the result in every lane of the row
#define PS_DPP_ROW_STEPS(COMBINE)                                                    \
    COMBINE(0xB1, 0xF)  /* quad_perm [1,0,3,2] */                                    \
    COMBINE(0x4E, 0xF)  /* quad_perm [2,3,0,1] */                                    \
    COMBINE(0x141, 0xF) /* row_half_mirror */                                        \
    COMBINE(0x140, 0xF) /* row_mirror */
__device__ __forceinline__ float row_sum(float v) {
#define PS_C(CTRL, RM) { const float o = __uint_as_float(dpp_u32<CTRL, RM>(0u, __float_as_uint(v))); v += o; }
    PS_DPP_ROW_STEPS(PS_C)
#undef PS_C
    return v;
}
__device__ __forceinline__ unsigned row_max_u32(unsigned v) {
#define PS_C(CTRL, RM) { const unsigned o = dpp_u32<CTRL, RM>(0u, v); v = o > v ? o : v; }
    PS_DPP_ROW_STEPS(PS_C)
#undef PS_C
    return v;
}
__device__ __forceinline__ float row_max(float v) {
    const unsigned u = __float_as_uint(v);
    const unsigned m = row_max_u32(u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u));
    return __uint_as_float(m ^ ((m >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}
__device__ __forceinline__ u64 row_max_u64(u64 v) {
    const unsigned hi = row_max_u32((unsigned)(v >> 32));
    const unsigned lo = row_max_u32((unsigned)(v >> 32) == hi ? (unsigned)v : 0u);
    return ((u64)hi << 32) | lo;
}
// over LPR = 64 (the wavefront) or 16 (a row) lanes
template <int LPR> __device__ __forceinline__ float grp_sum(float v) { if constexpr (LPR == 64) return wave_sum(v); else return row_sum(v); }
template <int LPR> __device__ __forceinline__ float grp_max(float v) { if constexpr (LPR == 64) return wave_max(v); else return row_max(v); }
template <int LPR> __device__ __forceinline__ u64 grp_max_u64(u64 v) { if constexpr (LPR == 64) return wave_max_u64(v); else return row_max_u64(v); }

// ---- top-k keys: (logit, id) packed so that unsigned comparison orders by larger logit first,
// equal logits by lower id.  Key 0 means "none".
__device__ __forceinline__ u64 make_key(float v, int id) {
    const unsigned u = __float_as_uint(v);
    const unsigned ord = u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
    return ((u64)ord << 32) | (unsigned)(0x7FFFFFFF - id);
}
__device__ __forceinline__ float key_value(u64 k) {
    const unsigned ord = (unsigned)(k >> 32);
    return __uint_as_float(ord ^ ((ord >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}
__device__ __forceinline__ int key_id(u64 k) { return 0x7FFFFFFF - (int)(unsigned)k; }

// The draw of the sampling epilogue (Algorithm 1's draft line samples from the draft distributions): the
// Gumbel-max construction, token = argmax_i (z_i + g_i) with g_i = -log(-log(u_i)), which is an exact sample of
// softmax(z).  u_i for output row `row` and token `id` comes from a counter-based generator: three rounds of
// MurmurHash3's 32-bit finaliser over the seed's low word plus 0x9E3779B9 (row + 1), then the seed's high word,
// then id * 0x9E3779B1 + 0x7F4A7C15; u = ((h >> 9) + 0.5) 2^-23 lies in (0, 1) and is exact in float32.
__device__ __forceinline__ unsigned fmix32(unsigned h) {
    h ^= h >> 16; h *= 0x85EBCA6Bu; h ^= h >> 13; h *= 0xC2B2AE35u; h ^= h >> 16;
    return h;
}
__device__ __forceinline__ float gumbel_of(const StepParams& P, int row, int id) {
    unsigned x = fmix32(P.seed_lo + 0x9E3779B9u * (unsigned)(row + 1));
    x = fmix32(x ^ P.seed_hi);
    x = fmix32(x ^ ((unsigned)id * 0x9E3779B1u + 0x7F4A7C15u));
    const float u = ((float)(x >> 9) + 0.5f) * 1.1920928955078125e-07f;
    return -logf(-logf(u));
}

// Row m of the step's activation matrix Z = [x rows ; mask embeddings] (Section 4.1: the k
// [MASK] tokens are appended after the sequence), element offset e.
// m / M for the small row counts of a step, with the reciprocal the host prepared
__device__ __forceinline__ int row_seq(const StepParams& P, int m) {
    return P.M == 1 ? m : (int)__umulhi((unsigned)m, P.m_magic);
}
// token id of real row (b, i) (token-id input modes)
__device__ __forceinline__ int tok_of(const StepParams& P, int b, int i) {
    return __builtin_amdgcn_readfirstlane(P.token_ids[b * P.n_new + i]);
}
// 4 elements of row m of Z from column e on, as floats.  Real rows: the caller's hidden states, a row of the
// embedding table, or the input projection's output (exchanged fp32, complete since that kernel ended).
template <typename WT>
__device__ __forceinline__ f32x4 load_z4(const StepParams& P, int m, int e) {
    const int b = row_seq(P, m), i = m - b * P.M;
    if (i >= P.n_new) return load4<WT>((const char*)P.mask_emb + ((long long)(i - P.n_new) * P.H + e) * Traits<WT>::ESZ);
    if (i < skipof(b)) return f32x4{0.f, 0.f, 0.f, 0.f};   // an unused slot: a zero row
    if (P.in_mode == PS_IN_HIDDEN) return load4<WT>((const char*)P.x + ((long long)(b * P.n_new + i) * P.H + e) * Traits<WT>::ESZ);
    if (P.in_mode == PS_IN_TOKENS)
        return load4<WT>((const char*)P.embed + ((long long)P.token_ids[b * P.n_new + i] * P.H + e) * Traits<WT>::ESZ);
    return *reinterpret_cast<const f32x4*>(act_ptr(P, P.x_buf) + ((size_t)m * P.H + e) * 4);
}

// Debugging aid (builds with -DPS_TIMELINE only): thread 0 of every workgroup notes the shader
// clock at point `ev` in the top 512 bytes of LDS; flush_stamps copies them out at the end
// together with the 100 MHz wall clock of the kernel's start and end.
#define PS_TL_OFF (PS_LDS_BYTES - 512)
#ifdef PS_TIMELINE
typedef __attribute__((address_space(3))) unsigned long long lds_u64;
// the kernels have no static LDS: dynamic LDS starts at LDS address 0
__device__ __forceinline__ volatile lds_u64* tl_slot(int ev) { return (volatile lds_u64*)(unsigned)(PS_TL_OFF + 8 * ev); }
#endif
__device__ __forceinline__ void stamp(const StepParams& P, int wg, int ev) {
#ifdef PS_TIMELINE
    if (P.timeline && threadIdx.x == 0) *tl_slot(ev) = __builtin_amdgcn_s_memtime();
#endif
}
__device__ __forceinline__ void stamp_wall(const StepParams& P, int wg, int ev) {
#ifdef PS_TIMELINE
    if (P.timeline && threadIdx.x == 0) *tl_slot(ev) = wall_clock64();
#endif
}
__device__ __forceinline__ void flush_stamps(const StepParams& P, int wg) {
#ifdef PS_TIMELINE
    __syncthreads();
    if (P.timeline && threadIdx.x < 64) P.timeline[(size_t)threadIdx.x * 1024 + wg] = *tl_slot(threadIdx.x);
#endif
}

// ------------------------------------------------------------------------------------------
// which weight row a lane of the init-time packing kernel copies
// ------------------------------------------------------------------------------------------
template <typename WT, int PH>
__device__ __forceinline__ const char* weight_row_ptr(const StepParams& P, int tau, int i) {
    constexpr int ESZ = Traits<WT>::ESZ;
    if (PH == PH_QKV) {
        // tile = 8 features of a head's first half + their 8 rotary partners in the second half
        const int tph = P.d >> 4;
        const int hh = tau / tph, sub = tau - hh * tph;
        const int rin = (i < 8) ? (8 * sub + i) : ((P.d >> 1) + 8 * sub + (i - 8));
        const char* base; int row;
        if (hh < P.nq) { base = (const char*)P.wq; row = hh * P.d + rin; }
        else if (hh < P.nq + P.nkv) { base = (const char*)P.wk; row = (hh - P.nq) * P.d + rin; }
        else { base = (const char*)P.wv; row = (hh - P.nq - P.nkv) * P.d + rin; }
        return base + (size_t)row * P.H * ESZ;
    } else if (PH == PH_OPROJ) {
        return (const char*)P.wo + (size_t)(16 * tau + i) * P.QD * ESZ;
    } else if (PH == PH_GATEUP) {
        // tile = 8 gate rows + the 8 up rows of the same features
        return (i < 8) ? (const char*)P.w_gate + (size_t)(8 * tau + i) * P.H * ESZ
                       : (const char*)P.w_up + (size_t)(8 * tau + i - 8) * P.H * ESZ;
    } else if (PH == PH_DOWN) {
        return (const char*)P.w_down + (size_t)(16 * tau + i) * P.F * ESZ;
    } else if (PH == PH_FC) {
        return (const char*)P.w_fc + (size_t)(16 * tau + i) * (2 * P.H) * ESZ;
    } else {
        int row = 16 * tau + i;
        if (row >= P.V) row = P.V - 1;   // ragged last vocabulary tile: clamp, masked in the epilogue
        return (const char*)P.w_lm + (size_t)row * P.H * ESZ;
    }
}

// Panel row r of the LM head is a decoding row: the last real row and the k mask rows of each
// sequence (or all rows).
__device__ __forceinline__ int lm_src_row(const StepParams& P, int r) {
    const int b = P.R == 1 ? r : (int)__umulhi((unsigned)r, P.r_magic), jj = r - b * P.R;
    return b * P.M + (P.all_rows ? jj : (P.n_new - 1 + jj));
}

// ------------------------------------------------------------------------------------------
// inner loop
// ------------------------------------------------------------------------------------------
// B operands (activation columns) of one step for all column tiles, read from the LDS panel
template <typename WT, int MT> struct BRegs { uint4 h[MT]; uint4 l[MT]; };

// (the panel's addresses are kept as LDS pointers, not generic ones: a generic pointer that the compiler
// cannot trace back to LDS becomes a flat load, which counts as a global-memory operation and makes every
// wait in the streaming loop wait for all the weight loads in flight)
typedef const __attribute__((address_space(3))) char* lds_cptr;
__device__ __forceinline__ uint4 ld16_lds(lds_cptr p) {
    const u32x4 v = *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(p);
    return make_uint4(v[0], v[1], v[2], v[3]);
}
template <typename WT, int MT>
__device__ __forceinline__ void load_b(BRegs<WT, MT>& b, const lds_cptr (&pa)[MT], const int (&pinc)[MT],
                                       const int (&plo)[MT], int t) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const lds_cptr p = pa[mt] + t * pinc[mt];
        b.h[mt] = ld16_lds(p);
        if constexpr (Traits<WT>::BF) b.l[mt] = ld16_lds(p + plo[mt]);
    }
}

template <typename WT, int MT>
__device__ __forceinline__ void mma_step(uint4 w, const BRegs<WT, MT>& b, f32x4 (&acc)[MT]) {
    if constexpr (Traits<WT>::BF) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, w);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, b.h[mt]), acc[mt], 0, 0, 0);
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, b.l[mt]), acc[mt], 0, 0, 0);
        }
    } else {
        const f32x4 a = __builtin_bit_cast(f32x4, w);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const f32x4 bv = __builtin_bit_cast(f32x4, b.h[mt]);
#pragma unroll
            for (int e = 0; e < 4; ++e)
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[e], bv[e], acc[mt], 0, 0, 0);
        }
    }
}

constexpr int PS_WS = 1024;   // prepacked weights: one step of a tile = 64 lanes x 16 B, contiguous

// Issues the first PS_U loads of a weight stream (base is wavefront-uniform, lane16 = 16 * lane).
// Weights do not depend on the activations, so this runs before the panel is staged: the HBM
// pipe stays busy while the activations arrive.
__device__ __forceinline__ void preload_weights(uint4 (&wb)[PS_U], const char* base, int lane16) {
#pragma unroll
    for (int u = 0; u < PS_U; ++u) wb[u] = ldg_stream16(base + u * PS_WS + lane16);
}

// Software pipeline over the n steps (a positive multiple of PS_U) of one weight stream: step t
// multiplies the weights loaded PS_U steps earlier with the B operands read one step earlier,
// then refills its register with step t + PS_U and reads the B operands of step t + 1.  The
// loads of the last group start the wavefront's next stream, so when this returns wb holds the
// head of that stream.  Every load is unconditional and only the oldest is waited for.
template <typename WT, int MT>
__device__ __forceinline__ void consume_weights(uint4 (&wb)[PS_U], const char* wp, int n, const char* next_wp, int lane16,
                                                const lds_cptr (&pa)[MT], const int (&pinc)[MT],
                                                const int (&plo)[MT], f32x4 (&acc)[MT]) {
    constexpr int U = PS_U;
    BRegs<WT, MT> bc, bn;
    load_b<WT, MT>(bc, pa, pinc, plo, 0);
    for (int t0 = 0; t0 < n; t0 += U) {
        const char* src = (t0 + U < n) ? wp + (size_t)(t0 + U) * PS_WS : next_wp;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            mma_step<WT, MT>(wb[u], bc, acc);
            wb[u] = ldg_stream16(src + u * PS_WS + lane16);   // reuses the register just consumed
            int tb = t0 + u + 1;
            if (u == U - 1 && tb >= n) tb = n - 1;            // nothing follows the last step
            load_b<WT, MT>(bn, pa, pinc, plo, tb);
            bc = bn;
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// Head of the stream of wavefront kw (of the 2^kw_log that share tile tau) inside the panel piece
// that covers groups [g_lo, g_lo + ng); a0 = the stream's first step relative to the piece,
// n = its length in steps.  The host makes sure every piece has at least 2^kw_log groups.
__device__ __forceinline__ const char* stream_ptr(const PhaseDesc& D, int tau, int g_lo, int ng, int kw, int& a0, int& n) {
    const int w0 = (kw * ng) >> D.kw_log, w1 = ((kw + 1) * ng) >> D.kw_log;
    a0 = w0 * PS_U;
    n = (w1 - w0) * PS_U;
    return D.wpack + ((size_t)tau * D.Kt + (size_t)(g_lo + w0) * PS_U) * PS_WS;
}
// The groups [lo, hi) of the contraction dimension that K-slice s of a phase covers, and the
// piece pc of it that is staged at a time.
__device__ __forceinline__ void slice_groups(const PhaseDesc& D, int s, int& lo, int& hi) {
    const int NG = D.Kt / PS_U;
    lo = (s * NG) >> D.s_log;
    hi = ((s + 1) * NG) >> D.s_log;
}
// The tile that slot `slot` of workgroup column j takes in round rd
__device__ __forceinline__ int tile_index(const PhaseDesc& D, int rd, int slot, int j) {
    return rd * D.per_round + slot * D.Gs + j;
}
// Head of the stream a wavefront reads first in phase ph (any readable address if it has none)
__device__ __forceinline__ const char* first_stream(const StepParams& P, int ph, int wg, int wave) {
    const PhaseDesc& D = P.ph[ph];
    const int s = wg & ((1 << D.s_log) - 1), j = wg >> D.s_log;
    const int tau = tile_index(D, 0, wave >> D.kw_log, j);
    if (tau >= D.T) return D.wpack;
    int lo, hi, a0, n;
    slice_groups(D, s, lo, hi);
    return stream_ptr(D, tau, lo, min(D.piece_groups, hi - lo), wave & ((1 << D.kw_log) - 1), a0, n);
}

// ------------------------------------------------------------------------------------------
// epilogues: lane (c = lane % 16, q = lane / 16) holds, for column tile mt, the outputs of
// activation row m = 16 mt + c and tile rows 4q .. 4q+3
// ------------------------------------------------------------------------------------------
template <typename WT, int MT>
__device__ __forceinline__ void epilogue_qkv(const StepParams& P, int tau, int lane, f32x4 (&acc)[MT]) {
    const int c = lane & 15, q = lane >> 4;
    const int half = P.d >> 1;
    const int hh = tau >> P.tph_log, sub = tau - (hh << P.tph_log);   // head_dim / 16 tiles per head
    const int jb = 8 * sub + 4 * (q & 1);            // rotary frequency index of this lane's 4 values
    const int f = jb + ((q >= 2) ? half : 0);        // feature inside the head
    const SxBuf rq = sx_buf(P, P.q_buf), rn = sx_buf(P, P.kvnew);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        f32x4 v = acc[mt], pv;
#pragma unroll
        for (int r = 0; r < 4; ++r) pv[r] = __shfl_xor(v[r], 32, 64);   // rotary partner (j <-> j + d/2)
        const int m = 16 * mt + c;
        if (m >= P.Mtot) continue;
        const int b = row_seq(P, m), i = m - b * P.M;
        const int sk = skipof(b);                    // unused leading slots of the sequence: they get no cache rows
        const int pos = max(kvlen(b) + i - sk, 0);   // positions continue after the valid cache rows
        f32x4 o = v;
        if (hh < P.nq + P.nkv) {
            const float2* cs = P.rope + (size_t)pos * half + jb;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float2 t = cs[r];
                o[r] = (q < 2) ? (v[r] * t.x - pv[r] * t.y) : (v[r] * t.x + pv[r] * t.y);
            }
        }
        if (hh < P.nq) {
            sx_st4(rq, (unsigned)((size_t)m * P.QD + hh * P.d + f), o);
        } else {
            // new K/V rows: into the cache in its storage type (for later steps), and - exactly as
            // stored - into the exchange buffer this step's attention reads
            const bool isk = hh < P.nq + P.nkv;
            const int hk = isk ? hh - P.nq : hh - P.nq - P.nkv;
            char* cache = (char*)(isk ? P.kc : P.vc);
            const size_t e = ((size_t)(P.kv_off[b] + pos) * P.nkv + hk) * P.d + f;
            const f32x4 stored = store4<WT>(cache + e * Traits<WT>::ESZ, o, i >= sk);
            sx_st4(rn, (unsigned)(((size_t)m * 2 + (isk ? 0 : 1)) * P.KVD + hk * P.d + f), stored);
        }
    }
}

template <typename WT, int MT>
__device__ __forceinline__ void epilogue_oproj(const StepParams& P, int tau, int lane, f32x4 (&acc)[MT]) {
    const int c = lane & 15, q = lane >> 4;
    const int n = 16 * tau + 4 * q;
    const SxBuf ry = sx_buf(P, P.y_buf);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = 16 * mt + c;
        if (m >= P.Mtot) continue;
        const f32x4 z = load_z4<WT>(P, m, n);
        sx_st4(ry, (unsigned)((size_t)m * P.H + n), z + acc[mt]);
    }
}

// input projection (Section 4.3, EAGLE integration): panel row r is real row (b, i) = (r / n_new, r % n_new);
// its output is row b M + i of Z, exchanged as fp32
template <typename WT, int MT>
__device__ __forceinline__ void epilogue_fc(const StepParams& P, int tau, int lane, f32x4 (&acc)[MT]) {
    const int c = lane & 15, q = lane >> 4;
    const int n = 16 * tau + 4 * q;
    const SxBuf rx = sx_buf(P, P.x_buf);
    f32x4 bias = {0.f, 0.f, 0.f, 0.f};
    if (P.b_fc) bias = load4<WT>((const char*)P.b_fc + (size_t)n * Traits<WT>::ESZ);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int r = 16 * mt + c;
        if (r >= P.B * P.n_new) continue;
        const int b = P.n_new == 1 ? r : (int)__umulhi((unsigned)r, P.n_magic), i = r - b * P.n_new;
        sx_st4(rx, (unsigned)((size_t)(b * P.M + i) * P.H + n), acc[mt] + bias);
    }
}

template <typename WT, int MT>
__device__ __forceinline__ void epilogue_gateup(const StepParams& P, int tau, int lane, f32x4 (&acc)[MT]) {
    const int c = lane & 15, q = lane >> 4;
    const SxBuf ru = sx_buf(P, P.u_buf);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        f32x4 up;
#pragma unroll
        for (int r = 0; r < 4; ++r) up[r] = __shfl_xor(acc[mt][r], 32, 64);   // lanes q<2: gate, q>=2: up
        const int m = 16 * mt + c;
        if (m >= P.Mtot || q >= 2) continue;
        f32x4 u;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float g = acc[mt][r];
            u[r] = g / (1.0f + expf(-g)) * up[r];
        }
        sx_st4(ru, (unsigned)((size_t)m * P.F + 8 * tau + 4 * q), u);
    }
}

template <typename WT, int MT>
__device__ __forceinline__ void epilogue_down(const StepParams& P, int tau, int lane, f32x4 (&acc)[MT]) {
    const int c = lane & 15, q = lane >> 4;
    const int n = 16 * tau + 4 * q;
    const rsrc_t ry = make_rsrc(act_ptr(P, P.y_buf));
    const SxBuf ry2 = sx_buf(P, P.y2_buf);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = 16 * mt + c;
        if (m >= P.Mtot) continue;
        const unsigned idx = (unsigned)((size_t)m * P.H + n);
        const f32x4 o = sx_wait4(P, ry, idx) + acc[mt];
        sx_st4(ry2, idx, o);
        if (P.hidden_out) *reinterpret_cast<f32x4*>(P.hidden_out + (size_t)m * P.H + n) = o;
    }
}

// LM head: logits of the workgroup's vocabulary tiles stay in LDS (s_lm[local tile][row][16])
template <typename WT, int MT>
__device__ __forceinline__ void epilogue_lm(const StepParams& P, int tau, int lane, f32x4 (&acc)[MT],
                                            float* s_lm, int lt) {
    const int c = lane & 15, q = lane >> 4;
    const int n = 16 * tau + 4 * q;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = 16 * mt + c;
        if (m >= P.Rtot) continue;
        f32x4 o = acc[mt] * P.inv_temp;      // what softmax, top-k and the draw see: logits / temperature
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (n + r >= P.V) o[r] = -INFINITY;
        *reinterpret_cast<f32x4*>(s_lm + ((size_t)lt * P.Rtot + m) * 16 + 4 * q) = o;
        if (P.logits_store) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (n + r < P.V) P.logits_store[(size_t)m * P.V + n + r] = acc[mt][r];
        }
    }
}

// ------------------------------------------------------------------------------------------
// the GEMM phase
// ------------------------------------------------------------------------------------------
__host__ __device__ inline int panel_row_stride(int panel_steps) {
    // rows are (steps x 64 B) long; the stride is padded to 64 (mod 256) bytes so the 16 rows a
    // wavefront reads in one ds_read_b128 spread over all LDS banks
    const int len = panel_steps * 64;
    return len + ((64 - (len & 255)) + 256) % 256;
}
// LDS layout of a GEMM phase (bytes from the start of dynamic LDS)
#define PS_LDS_SSQ PS_LDS_BASE   // [64 rows][8] partial sums of squares (RMSNorm); bytes below: see PS_LDS_BASE
#define PS_LDS_ZERO (PS_LDS_BASE + 2048)    // 64 zero bytes: B operand of unused MFMA columns
#define PS_LDS_RED (PS_LDS_BASE + 2304)     // [wavefronts][MT][64 lanes] f32x4: partial sums of wavefronts sharing a tile
__host__ __device__ inline int panel_offset(int mt) { return PS_LDS_RED + PS_WAVES * mt * 1024; }

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
// two floats -> two bf16 (round to nearest even) in one dword, first value in the low half
__device__ __forceinline__ unsigned pack_bf16x2(float a, float b) {
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}

// Stages steps [a_step, a_step + nsteps) of the activation panel.  The 16-byte groups of a row
// lie along 2^g2_log threads, the remaining threads take different rows; every thread requests
// its group of RB rows before it uses any of them (one memory round trip per RB rows), and
// re-requests them until none holds the "not written" pattern.  The panel holds x (.) gain
// (RMSNorm's 1/rms is applied in the epilogue); the sum of x^2 of row r over the groups a
// wavefront saw goes to s_ssq[8 r + w] (w = the wavefront's index along the row).
template <typename WT, int PH>
__device__ __forceinline__ void stage_piece(const StepParams& P, const PhaseDesc& D, int wave, char* smem,
                                            char* s_pa, char* s_pb, int a_step, int nsteps, bool first_piece,
                                            bool want_ssq) {
    constexpr bool BF = Traits<WT>::BF;
    constexpr int KSTEP = Traits<WT>::KSTEP, GE = Traits<WT>::GE, ESZ = Traits<WT>::ESZ;
    constexpr int NL = GE / 4;                       // 16-byte loads per group of exchanged fp32
    constexpr int RB = 8;                            // rows per thread requested before any is used
    constexpr bool from_x = PH == PH_QKV || PH == PH_FC;   // the step's inputs, complete at launch
    const int tid = threadIdx.x, lane = tid & 63;
    float* s_ssq = reinterpret_cast<float*>(smem + PS_LDS_SSQ);
    const int G = nsteps * 4;
    const int g2_log = D.g2_log, G2 = 1 << g2_log;
    // rows are wavefront-uniform (2^g2_log >= 64 threads lie along a row): everything that
    // depends only on the row is scalar arithmetic
    const int gi0 = tid & (G2 - 1), rsub = (wave << 6) >> g2_log, nrt = PS_WG_THREADS >> g2_log;
    const int wsub = wave & ((G2 >> 6) - 1);
    const int rows = D.rows, K = D.K, RS = D.rs, ld = D.src_ld;
    const bool norm = PH == PH_QKV || PH == PH_GATEUP || (PH == PH_LMHEAD && D.norm != 0);
    const int in_mode = P.in_mode;
    // where the rows come from.  QKV: the real rows of Z by input mode (see StepParams), the [MASK] rows from
    // mask_emb; input projection: features (columns < H) and the tokens' embedding rows (columns >= H)
    const rsrc_t rs = make_rsrc(PH == PH_FC ? P.features
                                : PH != PH_QKV ? (const void*)act_ptr(P, D.src)
                                : in_mode == PS_IN_HIDDEN ? P.x : in_mode == PS_IN_TOKENS ? P.embed : (const void*)act_ptr(P, P.x_buf));
    const rsrc_t rmask = make_rsrc(PH == PH_FC ? P.embed : P.mask_emb);
    // is row r of the QKV panel an fp32 row (the input projection's output)?
    auto fused_row = [&](int r) __attribute__((always_inline)) {
        return PH == PH_QKV && in_mode == PS_IN_FUSED && r - row_seq(P, r) * P.M < P.n_new;
    };
    for (int gc = 0; gc < G; gc += G2) {
        const int gi = gc + gi0;
        const bool gvalid = gi < G;
        const int gic = gvalid ? gi : G - 1;         // clamped: loads stay unconditional
        const int kk = a_step * KSTEP + gic * GE;
        const bool live = gvalid && kk < K;          // beyond K the packed weights are zero: so is the panel
        const int kkc = kk < K ? kk : 0;
        float gn[GE];
        if (norm) unpack_group<WT>(ld16((const char*)D.gain + (size_t)kkc * ESZ), gn);
        for (int rb = rsub; rb < rows; rb += nrt * RB) {
            u32x4 raw[RB][NL];
            int spins = 0;
            for (;;) {
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    const int r = min(rb + nrt * i, rows - 1);   // clamped: every load is unconditional
                    if (PH == PH_QKV) {
                        // row r of Z = [real rows ; mask embeddings] of its sequence
                        const int b = row_seq(P, r), ii = r - b * P.M;
                        if (ii >= P.n_new) {
                            raw[i][0] = __builtin_amdgcn_raw_buffer_load_b128(rmask, kkc * ESZ, (ii - P.n_new) * P.H * ESZ, 0);
                        } else if (in_mode == PS_IN_HIDDEN) {
                            raw[i][0] = __builtin_amdgcn_raw_buffer_load_b128(rs, kkc * ESZ, (b * P.n_new + ii) * P.H * ESZ, 0);
                        } else if (in_mode == PS_IN_TOKENS) {
                            const int tok = ii < P.skip[b] ? 0 : tok_of(P, b, ii);   // (an unused slot's token id is not read)
                            raw[i][0] = __builtin_amdgcn_raw_buffer_load_b128(rs, kkc * ESZ, tok * P.H * ESZ, 0);
                        } else {
#pragma unroll
                            for (int h = 0; h < NL; ++h)
                                raw[i][h] = __builtin_amdgcn_raw_buffer_load_b128(rs, (kkc + 4 * h) * 4, (b * P.M + ii) * P.H * 4, PS_SC1);
                        }
                    } else if (PH == PH_FC) {
                        // real row r = (b, ii): [features ; embedding of its token]
                        const int b = P.n_new == 1 ? r : (int)__umulhi((unsigned)r, P.n_magic), ii = r - b * P.n_new;
                        const int tok = ii < P.skip[b] ? 0 : tok_of(P, b, ii);
                        raw[i][0] = kkc < P.H
                            ? __builtin_amdgcn_raw_buffer_load_b128(rs, kkc * ESZ, r * P.H * ESZ, 0)
                            : __builtin_amdgcn_raw_buffer_load_b128(rmask, (kkc - P.H) * ESZ, tok * P.H * ESZ, 0);
                    } else {
                        const int srow = PH == PH_LMHEAD ? lm_src_row(P, r) : r;
#pragma unroll
                        for (int h = 0; h < NL; ++h)
                            raw[i][h] = __builtin_amdgcn_raw_buffer_load_b128(rs, (kkc + 4 * h) * 4, srow * ld * 4, PS_SC1);
                    }
                }
                if (from_x) break;
                bool ok = true;
#pragma unroll
                for (int i = 0; i < RB; ++i)
#pragma unroll
                    for (int h = 0; h < NL; ++h) ok = ok && sx_ok(raw[i][h]);
                if (__all(ok) || !spin_again(P, spins)) break;   // produced earlier in this step: wait for it
            }
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                const int r = rb + nrt * i;
                if (r >= rows) continue;
                float v[GE];
                if (from_x && !fused_row(r)) {
                    unpack_group<WT>(make_uint4(raw[i][0][0], raw[i][0][1], raw[i][0][2], raw[i][0][3]), v);
                } else {
#pragma unroll
                    for (int h = 0; h < NL; ++h)
#pragma unroll
                        for (int j = 0; j < 4; ++j) v[4 * h + j] = __uint_as_float(raw[i][h][j]);
                }
                // (the step's input rows of slots a sequence does not use are zero rows; the host array is read: this
                // runs before the workgroup's first barrier)
                bool zero_row = !live;
                if (PH == PH_QKV) {
                    const int b = row_seq(P, r), ii = r - b * P.M;
                    zero_row = zero_row || ii < P.skip[b];
                }
                float ss = 0.f;
#pragma unroll
                for (int e = 0; e < GE; ++e) {
                    if (zero_row) v[e] = 0.f;
                    if (norm) { ss += v[e] * v[e]; v[e] *= gn[e]; }
                }
                if (gvalid) {
                    if constexpr (BF) {
                        uint4 ph4, pl4;
                        unsigned* hp = &ph4.x;
                        unsigned* lp = &pl4.x;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const unsigned hi = pack_bf16x2(v[2 * j], v[2 * j + 1]);
                            hp[j] = hi;
                            lp[j] = pack_bf16x2(v[2 * j] - __uint_as_float(hi << 16), v[2 * j + 1] - __uint_as_float(hi & 0xFFFF0000u));
                        }
                        *reinterpret_cast<uint4*>(s_pa + r * RS + gi * 16) = ph4;
                        *reinterpret_cast<uint4*>(s_pb + r * RS + gi * 16) = pl4;
                    } else {
                        *reinterpret_cast<uint4*>(s_pa + r * RS + gi * 16) =
                            make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
                    }
                }
                if (norm && want_ssq) {
                    ss = wave_sum(ss);
                    if (lane == 0) s_ssq[r * 8 + wsub] = (first_piece && gc == 0) ? ss : s_ssq[r * 8 + wsub] + ss;
                }
            }
        }
    }
}

// Softmax statistics and top-k of the logits a workgroup holds in LDS (s_lm[local tile][row][16]) for its
// vocabulary tiles: per output row the maximum, the sum of exponentials against it and the topk largest keys
// in order go to lm_part as tagged data.  LPR lanes share a row; the keys are unique, so "the largest key below
// the previous winner" enumerates them in order.
template <int LPR>
__device__ __forceinline__ void lm_local_stats(const StepParams& P, const PhaseDesc& D, int j, int rows, const float* s_lm,
                                               int wave, int lane, int sl_log, int SL) {
    constexpr int GPW = 64 / LPR;               // rows a wavefront works on at a time
    constexpr int EPL = LPR == 64 ? 8 : 16;     // elements per lane kept in registers (more: re-read from LDS)
    const int n_el = D.rounds * SL * 16;
    const int li = lane & (LPR - 1), grp = lane / LPR;
    const int topk = P.topk;
    const rsrc_t rl = make_rsrc(P.lm_part);
    const unsigned stride = 4 + 2 * topk;       // tagged elements: max, sum exp, topk keys (low, high word), the draw's key
    const unsigned seq = ps_seq();
    for (int m0 = wave; m0 < rows; m0 += PS_WAVES * GPW) {
        const int mm = m0 + grp * PS_WAVES;
        const bool live = mm < rows;
        const int m = live ? mm : m0;           // lanes without a row of their own repeat the wavefront's first (and store nothing)
        u64 keys[EPL];
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
            const int x = li + LPR * i;
            keys[i] = 0;
            if (x < n_el) {
                const int lt = x >> 4;
                const float v = s_lm[(lt * rows + m) * 16 + (x & 15)];
                const int id = 16 * tile_index(D, lt >> sl_log, lt & (SL - 1), j) + (x & 15);
                if (v > -INFINITY) { keys[i] = make_key(v, id); mx = fmaxf(mx, v); }
            }
        }
        for (int x = li + LPR * EPL; x < n_el; x += LPR) mx = fmaxf(mx, s_lm[((x >> 4) * rows + m) * 16 + (x & 15)]);
        mx = grp_max<LPR>(mx);
        float se = 0.f;
        if (mx > -INFINITY)
            for (int x = li; x < n_el; x += LPR) se += expf(s_lm[((x >> 4) * rows + m) * 16 + (x & 15)] - mx);
        se = grp_sum<LPR>(se);
        const unsigned obase = (unsigned)((j * rows + m) * stride);
        if (live && li < 2) ll_st1(rl, obase + li, li ? se : mx, seq);
        const int nepl = min(EPL, (n_el + LPR - 1) / LPR);   // registers per lane that hold elements
        u64 prev = ~0ull;
        for (int t = 0; t < topk; ++t) {
            u64 best = 0;
#pragma unroll
            for (int i = 0; i < EPL; ++i)
                if (i < nepl && keys[i] < prev && keys[i] > best) best = keys[i];
            for (int x = li + LPR * EPL; x < n_el; x += LPR) {
                const int lt = x >> 4;
                const float v = s_lm[(lt * rows + m) * 16 + (x & 15)];
                const int id = 16 * tile_index(D, lt >> sl_log, lt & (SL - 1), j) + (x & 15);
                const u64 kx = v > -INFINITY ? make_key(v, id) : 0;
                if (kx < prev && kx > best) best = kx;
            }
            best = grp_max_u64<LPR>(best);
            if (live && li < 2)
                ll_st1(rl, obase + 2 + 2 * t + li, __uint_as_float(li ? (unsigned)(best >> 32) : (unsigned)best), seq);
            prev = best ? best : 0;   // 0: list exhausted, every later entry is "none"
        }
        if (P.sample_ids) {   // the workgroup's best perturbed logit (see gumbel_of)
            u64 gbest = 0;
#pragma unroll
            for (int i = 0; i < EPL; ++i)
                if (i < nepl && keys[i]) {
                    const int id = key_id(keys[i]);
                    const u64 kx = make_key(key_value(keys[i]) + gumbel_of(P, m, id), id);
                    gbest = kx > gbest ? kx : gbest;
                }
            for (int x = li + LPR * EPL; x < n_el; x += LPR) {
                const int lt = x >> 4;
                const float v = s_lm[(lt * rows + m) * 16 + (x & 15)];
                const int id = 16 * tile_index(D, lt >> sl_log, lt & (SL - 1), j) + (x & 15);
                const u64 kx = v > -INFINITY ? make_key(v + gumbel_of(P, m, id), id) : 0;
                gbest = kx > gbest ? kx : gbest;
            }
            gbest = grp_max_u64<LPR>(gbest);
            if (live && li < 2)
                ll_st1(rl, obase + 2 + 2 * topk + li, __uint_as_float(li ? (unsigned)(gbest >> 32) : (unsigned)gbest), seq);
        }
    }
}

// One phase for one workgroup.  wb: the wavefront's weight-load registers.  On entry they hold
// the preloaded head of first_stream(ph); on exit they hold PS_U loads from after_wp (the head of
// whatever this wavefront streams next, or any readable address).
template <typename WT, int MT, int PH>
__device__ __forceinline__ void gemm_phase(const StepParams& P, int wg, int wave, char* smem, uint4 (&wb)[PS_U],
                                           const char* after_wp, unsigned publish_seq = 0) {
    constexpr bool BF = Traits<WT>::BF;
    constexpr int ph = PH;
    constexpr bool sliceable = PH != PH_LMHEAD;   // see make_desc on the host
    const PhaseDesc& D = P.ph[ph];
    const int tid = threadIdx.x, lane = tid & 63, lane16 = lane * 16;
    const int c = lane & 15, kb = lane >> 4;
    const int rows = D.rows;
    const int kw_log = D.kw_log, KW = 1 << kw_log, SL = PS_WAVES >> kw_log, sl_log = PS_WAVES_LOG - kw_log;
    const int slot = wave >> kw_log, kw = wave & (KW - 1);
    const int S = sliceable ? 1 << D.s_log : 1, s = wg & (S - 1);   // K-slice and column of this workgroup
    const int j = S > 1 ? wg >> D.s_log : wg;
    const int RS = D.rs;

    char* s_zero = smem + PS_LDS_ZERO;
    char* s_red = smem + PS_LDS_RED;
    char* s_pa = smem + panel_offset(MT);                        // high parts (or f32 values)
    char* s_pb = s_pa + rows * RS;                               // low parts (bf16 only)
    float* s_lm = reinterpret_cast<float*>(s_pb + (BF ? rows * RS : 0));
    const float* s_ssq = reinterpret_cast<const float*>(smem + PS_LDS_SSQ);
    const int nsub = (1 << D.g2_log) >> 6;                       // entries of s_ssq per row
    const bool norm = PH == PH_QKV || PH == PH_GATEUP || (PH == PH_LMHEAD && D.norm != 0);

    constexpr int SB = PH == PH_FC ? 50 : 2 + PH * 6;   // this phase's clock stamps (timeline builds)
    stamp(P, wg, SB + 0);
    if (j >= D.T) {                   // more workgroup columns than tiles: nothing to do in this phase
        preload_weights(wb, after_wp, lane16);
        if (publish_seq) *(lds_u32*)(unsigned)PS_LDS_SEQ = publish_seq;
        return;
    }
    if (tid < 16) reinterpret_cast<uint32_t*>(s_zero)[tid] = 0u;
    if (ph == PH_LMHEAD) {
        const int n_lm = D.rounds * SL * rows * 16;
        for (int x = tid; x < n_lm; x += PS_WG_THREADS) s_lm[x] = -INFINITY;
    }

    // per-lane panel addressing: column c of column tile mt is activation row 16 mt + c
    lds_cptr pa[MT];
    int pinc[MT], plo[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = 16 * mt + c;
        if (m < rows) { pa[mt] = (lds_cptr)(s_pa + m * RS + kb * 16); pinc[mt] = 64; plo[mt] = (int)(s_pb - s_pa); }
        else { pa[mt] = (lds_cptr)(s_zero + kb * 16); pinc[mt] = 0; plo[mt] = 0; }
    }
    int sg_lo, sg_hi;
    slice_groups(D, s, sg_lo, sg_hi);

    // While the workgroup waits for its activations the memory is idle: besides the PS_U KiB per
    // wavefront that are already on their way into registers (wb), the next PS_PF * 8 KiB of the
    // wavefront's first weight stream are pulled into the L2 of this XCD, one 4-byte load per
    // 128-byte line (PS_PF is the most; the host says how many of these 8-KiB pieces: D.pf).  The
    // values are not used; they stay registers until the panel is staged.
    unsigned pf[PS_PF > 0 ? PS_PF : 1];
    if (PS_PF > 0 && tile_index(D, 0, slot, j) < D.T) {
        int a0, n;
        const char* wp0 = stream_ptr(D, tile_index(D, 0, slot, j), sg_lo, min(D.piece_groups, sg_hi - sg_lo), kw, a0, n);
        const int lines = (n - PS_U) * (PS_WS / 128);            // 128-byte lines that follow the preloaded steps
#pragma unroll
        for (int i = 0; i < PS_PF; ++i) {
            const int ln = min(64 * i + (lane16 >> 4), lines - 1);
            pf[i] = (lines > 0 && i < D.pf) ? *reinterpret_cast<const unsigned*>(wp0 + PS_U * PS_WS + (size_t)ln * 128) : 0u;
        }
    }

    bool streamed = false;
    for (int rd = 0; rd < D.rounds; ++rd) {
        const int tau = tile_index(D, rd, slot, j);
        const bool valid = tau < D.T;
        f32x4 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int pc = 0; pc < D.npieces; ++pc) {
            const int g_lo = sg_lo + pc * D.piece_groups;
            const int ng = min(D.piece_groups, sg_hi - g_lo);
            if (rd == 0 || D.npieces > 1) {   // a panel that fits as a whole is staged once
                if (rd > 0 || pc > 0) __syncthreads();   // everyone is done with the previous piece
                stage_piece<WT, PH>(P, D, wave, smem, s_pa, s_pb, g_lo * PS_U, ng * PS_U, pc == 0, rd == 0);
                if (publish_seq && rd == 0 && pc == 0) *(lds_u32*)(unsigned)PS_LDS_SEQ = publish_seq;   // see step_read
                __syncthreads();
                if (rd == 0 && pc == 0) {
#pragma unroll
                    for (int i = 0; i < (PS_PF > 0 ? PS_PF : 0); ++i) asm volatile("" ::"v"(pf[i]));
                    stamp(P, wg, SB + 1);
                }
            }
            if (valid) {
                int a0, n, na, nn;
                const char* wp = stream_ptr(D, tau, g_lo, ng, kw, a0, n);
                const char* next_wp = after_wp;
                if (pc + 1 < D.npieces) {
                    const int g2 = g_lo + D.piece_groups;
                    next_wp = stream_ptr(D, tau, g2, min(D.piece_groups, sg_hi - g2), kw, na, nn);
                } else if (rd + 1 < D.rounds && tile_index(D, rd + 1, slot, j) < D.T) {
                    next_wp = stream_ptr(D, tile_index(D, rd + 1, slot, j), sg_lo, min(D.piece_groups, sg_hi - sg_lo), kw, na, nn);
                }
                lds_cptr pa_t[MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) pa_t[mt] = pa[mt] + a0 * pinc[mt];
                consume_weights<WT, MT>(wb, wp, n, next_wp, lane16, pa_t, pinc, plo, acc);
                streamed = true;
            }
        }
        if (rd == D.rounds - 1) stamp(P, wg, SB + 2);

        // wavefronts sharing the tile: wavefront kw = 0 adds the others' partial sums in order
        if (KW > 1) {
            f32x4* red = reinterpret_cast<f32x4*>(s_red);
            if (valid && kw > 0) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) red[(wave * MT + mt) * 64 + lane] = acc[mt];
            }
            __syncthreads();
            if (valid && kw == 0) {
                for (int o = 1; o < KW; ++o) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) acc[mt] += red[((wave + o) * MT + mt) * 64 + lane];
                }
            }
            if (rd + 1 < D.rounds) __syncthreads();
        }
        if (rd == D.rounds - 1) stamp(P, wg, SB + 3);

        if (valid && kw == 0) {
            if (sliceable && S > 1) {
                // K-slices of other workgroups: publish this slice's part of the tile (and, once per
                // slice, its sums of squares); the sums are formed after the last round
                const SxBuf rfrag = sx_buf(P, D.frag), rssq = sx_buf(P, D.ssq_frag);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    sx_st4(rfrag, (unsigned)((((s * D.T + tau) * MT + mt) * 64 + lane) * 4), acc[mt]);
                if (norm && rd == 0 && j == 0 && slot == 0 && lane < rows) {
                    float t = 0.f;
                    for (int w = 0; w < nsub; ++w) t += s_ssq[lane * 8 + w];
                    sx_st1(rssq, (unsigned)(s * PS_MAX_ROWS + lane), t);
                }
            } else {
                if (norm) {   // RMSNorm: the panel held x (.) gain, 1/rms multiplies the result
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        const int m = 16 * mt + c;
                        float t = 0.f;
                        if (m < rows)
                            for (int w = 0; w < nsub; ++w) t += s_ssq[m * 8 + w];
                        acc[mt] *= 1.0f / sqrtf(t / (float)D.K + P.eps);
                    }
                }
                switch (ph) {
                    case PH_QKV: epilogue_qkv<WT, MT>(P, tau, lane, acc); break;
                    case PH_OPROJ: epilogue_oproj<WT, MT>(P, tau, lane, acc); break;
                    case PH_GATEUP: epilogue_gateup<WT, MT>(P, tau, lane, acc); break;
                    case PH_DOWN: epilogue_down<WT, MT>(P, tau, lane, acc); break;
                    case PH_FC: epilogue_fc<WT, MT>(P, tau, lane, acc); break;
                    default: epilogue_lm<WT, MT>(P, tau, lane, acc, s_lm, rd * SL + slot); break;
                }
            }
        }
    }
    if (sliceable && S > 1) {
        // Sum over the K-slices.  Of the tiles of this workgroup column, slice s completes every S-th;
        // its wavefronts take one each, wait for all S parts (its own included) and add them in slice
        // order, so the result does not depend on timing.  Then the phase's epilogue.
        const rsrc_t rf = make_rsrc(act_ptr(P, D.frag)), rq = make_rsrc(act_ptr(P, D.ssq_frag));
        const int ntl = D.rounds * SL;
        for (int lt = s + S * wave; lt < ntl; lt += S * PS_WAVES) {
            const int tau = tile_index(D, lt >> sl_log, lt & (SL - 1), j);
            if (tau >= D.T) continue;
            f32x4 acc[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                constexpr int SB = 8;                // slices requested per round trip (S <= 8)
                const int m = 16 * mt + c;
                u32x4 fr[SB];
                unsigned fq[SB];
                int spins = 0;
                for (;;) {
#pragma unroll
                    for (int i = 0; i < SB; ++i) {
                        const int ss = i < S ? i : S - 1;
                        fr[i] = coh_ld16(rf, (unsigned)((((ss * D.T + tau) * MT + mt) * 64 + lane) * 16));
                        fq[i] = norm ? coh_ld4(rq, (unsigned)((ss * PS_MAX_ROWS + (m < rows ? m : 0)) * 4)) : 0u;
                    }
                    unsigned bad = 0;   // all loads first, then all checks: no wait between the loads
#pragma unroll
                    for (int i = 0; i < SB; ++i) bad |= (unsigned)!sx_ok(fr[i]) | (unsigned)(fq[i] == PS_SENT);
                    if (__all(!bad) || !spin_again(P, spins)) break;
                }
                f32x4 sum = f32x4{0.f, 0.f, 0.f, 0.f};
                float t = 0.f;
#pragma unroll
                for (int i = 0; i < SB; ++i) {
                    if (i < S) { sum += __builtin_bit_cast(f32x4, fr[i]); t += __uint_as_float(fq[i]); }
                }
                if (norm) sum *= 1.0f / sqrtf(t / (float)D.K + P.eps);
                acc[mt] = sum;
            }
            switch (ph) {
                case PH_QKV: epilogue_qkv<WT, MT>(P, tau, lane, acc); break;
                case PH_OPROJ: epilogue_oproj<WT, MT>(P, tau, lane, acc); break;
                case PH_GATEUP: epilogue_gateup<WT, MT>(P, tau, lane, acc); break;
                case PH_FC: epilogue_fc<WT, MT>(P, tau, lane, acc); break;
                default: epilogue_down<WT, MT>(P, tau, lane, acc); break;
            }
        }
    }
    stamp(P, wg, SB + 4);
    if (!streamed) preload_weights(wb, after_wp, lane16);   // keep the contract on wb

    if (ph == PH_LMHEAD) {
        // per-workgroup softmax statistics and top-k over the logits held in LDS: a whole wavefront takes a
        // row; with more rows than wavefronts 16 lanes do (four rows per wavefront at a time) as long as a
        // lane's share of the row's logits fits its registers
        __syncthreads();
        if (rows > PS_WAVES && D.rounds * SL * 16 <= 16 * 16) lm_local_stats<16>(P, D, j, rows, s_lm, wave, lane, sl_log, SL);
        else lm_local_stats<64>(P, D, j, rows, s_lm, wave, lane, sl_log, SL);
    }
    stamp(P, wg, SB + 5);
}

// ------------------------------------------------------------------------------------------
// Init-time prepack: tile tau, step t of a phase's weight matrix becomes one contiguous KiB in
// the exact order the streaming loop reads it: lane (i = lane % 16, kb = lane / 16) gets bytes
// [64 t + 16 kb, +16) of tile row i, so a wavefront load is one contiguous 1 KiB burst.
// ------------------------------------------------------------------------------------------
// Steps Kreal .. Kt-1 (the padding of the contraction dimension to whole groups) hold zeros.
template <typename WT, int PH>
__global__ void __launch_bounds__(256) pack_kernel(const StepParams P, int T, int Kt, int Kreal, char* dst) {
    const size_t units = (size_t)T * Kt;
    const int lane = threadIdx.x & 63;
    for (size_t u = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6); u < units; u += (size_t)gridDim.x * 4) {
        const int tau = (int)(u / Kt), t = (int)(u - (size_t)tau * Kt);
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (t < Kreal) v = ld16(weight_row_ptr<WT, PH>(P, tau, lane & 15) + (size_t)t * 64 + (lane >> 4) * 16);
        *reinterpret_cast<uint4*>(dst + u * 1024 + lane * 16) = v;
    }
}

// ------------------------------------------------------------------------------------------
// attention: one work item = (sequence b, kv head hk, chunk of CH keys); all g*M query rows of
// the kv head are processed against the chunk.  Row i of the step sees cache positions
// 0 .. kv_len[b] + i (its own and earlier rows of this step included; Algorithm 1: distribution
// j is conditioned on [MASK]_1..j only).
//
// Each wavefront takes NK groups of 16 keys of the chunk (CH = 128 NK keys).  NK = 2 halves the
// number of work items; the host asks for it when that lets every workgroup get by with a single
// item (its registers only fit without the requests for a following item).  Scores are one MFMA tile per 16 keys and 16 query rows: the
// keys' K rows are the 16-row operand, loaded straight from the cache in its storage type; the
// query rows (fp32, split into bf16 high + low parts like every activation) are the 16-column
// operand.  The row maxima of the eight wavefronts meet in LDS, so all of them exponentiate
// against the same maximum and their partial sums and partial P.V products simply add up, in
// wavefront order.  P.V is plain FMA work: a lane owns D/64 adjacent output columns, reads the
// V rows of its wavefront's keys with coalesced loads and the probabilities as LDS broadcasts.
// Keys written in this very step come, exactly as stored in the cache, from the exchange buffer
// the QKV epilogue fills.
// ------------------------------------------------------------------------------------------
template <typename WT, int D, int NK> struct AttnCfg {
    static constexpr int CH = PS_ATTN_KEYS * NK;
    static constexpr int CH_LOG = PS_ATTN_KEYS_LOG + (NK == 2 ? 1 : 0);
    static constexpr int OFF_M = PS_LDS_BASE;                                // [waves][16] row maxima
    static constexpr int OFF_L = OFF_M + PS_WAVES * 16 * 4;          // [waves][16] row sums
    static constexpr int OFF_P = OFF_L + PS_WAVES * 16 * 4;          // [waves][NK][16 rows][16 keys]
    static constexpr int OFF_O = OFF_P + PS_WAVES * NK * 16 * 16 * 4;   // [waves][16 rows][D]
    static constexpr int OFF_Q = OFF_O + PS_WAVES * 16 * D * 4;      // 16 query rows as MFMA operands: [step][hi, lo][64 lanes] x 16 B
    static constexpr int LDS = OFF_Q + 16 * D * 4;
    static_assert(NK == 1 || NK == 2, "NK");
    static_assert(PS_ATTN_KEYS == 16 * PS_WAVES && LDS == ps_attn_lds_bytes(D, NK), "host and device agree on the layout");
};

// One attention work item: sequence b, kv head hk, key block ch of nch; L = valid cache rows
struct AttnItem { int b, hk, ch, nch, L; };
__device__ __forceinline__ AttnItem attn_decode(const StepParams& P, int item, int ch_log) {
    AttnItem it;
    int b = 0, rem = item, nch = 0;
    for (;; ++b) {
        nch = (kvlen_u(b) + P.attn_tail + (1 << ch_log) - 1) >> ch_log;
        if (rem < nch * P.nkv) break;
        rem -= nch * P.nkv;
    }
    it.b = b; it.nch = nch; it.hk = rem / nch; it.ch = rem - it.hk * nch; it.L = kvlen_u(b);
    return it;
}

// K rows of the wavefront's 16 keys key0 .. key0 + 15 as the MFMA operand: lane (c, kb) gets
// bytes [64 t + 16 kb, +16) of key c.  Keys beyond the sequence are clamped (masked later); keys
// written in this step are taken from the exchange buffer once the QKV phase has published them.
template <typename WT, int D>
__device__ __forceinline__ void attn_load_k(const StepParams& P, const AttnItem& it, int key0, int lane,
                                            uint4 (&kreg)[D / Traits<WT>::KSTEP], bool with_new = true) {
    constexpr bool BF = Traits<WT>::BF;
    constexpr int ESZ = Traits<WT>::ESZ, GE = Traits<WT>::GE, KSTEP = Traits<WT>::KSTEP, NL = GE / 4, STEPS = D / KSTEP;
    const int c = lane & 15, kb = lane >> 4;
    const int L = it.L, end = L + P.attn_tail;
    const int kpos = key0 + c;
    const int pc = kpos < L ? kpos : (L > 0 ? L - 1 : 0);
    const char* krow = (const char*)P.kc + (((size_t)P.kv_off[it.b] + pc) * P.nkv + it.hk) * D * ESZ + kb * 16;
#pragma unroll
    for (int t = 0; t < STEPS; ++t) kreg[t] = ld16(krow + t * 64);
    if (with_new && end > L && key0 + 15 >= L && key0 < end) {
        const rsrc_t rn = make_rsrc(act_ptr(P, P.kvnew));
        const bool k_new = kpos >= L;
        const int pn = kpos < L ? L : (kpos < end ? kpos : end - 1);
        const unsigned kbase = (unsigned)(((size_t)(it.b * P.M + (pn - L)) * 2) * P.KVD + it.hk * D + kb * GE);
        u32x4 kx[STEPS][NL];
        int spins = 0;
        const bool wanted = k_new && kpos < end;
        for (;;) {
#pragma unroll
            for (int t = 0; t < STEPS; ++t)
#pragma unroll
                for (int h = 0; h < NL; ++h) kx[t][h] = coh_ld16(rn, (kbase + t * KSTEP + 4 * h) * 4);
            unsigned bad = 0;   // all loads first, then all checks: no wait between the loads
#pragma unroll
            for (int t = 0; t < STEPS; ++t)
#pragma unroll
                for (int h = 0; h < NL; ++h) bad |= (unsigned)!sx_ok(kx[t][h]);
            if (__all(!wanted || !bad) || !spin_again(P, spins)) break;
        }
        if (k_new) {
#pragma unroll
            for (int t = 0; t < STEPS; ++t) {
                if constexpr (BF) {
                    kreg[t].x = pack_bf16x2(__uint_as_float(kx[t][0][0]), __uint_as_float(kx[t][0][1]));
                    kreg[t].y = pack_bf16x2(__uint_as_float(kx[t][0][2]), __uint_as_float(kx[t][0][3]));
                    kreg[t].z = pack_bf16x2(__uint_as_float(kx[t][1][0]), __uint_as_float(kx[t][1][1]));
                    kreg[t].w = pack_bf16x2(__uint_as_float(kx[t][1][2]), __uint_as_float(kx[t][1][3]));
                } else {
                    kreg[t] = make_uint4(kx[t][0][0], kx[t][0][1], kx[t][0][2], kx[t][0][3]);
                }
            }
        }
    }
}
// V rows of the same keys: a lane owns columns [DPL lane, DPL lane + DPL).  attn_issue_v requests
// them (unconditionally, positions clamped, so all 16 loads are in flight together) as raw bits and
// fetches the rows written in this step from the exchange buffer; attn_finish_v widens them and
// zeroes the keys beyond the sequence.
template <typename WT, int DPL> struct VRaw;
template <> struct VRaw<bf16_t, 2> { typedef uint32_t type; };
template <> struct VRaw<bf16_t, 1> { typedef uint16_t type; };
template <> struct VRaw<float, 2> { typedef float2 type; };
template <> struct VRaw<float, 1> { typedef float type; };
__device__ __forceinline__ void widen_v(uint32_t u, float* out) { out[0] = bf16_to_f32(u & 0xFFFFu); out[1] = bf16_to_f32(u >> 16); }
__device__ __forceinline__ void widen_v(uint16_t u, float* out) { out[0] = bf16_to_f32(u); }
__device__ __forceinline__ void widen_v(float2 u, float* out) { out[0] = u.x; out[1] = u.y; }
__device__ __forceinline__ void widen_v(float u, float* out) { out[0] = u; }
__device__ __forceinline__ void narrow_v(const float* in, uint32_t& u) { u = pack_bf16x2(in[0], in[1]); }
__device__ __forceinline__ void narrow_v(const float* in, uint16_t& u) { u = (uint16_t)f32_to_bf16(in[0]); }
__device__ __forceinline__ void narrow_v(const float* in, float2& u) { u = make_float2(in[0], in[1]); }
__device__ __forceinline__ void narrow_v(const float* in, float& u) { u = in[0]; }

template <typename WT, int D>
__device__ __forceinline__ void attn_issue_v(const StepParams& P, const AttnItem& it, int key0, int lane,
                                             typename VRaw<WT, D / 64>::type (&vraw)[16], bool with_new = true) {
    constexpr int ESZ = Traits<WT>::ESZ, DPL = D / 64;
    typedef typename VRaw<WT, DPL>::type raw_t;
    const int L = it.L, end = L + P.attn_tail;
    const size_t cache_row0 = (size_t)P.kv_off[it.b] * P.nkv + it.hk;   // in units of D elements
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
        const int pos = key0 + kk;                                // wavefront-uniform
        const int pc = pos < L ? pos : (L > 0 ? L - 1 : 0);
        vraw[kk] = *reinterpret_cast<const raw_t*>((const char*)P.vc + ((cache_row0 + (size_t)pc * P.nkv) * D + DPL * lane) * ESZ);
    }
    if (with_new && end > L && key0 + 15 >= L && key0 < end) {
        // rows written in this step: from the exchange buffer, as soon as the QKV phase has published
        // them; they are exactly representable in the storage type (they were rounded to it)
        const rsrc_t rn = make_rsrc(act_ptr(P, P.kvnew));
        float vx[16][DPL];
        int spins = 0;
        for (;;) {
#pragma unroll
            for (int kk = 0; kk < 16; ++kk) {
                const int pos = key0 + kk;
                const int pn = pos < L ? L : (pos < end ? pos : end - 1);   // clamped: every load is unconditional
                const unsigned vb = (unsigned)(((size_t)(it.b * P.M + (pn - L)) * 2 + 1) * P.KVD + it.hk * D + DPL * lane);
#pragma unroll
                for (int e = 0; e < DPL; ++e) vx[kk][e] = __uint_as_float(coh_ld4(rn, (vb + e) * 4));
            }
            unsigned bad = 0;   // clamped positions repeat a wanted row: checking them all is right
#pragma unroll
            for (int kk = 0; kk < 16; ++kk)
#pragma unroll
                for (int e = 0; e < DPL; ++e) bad |= (unsigned)(__float_as_uint(vx[kk][e]) == PS_SENT);
            if (__all(!bad) || !spin_again(P, spins)) break;
        }
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const int pos = key0 + kk;
            if (pos >= L && pos < end) narrow_v(vx[kk], vraw[kk]);
        }
    }
}
template <typename WT, int D>
__device__ __forceinline__ void attn_finish_v(const StepParams& P, const AttnItem& it, int key0, int lane,
                                              const typename VRaw<WT, D / 64>::type (&vraw)[16], float (&v)[16][D / 64]) {
    constexpr int DPL = D / 64;
    const int end = it.L + P.attn_tail;
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
        widen_v(vraw[kk], v[kk]);
        if (key0 + kk >= end) {                                   // beyond the sequence
#pragma unroll
            for (int e = 0; e < DPL; ++e) v[kk][e] = 0.f;
        }
    }
}
// The 16 query rows r0 .. r0 + 15 of an item are the same for all wavefronts: thread (row, group of
// 4 columns) requests its 16 bytes (attn_issue_q, no wait), and once they have arrived puts them
// into LDS as the 16-column MFMA operand (attn_store_q; bf16: split into high and low parts): lane
// (c, kb) of step t finds row r0 + c, elements [t KSTEP + kb GE, + GE) at ((t [* 2 + lo]) * 64 + lane) * 16.
template <typename WT, int D>
__device__ __forceinline__ u32x4 attn_issue_q(const StepParams& P, const AttnItem& it, int r0, int Ra, int grp, int tid) {
    constexpr int GPR = D / 4;                       // 16-byte groups per row
    const int r = tid / GPR < 16 ? tid / GPR : 15, g = tid % GPR;
    const rsrc_t rq = make_rsrc(act_ptr(P, P.q_buf));
    const int rho = r0 + r < Ra ? r0 + r : Ra - 1;
    const int gi = row_seq(P, rho), i = rho - gi * P.M;
    return coh_ld16(rq, (unsigned)((size_t)(it.b * P.M + i) * P.QD + (it.hk * grp + gi) * D + 4 * g) * 4);
}
template <typename WT, int D>
__device__ __forceinline__ void attn_store_q(char* sq, int tid, u32x4 x) {
    constexpr int GPR = D / 4;
    if (tid >= 16 * GPR) return;
    const int r = tid / GPR, e0 = 4 * (tid % GPR);
    if constexpr (Traits<WT>::BF) {
        const int t = e0 >> 5, kb = (e0 & 31) >> 3, half = (e0 & 7) >> 2;
        const float f0 = __uint_as_float(x[0]), f1 = __uint_as_float(x[1]), f2 = __uint_as_float(x[2]), f3 = __uint_as_float(x[3]);
        const unsigned h01 = pack_bf16x2(f0, f1), h23 = pack_bf16x2(f2, f3);
        const unsigned l01 = pack_bf16x2(f0 - __uint_as_float(h01 << 16), f1 - __uint_as_float(h01 & 0xFFFF0000u));
        const unsigned l23 = pack_bf16x2(f2 - __uint_as_float(h23 << 16), f3 - __uint_as_float(h23 & 0xFFFF0000u));
        char* p = sq + ((2 * t * 64) + kb * 16 + r) * 16 + half * 8;
        *reinterpret_cast<uint2*>(p) = make_uint2(h01, h23);
        *reinterpret_cast<uint2*>(p + 64 * 16) = make_uint2(l01, l23);
    } else {
        const int t = e0 >> 4, kb = (e0 & 15) >> 2;
        *reinterpret_cast<uint4*>(sq + (t * 64 + kb * 16 + r) * 16) = make_uint4(x[0], x[1], x[2], x[3]);
    }
}

// qx: the rows requested earlier with attn_issue_q(it, r0)
template <typename WT, int D>
__device__ __forceinline__ void attn_place_q(const StepParams& P, const AttnItem it, int r0, int Ra, int grp, int tid,
                                             u32x4& qx, char* sq) {
    if (!__all(sx_ok(qx))) {
        int spins = 0;
        do qx = attn_issue_q<WT, D>(P, it, r0, Ra, grp, tid); while (!__all(sx_ok(qx)) && spin_again(P, spins));
    }
    attn_store_q<WT, D>(sq, tid, qx);
}

// ------------------------------------------------------------------------------------------
// Sequences cut into several key blocks: the work items that put the blocks' partial results together.
// sM, sL: at least 72 floats each; sW: [PS_WAVES][256] floats; sO: [PS_WAVES][D] floats.
// ------------------------------------------------------------------------------------------
// key blocks of sequence b.  V2 (see attn_phase2): blocks of cache keys, the rows of this step ride on the
// last one (an empty cache still has that one); else the blocks cover valid rows + attn_tail
template <bool V2> __device__ __forceinline__ int attn_nch(const StepParams& P, int b, int ch_log) {
    const int CH = 1 << ch_log;
    if constexpr (V2) return max(1, (kvlen_u(b) + CH - 1) >> ch_log);
    else return (kvlen_u(b) + P.attn_tail + CH - 1) >> ch_log;
}
template <typename WT, int D, bool V2>
__device__ __forceinline__ void attn_merge(const StepParams& P, int wg, int nwg, int wave, int n_merge, int ch_log,
                                           float* sM, float* sL, float* sW, float* sO) {
    constexpr int DPL = D / 64;                     // output columns per lane
    const int tid = threadIdx.x, lane = tid & 63;
    const int grp = P.nq / P.nkv;
    const int Ra = grp * P.M;
    const rsrc_t racc = make_rsrc(P.attn_acc), rml = make_rsrc(P.attn_ml);
    const SxBuf ro = sx_buf(P, P.o_buf);
    const unsigned seq = ps_seq();
    const bool sep = !V2 && P.attn_sep;
    // ---- sequences cut into several blocks: put the blocks' partial results together.  One work
    // item = (sequence, kv head, 8 query rows).  Wavefront w turns the (max, sum) pairs of row w
    // into one weight per block (in LDS); then thread (row, column pair) adds up the blocks'
    // outputs with these weights, 16 blocks per round of loads.  Blocks are taken in groups of
    // 256; groups are folded with a running maximum, so any number of blocks works.
    constexpr int MR = PS_WAVES;                     // rows per work item: one wavefront per row
    constexpr int GRP = 256, CB = 16;
    constexpr int PP = D / 2;                        // column pairs per row
    const int RT = (Ra + MR - 1) / MR;
    constexpr int SEP_ML = 64;                       // (max, sum) of the step's own rows: sM / sL [SEP_ML + row], beside the groups' [row]
    for (int mi = wg; mi < n_merge; mi += nwg) {
        int b = 0, rem = mi, nch = 0, item_base = 0;
        for (;; ++b) {
            nch = attn_nch<V2>(P, b, ch_log);
            const int n = (nch > 1 || sep) ? P.nkv * RT : 0;
            if (rem < n) break;
            rem -= n;
            item_base += nch * P.nkv;
        }
        const int hk = rem / RT, rt = rem - hk * RT;
        const int item0 = item_base + hk * nch;      // block 0 of this (b, hk)
        const int r0 = rt * MR, nr = min(MR, Ra - r0);
        const int myrow = tid / PP, dp = tid - myrow * PP;
        const bool active = myrow < nr;
        float num0 = 0.f, num1 = 0.f, den = 0.f, mrun = -INFINITY;
        if (sep) {
            // The rows written in this step are not part of any block: wavefront w works out row w's
            // attention over them (at most 16 keys, a lane owns DPL columns of q, K and V, the dot
            // products are wavefront sums); the result is folded in after the blocks like one more group of
            // them.  This comes first: its inputs (the QKV phase's outputs) are there long before the last
            // block's partial results, so it runs while those are still being produced.
            __syncthreads();                         // the previous item is done with the output area
            if (wave < nr) {
                const int rho = r0 + wave;
                const int gi = row_seq(P, rho), i = rho - gi * P.M;
                const int sk = skipof_u(b), i_hi = max(i, sk);   // the row sees rows sk .. max(i, sk) of this step
                const rsrc_t rq = make_rsrc(act_ptr(P, P.q_buf)), rn = make_rsrc(act_ptr(P, P.kvnew));
                const unsigned qo = (unsigned)((size_t)(b * P.M + i) * P.QD + (hk * grp + gi) * D + DPL * lane);
                float q[DPL], kx[16][DPL], vx[16][DPL];
                auto issue_new = [&]() __attribute__((always_inline)) {
#pragma unroll
                    for (int e = 0; e < DPL; ++e) q[e] = coh_ld_f(rq, (qo + e) * 4);
#pragma unroll
                    for (int jj = 0; jj < 16; ++jj) {
                        const int jc = jj < P.M ? jj : P.M - 1;     // clamped: every load is unconditional
                        const unsigned ko = (unsigned)(((size_t)(b * P.M + jc) * 2) * P.KVD + hk * D + DPL * lane);
#pragma unroll
                        for (int e = 0; e < DPL; ++e) {
                            kx[jj][e] = coh_ld_f(rn, (ko + e) * 4);
                            vx[jj][e] = coh_ld_f(rn, (ko + P.KVD + e) * 4);
                        }
                    }
                };
                auto bad_new = [&]() __attribute__((always_inline)) {
                    unsigned bad = 0;
#pragma unroll
                    for (int e = 0; e < DPL; ++e) bad |= (unsigned)(__float_as_uint(q[e]) == PS_SENT);
#pragma unroll
                    for (int jj = 0; jj < 16; ++jj)
#pragma unroll
                        for (int e = 0; e < DPL; ++e)
                            bad |= (unsigned)(__float_as_uint(kx[jj][e]) == PS_SENT) | (unsigned)(__float_as_uint(vx[jj][e]) == PS_SENT);
                    return bad;
                };
                issue_new();
                if (!__all(!bad_new())) {
                    int spins = 0;
                    do issue_new(); while (!__all(!bad_new()) && spin_again(P, spins));
                }
                float sc[16], mn = -INFINITY;
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) {
                    sc[jj] = -INFINITY;
                    if (jj >= sk && jj <= i_hi) {    // wavefront-uniform
                        float part = 0.f;
#pragma unroll
                        for (int e = 0; e < DPL; ++e) part += q[e] * kx[jj][e];
                        sc[jj] = wave_sum(part) * P.inv_sqrt_d;
                        mn = fmaxf(mn, sc[jj]);
                    }
                }
                float ln = 0.f, on[DPL];
#pragma unroll
                for (int e = 0; e < DPL; ++e) on[e] = 0.f;
#pragma unroll
                for (int jj = 0; jj < 16; ++jj) {
                    if (jj >= sk && jj <= i_hi) {
                        const float pj = expf(sc[jj] - mn);
                        ln += pj;
#pragma unroll
                        for (int e = 0; e < DPL; ++e) on[e] += pj * vx[jj][e];
                    }
                }
#pragma unroll
                for (int e = 0; e < DPL; ++e) sO[wave * D + DPL * lane + e] = on[e];
                if (lane == 0) { sM[SEP_ML + wave] = mn; sL[SEP_ML + wave] = ln; }
            }
        }
        for (int g0 = 0; g0 < nch; g0 += GRP) {
            const int gn = min(GRP, nch - g0);
            __syncthreads();                         // the weights of the previous group (or item) are no longer read
            // Both kinds of loads are requested at once, the (max, sum) pairs first: the outputs of the
            // first 16 blocks are on their way while the weights are worked out.  The first look at
            // either is straight-line code (see the query rows above); only a failed look loops.
            u32x4 ml[GRP / 64];
            u32x4 av[CB];
            const int rho_w = r0 + (wave < nr ? wave : 0);
            auto issue_ml = [&]() __attribute__((always_inline)) {
#pragma unroll
                for (int q = 0; q < GRP / 64; ++q) {
                    const int cx = lane + 64 * q;
                    const int cc = g0 + (cx < gn ? cx : gn - 1);
                    ml[q] = coh_ld16(rml, (unsigned)(((size_t)(item0 + cc) * Ra + rho_w) * 2) * 8);   // {max, tag, sum, tag}
                }
            };
            auto bad_ml = [&]() __attribute__((always_inline)) {
                unsigned bad = 0;
#pragma unroll
                for (int q = 0; q < GRP / 64; ++q) bad |= (unsigned)(ml[q][1] != seq) | (unsigned)(ml[q][3] != seq);
                return bad;
            };
            auto issue_av = [&](int cb) __attribute__((always_inline)) {
#pragma unroll
                for (int i = 0; i < CB; ++i) {
                    const int cc = g0 + (cb + i < gn ? cb + i : gn - 1);
                    const int rho = r0 + (active ? myrow : 0);
                    av[i] = coh_ld16(racc, (unsigned)(((size_t)(item0 + cc) * Ra + rho) * D + 2 * dp) * 8);   // {o, tag, o', tag}
                }
            };
            auto bad_av = [&]() __attribute__((always_inline)) {
                unsigned bad = 0;
#pragma unroll
                for (int i = 0; i < CB; ++i) bad |= (unsigned)(av[i][1] != seq) | (unsigned)(av[i][3] != seq);
                return bad;
            };
            if (wave < nr) issue_ml();
            issue_av(0);
            if (wave < nr) {
                if (!__all(!bad_ml())) {
                    int spins = 0;
                    do issue_ml(); while (!__all(!bad_ml()) && spin_again(P, spins));
                }
                float mloc = -INFINITY;
#pragma unroll
                for (int q = 0; q < GRP / 64; ++q)
                    if (lane + 64 * q < gn && __uint_as_float(ml[q][2]) > 0.f) mloc = fmaxf(mloc, __uint_as_float(ml[q][0]));
                const float mg = wave_max(mloc);
                float lsum = 0.f;
#pragma unroll
                for (int q = 0; q < GRP / 64; ++q) {
                    const float l_c = __uint_as_float(ml[q][2]);
                    const float w = (lane + 64 * q < gn && l_c > 0.f) ? expf(__uint_as_float(ml[q][0]) - mg) : 0.f;
                    sW[wave * GRP + lane + 64 * q] = w;
                    lsum += l_c * w;
                }
                lsum = wave_sum(lsum);
                if (lane == 0) { sM[wave] = mg; sL[wave] = lsum; }
            }
            __syncthreads();
            float o0 = 0.f, o1 = 0.f;
            for (int cb = 0; cb < gn; cb += CB) {
                if (cb > 0) issue_av(cb);
                if (!__all(!bad_av() || !active)) {
                    int spins = 0;
                    do issue_av(cb); while (!__all(!bad_av() || !active) && spin_again(P, spins));
                }
#pragma unroll
                for (int i = 0; i < CB; ++i) {
                    if (cb + i < gn && active) {
                        const float w = sW[myrow * GRP + cb + i];
                        o0 += __uint_as_float(av[i][0]) * w;
                        o1 += __uint_as_float(av[i][2]) * w;
                    }
                }
            }
            if (active) {
                const float mg = sM[myrow], lg = sL[myrow];
                if (lg > 0.f) {
                    const float mnew = fmaxf(mrun, mg);
                    const float so = expf(mrun - mnew), sn = expf(mg - mnew);   // exp(-inf) = 0 at the start
                    num0 = num0 * so + o0 * sn;
                    num1 = num1 * so + o1 * sn;
                    den = den * so + lg * sn;
                    mrun = mnew;
                }
            }
        }
        if (sep) {
            // fold in the attention over the rows written in this step (worked out first, see above)
            __syncthreads();
            if (active) {
                const float mg = sM[SEP_ML + myrow], lg = sL[SEP_ML + myrow];
                const float mnew = fmaxf(mrun, mg);
                const float so = expf(mrun - mnew), sn = expf(mg - mnew);
                num0 = num0 * so + sO[myrow * D + 2 * dp] * sn;
                num1 = num1 * so + sO[myrow * D + 2 * dp + 1] * sn;
                den = den * so + lg * sn;
                mrun = mnew;
            }
        }
        if (active) {
            const int rho = r0 + myrow;
            const int gi = row_seq(P, rho), i = rho - gi * P.M;
            const unsigned oi = (unsigned)((size_t)(b * P.M + i) * P.QD + (hk * grp + gi) * D + 2 * dp);
            sx_st1(ro, oi, num0 / den);
            sx_st1(ro, oi + 1, num1 / den);
        }
    }
}

template <typename WT, int D, int NK, bool SINGLE>
__device__ __forceinline__ void attn_phase(const StepParams& P, int wg, int nwg, int wave, char* smem) {
    typedef AttnCfg<WT, D, NK> C;
    constexpr bool BF = Traits<WT>::BF;
    constexpr int CH = C::CH, CH_LOG = C::CH_LOG, GE = Traits<WT>::GE, KSTEP = Traits<WT>::KSTEP;
    constexpr int NL = GE / 4;                      // 16-byte loads per group of exchanged fp32
    constexpr int STEPS = D / KSTEP;                // MFMA steps along the head dimension
    constexpr int DPL = D / 64;                     // output columns per lane
    const int tid = threadIdx.x, lane = tid & 63;
    const int c = lane & 15, kb = lane >> 4;
    const int grp = P.nq / P.nkv;
    const int Ra = grp * P.M;
    float* sM = reinterpret_cast<float*>(smem + C::OFF_M);
    float* sL = reinterpret_cast<float*>(smem + C::OFF_L);
    float* sP = reinterpret_cast<float*>(smem + C::OFF_P);
    float* sO = reinterpret_cast<float*>(smem + C::OFF_O);
    char* sQ = smem + C::OFF_Q;
    const rsrc_t racc = make_rsrc(P.attn_acc), rml = make_rsrc(P.attn_ml);
    const SxBuf ro = sx_buf(P, P.o_buf);
    const unsigned seq = ps_seq();

    // The loads of a work item are requested while the previous item is still being computed: the
    // K rows and the first query rows right after the score MFMAs, the V rows right after P.V.
    // For these loads to stay in flight the waits in front of their uses must count exactly the
    // younger memory operations, and the compiler can only do that along straight-line code: so a
    // workgroup's last item requests (harmless, clamped) loads as if another one followed; the
    // stores of an item's results are a fixed number per thread; and SINGLE (all g*M query rows
    // fit in one pass of 16: the host knows) removes the loop over the passes.
    uint4 kreg[NK][STEPS];
    typename VRaw<WT, DPL>::type vraw[NK][16];
    u32x4 qx;
    // The query rows of a pass are requested during the previous pass (or item) and put into LDS at
    // its end.  The first look at them is straight-line code, not behind a loop's back edge, so
    // that the wait in front of it counts exactly the younger operations (the V rows) and leaves
    // them in flight.  Only a failed look (the QKV phase has not published the rows yet) asks
    // again, in a loop.
    AttnItem cur = {0, 0, 0, 1, 0};
    const int wkey = 16 * NK * wave;                // this wavefront's keys within a chunk: wkey .. wkey + 16 NK - 1
    // work items: the host's counts, unless the lengths are device data (then the host only knew upper bounds)
    int n_items = P.attn_items, n_merge = P.attn_merge_items;
    if (P.kv_len_dev) {
        n_items = 0; n_merge = 0;
        for (int b = 0; b < P.B; ++b) {
            const int nch = (kvlen_u(b) + P.attn_tail + CH - 1) >> CH_LOG;
            n_items += nch * P.nkv;
            if (nch > 1 || P.attn_sep) n_merge += P.nkv * ((Ra + PS_WAVES - 1) / PS_WAVES);
        }
    }
    if (wg < n_items) {
        cur = attn_decode(P, wg, CH_LOG);
#pragma unroll
        for (int j = 0; j < NK; ++j) attn_load_k<WT, D>(P, cur, cur.ch * CH + wkey + 16 * j, lane, kreg[j]);
        qx = attn_issue_q<WT, D>(P, cur, 0, Ra, grp, tid);   // same order as in the loop: K, Q, then V
#pragma unroll
        for (int j = 0; j < NK; ++j) attn_issue_v<WT, D>(P, cur, cur.ch * CH + wkey + 16 * j, lane, vraw[j]);
        attn_place_q<WT, D>(P, cur, 0, Ra, grp, tid, qx, sQ);
    }
    __syncthreads();
    // One work item.  RQ: the loads of a following item nx are requested here: if there is none
    // (has_next false) they are harmless, clamped loads of the same item, so that the body stays
    // straight-line code.  A workgroup with a single item uses the variant without requests.
    auto do_item = [&](int item, const AttnItem nx, bool has_next, auto RQ) __attribute__((always_inline)) {
        constexpr bool requests = decltype(RQ)::value;
        const int b = cur.b, hk = cur.hk, ch = cur.ch, nch = cur.nch, L = cur.L;
        const int key0 = ch * CH + wkey;            // this wavefront's keys: positions key0 .. key0 + 16 NK - 1
        const int end = L + P.attn_tail;            // positions the blocks cover (see attn_sep)
        const int sk = skipof_u(b);
        stamp(P, wg, 44);

        for (int r0 = 0; r0 < (SINGLE ? 16 : Ra); r0 += 16) {       // 16 query rows per pass
            const int nr = min(16, Ra - r0);
            const bool last_pass = SINGLE || r0 + 16 >= Ra;
            const int rho = r0 + c < Ra ? r0 + c : Ra - 1;
            const int i = rho - row_seq(P, rho) * P.M;
            BRegs<WT, 1> bq[STEPS];
#pragma unroll
            for (int t = 0; t < STEPS; ++t) {
                if constexpr (BF) {
                    bq[t].h[0] = ld16(sQ + (2 * t * 64 + lane) * 16);
                    bq[t].l[0] = ld16(sQ + ((2 * t + 1) * 64 + lane) * 16);
                } else {
                    bq[t].h[0] = ld16(sQ + (t * 64 + lane) * 16);
                }
            }
            // ---- scores of keys 4 kb .. 4 kb + 3 (of each of this wavefront's groups of 16) for query row c
            f32x4 acc[NK][1];
#pragma unroll
            for (int j = 0; j < NK; ++j) {
                acc[j][0] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int t = 0; t < STEPS; ++t) mma_step<WT, 1>(kreg[j][t], bq[t], acc[j]);
            }
            if (!last_pass) {              // request the query rows of the next pass,
                qx = attn_issue_q<WT, D>(P, cur, r0 + 16, Ra, grp, tid);
            } else if constexpr (requests) {   // or, the K rows being consumed, the next item's K and query rows
#pragma unroll
                for (int j = 0; j < NK; ++j) attn_load_k<WT, D>(P, nx, nx.ch * CH + wkey + 16 * j, lane, kreg[j], has_next);
                qx = attn_issue_q<WT, D>(P, nx, 0, Ra, grp, tid);
            }
            stamp(P, wg, 45);
            float sc[NK][4], mloc = -INFINITY;
#pragma unroll
            for (int j = 0; j < NK; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int pos = key0 + 16 * j + 4 * kb + r;
                    // (row i sees the cache and rows sk .. i of this step, sk = the sequence's unused slots; a row of an
                    // unused slot sees what the first used one does, so that it stays finite)
                    const bool vis = r0 + c < Ra && pos < end && pos <= L + max(i, sk) && (pos < L || pos >= L + sk);
                    sc[j][r] = vis ? acc[j][0][r] * P.inv_sqrt_d : -INFINITY;
                    mloc = fmaxf(mloc, sc[j][r]);
                }
            mloc = fmaxf(mloc, __shfl_xor(mloc, 16, 64));
            mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
            __syncthreads();                        // the previous pass is done with the LDS areas
            if (kb == 0) sM[wave * 16 + c] = mloc;
            __syncthreads();
            stamp(P, wg, 46);
            float mrow = -INFINITY;
#pragma unroll
            for (int w = 0; w < PS_WAVES; ++w) mrow = fmaxf(mrow, sM[w * 16 + c]);
            float lloc = 0.f;
#pragma unroll
            for (int j = 0; j < NK; ++j) {
                f32x4 pr;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    pr[r] = sc[j][r] > -INFINITY ? expf(sc[j][r] - mrow) : 0.f;
                    lloc += pr[r];
                }
                *reinterpret_cast<f32x4*>(sP + ((wave * NK + j) * 16 + c) * 16 + 4 * kb) = pr;
            }
            lloc += __shfl_xor(lloc, 16, 64);
            lloc += __shfl_xor(lloc, 32, 64);
            if (kb == 0) sL[wave * 16 + c] = lloc;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // written and read by this wavefront only
            __builtin_amdgcn_wave_barrier();
            // ---- this wavefront's part of P.V for every row of the pass
            if constexpr (NK == 1) {
                float v[16][DPL];
                attn_finish_v<WT, D>(P, cur, key0, lane, vraw[0], v);
                // the raw V rows are consumed: request the next item's, ahead of the arithmetic
                if constexpr (requests)
                    if (last_pass) attn_issue_v<WT, D>(P, nx, nx.ch * CH + wkey, lane, vraw[0], has_next);
                for (int rr = 0; rr < nr; ++rr) {
                    const f32x4* prow = reinterpret_cast<const f32x4*>(sP + (wave * 16 + rr) * 16);
                    float o[DPL];
#pragma unroll
                    for (int e = 0; e < DPL; ++e) o[e] = 0.f;
#pragma unroll
                    for (int k4 = 0; k4 < 4; ++k4) {
                        const f32x4 p4 = prow[k4];
#pragma unroll
                        for (int r = 0; r < 4; ++r)
#pragma unroll
                            for (int e = 0; e < DPL; ++e) o[e] += p4[r] * v[4 * k4 + r][e];
                    }
#pragma unroll
                    for (int e = 0; e < DPL; ++e) sO[(wave * 16 + rr) * D + DPL * lane + e] = o[e];
                }
            } else {
                // the rows' sums stay in registers while the groups of 16 keys are widened one at a time
                float o[16][DPL];
#pragma unroll
                for (int rr = 0; rr < 16; ++rr)
#pragma unroll
                    for (int e = 0; e < DPL; ++e) o[rr][e] = 0.f;
#pragma unroll
                for (int j = 0; j < NK; ++j) {
                    float v[16][DPL];
                    attn_finish_v<WT, D>(P, cur, key0 + 16 * j, lane, vraw[j], v);
                    if constexpr (requests)
                        if (last_pass) attn_issue_v<WT, D>(P, nx, nx.ch * CH + wkey + 16 * j, lane, vraw[j], has_next);
#pragma unroll
                    for (int rr = 0; rr < 16; ++rr) {
                        if (rr < nr) {   // wavefront-uniform
                            const f32x4* prow = reinterpret_cast<const f32x4*>(sP + ((wave * NK + j) * 16 + rr) * 16);
#pragma unroll
                            for (int k4 = 0; k4 < 4; ++k4) {
                                const f32x4 p4 = prow[k4];
#pragma unroll
                                for (int r = 0; r < 4; ++r)
#pragma unroll
                                    for (int e = 0; e < DPL; ++e) o[rr][e] += p4[r] * v[4 * k4 + r][e];
                            }
                        }
                    }
                }
#pragma unroll
                for (int rr = 0; rr < 16; ++rr)
                    if (rr < nr) {
#pragma unroll
                        for (int e = 0; e < DPL; ++e) sO[(wave * 16 + rr) * D + DPL * lane + e] = o[rr][e];
                    }
            }
            stamp(P, wg, 47);
            // every wavefront has read this pass's query rows (before the pass's first barrier):
            // the next ones take their place; they are read after the barrier below
            if (!last_pass) attn_place_q<WT, D>(P, cur, r0 + 16, Ra, grp, tid, qx, sQ);
            else if (requests && has_next) attn_place_q<WT, D>(P, nx, 0, Ra, grp, tid, qx, sQ);
            __syncthreads();
            stamp(P, wg, 48);
            // ---- add the wavefronts' parts in order.  SINGLE: a fixed number of rounds; threads beyond
            // the last element repeat it (same value to the same place)
            constexpr int XR = (16 * D + PS_WG_THREADS - 1) / PS_WG_THREADS;
#pragma unroll
            for (int xi = 0; xi < XR; ++xi) {
                int x = tid + xi * PS_WG_THREADS;
                if constexpr (SINGLE) {
                    x = min(x, nr * D - 1);
                } else {
                    if (x >= nr * D) break;
                }
                const int rr = x / D, dd = x - rr * D;
                float o = 0.f, l = 0.f;
#pragma unroll
                for (int w = 0; w < PS_WAVES; ++w) { o += sO[(w * 16 + rr) * D + dd]; l += sL[w * 16 + rr]; }
                const int rho2 = r0 + rr;
                const int gi2 = row_seq(P, rho2), i2 = rho2 - gi2 * P.M;
                if (nch == 1 && !P.attn_sep) {
                    // the only chunk: normalise and hand the row to the output projection
                    sx_st1(ro, (unsigned)((size_t)(b * P.M + i2) * P.QD + (hk * grp + gi2) * D + dd), o / l);
                } else {
                    // partial (max, sum, unnormalised output) of this chunk, as tagged data
                    ll_st1(racc, (unsigned)(((size_t)item * Ra + rho2) * D + dd), o, seq);
                    if constexpr (!SINGLE) {
                        if (dd < 2) {
                            float mr = -INFINITY;
#pragma unroll
                            for (int w = 0; w < PS_WAVES; ++w) mr = fmaxf(mr, sM[w * 16 + rr]);
                            ll_st1(rml, (unsigned)(((size_t)item * Ra + rho2) * 2 + dd), dd ? l : mr, seq);
                        }
                    }
                }
            }
            if constexpr (SINGLE) {
                if (nch > 1 || P.attn_sep) {   // (max, sum) of row tid / 2: one store per thread, the surplus threads repeat the last
                    const int e = min(tid, 2 * nr - 1), rr = e >> 1;
                    float mr = -INFINITY, l = 0.f;
#pragma unroll
                    for (int w = 0; w < PS_WAVES; ++w) { mr = fmaxf(mr, sM[w * 16 + rr]); l += sL[w * 16 + rr]; }
                    ll_st1(rml, (unsigned)(((size_t)item * Ra + r0 + rr) * 2 + (e & 1)), (e & 1) ? l : mr, seq);
                }
            }
        }
        cur = nx;
        stamp(P, wg, 34);
    };
    if (wg + nwg >= n_items) {
        if (wg < n_items) do_item(wg, cur, false, std::false_type());
    } else if constexpr (NK == 1) {   // (the host uses two key groups per wavefront only when no workgroup gets a second item)
        for (int item = wg; item < n_items; item += nwg) {
            const bool has_next = item + nwg < n_items;
            do_item(item, has_next ? attn_decode(P, item + nwg, CH_LOG) : cur, has_next, std::true_type());
        }
    }

    attn_merge<WT, D, false>(P, wg, nwg, wave, n_merge, CH_LOG, sM, sL, sP, sO);
}

// ------------------------------------------------------------------------------------------
// attention, bf16 storage.  One work unit = (sequence b, kv head hk, block ch of 2^ch_log cache keys, pass of
// 16 query rows); the rows written in this step ride on the sequence's last block.  The wavefronts of the
// workgroup take the block's groups of 16 keys in turn, each with its own running maximum, sum and output
// (online softmax), the next group's K and V rows requested one group ahead; their results meet in LDS once,
// at the end of the unit.  Scores are one MFMA tile per group (K rows = the 16-row operand straight from the
// cache, the query rows split into bf16 high + low parts = the 16-column operand in LDS).  P.V is MFMA work
// too: the score tile leaves the matrix core with a lane holding four consecutive keys of one query row,
// which is the 16-row operand layout of v_mfma_f32_16x16x16_bf16 (P, split into high and low parts); the
// other operand needs four consecutive keys of one value column per lane, so a wavefront passes its 16 value
// rows through LDS with the two rows of a key pair interleaved (one dword = the same column of two keys).
// The host picks the block size so that the units fill the compute units once; a sequence that is a single
// block hands its rows straight to the output projection, else (max, sum, output) per block go to memory
// and attn_merge puts them together.
// ------------------------------------------------------------------------------------------
// LDS data that one wavefront writes and the same wavefront reads: its LDS operations complete in order, so
// all that is needed is that the compiler keeps the order too and that the writes have left the queue.  (A
// workgroup-scope fence would also wait for every global load in flight - the next group's, requested ahead.)
__device__ __forceinline__ void lds_sync_wave() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

template <int D> struct Attn2Cfg {
    static constexpr int G = 2;                                          // groups of 16 keys a wavefront works on at a time
    static constexpr int VSTR = D + 8;                                   // dwords between key pairs of the staged values (no bank conflicts)
    static constexpr int OSTR = D + 4;                                   // floats between rows of a wavefront's output
    static constexpr int OFF_Q = PS_LDS_BASE;                            // 16 query rows as MFMA operands (hi, lo)
    static constexpr int OFF_V = OFF_Q + 16 * D * 4;                     // [waves][G][8 key pairs][VSTR] dwords
    static constexpr int OFF_A = OFF_V + PS_WAVES * G * 8 * VSTR * 4;    // [waves][16] rescale factors of the running output
    static constexpr int OFF_ML = OFF_A + PS_WAVES * 16 * 4;             // [waves][16][2] final (max, sum); attn_merge: sM, sL
    static constexpr int OFF_O = OFF_ML + PS_WAVES * 16 * 2 * 4;         // [waves][16][OSTR] final outputs; attn_merge: weights
    static constexpr int LDS = OFF_O + PS_WAVES * 16 * OSTR * 4;
    static_assert(LDS == ps_attn2_lds_bytes(D), "host and device agree on the layout");
    static_assert(PS_WAVES * 16 * OSTR >= PS_WAVES * 256 + PS_WAVES * D, "attn_merge's weights and rows fit the output area");
};

// block item -> (sequence, kv head, block): the blocks of a sequence are those of attn_nch<true>
__device__ __forceinline__ AttnItem attn_decode2(const StepParams& P, int item, int ch_log) {
    AttnItem it;
    int b = 0, rem = item, nch = 0;
    for (;; ++b) {
        nch = attn_nch<true>(P, b, ch_log);
        if (rem < nch * P.nkv || b + 1 >= P.B) break;
        rem -= nch * P.nkv;
    }
    it.b = b; it.nch = nch; it.hk = rem / nch; it.ch = rem - it.hk * nch; it.L = kvlen_u(b);
    return it;
}

// Maximum / sum over the four lanes (c, 0 .. 3) that share a query row c, returned to all four: two row swaps
// (v_permlane32_swap exchanges the upper half of one register with the lower half of another, v_permlane16_swap
// the odd 16-lane rows of one with the even rows of another; fed the same value twice they yield the value of
// lane ^ 32 resp. lane ^ 16 beside the lane's own)
__device__ __forceinline__ float quad_rows_max(float v) {
    auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float quad_rows_sum(float v) {
    auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// K rows (MFMA operand) and value rows of one group of 16 keys, as they come from memory
template <int STEPS> struct KvRegs { uint4 k[STEPS]; uint4 va[2], vb[2]; };

template <typename WT, int D>
__device__ __forceinline__ void attn_phase2(const StepParams& P, int wg, int nwg, int wave, char* smem) {
    static_assert(Traits<WT>::BF, "bf16 storage");
    typedef Attn2Cfg<D> C;
    constexpr int STEPS = D / 32;                   // MFMA steps along the head dimension
    constexpr int CBN = D / 16;                     // blocks of 16 output columns
    constexpr int VSTR = C::VSTR, OSTR = C::OSTR, G = C::G;
    constexpr float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef KvRegs<STEPS> Kv;
    const int tid = threadIdx.x, lane = tid & 63;
    const int c = lane & 15, kb = lane >> 4;
    const int grp = P.nq / P.nkv;
    const int Ra = grp * P.M;
    const int ch_log = P.attn_ch_log, CH = 1 << ch_log, npass = P.attn_npass;
    const float scale2 = P.inv_sqrt_d * LOG2E;     // scores are kept in units of ln 2: exponentials are v_exp_f32
    char* sQ = smem + C::OFF_Q;
    unsigned* sV = reinterpret_cast<unsigned*>(smem + C::OFF_V) + wave * G * 8 * VSTR;
    float* sA = reinterpret_cast<float*>(smem + C::OFF_A) + wave * 16;
    float* sML = reinterpret_cast<float*>(smem + C::OFF_ML);
    float* sO = reinterpret_cast<float*>(smem + C::OFF_O);
    const rsrc_t racc = make_rsrc(P.attn_acc), rml = make_rsrc(P.attn_ml), rn = make_rsrc(act_ptr(P, P.kvnew));
    const SxBuf ro = sx_buf(P, P.o_buf);
    const unsigned seq = ps_seq();
    const int vm = min(lane / CBN, 7), vcb = lane % CBN;   // this lane's key pair and column block of the value rows
    const bool vlive = lane / CBN < 8;

    // work units and merge items: the host's counts, unless the lengths are device data (then it only knew upper bounds)
    int n_units = P.attn_units, n_merge = P.attn_merge_items;
    if (P.kv_len_dev) {
        n_units = 0; n_merge = 0;
        for (int b = 0; b < P.B; ++b) {
            const int nch = attn_nch<true>(P, b, ch_log);
            n_units += nch * P.nkv * npass;
            if (nch > 1) n_merge += P.nkv * ((Ra + PS_WAVES - 1) / PS_WAVES);
        }
    }
    const int n_items = npass == 1 ? n_units : (int)__umulhi((unsigned)n_units, P.pass_magic);
    for (int u = wg; u < n_units; u += nwg) {
        // unit -> (pass, block item), the passes of a block n_items units apart (workgroups on the same XCD when that
        // is a multiple of 8: they read the same K and V rows)
        int item = u, pass = 0;
        while (item >= n_items) { item -= n_items; ++pass; }
        const AttnItem it = attn_decode2(P, item, ch_log);
        const int r0 = 16 * pass, nr = min(16, Ra - r0);
        const int k_lo = it.ch << ch_log, k_hi = min(it.L, k_lo + CH);
        const int ncs = (k_hi - k_lo + 15) >> 4;                    // groups of 16 cache keys (none: empty cache)
        const int nts = it.ch == it.nch - 1 ? (P.M + 15) >> 4 : 0;  // groups of rows written in this step
        const size_t cache_row0 = (size_t)P.kv_off[it.b] * P.nkv + it.hk;   // in units of D elements
        stamp(P, wg, 44);

        // K rows of cache keys key0 .. key0 + 15 as the MFMA operand (lane (c, kb): bytes [64 t + 16 kb, +16) of key
        // c) and the value rows (lane (vm, vcb): columns [16 vcb, +16) of keys 2 vm and 2 vm + 1); keys beyond the
        // block are clamped (masked later)
        auto load_cache = [&](int s, Kv& r) __attribute__((always_inline)) {
            const int key0 = k_lo + 16 * s, k_last = max(k_hi - 1, 0);
            const int kp = min(key0 + c, k_last);
            const char* krow = (const char*)P.kc + ((cache_row0 + (size_t)kp * P.nkv) * D) * 2 + kb * 16;
#pragma unroll
            for (int t = 0; t < STEPS; ++t) r.k[t] = ld16(krow + t * 64);
            const int pa = min(key0 + 2 * vm, k_last), pb = min(key0 + 2 * vm + 1, k_last);
            const char* pa_ = (const char*)P.vc + ((cache_row0 + (size_t)pa * P.nkv) * D) * 2 + vcb * 32;
            const char* pb_ = (const char*)P.vc + ((cache_row0 + (size_t)pb * P.nkv) * D) * 2 + vcb * 32;
            r.va[0] = ld16(pa_); r.va[1] = ld16(pa_ + 16);
            r.vb[0] = ld16(pb_); r.vb[1] = ld16(pb_ + 16);
        };
        // the same for rows 16 ts .. 16 ts + 15 of this step: from the exchange buffer, once the QKV phase has
        // published them (fp32, exactly representable in bf16: they were rounded when they went to the cache)
        auto load_tail = [&](int ts, Kv& r) __attribute__((always_inline)) {
            const int jk = min(16 * ts + c, P.M - 1);
            const int ja = min(16 * ts + 2 * vm, P.M - 1), jb = min(16 * ts + 2 * vm + 1, P.M - 1);
            const unsigned kbase = (unsigned)(((size_t)(it.b * P.M + jk) * 2) * P.KVD + it.hk * D + kb * 8);
            const unsigned abase = (unsigned)(((size_t)(it.b * P.M + ja) * 2 + 1) * P.KVD + it.hk * D + vcb * 16);
            const unsigned bbase = (unsigned)(((size_t)(it.b * P.M + jb) * 2 + 1) * P.KVD + it.hk * D + vcb * 16);
            u32x4 kx[STEPS][2], ax[4], bx[4];
            int spins = 0;
            for (;;) {
#pragma unroll
                for (int t = 0; t < STEPS; ++t)
#pragma unroll
                    for (int h = 0; h < 2; ++h) kx[t][h] = coh_ld16(rn, (kbase + 32 * t + 4 * h) * 4);
#pragma unroll
                for (int h = 0; h < 4; ++h) { ax[h] = coh_ld16(rn, (abase + 4 * h) * 4); bx[h] = coh_ld16(rn, (bbase + 4 * h) * 4); }
                unsigned bad = 0;   // all loads first, then all checks: no wait between the loads
#pragma unroll
                for (int t = 0; t < STEPS; ++t) bad |= (unsigned)!sx_ok(kx[t][0]) | (unsigned)!sx_ok(kx[t][1]);
#pragma unroll
                for (int h = 0; h < 4; ++h) bad |= (unsigned)!sx_ok(ax[h]) | (unsigned)!sx_ok(bx[h]);
                if (__all(!bad) || !spin_again(P, spins)) break;
            }
            auto pk = [](u32x4 lo, u32x4 hi) __attribute__((always_inline)) {
                return make_uint4(pack_bf16x2(__uint_as_float(lo[0]), __uint_as_float(lo[1])), pack_bf16x2(__uint_as_float(lo[2]), __uint_as_float(lo[3])),
                                  pack_bf16x2(__uint_as_float(hi[0]), __uint_as_float(hi[1])), pack_bf16x2(__uint_as_float(hi[2]), __uint_as_float(hi[3])));
            };
#pragma unroll
            for (int t = 0; t < STEPS; ++t) r.k[t] = pk(kx[t][0], kx[t][1]);
            r.va[0] = pk(ax[0], ax[1]); r.va[1] = pk(ax[2], ax[3]);
            r.vb[0] = pk(bx[0], bx[1]); r.vb[1] = pk(bx[2], bx[3]);
        };

        // A wavefront works on G = 2 groups at a time (groups s and s + 8 of the block), and the K and V rows of the
        // next two are requested while it does: two sets of registers take turns.  Every request is unconditional
        // (beyond the last group it repeats a row of the block: nobody uses it), so that the waits in front of the
        // uses count exactly the younger requests and leave them in flight.
        Kv ra[G], rb[G];
#pragma unroll
        for (int g = 0; g < G; ++g) load_cache(wave + g * PS_WAVES, ra[g]);      // ahead of the wait for the query rows
        u32x4 qx = attn_issue_q<WT, D>(P, it, r0, Ra, grp, tid);
#pragma unroll
        for (int g = 0; g < G; ++g) load_cache(wave + (G + g) * PS_WAVES, rb[g]);
        attn_place_q<WT, D>(P, it, r0, Ra, grp, tid, qx, sQ);
        __syncthreads();                                             // (also: the previous unit's results have been read)
        stamp(P, wg, 45);
        // this lane's query row (column c of the score tile) and its index among the M rows of its sequence
        const bool qlive = c < nr;
        const int sk = skipof_u(it.b);               // unused leading slots of the sequence: no keys; their rows see what the first used row does
        const int rho_c = min(r0 + c, Ra - 1);
        const int qi = rho_c - row_seq(P, rho_c) * P.M;
        float m_run = -INFINITY, l_run = 0.f;                        // of query c (the same in the four lanes that share it); m in units of ln 2
        f32x4 oacc[CBN];                                             // lane (c, kb): column 16 j + c of rows 4 kb .. 4 kb + 3
#pragma unroll
        for (int j = 0; j < CBN; ++j) oacc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

        // NG groups of 16 keys at once.  TAIL: rows base .. base + 15 of this step (row qi sees rows sk .. qi); else
        // cache positions base + 128 g .. + 15 (every row of the step sees all valid cache positions)
        auto process = [&](const Kv* r, int base, auto NG_, auto TAIL) __attribute__((always_inline)) {
            constexpr bool tail = decltype(TAIL)::value;
            constexpr int NG = decltype(NG_)::value;
            f32x4 acc[NG][1];
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[g][0] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < STEPS; ++t) {
                BRegs<WT, 1> bq;                                     // the query rows (read per step: registers are scarce)
                bq.h[0] = ld16(sQ + (2 * t * 64 + lane) * 16);
                bq.l[0] = ld16(sQ + ((2 * t + 1) * 64 + lane) * 16);
#pragma unroll
                for (int g = 0; g < NG; ++g) mma_step<WT, 1>(r[g].k[t], bq, acc[g]);
            }
            float sc[NG][4], mt = -INFINITY;
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int j = base + 16 * PS_WAVES * g + 4 * kb + e;
                    const bool vis = qlive && (tail ? (j >= sk && j <= max(qi, sk) && j < P.M) : j < k_hi);
                    sc[g][e] = vis ? acc[g][0][e] * scale2 : -INFINITY;
                    mt = fmaxf(mt, sc[g][e]);
                }
            mt = quad_rows_max(mt);
            const float m_new = fmaxf(m_run, mt);
            const float alpha = m_new > -INFINITY ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.f;   // 2^-inf = 0 when nothing was seen before
            const float m_use = m_new > -INFINITY ? m_new : 0.f;     // (all masked: every exponent is -inf)
            f32x4 pr[NG];
            float ls = 0.f;
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    pr[g][e] = __builtin_amdgcn_exp2f(sc[g][e] - m_use);
                    ls += pr[g][e];
                }
            ls = quad_rows_sum(ls);
            l_run = l_run * alpha + ls;
            m_run = m_new;
            if (kb == 0) sA[c] = alpha;
            // the value rows into LDS, the two keys of a pair interleaved column by column
            if (vlive) {
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    unsigned ov[16];
#pragma unroll
                    for (int w = 0; w < 8; ++w) {
                        const unsigned a2 = w < 4 ? (&r[g].va[0].x)[w] : (&r[g].va[1].x)[w - 4], b2 = w < 4 ? (&r[g].vb[0].x)[w] : (&r[g].vb[1].x)[w - 4];
                        ov[2 * w] = __builtin_amdgcn_perm(b2, a2, 0x05040100u);       // (low half of a2, low half of b2)
                        ov[2 * w + 1] = __builtin_amdgcn_perm(b2, a2, 0x07060302u);   // (high half of a2, high half of b2)
                    }
                    uint4* dst = reinterpret_cast<uint4*>(sV + (g * 8 + vm) * VSTR + 16 * vcb);
#pragma unroll
                    for (int w = 0; w < 4; ++w) dst[w] = make_uint4(ov[4 * w], ov[4 * w + 1], ov[4 * w + 2], ov[4 * w + 3]);
                }
            }
            lds_sync_wave();                                         // written and read by this wavefront only
            __builtin_amdgcn_wave_barrier();
            // rescale the running output (rows 4 kb .. 4 kb + 3) unless no row's maximum moved
            const f32x4 al = *reinterpret_cast<const f32x4*>(sA + 4 * kb);
            if (__any(alpha != 1.f)) {
#pragma unroll
                for (int j = 0; j < CBN; ++j) oacc[j] *= al;
            }
            // P (query c, keys 4 kb .. 4 kb + 3 of every group) as the 16-row operand, split into bf16 high and low parts
            unsigned ph2[NG][2], pl2[NG][2];
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                ph2[g][0] = pack_bf16x2(pr[g][0], pr[g][1]); ph2[g][1] = pack_bf16x2(pr[g][2], pr[g][3]);
                pl2[g][0] = pack_bf16x2(pr[g][0] - __uint_as_float(ph2[g][0] << 16), pr[g][1] - __uint_as_float(ph2[g][0] & 0xFFFF0000u));
                pl2[g][1] = pack_bf16x2(pr[g][2] - __uint_as_float(ph2[g][1] << 16), pr[g][3] - __uint_as_float(ph2[g][1] & 0xFFFF0000u));
            }
            if constexpr (NG == 2) {
                // two groups = 32 keys: one v_mfma_f32_16x16x32_bf16 per part and column block; its contraction index
                // 8 kb + e is key 4 kb + e of the first group (e < 4) or key 4 kb + e - 4 of the second
                const bf16x8 pa = __builtin_bit_cast(bf16x8, make_uint4(ph2[0][0], ph2[0][1], ph2[1][0], ph2[1][1]));
                const bf16x8 pb = __builtin_bit_cast(bf16x8, make_uint4(pl2[0][0], pl2[0][1], pl2[1][0], pl2[1][1]));
#pragma unroll
                for (int j = 0; j < CBN; ++j) {
                    const bf16x8 vv = __builtin_bit_cast(bf16x8, make_uint4(sV[(2 * kb) * VSTR + 16 * j + c], sV[(2 * kb + 1) * VSTR + 16 * j + c],
                                                                            sV[(8 + 2 * kb) * VSTR + 16 * j + c], sV[(8 + 2 * kb + 1) * VSTR + 16 * j + c]));
                    const f32x4 t = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, vv, oacc[j], 0, 0, 0);
                    oacc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pb, vv, t, 0, 0, 0);
                }
            } else {
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    const s16x4 ph_ = __builtin_bit_cast(s16x4, make_uint2(ph2[g][0], ph2[g][1])), pl_ = __builtin_bit_cast(s16x4, make_uint2(pl2[g][0], pl2[g][1]));
#pragma unroll
                    for (int j = 0; j < CBN; ++j) {
                        // values of keys 4 kb .. 4 kb + 3, column 16 j + c: the key pairs 2 kb and 2 kb + 1
                        const unsigned w0 = sV[(g * 8 + 2 * kb) * VSTR + 16 * j + c], w1 = sV[(g * 8 + 2 * kb + 1) * VSTR + 16 * j + c];
                        const s16x4 vv = __builtin_bit_cast(s16x4, make_uint2(w0, w1));
                        const f32x4 t = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ph_, vv, oacc[j], 0, 0, 0);
                        oacc[j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pl_, vv, t, 0, 0, 0);
                    }
                }
            }
            lds_sync_wave();
            __builtin_amdgcn_wave_barrier();                         // the next groups overwrite the staged values
        };
        typedef std::integral_constant<int, G> NGG;
        typedef std::integral_constant<int, 1> NG1;
        // ra holds groups (s, s + 8), rb groups (s + 16, s + 24); requests only while ra has a successor, so a
        // block of up to 32 groups requests nothing it does not use
        int s = wave;
        for (; s + 2 * G * PS_WAVES < ncs; s += 2 * G * PS_WAVES) {
            process(ra, k_lo + 16 * s, NGG(), std::false_type());
#pragma unroll
            for (int g = 0; g < G; ++g) load_cache(s + (2 * G + g) * PS_WAVES, ra[g]);
            process(rb, k_lo + 16 * (s + G * PS_WAVES), NGG(), std::false_type());
#pragma unroll
            for (int g = 0; g < G; ++g) load_cache(s + (3 * G + g) * PS_WAVES, rb[g]);
        }
        if (s < ncs) process(ra, k_lo + 16 * s, NGG(), std::false_type());
        if (s + G * PS_WAVES < ncs) process(rb, k_lo + 16 * (s + G * PS_WAVES), NGG(), std::false_type());
        // the rows of this step come last (they are the last to arrive), taken by the wavefronts next in turn
        for (int ts = 0; ts < nts; ++ts) {
            if (((ncs + ts) & (PS_WAVES - 1)) != wave) continue;
            load_tail(ts, ra[0]);
            process(ra, 16 * ts, NG1(), std::true_type());
        }
        stamp(P, wg, 47);
        // ---- the wavefronts' results meet in LDS
        if (kb == 0) { sML[(wave * 16 + c) * 2] = m_run; sML[(wave * 16 + c) * 2 + 1] = l_run; }
#pragma unroll
        for (int j = 0; j < CBN; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) sO[(wave * 16 + 4 * kb + e) * OSTR + 16 * j + c] = oacc[j][e];
        __syncthreads();
        for (int x = tid; x < nr * (D / 4); x += PS_WG_THREADS) {
            const int rr = x / (D / 4), dd = 4 * (x - rr * (D / 4));
            float mx = -INFINITY;
#pragma unroll
            for (int w = 0; w < PS_WAVES; ++w) mx = fmaxf(mx, sML[(w * 16 + rr) * 2]);
            f32x4 num = {0.f, 0.f, 0.f, 0.f};
            float den = 0.f;
#pragma unroll
            for (int w = 0; w < PS_WAVES; ++w) {
                const float mw = sML[(w * 16 + rr) * 2];
                const float f = mw > -INFINITY ? __builtin_amdgcn_exp2f(mw - mx) : 0.f;
                num += *reinterpret_cast<const f32x4*>(sO + (w * 16 + rr) * OSTR + dd) * f;
                den += sML[(w * 16 + rr) * 2 + 1] * f;
            }
            const int rho = r0 + rr;
            const int gi = row_seq(P, rho), i = rho - gi * P.M;
            if (it.nch == 1) {
                // the only block: normalise and hand the row to the output projection (every row sees at least itself)
                sx_st4(ro, (unsigned)((size_t)(it.b * P.M + i) * P.QD + (it.hk * grp + gi) * D + dd), num * (1.0f / den));
            } else {
                // partial (max, sum, unnormalised output) of this block, as tagged data; the maximum in natural units
                ll_st4(racc, (unsigned)(((size_t)item * Ra + rho) * D + dd), num, seq);
                if (dd == 0) {
                    ll_st1(rml, (unsigned)(((size_t)item * Ra + rho) * 2), mx * LN2, seq);
                    ll_st1(rml, (unsigned)(((size_t)item * Ra + rho) * 2 + 1), den, seq);
                }
            }
        }
        stamp(P, wg, 48);
    }
    stamp(P, wg, 34);
    float* sM = sML;
    attn_merge<WT, D, true>(P, wg, nwg, wave, n_merge, ch_log, sM, sM + 128, sO, sO + PS_WAVES * 256);
}

// ------------------------------------------------------------------------------------------
// LM-head merge of one output row by one workgroup.  Thread p fetches workgroup p's statistics
// of the row (max, sum of exponentials, its sorted top-k keys) in one round of loads; every
// wavefront merges the lists of its 64 threads into a sorted top-k, wavefront 0 merges those.
// Keys are unique, so "the largest key below the previous winner" enumerates them in order.
// sk: LDS scratch of PS_MERGE_BYTES.
// ------------------------------------------------------------------------------------------
#define PS_MAX_TOPK 32
#define PS_MERGE_BYTES (PS_WAVES * PS_MAX_TOPK * 8 + PS_WAVES * 8 + PS_WAVES * 8)
__device__ __forceinline__ void lm_merge_row(const StepParams& P, int m, int wave, char* scratch) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int nparts = min(P.ph[PH_LMHEAD].nwg, P.ph[PH_LMHEAD].T);   // workgroups that had vocabulary tiles
    const int topk = P.topk;
    const unsigned stride = 4 + 2 * topk;                  // tagged elements per (workgroup, row)
    const unsigned pstride = (unsigned)P.Rtot * stride;
    const rsrc_t rl = make_rsrc(P.lm_part);
    const unsigned seq = ps_seq();
    u64* sk = reinterpret_cast<u64*>(scratch);                              // [waves][PS_MAX_TOPK] keys
    float* sf = reinterpret_cast<float*>(scratch + PS_WAVES * PS_MAX_TOPK * 8);   // [waves] max, [waves] sum
    u64* sg = reinterpret_cast<u64*>(scratch + PS_WAVES * PS_MAX_TOPK * 8 + PS_WAVES * 8);   // [waves] the draw's keys
    const bool mine = tid < nparts;                        // host: nparts <= PS_WG_THREADS
    const unsigned base = ((unsigned)m * stride + (mine ? tid : 0) * pstride) * 8;   // bytes
    constexpr int KB = 8;                                  // keys requested per round trip
    u64 keys[PS_MAX_TOPK], gkey = 0;
    float pmax = -INFINITY, psum = 0.f;
#pragma unroll
    for (int t0 = 0; t0 < PS_MAX_TOPK; t0 += KB) {
        if (t0 >= topk) {
#pragma unroll
            for (int i = 0; i < KB; ++i) keys[t0 + i] = 0;
            continue;
        }
        u32x4 hd, kr[KB], gk;
        int spins = 0;
        for (;;) {
            hd = coh_ld16(rl, base);                       // {max, tag, sum, tag}
#pragma unroll
            for (int i = 0; i < KB; ++i) {
                const int t = t0 + i < topk ? t0 + i : topk - 1;
                kr[i] = coh_ld16(rl, base + (2 + 2 * t) * 8);   // {low, tag, high, tag}
            }
            gk = coh_ld16(rl, base + ((t0 == 0 && P.sample_ids) ? 2 + 2 * topk : 0) * 8);   // the draw's key (else the head again)
            unsigned bad = (unsigned)(hd[1] != seq) | (unsigned)(hd[3] != seq) | (unsigned)(gk[1] != seq) | (unsigned)(gk[3] != seq);   // all loads first, then all checks
#pragma unroll
            for (int i = 0; i < KB; ++i) bad |= (unsigned)(kr[i][1] != seq) | (unsigned)(kr[i][3] != seq);
            if (__all(!bad || !mine) || !spin_again(P, spins)) break;
        }
        if (t0 == 0 && mine) { pmax = __uint_as_float(hd[0]); psum = __uint_as_float(hd[2]); gkey = ((u64)gk[2] << 32) | gk[0]; }
#pragma unroll
        for (int i = 0; i < KB; ++i)
            keys[t0 + i] = (mine && t0 + i < topk) ? (((u64)kr[i][2] << 32) | kr[i][0]) : 0;
    }
    stamp(P, blockIdx.x, 41);
    // Has any wait of this step been given up (see spin_again)?  Whoever gave up raised the flag before it
    // published anything, so now that all statistics of the row are here the flag tells; requested here,
    // looked at when the outputs are written.
    const unsigned gave_up = ld_agent_u32(P.error_flag);
    // this wavefront's share of the log-sum-exp and its sorted top-k
    const float wmax = wave_max(pmax);
    if (lane == 0) sf[wave] = wmax;
    if (P.sample_ids) {
        const u64 wg_best = wave_max_u64(gkey);
        if (lane == 0) sg[wave] = wg_best;
    }
    u64 prev = ~0ull;
    for (int t = 0; t < topk; ++t) {
        u64 best = 0;
#pragma unroll
        for (int i0 = 0; i0 < PS_MAX_TOPK; i0 += KB) {
            if (i0 < topk) {   // entries beyond topk are "none"
#pragma unroll
                for (int i = i0; i < i0 + KB; ++i)
                    if (keys[i] < prev && keys[i] > best) best = keys[i];
            }
        }
        best = wave_max_u64(best);
        if (lane == 0) sk[wave * PS_MAX_TOPK + t] = best;
        prev = best;                                       // 0: exhausted, every later entry is "none"
    }
    stamp(P, blockIdx.x, 43);
    __syncthreads();
    stamp(P, blockIdx.x, 49);
    float mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < PS_WAVES; ++w) mx = fmaxf(mx, sf[w]);
    const float wsum = wave_sum(pmax > -INFINITY ? psum * expf(pmax - mx) : 0.f);
    if (lane == 0) sf[PS_WAVES + wave] = wsum;
    __syncthreads();
    stamp(P, blockIdx.x, 42);
    if (wave == 0) {
        float se = 0.f;
#pragma unroll
        for (int w = 0; w < PS_WAVES; ++w) se += sf[PS_WAVES + w];
        const float lse = gave_up ? __uint_as_float(0x7FC00000u) : mx + logf(se);   // a step that gave up a wait: NaN, ids -1
        if (lane == 0) P.lse[m] = lse;
        if (P.sample_ids && lane == 0) {
            u64 best = 0;
#pragma unroll
            for (int w = 0; w < PS_WAVES; ++w) best = sg[w] > best ? sg[w] : best;
            const int id = key_id(best);
            // the winner's own logit: its perturbed value minus its Gumbel number
            P.sample_ids[m] = (gave_up || !best) ? -1 : id;
            if (P.sample_p) P.sample_p[m] = (gave_up || !best) ? 0.f : expf(key_value(best) - gumbel_of(P, m, id) - lse);
        }
        // PS_WAVES sorted lists of topk keys: 4 candidates per lane
        constexpr int CPL = PS_WAVES * PS_MAX_TOPK / 64;
        u64 cand[CPL];
#pragma unroll
        for (int i = 0; i < CPL; ++i) {
            const int x = lane + 64 * i, w = x / PS_MAX_TOPK, t = x - w * PS_MAX_TOPK;
            cand[i] = t < topk ? sk[x] : 0;
        }
        u64 prev2 = ~0ull;
        for (int t = 0; t < topk; ++t) {
            u64 best = 0;
#pragma unroll
            for (int i = 0; i < CPL; ++i)
                if (cand[i] < prev2 && cand[i] > best) best = cand[i];
            best = wave_max_u64(best);
            if (lane == 0) {
                P.top_ids[(size_t)m * topk + t] = gave_up ? -1 : (best ? key_id(best) : 0x7FFFFFFF);
                P.top_p[(size_t)m * topk + t] = (best && !gave_up) ? expf(key_value(best) - lse) : 0.f;
            }
            prev2 = best;
        }
        stamp(P, blockIdx.x, 56);
    }
    __syncthreads();   // the scratch is reused by the next row
}

// ------------------------------------------------------------------------------------------
// kernels
// ------------------------------------------------------------------------------------------
// Every kernel starts by reading the step counter: the step's number goes to LDS.  In the kernel
// that ends a step (count = true) every workgroup also takes a ticket; the workgroup with the
// last ticket - by then all of them have read the counter - advances it in step_end.  The ticket
// is only looked at when the kernel ends, so its round trip costs nothing.  step_read only
// requests (thread 0 returns the number, the others 0); the persistent kernel hands the number to
// its first phase, which stores it to LDS just before its first barrier: the first phase reads
// only the step's inputs, so the counter's round trip hides behind the first activation loads.
__device__ __forceinline__ unsigned step_read(const StepParams& P, bool count, unsigned& ticket) {
    unsigned seq = 0;
    ticket = 0xFFFFFFFFu;
    if (threadIdx.x == 0) {
        seq = ld_agent_u32(P.step_ctr) + 1u;
        if (seq == 0u) seq = 2u;   // 0 is what cleared exchange buffers hold; even, so the copies keep alternating
        if (count) ticket = __hip_atomic_fetch_add(P.done_ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return seq;
}
__device__ __forceinline__ unsigned step_begin(const StepParams& P, bool count) {
    unsigned ticket;
    const unsigned seq = step_read(P, count, ticket);
    if (threadIdx.x == 0) *(lds_u32*)(unsigned)PS_LDS_SEQ = seq;
    kv_fill(P);
    __syncthreads();
    return ticket;
}
__device__ __forceinline__ void step_end(const StepParams& P, unsigned ticket, unsigned nwg) {
    if (threadIdx.x == 0 && ticket == nwg - 1u) {
        unsigned* foot = P.foot_mem + (ps_seq() & 1u) * PS_FOOT_INTS;   // read by the next step (sx_reset_stale)
        for (int i = 0; i < PS_FOOT_INTS; ++i) st_agent_u32(foot + i, P.foot[i]);
        st_agent_u32(P.done_ctr, 0u);
        st_agent_u32(P.step_ctr, ps_seq());
    }
}

template <typename WT, int MT, int PH>
__global__ void __launch_bounds__(PS_WG_THREADS, 1) gemm_kernel(const StepParams P) {
    extern __shared__ __attribute__((aligned(256))) char smem[];
    uint4 wb[PS_U];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    step_begin(P, false);
    preload_weights(wb, first_stream(P, PH, blockIdx.x, wave), (threadIdx.x & 63) * 16);
    gemm_phase<WT, MT, PH>(P, blockIdx.x, wave, smem, wb, P.ph[PH].wpack);
}

template <typename WT, int D, int NK, bool SINGLE>
__global__ void __launch_bounds__(PS_WG_THREADS) attn_kernel(const StepParams P) {
    extern __shared__ __attribute__((aligned(256))) char smem[];
    step_begin(P, false);
    sx_reset_stale(P, blockIdx.x, gridDim.x);
    attn_phase<WT, D, NK, SINGLE>(P, blockIdx.x, gridDim.x, __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), smem);
}

template <typename WT, int D>
__global__ void __launch_bounds__(PS_WG_THREADS) attn2_kernel(const StepParams P) {
    extern __shared__ __attribute__((aligned(256))) char smem[];
    step_begin(P, false);
    sx_reset_stale(P, blockIdx.x, gridDim.x);
    attn_phase2<WT, D>(P, blockIdx.x, gridDim.x, __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), smem);
}

static __global__ void __launch_bounds__(PS_WG_THREADS) lm_merge_kernel(const StepParams P) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const unsigned ticket = step_begin(P, true);   // the last kernel of a step in this mode
    lm_merge_row(P, blockIdx.x, __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), smem + PS_LDS_BASE);
    step_end(P, ticket, gridDim.x);
}

static __global__ void __launch_bounds__(256) probs_kernel(const StepParams P) {
    const int m = blockIdx.y;
    const float lse = P.lse[m];
    for (int n = blockIdx.x * 256 + threadIdx.x; n < P.V; n += gridDim.x * 256)
        P.probs[(size_t)m * P.V + n] = expf(P.logits_store[(size_t)m * P.V + n] * P.inv_temp - lse);
}

// The whole step in one persistent kernel: gridDim.x workgroups, all resident.  No grid-wide
// synchronisation: the phases are chained by the exchanged data itself.  While a workgroup waits
// for the activations of its next phase, the first weight loads of that phase are already in
// flight.
template <typename WT, int D, int MT>
__global__ void __launch_bounds__(PS_WG_THREADS, 1) fused_kernel(const StepParams P) {
    extern __shared__ __attribute__((aligned(256))) char smem[];
    const int wg = blockIdx.x, lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint4 wb[PS_U];
#ifdef PS_TIMELINE
    if (threadIdx.x < 64) *tl_slot(threadIdx.x) = 0;    // a stamp nobody takes reads as 0
    __syncthreads();
#endif
    stamp_wall(P, wg, 0);
    stamp(P, wg, 1);
    unsigned ticket;
    const unsigned my_seq = step_read(P, false, ticket);
    kv_fill(P);                                  // (read after the first phase's barriers at the earliest)
    preload_weights(wb, first_stream(P, PH_QKV, wg, wave), lane * 16);
    // (bf16 storage: the attention needs the registers; the output projection's first weight loads are
    // requested after it - a workgroup without attention work gets there at once)
    gemm_phase<WT, MT, PH_QKV>(P, wg, wave, smem, wb, Traits<WT>::BF ? P.ph[PH_OPROJ].wpack : first_stream(P, PH_OPROJ, wg, wave), my_seq);
    __syncthreads();
    stamp(P, wg, 32);
    if constexpr (Traits<WT>::BF) {
        attn_phase2<WT, D>(P, wg, gridDim.x, wave, smem);
        preload_weights(wb, first_stream(P, PH_OPROJ, wg, wave), lane * 16);
    } else {
        switch (2 * P.attn_nk + P.attn_single) {
            case 2: attn_phase<WT, D, 1, false>(P, wg, gridDim.x, wave, smem); break;
            case 3: attn_phase<WT, D, 1, true>(P, wg, gridDim.x, wave, smem); break;
            default: attn_phase<WT, D, 2, true>(P, wg, gridDim.x, wave, smem); break;   // (host: two key groups only with a single pass)
        }
    }
    __syncthreads();
    stamp(P, wg, 36);
    // the ticket (see step_read) is taken here: the next thing this workgroup does is wait for the
    // attention outputs of all the others, so the atomic's round trip delays nothing
    if (threadIdx.x == 0) ticket = __hip_atomic_fetch_add(P.done_ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    gemm_phase<WT, MT, PH_OPROJ>(P, wg, wave, smem, wb, first_stream(P, PH_GATEUP, wg, wave));
    __syncthreads();
    gemm_phase<WT, MT, PH_GATEUP>(P, wg, wave, smem, wb, first_stream(P, PH_DOWN, wg, wave));
    __syncthreads();
    gemm_phase<WT, MT, PH_DOWN>(P, wg, wave, smem, wb, first_stream(P, PH_LMHEAD, wg, wave));
    __syncthreads();
    gemm_phase<WT, MT, PH_LMHEAD>(P, wg, wave, smem, wb, P.ph[PH_QKV].wpack);
    __syncthreads();
    // output row m is merged by the m-th workgroup from the end: the last workgroups have the fewest
    // vocabulary tiles (the last round of tiles is not full), so they are the first to be ready for it
    stamp(P, wg, 40);
    // here most workgroups have nothing left to do, and those that merge an output row would only wait for the
    // slowest workgroup's statistics
    sx_reset_stale(P, wg, gridDim.x);
    for (int m = (int)gridDim.x - 1 - wg; m < P.Rtot; m += gridDim.x) lm_merge_row(P, m, wave, smem + PS_LDS_BASE);
    step_end(P, ticket, gridDim.x);
    stamp(P, wg, 62);
    stamp_wall(P, wg, 63);
    flush_stamps(P, wg);
}
