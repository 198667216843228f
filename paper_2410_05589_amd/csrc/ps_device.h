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
// They run either as one persistent kernel (one 1024-thread workgroup per compute unit, grid
// barriers between phases, the next phase's first weight loads already in flight across each
// barrier) or as one kernel per phase (profiling and fallback).
//
// GEMM engine.  Weights are the 16-row MFMA operand.  At init they are repacked so that one
// step (64 bytes of each of a tile's 16 rows) is one contiguous KiB in lane order; a wavefront
// streams its tiles with 16-byte non-temporal loads, 8 in flight per lane, waiting only for the
// oldest.  The few activation rows are the 16-column operand, staged once per workgroup in LDS.
// bf16 weights use v_mfma_f32_16x16x32_bf16 twice per step: the fp32 activations are split into
// a bf16 high and a bf16 low part (x = hi + lo to ~2^-17), so products with the exactly-bf16
// weights keep fp32-class accuracy at no extra weight traffic.  f32 weights use
// v_mfma_f32_16x16x4_f32.  Accumulation is fp32.  RMSNorm is folded in: the panel holds
// x (.) gain, the per-row factor 1/rms multiplies the accumulator in the epilogue.
// The contraction dimension is cut across workgroups (S slices) and/or across the wavefronts of
// a workgroup (KW).  Slices meet through global fragments; the wavefront that arrives last at a
// tile's counter adds the S fragments in slice order (results do not depend on arrival order)
// and runs the phase epilogue.
//
// Data that one workgroup writes and another reads inside the same step (activations between
// phases, split-K fragments, attention partials, LM-head statistics) is exchanged WITHOUT
// barriers, counters or fences: every 4-byte value travels with a 4-byte sequence number of the
// step in one 8-byte unit, written and read with agent-scope (sc1) buffer accesses that write
// through / bypass the per-XCD L2.  A consumer simply re-reads a unit until its sequence number
// is the current step's.  The persistent kernel therefore has no grid-wide synchronisation:
// each workgroup walks through the phases at its own pace and waits only for the data it needs.
#pragma once
#include "ps_internal.h"

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
// Bounded wait: a consumer that never sees its data (possible only after a fault elsewhere)
// raises the error flag and goes on, so the kernel always terminates.
#define PS_SPIN_LIMIT (1 << 20)
__device__ __forceinline__ bool spin_again(const StepParams& P, int& spins) {
    __builtin_amdgcn_s_sleep(2);
    if (++spins > PS_SPIN_LIMIT) {
        __hip_atomic_store(P.error_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return false;
    }
    return true;
}
// one element / four elements, waiting until they carry this step's sequence number
__device__ __forceinline__ float ll_wait1(const StepParams& P, rsrc_t r, unsigned i) {
    int spins = 0;
    for (;;) {
        const u32x2 x = coh_ld8(r, i * 8);
        if (__all(x[1] == P.seq) || !spin_again(P, spins)) return __uint_as_float(x[0]);
    }
}
__device__ __forceinline__ f32x4 ll_wait4(const StepParams& P, rsrc_t r, unsigned i) {
    int spins = 0;
    for (;;) {
        const LL4 x = ll_ld4(r, i);
        if (__all(ll_ok(x, P.seq)) || !spin_again(P, spins)) return ll_val(x);
    }
}

// ---- sentinel-coded exchange for the activation buffers (the bulk of the exchanged bytes, read
// by every workgroup): plain fp32 values, "not written yet" is the bit pattern 0xFFFFFFFF (a NaN no
// computation on finite inputs produces).  Each buffer exists twice; step n uses copy n & 1, and
// whoever writes element i of the current copy also resets element i of the other copy, so the
// copy the next step uses is clean again without a separate clearing pass.
#define PS_SENT 0xFFFFFFFFu
struct SxBuf { rsrc_t cur, alt; };
__device__ __forceinline__ SxBuf sx_buf(const StepParams& P, const float* cur) {
    SxBuf b;
    b.cur = make_rsrc(cur);
    b.alt = make_rsrc(reinterpret_cast<const char*>(cur) + P.alt_delta);
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

// per-lane 64-bit addresses (KV-cache rows): relaxed agent-scope atomics, dword granularity
__device__ __forceinline__ void st_agent_u32(void* p, unsigned v) {
    __hip_atomic_store((unsigned*)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned ld_agent_u32(const void* p) {
    return __hip_atomic_load((const unsigned*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 4 values -> the cache's storage type: stores them, returns them as stored (widened again)
template <typename WT> __device__ __forceinline__ f32x4 store4(void* p, f32x4 v);
template <> __device__ __forceinline__ f32x4 store4<float>(void* p, f32x4 v) {
    *reinterpret_cast<f32x4*>(p) = v;
    return v;
}
template <> __device__ __forceinline__ f32x4 store4<bf16_t>(void* p, f32x4 v) {
    const unsigned b0 = f32_to_bf16(v[0]), b1 = f32_to_bf16(v[1]), b2 = f32_to_bf16(v[2]), b3 = f32_to_bf16(v[3]);
    uint2 o;
    o.x = b0 | (b1 << 16);
    o.y = b2 | (b3 << 16);
    *reinterpret_cast<uint2*>(p) = o;
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
__device__ __forceinline__ float wave_max(float v) {
#define PS_C(CTRL, RM) { const float o = __uint_as_float(dpp_u32<CTRL, RM>(__float_as_uint(v), __float_as_uint(v))); v = fmaxf(v, o); }
    PS_DPP_STEPS(PS_C)
#undef PS_C
    return __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(v), 63));
}
__device__ __forceinline__ u64 wave_max_u64(u64 v) {
#define PS_C(CTRL, RM) { const unsigned lo = dpp_u32<CTRL, RM>((unsigned)v, (unsigned)v);                 \
                         const unsigned hi = dpp_u32<CTRL, RM>((unsigned)(v >> 32), (unsigned)(v >> 32)); \
                         const u64 o = ((u64)hi << 32) | lo; v = o > v ? o : v; }
    PS_DPP_STEPS(PS_C)
#undef PS_C
    const unsigned lo = __builtin_amdgcn_readlane((unsigned)v, 63);
    const unsigned hi = __builtin_amdgcn_readlane((unsigned)(v >> 32), 63);
    return ((u64)hi << 32) | lo;
}

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

// Row m of the step's activation matrix Z = [x rows ; mask embeddings] (Section 4.1: the k
// [MASK] tokens are appended after the sequence), element offset e.
template <typename WT>
__device__ __forceinline__ const char* z_ptr(const StepParams& P, int m, int e) {
    const int b = m / P.M, i = m - b * P.M;
    const char* base;
    long long off;
    if (i < P.n_new) { base = (const char*)P.x; off = ((long long)(b * P.n_new + i)) * P.H + e; }
    else { base = (const char*)P.mask_emb; off = ((long long)(i - P.n_new)) * P.H + e; }
    return base + off * Traits<WT>::ESZ;
}

// Debugging aid: thread 0 of every workgroup stamps the 100 MHz wall clock at point `ev`.
__device__ __forceinline__ void stamp(const StepParams& P, int wg, int ev) {
#ifdef PS_TIMELINE
    if (P.timeline && threadIdx.x == 0) P.timeline[(size_t)ev * 1024 + wg] = wall_clock64();
#endif
}

// ------------------------------------------------------------------------------------------
// GEMM phase descriptors: which weight row a lane streams, where activations come from
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
    } else {
        int row = 16 * tau + i;
        if (row >= P.V) row = P.V - 1;   // ragged last vocabulary tile: clamp, masked in the epilogue
        return (const char*)P.w_lm + (size_t)row * P.H * ESZ;
    }
}

template <int PH> __device__ __forceinline__ int phase_K(const StepParams& P) {
    return PH == PH_OPROJ ? P.QD : (PH == PH_DOWN ? P.F : P.H);
}
template <int PH> __device__ __forceinline__ int phase_rows(const StepParams& P) {
    return PH == PH_LMHEAD ? P.Rtot : P.Mtot;
}
template <int PH> __device__ __forceinline__ bool phase_norm(const StepParams& P) {
    return PH == PH_QKV || PH == PH_GATEUP || (PH == PH_LMHEAD && P.final_norm);
}
template <int PH> __device__ __forceinline__ const void* phase_gain(const StepParams& P) {
    return PH == PH_QKV ? P.g_in : (PH == PH_GATEUP ? P.g_post : P.g_final);
}
// fp32 source buffer of the phase's activations (phases other than QKV) and its row stride
template <int PH> __device__ __forceinline__ const float* phase_src(const StepParams& P) {
    return PH == PH_OPROJ ? P.o_buf : (PH == PH_GATEUP ? P.y_buf : (PH == PH_DOWN ? P.u_buf : P.y2_buf));
}
template <int PH> __device__ __forceinline__ int phase_src_row(const StepParams& P, int r) {
    if (PH != PH_LMHEAD) return r;
    // decoding rows: last real row and the k mask rows of each sequence (or all rows)
    const int b = r / P.R, jj = r - b * P.R;
    return b * P.M + (P.all_rows ? jj : (P.n_new - 1 + jj));
}

// ------------------------------------------------------------------------------------------
// inner loop
// ------------------------------------------------------------------------------------------
// B operands (activation columns) of one step for all column tiles, read from the LDS panel
template <typename WT, int MT> struct BRegs { uint4 h[MT]; uint4 l[MT]; };

template <typename WT, int MT>
__device__ __forceinline__ void load_b(BRegs<WT, MT>& b, const char* const (&pa)[MT], const int (&pinc)[MT],
                                       const int (&plo)[MT], int t) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const char* p = pa[mt] + t * pinc[mt];
        b.h[mt] = ld16(p);
        if constexpr (Traits<WT>::BF) b.l[mt] = ld16(p + plo[mt]);
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

// Issues the first PS_U loads of a weight stream.  Weights do not depend on the activations, so
// this can run before the panel is staged (and before the grid barrier that ends the previous
// phase): the HBM pipe stays busy while the activations arrive.  Every load is unconditional
// (streams shorter than PS_U steps read on into the following KiBs, which always exist: the
// packed buffers are padded), so the compiler can count outstanding loads exactly.
__device__ __forceinline__ void preload_weights(uint4 (&wb)[PS_U], const char* wp) {
#pragma unroll
    for (int u = 0; u < PS_U; ++u) wb[u] = ldg_stream16(wp + u * PS_WS);
}

// Software pipeline over the n steps of one weight stream: step t multiplies the weights loaded
// PS_U steps earlier with the B operands read one step earlier, then refills its register with
// step t + PS_U and reads the B operands of step t + 1.  Loads past the end of the stream
// continue at next_wp (the wavefront's next stream), so when this returns wb holds the
// preloaded head of that stream.  Only the oldest load is waited for at each step.
template <typename WT, int MT>
__device__ __forceinline__ void consume_weights(uint4 (&wb)[PS_U], const char* wp, int n_, const char* next_wp,
                                                const char* const (&pa)[MT], const int (&pinc)[MT],
                                                const int (&plo)[MT], f32x4 (&acc)[MT]) {
    constexpr int U = PS_U;
    const int n = __builtin_amdgcn_readfirstlane(n_);   // wavefront-uniform: keep the loop control scalar
    const int n_main = n & ~(U - 1), r = n - n_main;
    BRegs<WT, MT> bc, bn;
    load_b<WT, MT>(bc, pa, pinc, plo, 0);
    const int last = n > 0 ? n - 1 : 0;
    int t0 = 0;
    for (; t0 + 2 * U <= n_main; t0 += U) {   // steady state: every load is inside this stream
#pragma unroll
        for (int u = 0; u < U; ++u) {
            mma_step<WT, MT>(wb[u], bc, acc);
            wb[u] = ldg_stream16(wp + (size_t)(t0 + u + U) * PS_WS);   // reuses the register just consumed
            load_b<WT, MT>(bn, pa, pinc, plo, t0 + u + 1);
            bc = bn;
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (t0 < n_main) {   // last full group: its loads start the next stream (or fetch the tail steps)
#pragma unroll
        for (int u = 0; u < U; ++u) {
            mma_step<WT, MT>(wb[u], bc, acc);
            const int idx = t0 + u + U;
            const char* src = r == 0 ? next_wp + (size_t)u * PS_WS
                                     : wp + (size_t)(idx < n ? idx : last) * PS_WS;   // tail, then harmless re-reads
            wb[u] = ldg_stream16(src);
            const int tb = t0 + u + 1;
            load_b<WT, MT>(bn, pa, pinc, plo, tb < n ? tb : last);
            bc = bn;
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (r != 0 || n == 0) {   // K not a multiple of PS_U steps: finish the tail, then start the next stream afresh
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (u < r) {
                mma_step<WT, MT>(wb[u], bc, acc);
                const int tb = n_main + u + 1;
                load_b<WT, MT>(bn, pa, pinc, plo, tb < n ? tb : last);
                bc = bn;
            }
        }
        preload_weights(wb, next_wp);
    }
}

// Where the weight stream of segment q of this wavefront starts, and its length in steps.
// A phase is cut into rounds (one tile per wavefront slot per round) and, inside a round, into
// the K-pieces whose activation panel fits in LDS; segment q = round * pieces + piece.
struct PhaseGeom {
    int S, KW, s, j, Gs, k_lo, k_hi, SL, slot, kw, per_round, rounds, nsub, nseg;
    bool active;
};
template <int PH>
__device__ __forceinline__ PhaseGeom phase_geom(const StepParams& P, int wg, int wave) {
    const PhasePlan& pl = P.plan[PH];
    PhaseGeom g;
    g.S = pl.S; g.KW = pl.KW;
    g.s = wg % g.S; g.j = wg / g.S; g.Gs = pl.nwg / g.S;
    g.active = g.j < g.Gs;
    g.k_lo = (int)((long long)g.s * pl.Kt / g.S); g.k_hi = (int)((long long)(g.s + 1) * pl.Kt / g.S);
    g.SL = PS_WAVES / g.KW; g.slot = wave / g.KW; g.kw = wave - g.slot * g.KW;
    g.per_round = g.Gs * g.SL;
    g.rounds = g.active ? (pl.T + g.per_round - 1) / g.per_round : 0;
    g.nsub = (g.k_hi - g.k_lo + pl.panel_steps - 1) / pl.panel_steps;
    g.nseg = g.rounds * g.nsub;
    return g;
}
struct WeightSeg { const char* wp; int n; int tau; int a; int b; bool valid; };
template <int PH>
__device__ __forceinline__ WeightSeg segment(const StepParams& P, const PhaseGeom& g, int q, int lane) {
    const PhasePlan& pl = P.plan[PH];
    WeightSeg sg;
    const int rd = q / g.nsub, si = q - rd * g.nsub;
    sg.tau = rd * g.per_round + g.slot * g.Gs + g.j;
    sg.valid = q < g.nseg && sg.tau < pl.T;
    sg.a = g.k_lo + si * pl.panel_steps;
    sg.b = min(sg.a + pl.panel_steps, g.k_hi);
    const int n = sg.b - sg.a;
    const int t0 = (int)((long long)g.kw * n / g.KW), t1 = (int)((long long)(g.kw + 1) * n / g.KW);
    sg.n = sg.valid ? t1 - t0 : 0;
    // invalid segments point at the start of the packed matrix: always readable, always cached
    sg.wp = P.wpack[PH] + (sg.valid ? ((size_t)sg.tau * pl.Kt + sg.a + t0) * PS_WS : (size_t)0) + lane * 16;
    return sg;
}
// head of the stream a wavefront reads first in phase PH
template <int PH>
__device__ __forceinline__ const char* first_stream(const StepParams& P, int wg, int wave, int lane) {
    const PhaseGeom g = phase_geom<PH>(P, wg, wave);
    return segment<PH>(P, g, 0, lane).wp;
}

// ------------------------------------------------------------------------------------------
// epilogues: lane (c = lane % 16, q = lane / 16) holds, for column tile mt, the outputs of
// activation row m = 16 mt + c and tile rows 4q .. 4q+3
// ------------------------------------------------------------------------------------------
template <typename WT, int MT>
__device__ __forceinline__ void epilogue_qkv(const StepParams& P, int tau, int lane, f32x4 (&acc)[MT]) {
    const int c = lane & 15, q = lane >> 4;
    const int tph = P.d >> 4, half = P.d >> 1;
    const int hh = tau / tph, sub = tau - hh * tph;
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
        const int b = m / P.M, i = m - b * P.M;
        const int pos = P.kv_len[b] + i;             // positions continue after the valid cache rows
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
            // stored - into the tagged side buffer this step's attention reads
            const bool isk = hh < P.nq + P.nkv;
            const int hk = isk ? hh - P.nq : hh - P.nq - P.nkv;
            char* cache = (char*)(isk ? P.kc : P.vc);
            const size_t e = ((size_t)(P.kv_off[b] + pos) * P.nkv + hk) * P.d + f;
            const f32x4 stored = store4<WT>(cache + e * Traits<WT>::ESZ, o);
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
        const f32x4 z = load4<WT>(z_ptr<WT>(P, m, n));
        sx_st4(ry, (unsigned)((size_t)m * P.H + n), z + acc[mt]);
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
    const rsrc_t ry = make_rsrc(P.y_buf);
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
        f32x4 o = acc[mt];
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (n + r >= P.V) o[r] = -INFINITY;
        *reinterpret_cast<f32x4*>(s_lm + ((size_t)lt * P.Rtot + m) * 16 + 4 * q) = o;
        if (P.logits_store) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (n + r < P.V) P.logits_store[(size_t)m * P.V + n + r] = o[r];
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
#define PS_LDS_SSQ 0        // [64 units] partial sums of squares (RMSNorm)
#define PS_LDS_ZERO 256     // 64 zero bytes: B operand of unused MFMA columns
#define PS_LDS_RED 512      // [16 wavefronts][MT][64 lanes] f32x4: K-split inside the workgroup
__host__ __device__ inline int panel_offset(int mt) { return PS_LDS_RED + PS_WAVES * mt * 1024; }

// Stages steps [a, b) of the activation panel: rows x (b-a) x 4 groups of 16 bytes.  A unit is
// (row, part of the row's groups); wavefronts take units round-robin, lanes stride over the
// groups, four groups per lane are loaded before any is processed.  The panel holds x (.) gain
// (RMSNorm's 1/rms is applied in the epilogue); the unit's sum of x^2 goes to s_ssq[unit].
template <typename WT, int PH>
__device__ __forceinline__ void stage_panel(const StepParams& P, char* smem, int RS, char* s_pa, char* s_pb,
                                            int rows, int a, int b, bool norm, bool first_piece, bool want_ssq) {
    constexpr bool BF = Traits<WT>::BF;
    constexpr int KSTEP = Traits<WT>::KSTEP, GE = Traits<WT>::GE, ESZ = Traits<WT>::ESZ;
    constexpr int BATCH = 4;                         // groups per lane requested before any is used
    constexpr int NL = GE / 4;                       // 4-element loads per group
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float* s_ssq = reinterpret_cast<float*>(smem + PS_LDS_SSQ);
    const int groups = (b - a) * 4;
    const int wpr = rows >= PS_WAVES ? 1 : PS_WAVES / rows;      // units per row
    const int units = rows * wpr;
    const void* gain = phase_gain<PH>(P);
    const rsrc_t rs = make_rsrc(PH == PH_QKV ? (const void*)P.x : (const void*)phase_src<PH>(P));
    const int ld = phase_K<PH>(P);
    for (int u = wave; u < units; u += PS_WAVES) {
        const int r = u / wpr, sub = u - r * wpr;
        const int g0 = (int)((long long)sub * groups / wpr), g1 = (int)((long long)(sub + 1) * groups / wpr);
        const int srow = phase_src_row<PH>(P, r);
        float ss = 0.f;
        for (int gb = g0 + lane; gb - lane < g1; gb += 64 * BATCH) {
            uint4 zraw[BATCH], graw[BATCH];
            u32x4 araw[BATCH][NL];
            int spins = 0;
            for (;;) {
                bool ok = true;
#pragma unroll
                for (int i = 0; i < BATCH; ++i) {
                    int gi = gb + 64 * i;
                    if (gi >= g1) gi = g1 - 1;                   // clamped: loads stay unconditional
                    const int kk = a * KSTEP + gi * GE;
                    if (PH == PH_QKV) {
                        zraw[i] = ld16(z_ptr<WT>(P, r, kk));
                    } else {
#pragma unroll
                        for (int h = 0; h < NL; ++h) araw[i][h] = coh_ld16(rs, (unsigned)((size_t)srow * ld + kk + 4 * h) * 4);
                    }
                    if (norm) graw[i] = ld16((const char*)gain + (size_t)kk * ESZ);
                }
                if (PH == PH_QKV) break;                         // the step's inputs were complete at launch
#pragma unroll
                for (int i = 0; i < BATCH; ++i)
#pragma unroll
                    for (int h = 0; h < NL; ++h) ok = ok && sx_ok(araw[i][h]);
                if (__all(ok) || !spin_again(P, spins)) break;   // produced earlier in this step: wait for it
            }
#pragma unroll
            for (int i = 0; i < BATCH; ++i) {
                const int gi = gb + 64 * i;
                if (gi >= g1) continue;
                float v[GE];
                if (PH == PH_QKV) {
                    unpack_group<WT>(zraw[i], v);
                } else {
#pragma unroll
                    for (int h = 0; h < NL; ++h) {
                        const f32x4 t = __builtin_bit_cast(f32x4, araw[i][h]);
                        v[4 * h] = t[0]; v[4 * h + 1] = t[1]; v[4 * h + 2] = t[2]; v[4 * h + 3] = t[3];
                    }
                }
                if (norm) {
                    float gn[GE];
                    unpack_group<WT>(graw[i], gn);
#pragma unroll
                    for (int e = 0; e < GE; ++e) { ss += v[e] * v[e]; v[e] *= gn[e]; }
                }
                if constexpr (BF) {
                    uint32_t hi[GE], lo[GE];
#pragma unroll
                    for (int e = 0; e < GE; ++e) {
                        hi[e] = f32_to_bf16(v[e]);
                        lo[e] = f32_to_bf16(v[e] - bf16_to_f32(hi[e]));
                    }
                    uint4 ph, plw;
                    ph.x = hi[0] | (hi[1] << 16); ph.y = hi[2] | (hi[3] << 16);
                    ph.z = hi[4] | (hi[5] << 16); ph.w = hi[6] | (hi[7] << 16);
                    plw.x = lo[0] | (lo[1] << 16); plw.y = lo[2] | (lo[3] << 16);
                    plw.z = lo[4] | (lo[5] << 16); plw.w = lo[6] | (lo[7] << 16);
                    *reinterpret_cast<uint4*>(s_pa + (size_t)r * RS + gi * 16) = ph;
                    *reinterpret_cast<uint4*>(s_pb + (size_t)r * RS + gi * 16) = plw;
                } else {
                    uint4 pv;
                    pv.x = __float_as_uint(v[0]); pv.y = __float_as_uint(v[1]);
                    pv.z = __float_as_uint(v[2]); pv.w = __float_as_uint(v[3]);
                    *reinterpret_cast<uint4*>(s_pa + (size_t)r * RS + gi * 16) = pv;
                }
            }
        }
        if (norm && want_ssq) {
            ss = wave_sum(ss);
            if (lane == 0) s_ssq[u] = first_piece ? ss : s_ssq[u] + ss;
        }
    }
}

// 1/rms of panel row m from the per-unit sums in LDS (this workgroup's K-slice)
__device__ __forceinline__ float slice_ssq(const char* smem, int rows, int m) {
    const float* s_ssq = reinterpret_cast<const float*>(smem + PS_LDS_SSQ);
    const int wpr = rows >= PS_WAVES ? 1 : PS_WAVES / rows;
    float t = 0.f;
    for (int sub = 0; sub < wpr; ++sub) t += s_ssq[m * wpr + sub];
    return t;
}

// wb: the wavefront's weight-load registers.  On entry they hold the preloaded head of segment 0
// (preload_weights(first_stream<PH>(..))); on exit they hold PS_U loads from after_wp (the head of
// whatever this wavefront streams next, or any readable address).
template <typename WT, int MT, int PH>
__device__ void gemm_phase(const StepParams& P, int wg, char* smem, uint4 (&wb)[PS_U], const char* after_wp) {
    constexpr bool BF = Traits<WT>::BF;
    const PhasePlan pl = P.plan[PH];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, kb = lane >> 4;
    const int rows = phase_rows<PH>(P);
    const int K = phase_K<PH>(P);
    const PhaseGeom g = phase_geom<PH>(P, wg, wave);
    const int S = g.S, KW = g.KW, s = g.s, SL = g.SL, slot = g.slot, kw = g.kw;
    const bool norm = phase_norm<PH>(P);

    char* s_zero = smem + PS_LDS_ZERO;
    char* s_red = smem + PS_LDS_RED;
    const int RS = panel_row_stride(pl.panel_steps);
    char* s_pa = smem + panel_offset(MT);                        // high parts (or f32 values)
    char* s_pb = s_pa + (size_t)rows * RS;                       // low parts (bf16 only)
    float* s_lm = reinterpret_cast<float*>(s_pb + (BF ? (size_t)rows * RS : 0));

    stamp(P, wg, PH * 4 + 0);
    if (g.active) {
    if (tid < 16) reinterpret_cast<uint32_t*>(s_zero)[tid] = 0u;
    if (PH == PH_LMHEAD) {
        const int n_lm = g.rounds * SL * rows * 16;
        for (int x = tid; x < n_lm; x += PS_WG_THREADS) s_lm[x] = -INFINITY;
    }

    // per-lane panel addressing: column c of column tile mt is activation row 16 mt + c
    const char* pa[MT];
    int pinc[MT], plo[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = 16 * mt + c;
        if (m < rows) { pa[mt] = s_pa + (size_t)m * RS + kb * 16; pinc[mt] = 64; plo[mt] = (int)(s_pb - s_pa); }
        else { pa[mt] = s_zero + kb * 16; pinc[mt] = 0; plo[mt] = 0; }
    }

    int staged_a = -1, staged_b = -1;
    f32x4 acc[MT];
    for (int q = 0; q < g.nseg; ++q) {
        const WeightSeg sg = segment<PH>(P, g, q, lane);
        const int rd = q / g.nsub, si = q - rd * g.nsub;
        const int tau = sg.tau;
        const bool valid = sg.valid;
        if (si == 0) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        const int a = sg.a, b = sg.b;
        if (a != staged_a || b != staged_b) {
            if (q > 0) __syncthreads();   // everyone is done with the previous panel
            stage_panel<WT, PH>(P, smem, RS, s_pa, s_pb, rows, a, b, norm, si == 0, rd == 0);
            __syncthreads();
            staged_a = a; staged_b = b;
        }
        if (q == 0) stamp(P, wg, PH * 4 + 1);
        {
            // this wavefront's share [t0, t1) of the staged piece; the stream continues in segment q + 1
            const int n = b - a;
            const int t0 = (int)((long long)kw * n / KW);
            const char* next_wp = (q + 1 < g.nseg) ? segment<PH>(P, g, q + 1, lane).wp : after_wp;
            const char* pa_t[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) pa_t[mt] = pa[mt] + t0 * pinc[mt];
            consume_weights<WT, MT>(wb, sg.wp, sg.n, next_wp, pa_t, pinc, plo, acc);
        }
        if (si != g.nsub - 1) continue;
        if (q == g.nseg - 1) stamp(P, wg, PH * 4 + 2);

        // K-split inside the workgroup: wavefront kw = 0 of each slot adds the others in order
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
            __syncthreads();
        }

        if (valid && kw == 0) {
            // sum of squares of this lane's activation rows over the workgroup's K-slice
            float ssq[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int m = 16 * mt + c;
                ssq[mt] = (norm && m < rows) ? slice_ssq(smem, rows, m) : 0.f;
            }
            bool run_epilogue = true;
            if (S > 1) {
                // K-slices of other workgroups meet here.  Every slice publishes its fragment (and its
                // sums of squares) as tagged data; the wavefront of slice tau % S waits for the other
                // S - 1 fragments and adds all S in slice order, so the result does not depend on timing.
                const rsrc_t rp = make_rsrc(P.part), rq = make_rsrc(P.ssq_part);
                // all phases share the fragment buffer: the tag names the phase as well as the step
                const unsigned ftag = P.seq * 8u + PH + 1u;
                const int s_red = tau % S;
                run_epilogue = (s == s_red);
                if (!run_epilogue) {
                    const unsigned fb = (unsigned)((size_t)s * pl.T + tau);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        ll_st4(rp, ((fb * MT + mt) * 64 + lane) * 4, acc[mt], ftag);
                        if (norm && lane < 16) ll_st1(rq, fb * PS_MAX_ROWS + 16 * mt + lane, ssq[mt], ftag);
                    }
                } else {
                    f32x4 own[MT];
                    float own_q[MT];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        own[mt] = acc[mt]; own_q[mt] = ssq[mt];
                        acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f}; ssq[mt] = 0.f;
                    }
                    for (int s0 = 0; s0 < S; s0 += 4) {   // four slices are requested per round trip
                        LL4 fr[4][MT];
                        u32x2 fq[4][MT];
                        int spins = 0;
                        for (;;) {
                            bool ok = true;
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                int ss = s0 + i < S ? s0 + i : S - 1;
                                const bool mine = ss == s;
                                if (mine) ss = (s + 1) % S;   // placeholder load, never used
                                const unsigned fb = (unsigned)((size_t)ss * pl.T + tau);
#pragma unroll
                                for (int mt = 0; mt < MT; ++mt) {
                                    fr[i][mt] = ll_ld4(rp, ((fb * MT + mt) * 64 + lane) * 4);
                                    fq[i][mt] = coh_ld8(rq, (fb * PS_MAX_ROWS + 16 * mt + c) * 8);
                                    if (!mine) {
                                        ok = ok && ll_ok(fr[i][mt], ftag);
                                        if (norm && 16 * mt + c < rows) ok = ok && fq[i][mt][1] == ftag;
                                    }
                                }
                            }
                            if (__all(ok) || !spin_again(P, spins)) break;
                        }
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int ss = s0 + i;
                            if (ss >= S) continue;
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt) {
                                if (ss == s) { acc[mt] += own[mt]; ssq[mt] += own_q[mt]; }
                                else { acc[mt] += ll_val(fr[i][mt]); ssq[mt] += __uint_as_float(fq[i][mt][0]); }
                            }
                        }
                    }
                }
            }
            if (run_epilogue) {
                if (norm) {   // RMSNorm: the panel held x (.) gain, 1/rms multiplies the result
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        const float rinv = 1.0f / sqrtf(ssq[mt] / (float)K + P.eps);
                        acc[mt] *= rinv;
                    }
                }
                if (PH == PH_QKV) epilogue_qkv<WT, MT>(P, tau, lane, acc);
                else if (PH == PH_OPROJ) epilogue_oproj<WT, MT>(P, tau, lane, acc);
                else if (PH == PH_GATEUP) epilogue_gateup<WT, MT>(P, tau, lane, acc);
                else if (PH == PH_DOWN) epilogue_down<WT, MT>(P, tau, lane, acc);
                else epilogue_lm<WT, MT>(P, tau, lane, acc, s_lm, rd * SL + slot);
            }
        }
    }
    stamp(P, wg, PH * 4 + 3);

    if (PH == PH_LMHEAD) {
        // per-workgroup softmax statistics and top-k over the logits held in LDS: one wavefront per row
        __syncthreads();
        const int n_el = g.rounds * SL * 16;
        const int topk = P.topk;
        const rsrc_t rl = make_rsrc(P.lm_part);
        const unsigned stride = 2 + 2 * topk;   // tagged elements: max, sum exp, topk keys (low, high word)
        for (int m = wave; m < rows; m += PS_WAVES) {
            constexpr int EPL = 8;   // elements per lane kept in registers (more: re-read from LDS)
            u64 keys[EPL];
            float mx = -INFINITY;
#pragma unroll
            for (int i = 0; i < EPL; ++i) {
                const int x = lane + 64 * i;
                keys[i] = 0;
                if (x < n_el) {
                    const int lt = x >> 4;
                    const float v = s_lm[((size_t)lt * rows + m) * 16 + (x & 15)];
                    const int rd2 = lt / SL, sl2 = lt - rd2 * SL;
                    const int id = 16 * (rd2 * g.per_round + sl2 * g.Gs + g.j) + (x & 15);
                    if (v > -INFINITY) { keys[i] = make_key(v, id); mx = fmaxf(mx, v); }
                }
            }
            for (int x = lane + 64 * EPL; x < n_el; x += 64) mx = fmaxf(mx, s_lm[((size_t)(x >> 4) * rows + m) * 16 + (x & 15)]);
            mx = wave_max(mx);
            float se = 0.f;
            if (mx > -INFINITY)
                for (int x = lane; x < n_el; x += 64) se += expf(s_lm[((size_t)(x >> 4) * rows + m) * 16 + (x & 15)] - mx);
            se = wave_sum(se);
            const unsigned obase = (unsigned)(((size_t)wg * rows + m) * stride);
            if (lane < 2) ll_st1(rl, obase + lane, lane ? se : mx, P.seq);
            u64 prev = ~0ull;   // keys are unique: the next winner is the largest key below the previous one
            for (int t = 0; t < topk; ++t) {
                u64 best = 0;
#pragma unroll
                for (int i = 0; i < EPL; ++i)
                    if (keys[i] < prev && keys[i] > best) best = keys[i];
                for (int x = lane + 64 * EPL; x < n_el; x += 64) {
                    const int lt = x >> 4;
                    const float v = s_lm[((size_t)lt * rows + m) * 16 + (x & 15)];
                    const int rd2 = lt / SL, sl2 = lt - rd2 * SL;
                    const int id = 16 * (rd2 * g.per_round + sl2 * g.Gs + g.j) + (x & 15);
                    const u64 kx = v > -INFINITY ? make_key(v, id) : 0;
                    if (kx < prev && kx > best) best = kx;
                }
                best = wave_max_u64(best);
                if (lane < 2)
                    ll_st1(rl, obase + 2 + 2 * t + lane, __uint_as_float(lane ? (unsigned)(best >> 32) : (unsigned)best), P.seq);
                prev = best ? best : 0;   // 0: list exhausted, every later entry is "none"
            }
        }
    }
    } else {
        preload_weights(wb, after_wp);   // keep the contract on wb for workgroups without work here
    }
    stamp(P, wg, 20 + PH);
}

// ------------------------------------------------------------------------------------------
// Init-time prepack: tile tau, step t of a phase's weight matrix becomes one contiguous KiB in
// the exact order the streaming loop reads it: lane (i = lane % 16, kb = lane / 16) gets bytes
// [64 t + 16 kb, +16) of tile row i, so a wavefront load is one contiguous 1 KiB burst.
// ------------------------------------------------------------------------------------------
template <typename WT, int PH>
__global__ void __launch_bounds__(256) pack_kernel(const StepParams P, int T, int Kt, char* dst) {
    const size_t units = (size_t)T * Kt;
    const int lane = threadIdx.x & 63;
    for (size_t u = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6); u < units; u += (size_t)gridDim.x * 4) {
        const int tau = (int)(u / Kt), t = (int)(u - (size_t)tau * Kt);
        const char* src = weight_row_ptr<WT, PH>(P, tau, lane & 15) + (size_t)t * 64 + (lane >> 4) * 16;
        *reinterpret_cast<uint4*>(dst + u * 1024 + lane * 16) = ld16(src);
    }
}

// ------------------------------------------------------------------------------------------
// attention: one work item = (sequence b, kv head hk, chunk of CH keys); all g*M query rows
// of the kv head are processed against the chunk; K/V tiles are staged in LDS; row i of the
// step sees cache positions 0 .. kv_len[b] + i (its own and earlier rows of this step
// included; Algorithm 1: distribution j is conditioned on [MASK]_1..j only).
// ------------------------------------------------------------------------------------------
template <typename WT, int D> struct AttnCfg {
    static constexpr int CH = Traits<WT>::BF ? 128 : (D == 64 ? 128 : 64);
    static constexpr int LDS = 256 + PS_MAX_ROWS * D * 4 + PS_MAX_ROWS * CH * 4 + 2 * CH * (D * Traits<WT>::ESZ + 16);
};

template <typename WT, int D>
__device__ void attn_phase(const StepParams& P, int wg, int nwg, char* smem) {
    constexpr int CH = AttnCfg<WT, D>::CH;
    constexpr int ESZ = Traits<WT>::ESZ, GE = Traits<WT>::GE;
    constexpr int KSTR = D * ESZ + 16;              // padded K/V row stride in LDS (bytes)
    constexpr int DPL = D / 64;                     // output columns per lane
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = P.nq / P.nkv;
    const int Ra = grp * P.M;
    float* sQ = reinterpret_cast<float*>(smem + 256);           // [Ra][D]
    float* sP = sQ + PS_MAX_ROWS * D;                           // [Ra][CH]
    char* sK = reinterpret_cast<char*>(sP + PS_MAX_ROWS * CH);  // [CH][KSTR]
    char* sV = sK + CH * KSTR;
    const rsrc_t rq = make_rsrc(P.q_buf), rn = make_rsrc(P.kvnew), racc = make_rsrc(P.attn_acc),
                 rml = make_rsrc(P.attn_ml);
    const SxBuf ro = sx_buf(P, P.o_buf);

    for (int item = wg; item < P.attn_items; item += nwg) {
        // decode item -> (b, hk, chunk)
        int b = 0, rem = item, nch = 0;
        for (;; ++b) {
            nch = (P.kv_len[b] + P.M + CH - 1) / CH;
            if (rem < nch * P.nkv) break;
            rem -= nch * P.nkv;
        }
        const int hk = rem / nch, ch = rem - hk * nch;
        const int L = P.kv_len[b];
        const int c0 = ch * CH, c1 = min(c0 + CH, L + P.M);
        const int nk = c1 - c0;
        __syncthreads();   // previous item's LDS use is over
        // stage the K/V chunk: rows already in the cache come from there; rows of this step come,
        // exactly as stored, from the tagged side buffer the QKV epilogue fills
        constexpr int GPR = D / GE;   // 16-byte groups per key row
        for (int x = tid; x < nk * GPR; x += PS_WG_THREADS) {
            const int key = x / GPR, gg = x - key * GPR;
            if (c0 + key < L) {
                const size_t e = ((size_t)(P.kv_off[b] + c0 + key) * P.nkv + hk) * D + gg * GE;
                *reinterpret_cast<uint4*>(sK + key * KSTR + gg * 16) = ld16((const char*)P.kc + e * ESZ);
                *reinterpret_cast<uint4*>(sV + key * KSTR + gg * 16) = ld16((const char*)P.vc + e * ESZ);
            }
        }
        const int n_old = L > c0 ? min(L - c0, nk) : 0;          // keys of this chunk that were cached
        for (int x = tid; x < (nk - n_old) * 2 * (D / 4); x += PS_WG_THREADS) {
            const int kn = x / (2 * (D / 4)), rest = x - kn * (2 * (D / 4));
            const int isv = rest / (D / 4), dd = (rest - isv * (D / 4)) * 4;
            const int key = n_old + kn;
            const int m = b * P.M + (c0 + key - L);
            const f32x4 v = sx_wait4(P, rn, (unsigned)(((size_t)m * 2 + isv) * P.KVD + hk * D + dd));
            char* dst = (isv ? sV : sK) + key * KSTR + dd * ESZ;
            if constexpr (Traits<WT>::BF) {
                uint2 o;
                o.x = f32_to_bf16(v[0]) | (f32_to_bf16(v[1]) << 16);
                o.y = f32_to_bf16(v[2]) | (f32_to_bf16(v[3]) << 16);
                *reinterpret_cast<uint2*>(dst) = o;
            } else {
                *reinterpret_cast<f32x4*>(dst) = v;
            }
        }
        // Q rows of the head group
        for (int x = tid; x < Ra * (D / 4); x += PS_WG_THREADS) {
            const int rho = x / (D / 4), dd = (x - rho * (D / 4)) * 4;
            const int gi = rho / P.M, i = rho - gi * P.M;
            const f32x4 v = sx_wait4(P, rq, (unsigned)((size_t)(b * P.M + i) * P.QD + (hk * grp + gi) * D + dd));
            *reinterpret_cast<f32x4*>(sQ + rho * D + dd) = v;
        }
        __syncthreads();
        for (int rho = wave; rho < Ra; rho += PS_WAVES) {
            const int gi = rho / P.M, i = rho - gi * P.M;
            const int last_visible = L + i;            // absolute position
            // scores: lane handles keys lane, lane + 64, ...
            constexpr int KPL = CH / 64;
            float sc[KPL];
            float mx = -INFINITY;
#pragma unroll
            for (int kk = 0; kk < KPL; ++kk) {
                const int key = lane + 64 * kk;
                float dot = 0.f;
                if (key < nk && c0 + key <= last_visible) {
                    const char* krow = sK + key * KSTR;
#pragma unroll 4
                    for (int gg = 0; gg < GPR; ++gg) {
                        float kv[GE];
                        load_group<WT>(krow + gg * 16, kv);
#pragma unroll
                        for (int e = 0; e < GE; e += 4) {
                            const f32x4 qv = *reinterpret_cast<const f32x4*>(sQ + rho * D + gg * GE + e);
                            dot += qv[0] * kv[e] + qv[1] * kv[e + 1] + qv[2] * kv[e + 2] + qv[3] * kv[e + 3];
                        }
                    }
                    sc[kk] = dot * P.inv_sqrt_d;
                } else {
                    sc[kk] = -INFINITY;                // masked in-register
                }
                mx = fmaxf(mx, sc[kk]);
            }
            mx = wave_max(mx);
            float l = 0.f;
#pragma unroll
            for (int kk = 0; kk < KPL; ++kk) {
                const float p = (sc[kk] > -INFINITY) ? expf(sc[kk] - mx) : 0.f;
                l += p;
                sP[rho * CH + lane + 64 * kk] = p;
            }
            l = wave_sum(l);
            // P.V: lane owns DPL adjacent output columns
            float o[DPL];
#pragma unroll
            for (int e = 0; e < DPL; ++e) o[e] = 0.f;
#pragma unroll 4
            for (int key = 0; key < nk; ++key) {
                const float p = sP[rho * CH + key];
                const char* vrow = sV + key * KSTR + lane * DPL * ESZ;
#pragma unroll
                for (int e = 0; e < DPL; ++e) {
                    float vv;
                    if constexpr (Traits<WT>::BF) vv = bf16_to_f32(*reinterpret_cast<const uint16_t*>(vrow + e * 2));
                    else vv = *reinterpret_cast<const float*>(vrow + e * 4);
                    o[e] += p * vv;
                }
            }
            const unsigned orow = (unsigned)((size_t)(b * P.M + i) * P.QD + (hk * grp + gi) * D + lane * DPL);
            if (nch == 1) {
                // the only chunk: normalise and hand the row to the output projection
#pragma unroll
                for (int e = 0; e < DPL; ++e) sx_st1(ro, orow + e, o[e] / l);
            } else {
                // partial (max, sum, unnormalised output) of this chunk, as tagged data
                const unsigned abase = (unsigned)(((size_t)item * Ra + rho) * D + lane * DPL);
#pragma unroll
                for (int e = 0; e < DPL; ++e) ll_st1(racc, abase + e, o[e], P.seq);
                if (lane < 2) ll_st1(rml, (unsigned)(((size_t)item * Ra + rho) * 2 + lane), lane ? l : mx, P.seq);
            }
        }
        // several chunks: the workgroup of the last chunk waits for the others' partials and merges
        if (nch > 1 && ch == nch - 1) {
            const int item0 = item - ch;   // chunk 0 of this (b, hk)
            for (int x = tid; x < Ra * D; x += PS_WG_THREADS) {
                const int rho = x / D, dd = x - rho * D;
                // chunks are folded in order with a running maximum; four chunks per round trip
                float mrun = -INFINITY, num = 0.f, den = 0.f;
                for (int cb = 0; cb < nch; cb += 4) {
                    u32x2 ml0[4], ml1[4], av[4];
                    int spins = 0;
                    for (;;) {
                        bool ok = true;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int cc = cb + i < nch ? cb + i : nch - 1;
                            const unsigned mb = (unsigned)(((size_t)(item0 + cc) * Ra + rho) * 2);
                            ml0[i] = coh_ld8(rml, mb * 8);
                            ml1[i] = coh_ld8(rml, (mb + 1) * 8);
                            av[i] = coh_ld8(racc, (unsigned)(((size_t)(item0 + cc) * Ra + rho) * D + dd) * 8);
                            ok = ok && ml0[i][1] == P.seq && ml1[i][1] == P.seq && av[i][1] == P.seq;
                        }
                        if (__all(ok) || !spin_again(P, spins)) break;
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (cb + i >= nch) continue;
                        const float m_c = __uint_as_float(ml0[i][0]), l_c = __uint_as_float(ml1[i][0]);
                        if (l_c > 0.f) {
                            const float mnew = fmaxf(mrun, m_c);
                            const float so = expf(mrun - mnew), sn = expf(m_c - mnew);   // exp(-inf) = 0 at the start
                            num = num * so + __uint_as_float(av[i][0]) * sn;
                            den = den * so + l_c * sn;
                            mrun = mnew;
                        }
                    }
                }
                const int gi = rho / P.M, i = rho - gi * P.M;
                sx_st1(ro, (unsigned)((size_t)(b * P.M + i) * P.QD + (hk * grp + gi) * D + dd), num / den);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// LM-head merge of one output row by one wavefront.  Every workgroup's list is sorted, so the
// topk-th largest of the list HEADS is a lower bound of the global topk-th key: candidates below
// it are dropped in one pass (at most topk^2 survive) and only those go through the selection.
// sk: LDS scratch of PS_MERGE_BYTES, private to the calling wavefront.
// ------------------------------------------------------------------------------------------
#define PS_MAX_PARTS 512
#define PS_MERGE_CAP 1024
#define PS_MERGE_BYTES (PS_MERGE_CAP * 8 + 128)
__device__ void lm_merge_row(const StepParams& P, int m, int lane, u64* sk) {
    const int nparts = P.plan[PH_LMHEAD].nwg;
    const int topk = P.topk;
    const unsigned stride = 2 + 2 * topk;                  // tagged elements per (workgroup, row)
    const unsigned pstride = (unsigned)P.Rtot * stride;
    const rsrc_t rl = make_rsrc(P.lm_part);
    const unsigned base = (unsigned)m * stride;
    constexpr int HPL = PS_MAX_PARTS / 64;   // lists per lane
    float hmax[HPL], hsum[HPL];
    u64 hk[HPL];
    {
        LL4 hd[HPL];
        int spins = 0;
        for (;;) {   // every workgroup's statistics of this row, once they have arrived
            bool ok = true;
#pragma unroll
            for (int u = 0; u < HPL; ++u) {
                const int gp = lane + 64 * u;
                hd[u] = ll_ld4(rl, base + (gp < nparts ? gp : 0) * pstride);   // max, sum exp, first key
                ok = ok && ll_ok(hd[u], P.seq);
            }
            if (__all(ok) || !spin_again(P, spins)) break;
        }
#pragma unroll
        for (int u = 0; u < HPL; ++u) {
            const bool ok = lane + 64 * u < nparts;
            const f32x4 v = ll_val(hd[u]);
            hmax[u] = ok ? v[0] : -INFINITY;
            hsum[u] = ok ? v[1] : 0.f;
            hk[u] = ok ? (((u64)__float_as_uint(v[3]) << 32) | __float_as_uint(v[2])) : 0;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int u = 0; u < HPL; ++u) mx = fmaxf(mx, hmax[u]);
    mx = wave_max(mx);
    float se = 0.f;
#pragma unroll
    for (int u = 0; u < HPL; ++u)
        if (hmax[u] > -INFINITY) se += hsum[u] * expf(hmax[u] - mx);
    se = wave_sum(se);
    const float lse = mx + logf(se);
    if (lane == 0) P.lse[m] = lse;
    // threshold: the topk-th largest head
    u64 thr = ~0ull;
    for (int t = 0; t < topk; ++t) {
        u64 best = 0;
#pragma unroll
        for (int u = 0; u < HPL; ++u)
            if (hk[u] < thr && hk[u] > best) best = hk[u];
        thr = wave_max_u64(best);
        if (thr == 0) break;   // fewer than topk non-empty lists: keep everything
    }
    // only lists whose head reaches the threshold can contribute: at most topk of them.  Their
    // indices are compacted into LDS, then every (list, entry) pair is fetched in one round.
    int* sl = reinterpret_cast<int*>(sk + PS_MERGE_CAP);   // [32] qualifying list indices (behind the keys)
    int nl = 0;
#pragma unroll
    for (int u = 0; u < HPL; ++u) {
        const bool q = hk[u] != 0 && hk[u] >= thr;
        const u64 mask = __ballot(q);
        const int pos = nl + __popcll(mask & ((1ull << lane) - 1ull));
        if (q && pos < 32) sl[pos] = lane + 64 * u;
        nl += __popcll(mask);
    }
    if (nl > 32) nl = 32;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    int ns = 0;
    const int npair = nl * topk;
    for (int x0 = 0; x0 < npair; x0 += 64 * 4) {
        u32x4 raw[4];
        int spins = 0;
        for (;;) {
            bool ok = true;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int x = x0 + 64 * i + lane;
                if (x >= npair) x = npair - 1;
                const int li = x / topk, tt = x - li * topk;
                raw[i] = coh_ld16(rl, (base + sl[li] * pstride + 2 + 2 * tt) * 8);   // {low, seq, high, seq}
                ok = ok && raw[i][1] == P.seq && raw[i][3] == P.seq;
            }
            if (__all(ok) || !spin_again(P, spins)) break;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int x = x0 + 64 * i + lane;
            const u64 kx = ((u64)raw[i][2] << 32) | raw[i][0];
            const bool keep = x < npair && kx != 0 && kx >= thr;
            const u64 mask = __ballot(keep);
            const int pos = ns + __popcll(mask & ((1ull << lane) - 1ull));
            if (keep && pos < PS_MERGE_CAP) sk[pos] = kx;
            ns += __popcll(mask);
        }
    }
    if (ns > PS_MERGE_CAP) ns = PS_MERGE_CAP;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // survivors written by this wavefront, read by it below
    u64 prev = ~0ull;
    for (int t = 0; t < topk; ++t) {
        u64 best = 0;
        for (int x = lane; x < ns; x += 64) {
            const u64 kx = sk[x];
            if (kx < prev && kx > best) best = kx;
        }
        best = wave_max_u64(best);
        if (lane == 0) {
            P.top_ids[(size_t)m * topk + t] = best ? key_id(best) : 0x7FFFFFFF;
            P.top_p[(size_t)m * topk + t] = best ? expf(key_value(best) - lse) : 0.f;
        }
        prev = best;
    }
}

// ------------------------------------------------------------------------------------------
// kernels
// ------------------------------------------------------------------------------------------
template <typename WT, int MT, int PH>
__global__ void __launch_bounds__(PS_WG_THREADS, 1) gemm_kernel(const StepParams P) {
    extern __shared__ __attribute__((aligned(256))) char smem[];
    uint4 wb[PS_U];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    preload_weights(wb, first_stream<PH>(P, blockIdx.x, wave, lane));
    gemm_phase<WT, MT, PH>(P, blockIdx.x, smem, wb, P.wpack[PH] + lane * 16);
}

template <typename WT, int D>
__global__ void __launch_bounds__(PS_WG_THREADS) attn_kernel(const StepParams P) {
    extern __shared__ __attribute__((aligned(256))) char smem[];
    attn_phase<WT, D>(P, blockIdx.x, gridDim.x, smem);
}

static __global__ void __launch_bounds__(64) lm_merge_kernel(const StepParams P) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    lm_merge_row(P, blockIdx.x, threadIdx.x, reinterpret_cast<u64*>(smem));
}

static __global__ void __launch_bounds__(256) probs_kernel(const StepParams P) {
    const int m = blockIdx.y;
    const float lse = P.lse[m];
    for (int n = blockIdx.x * 256 + threadIdx.x; n < P.V; n += gridDim.x * 256)
        P.probs[(size_t)m * P.V + n] = expf(P.logits_store[(size_t)m * P.V + n] - lse);
}

// The whole step in one persistent kernel: gridDim.x workgroups, all resident (cooperative
// launch).  No grid-wide synchronisation: the phases are chained by the tagged data itself.
// While a workgroup waits for the activations of its next phase, the first weight loads of that
// phase are already in flight.
template <typename WT, int D, int MT>
__global__ void __launch_bounds__(PS_WG_THREADS, 1) fused_kernel(const StepParams P) {
    extern __shared__ __attribute__((aligned(256))) char smem[];
    const int wg = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint4 wb[PS_U];
    stamp(P, wg, 30);
    preload_weights(wb, first_stream<PH_QKV>(P, wg, wave, lane));
    gemm_phase<WT, MT, PH_QKV>(P, wg, smem, wb, P.wpack[PH_QKV] + lane * 16);
    __syncthreads();
    stamp(P, wg, 25);
    attn_phase<WT, D>(P, wg, gridDim.x, smem);
    __syncthreads();
    stamp(P, wg, 26);
    preload_weights(wb, first_stream<PH_OPROJ>(P, wg, wave, lane));
    gemm_phase<WT, MT, PH_OPROJ>(P, wg, smem, wb, first_stream<PH_GATEUP>(P, wg, wave, lane));
    __syncthreads();
    gemm_phase<WT, MT, PH_GATEUP>(P, wg, smem, wb, first_stream<PH_DOWN>(P, wg, wave, lane));
    __syncthreads();
    gemm_phase<WT, MT, PH_DOWN>(P, wg, smem, wb, first_stream<PH_LMHEAD>(P, wg, wave, lane));
    __syncthreads();
    gemm_phase<WT, MT, PH_LMHEAD>(P, wg, smem, wb, P.wpack[PH_LMHEAD] + lane * 16);
    __syncthreads();
    // output row m is merged by wavefront 0 of workgroup m mod gridDim.x
    if (wave == 0) {
        u64* sk = reinterpret_cast<u64*>(smem + 256);
        for (int m = wg; m < P.Rtot; m += gridDim.x) lm_merge_row(P, m, lane, sk);
    }
    stamp(P, wg, 31);
}
