// HIP kernels of the parallel draft step for CDNA4 (gfx950, 64-lane wavefronts).
//
// The step (Section 4.1 "Inference": one drafter forward over the n_new real rows plus k
// [MASK] rows; Section 5.1: the drafter is one Llama-style layer; Section 4.3: shared LM
// head) is five weight-streaming small-M GEMM phases plus attention:
//
//   QKV     RMSNorm(Z; g_in) . [Wq;Wk;Wv]^T   -> rotary -> q_buf, K/V cache rows
//   ATTN    per (sequence, kv head, key chunk) partial softmax.V, merged by the last chunk
//   OPROJ   Y  = Z + O . Wo^T
//   GATEUP  U  = silu(RMSNorm(Y; g_post) . Wg^T) * (RMSNorm(Y; g_post) . Wu^T)
//   DOWN    Y2 = Y + U . Wd^T
//   LMHEAD  logits = RMSNorm(Y2[rows]; g_final) . Wlm^T -> per-workgroup (max, sum exp, top-k)
//   MERGE   per row: log-sum-exp, top-k ids and probabilities
//
// GEMM engine.  Weights are the 16-row MFMA operand, read straight from HBM into
// registers with 16-byte non-temporal loads (each wavefront load covers 16 rows x 64
// contiguous bytes); the few activation rows are the 16-column operand, staged once per
// workgroup in LDS.  bf16 weights use v_mfma_f32_16x16x32_bf16 twice per step: the fp32
// activations are split into a bf16 high part and a bf16 low part (x = hi + lo to ~2^-17),
// so products with the exactly-bf16 weights keep fp32-class accuracy at no extra weight
// traffic.  f32 weights use v_mfma_f32_16x16x4_f32.  Accumulation is always fp32.
// The contraction dimension is cut across workgroups (S slices) and/or across the
// wavefronts of a workgroup (KW).  Slices meet through global partial fragments; the
// wavefront that arrives last at a tile's counter adds the S fragments in slice order
// (so results do not depend on arrival order) and runs the phase epilogue.
#include "ps_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

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
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ldg_stream16(const void* p) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ uint4 ld16(const void* p) { return *reinterpret_cast<const uint4*>(p); }

// GE stored elements starting at p -> floats
template <typename WT> __device__ __forceinline__ void load_group(const void* p, float* out);
template <> __device__ __forceinline__ void load_group<float>(const void* p, float* out) {
    uint4 v = ld16(p);
    out[0] = __uint_as_float(v.x); out[1] = __uint_as_float(v.y);
    out[2] = __uint_as_float(v.z); out[3] = __uint_as_float(v.w);
}
template <> __device__ __forceinline__ void load_group<bf16_t>(const void* p, float* out) {
    uint4 v = ld16(p);
    out[0] = bf16_to_f32(v.x & 0xFFFFu); out[1] = bf16_to_f32(v.x >> 16);
    out[2] = bf16_to_f32(v.y & 0xFFFFu); out[3] = bf16_to_f32(v.y >> 16);
    out[4] = bf16_to_f32(v.z & 0xFFFFu); out[5] = bf16_to_f32(v.z >> 16);
    out[6] = bf16_to_f32(v.w & 0xFFFFu); out[7] = bf16_to_f32(v.w >> 16);
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
template <typename WT> __device__ __forceinline__ void store4(void* p, f32x4 v);
template <> __device__ __forceinline__ void store4<float>(void* p, f32x4 v) { *reinterpret_cast<f32x4*>(p) = v; }
template <> __device__ __forceinline__ void store4<bf16_t>(void* p, f32x4 v) {
    uint2 o;
    o.x = f32_to_bf16(v[0]) | (f32_to_bf16(v[1]) << 16);
    o.y = f32_to_bf16(v[2]) | (f32_to_bf16(v[3]) << 16);
    *reinterpret_cast<uint2*>(p) = o;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// (value, id) ordering of the top-k: larger logit first, equal logits by lower id
__device__ __forceinline__ bool cand_better(float v, int id, float bv, int bid) {
    return v > bv || (v == bv && id < bid);
}
__device__ __forceinline__ void wave_best(float& v, int& id) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        float ov = __shfl_xor(v, o, 64);
        int oid = __shfl_xor(id, o, 64);
        if (cand_better(ov, oid, v, id)) { v = ov; id = oid; }
    }
}

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

// GE activation values of panel row r starting at contraction index kk (before norm/gain)
template <typename WT, int PH>
__device__ __forceinline__ void act_group(const StepParams& P, int r, int kk, float* out) {
    constexpr int GE = Traits<WT>::GE;
    if (PH == PH_QKV) {
        load_group<WT>(z_ptr<WT>(P, r, kk), out);
    } else {
        const float* src;
        if (PH == PH_OPROJ) src = P.o_buf + (size_t)r * P.QD + kk;
        else if (PH == PH_GATEUP) src = P.y_buf + (size_t)r * P.H + kk;
        else if (PH == PH_DOWN) src = P.u_buf + (size_t)r * P.F + kk;
        else {   // decoding rows: last real row and the k mask rows of each sequence (or all rows)
            const int b = r / P.R, jj = r - b * P.R;
            const int m = b * P.M + (P.all_rows ? jj : (P.n_new - 1 + jj));
            src = P.y2_buf + (size_t)m * P.H + kk;
        }
#pragma unroll
        for (int g = 0; g < GE; g += 4) {
            f32x4 v = *reinterpret_cast<const f32x4*>(src + g);
            out[g] = v[0]; out[g + 1] = v[1]; out[g + 2] = v[2]; out[g + 3] = v[3];
        }
    }
}

// ------------------------------------------------------------------------------------------
// inner loop: stream nsteps x 64 B of one weight row per lane, multiply with the LDS panel
// ------------------------------------------------------------------------------------------
template <typename WT, int MT>
__device__ __forceinline__ void mma_step(uint4 w, const char* const (&pa)[MT], const int (&pinc)[MT],
                                         const int (&plo)[MT], int t, f32x4 (&acc)[MT]) {
    if constexpr (Traits<WT>::BF) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, w);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const char* p = pa[mt] + t * pinc[mt];
            const bf16x8 bh = __builtin_bit_cast(bf16x8, ld16(p));
            const bf16x8 bl = __builtin_bit_cast(bf16x8, ld16(p + plo[mt]));
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bh, acc[mt], 0, 0, 0);
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bl, acc[mt], 0, 0, 0);
        }
    } else {
        const f32x4 a = __builtin_bit_cast(f32x4, w);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const f32x4 b = __builtin_bit_cast(f32x4, ld16(pa[mt] + t * pinc[mt]));
#pragma unroll
            for (int e = 0; e < 4; ++e)
                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[e], b[e], acc[mt], 0, 0, 0);
        }
    }
}

template <typename WT, int MT>
__device__ __forceinline__ void accumulate(const char* wp, int n, const char* const (&pa)[MT],
                                           const int (&pinc)[MT], const int (&plo)[MT], f32x4 (&acc)[MT]) {
    constexpr int U = 8;   // weight loads in flight per lane (8 x 16 B)
    uint4 wb[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (u < n) wb[u] = ldg_stream16(wp + u * 64);
    int t0 = 0;
    for (; t0 + 2 * U <= n; t0 += U) {   // steady state: every prefetch is in range
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint4 w = wb[u];
            wb[u] = ldg_stream16(wp + (t0 + u + U) * 64);
            mma_step<WT, MT>(w, pa, pinc, plo, t0 + u, acc);
        }
    }
    for (; t0 < n; t0 += U) {            // drain
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u;
            if (t < n) {
                const uint4 w = wb[u];
                if (t + U < n) wb[u] = ldg_stream16(wp + (t + U) * 64);
                mma_step<WT, MT>(w, pa, pinc, plo, t, acc);
            }
        }
    }
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
            *reinterpret_cast<f32x4*>(P.q_buf + (size_t)m * P.QD + hh * P.d + f) = o;
        } else {
            const bool isk = hh < P.nq + P.nkv;
            const int hk = isk ? hh - P.nq : hh - P.nq - P.nkv;
            char* cache = (char*)(isk ? P.kc : P.vc);
            const size_t e = ((size_t)(P.kv_off[b] + pos) * P.nkv + hk) * P.d + f;
            store4<WT>(cache + e * Traits<WT>::ESZ, o);
        }
    }
}

template <typename WT, int MT>
__device__ __forceinline__ void epilogue_oproj(const StepParams& P, int tau, int lane, f32x4 (&acc)[MT]) {
    const int c = lane & 15, q = lane >> 4;
    const int n = 16 * tau + 4 * q;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = 16 * mt + c;
        if (m >= P.Mtot) continue;
        const f32x4 z = load4<WT>(z_ptr<WT>(P, m, n));
        *reinterpret_cast<f32x4*>(P.y_buf + (size_t)m * P.H + n) = z + acc[mt];
    }
}

template <typename WT, int MT>
__device__ __forceinline__ void epilogue_gateup(const StepParams& P, int tau, int lane, f32x4 (&acc)[MT]) {
    const int c = lane & 15, q = lane >> 4;
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
        *reinterpret_cast<f32x4*>(P.u_buf + (size_t)m * P.F + 8 * tau + 4 * q) = u;
    }
}

template <typename WT, int MT>
__device__ __forceinline__ void epilogue_down(const StepParams& P, int tau, int lane, f32x4 (&acc)[MT]) {
    const int c = lane & 15, q = lane >> 4;
    const int n = 16 * tau + 4 * q;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = 16 * mt + c;
        if (m >= P.Mtot) continue;
        const f32x4 y = *reinterpret_cast<const f32x4*>(P.y_buf + (size_t)m * P.H + n);
        const f32x4 o = y + acc[mt];
        *reinterpret_cast<f32x4*>(P.y2_buf + (size_t)m * P.H + n) = o;
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

template <typename WT, int MT, int PH>
__device__ void gemm_phase(const StepParams& P, int wg, char* smem) {
    constexpr bool BF = Traits<WT>::BF;
    constexpr int KSTEP = Traits<WT>::KSTEP, GE = Traits<WT>::GE, ESZ = Traits<WT>::ESZ;
    const PhasePlan pl = P.plan[PH];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, kb = lane >> 4;
    const int rows = phase_rows<PH>(P);
    const int K = phase_K<PH>(P);

    const int S = pl.S, KW = pl.KW;
    const int s = wg % S, j = wg / S, Gs = pl.nwg / S;
    if (j >= Gs) return;
    const int k_lo = (int)((long long)s * pl.Kt / S), k_hi = (int)((long long)(s + 1) * pl.Kt / S);
    const int SL = PS_WAVES / KW, slot = wave / KW, kw = wave - slot * KW;
    const int per_round = Gs * SL;
    const int rounds = (pl.T + per_round - 1) / per_round;

    // LDS carve-up
    float* s_scale = reinterpret_cast<float*>(smem);             // [64] per-row 1/rms
    char* s_zero = smem + 256;                                   // 64 zero bytes for unused columns
    char* s_red = smem + 512;                                    // [16 waves][MT][64 lanes] f32x4
    const int RS = panel_row_stride(pl.panel_steps);
    char* s_pa = s_red + PS_WAVES * MT * 1024;                   // high parts (or f32 values)
    char* s_pb = s_pa + (size_t)rows * RS;                       // low parts (bf16 only)
    float* s_lm = reinterpret_cast<float*>(s_pb + (BF ? (size_t)rows * RS : 0));

    if (tid < 16) reinterpret_cast<uint32_t*>(s_zero)[tid] = 0u;
    if (PH == PH_LMHEAD) {
        const int n_lm = rounds * SL * rows * 16;
        for (int x = tid; x < n_lm; x += PS_WG_THREADS) s_lm[x] = -INFINITY;
    }
    // per-row 1/rms over the FULL row (RMSNorm), whatever K-slice this workgroup owns
    const bool norm = phase_norm<PH>(P);
    if (norm) {
        for (int r = wave; r < rows; r += PS_WAVES) {
            float ss = 0.f;
            for (int kk = lane * GE; kk < K; kk += 64 * GE) {
                float v[GE];
                act_group<WT, PH>(P, r, kk, v);
#pragma unroll
                for (int e = 0; e < GE; ++e) ss += v[e] * v[e];
            }
            ss = wave_sum(ss);
            if (lane == 0) s_scale[r] = 1.0f / sqrtf(ss / (float)K + P.eps);
        }
    }
    __syncthreads();

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
    for (int rd = 0; rd < rounds; ++rd) {
        const int tau = rd * per_round + slot * Gs + j;
        const bool valid = tau < pl.T;
        const char* wrow = valid ? weight_row_ptr<WT, PH>(P, tau, c) + kb * 16 : nullptr;
        f32x4 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};

        for (int a = k_lo; a < k_hi; a += pl.panel_steps) {
            const int b = min(a + pl.panel_steps, k_hi);
            if (a != staged_a || b != staged_b) {
                __syncthreads();   // everyone is done with the previous panel
                // stage steps [a, b): 4 groups of 16 B per (row, step)
                const int groups = (b - a) * 4;
                const void* gain = phase_gain<PH>(P);
                for (int x = tid; x < rows * groups; x += PS_WG_THREADS) {
                    const int r = x / groups, g = x - r * groups;
                    const int kk = a * KSTEP + g * GE;
                    float v[GE];
                    act_group<WT, PH>(P, r, kk, v);
                    if (norm) {
                        float gn[GE];
                        load_group<WT>((const char*)gain + (size_t)kk * ESZ, gn);
                        const float sc = s_scale[r];
#pragma unroll
                        for (int e = 0; e < GE; ++e) v[e] = v[e] * sc * gn[e];
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
                        *reinterpret_cast<uint4*>(s_pa + (size_t)r * RS + g * 16) = ph;
                        *reinterpret_cast<uint4*>(s_pb + (size_t)r * RS + g * 16) = plw;
                    } else {
                        uint4 pv;
                        pv.x = __float_as_uint(v[0]); pv.y = __float_as_uint(v[1]);
                        pv.z = __float_as_uint(v[2]); pv.w = __float_as_uint(v[3]);
                        *reinterpret_cast<uint4*>(s_pa + (size_t)r * RS + g * 16) = pv;
                    }
                }
                __syncthreads();
                staged_a = a; staged_b = b;
            }
            if (valid) {
                const int n = b - a;
                const int t0 = (int)((long long)kw * n / KW), t1 = (int)((long long)(kw + 1) * n / KW);
                const char* pa_t[MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) pa_t[mt] = pa[mt] + t0 * pinc[mt];
                accumulate<WT, MT>(wrow + (size_t)(a + t0) * 64, t1 - t0, pa_t, pinc, plo, acc);
            }
        }

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
            bool run_epilogue = true;
            if (S > 1) {
                // K-slices of other workgroups: publish this fragment, the last arrival sums all S
                f32x4* part = reinterpret_cast<f32x4*>(P.part);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    part[(((size_t)s * pl.T + tau) * MT + mt) * 64 + lane] = acc[mt];
                __threadfence();   // release: fragment visible device-wide before the count
                int old = 0;
                if (lane == 0) old = atomicAdd(P.counters + pl.cnt_base + tau, 1);
                old = __shfl(old, 0, 64);
                run_epilogue = (old == S - 1);
                if (run_epilogue) {
                    __threadfence();   // acquire: see the other slices' fragments
                    if (lane == 0) P.counters[pl.cnt_base + tau] = 0;   // ready for the next step
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
                    for (int ss = 0; ss < S; ++ss) {
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt)
                            acc[mt] += __builtin_nontemporal_load(
                                &part[(((size_t)ss * pl.T + tau) * MT + mt) * 64 + lane]);
                    }
                }
            }
            if (run_epilogue) {
                if (PH == PH_QKV) epilogue_qkv<WT, MT>(P, tau, lane, acc);
                else if (PH == PH_OPROJ) epilogue_oproj<WT, MT>(P, tau, lane, acc);
                else if (PH == PH_GATEUP) epilogue_gateup<WT, MT>(P, tau, lane, acc);
                else if (PH == PH_DOWN) epilogue_down<WT, MT>(P, tau, lane, acc);
                else epilogue_lm<WT, MT>(P, tau, lane, acc, s_lm, rd * SL + slot);
            }
        }
    }

    if (PH == PH_LMHEAD) {
        // per-workgroup softmax statistics and top-k over the logits held in LDS
        __syncthreads();
        const int n_el = rounds * SL * 16;
        const int topk = P.topk;
        const int stride = 2 + 2 * topk;
        for (int m = wave; m < rows; m += PS_WAVES) {
            float mx = -INFINITY;
            for (int x = lane; x < n_el; x += 64) mx = fmaxf(mx, s_lm[((size_t)(x >> 4) * rows + m) * 16 + (x & 15)]);
            mx = wave_max(mx);
            float se = 0.f;
            if (mx > -INFINITY)
                for (int x = lane; x < n_el; x += 64) se += expf(s_lm[((size_t)(x >> 4) * rows + m) * 16 + (x & 15)] - mx);
            se = wave_sum(se);
            float* out = P.lm_part + ((size_t)wg * rows + m) * stride;
            if (lane == 0) { out[0] = mx; out[1] = se; }
            float pv = INFINITY; int pid = -1;   // previous winner: candidates must come strictly after it
            for (int t = 0; t < topk; ++t) {
                float bv = -INFINITY; int bid = 0x7FFFFFFF;
                for (int x = lane; x < n_el; x += 64) {
                    const int lt = x >> 4;
                    const float v = s_lm[((size_t)lt * rows + m) * 16 + (x & 15)];
                    const int rd2 = lt / SL, sl2 = lt - rd2 * SL;
                    const int id = 16 * (rd2 * per_round + sl2 * Gs + j) + (x & 15);
                    const bool after_prev = v < pv || (v == pv && id > pid);
                    if (v > -INFINITY && after_prev && cand_better(v, id, bv, bid)) { bv = v; bid = id; }
                }
                wave_best(bv, bid);
                if (lane == 0) { out[2 + t] = bv; reinterpret_cast<int*>(out)[2 + topk + t] = bid; }
                pv = bv; pid = bid;
                if (!(bv > -INFINITY)) { pv = -INFINITY; pid = 0x7FFFFFFF; }
            }
        }
    }
}

template <typename WT, int MT, int PH>
__global__ void __launch_bounds__(PS_WG_THREADS) gemm_kernel(const StepParams P) {
    extern __shared__ __attribute__((aligned(256))) char smem[];
    gemm_phase<WT, MT, PH>(P, blockIdx.x, smem);
}

// ------------------------------------------------------------------------------------------
// attention: one work item = (sequence b, kv head hk, chunk of CH keys); all g*M query rows
// of the kv head are processed against the chunk; K/V tiles are staged in LDS; row i of the
// step sees cache positions 0 .. kv_len[b] + i (its own and earlier rows of this step
// included; Algorithm 1: distribution j is conditioned on [MASK]_1..j only).
// ------------------------------------------------------------------------------------------
template <typename WT, int D, int CH>
__device__ void attn_phase(const StepParams& P, int wg, int nwg, char* smem) {
    constexpr int ESZ = Traits<WT>::ESZ, GE = Traits<WT>::GE;
    constexpr int KSTR = D * ESZ + 16;              // padded K/V row stride in LDS (bytes)
    constexpr int DPL = D / 64;                     // output columns per lane
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = P.nq / P.nkv;
    const int Ra = grp * P.M;
    int& s_last = *reinterpret_cast<int*>(smem);                // completion flag of the current item
    float* sQ = reinterpret_cast<float*>(smem + 256);           // [Ra][D]
    float* sP = sQ + PS_MAX_ROWS * D;                           // [Ra][CH]
    char* sK = reinterpret_cast<char*>(sP + PS_MAX_ROWS * CH);  // [CH][KSTR]
    char* sV = sK + CH * KSTR;

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
        // stage Q rows of the head group, and the K/V chunk
        for (int x = tid; x < Ra * (D / 4); x += PS_WG_THREADS) {
            const int rho = x / (D / 4), dd = (x - rho * (D / 4)) * 4;
            const int gi = rho / P.M, i = rho - gi * P.M;
            const f32x4 v = *reinterpret_cast<const f32x4*>(P.q_buf + (size_t)(b * P.M + i) * P.QD + (hk * grp + gi) * D + dd);
            *reinterpret_cast<f32x4*>(sQ + rho * D + dd) = v;
        }
        constexpr int GPR = D / GE;   // 16-byte groups per key row
        for (int x = tid; x < nk * GPR; x += PS_WG_THREADS) {
            const int key = x / GPR, g = x - key * GPR;
            const size_t e = ((size_t)(P.kv_off[b] + c0 + key) * P.nkv + hk) * D + g * GE;
            *reinterpret_cast<uint4*>(sK + key * KSTR + g * 16) = ld16((const char*)P.kc + e * ESZ);
            *reinterpret_cast<uint4*>(sV + key * KSTR + g * 16) = ld16((const char*)P.vc + e * ESZ);
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
                    for (int g = 0; g < GPR; ++g) {
                        float kv[GE];
                        load_group<WT>(krow + g * 16, kv);
#pragma unroll
                        for (int e = 0; e < GE; e += 4) {
                            const f32x4 qv = *reinterpret_cast<const f32x4*>(sQ + rho * D + g * GE + e);
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
            float* acc = P.attn_acc + ((size_t)item * Ra + rho) * D + lane * DPL;
#pragma unroll
            for (int e = 0; e < DPL; ++e) acc[e] = o[e];
            if (lane == 0) P.attn_ml[(size_t)item * Ra + rho] = make_float2(mx, l);
        }
        // completion of (b, hk): the workgroup that finishes the last chunk merges all chunks
        __threadfence();
        __syncthreads();
        if (tid == 0) {
            int* cnt = P.counters + P.attn_cnt_base + b * P.nkv + hk;
            const int old = atomicAdd(cnt, 1);
            s_last = (old == nch - 1);
            if (s_last) *cnt = 0;
        }
        __syncthreads();
        if (s_last) {
            __threadfence();
            const int item0 = item - ch;   // chunk 0 of this (b, hk)
            for (int x = tid; x < Ra * D; x += PS_WG_THREADS) {
                const int rho = x / D, dd = x - rho * D;
                float mstar = -INFINITY;
                for (int cc = 0; cc < nch; ++cc)
                    mstar = fmaxf(mstar, P.attn_ml[(size_t)(item0 + cc) * Ra + rho].x);
                float num = 0.f, den = 0.f;
                for (int cc = 0; cc < nch; ++cc) {
                    const float2 ml = P.attn_ml[(size_t)(item0 + cc) * Ra + rho];
                    if (ml.y > 0.f) {
                        const float w = expf(ml.x - mstar);
                        den += ml.y * w;
                        num += __builtin_nontemporal_load(&P.attn_acc[((size_t)(item0 + cc) * Ra + rho) * D + dd]) * w;
                    }
                }
                const int gi = rho / P.M, i = rho - gi * P.M;
                P.o_buf[(size_t)(b * P.M + i) * P.QD + (hk * grp + gi) * D + dd] = num / den;
            }
        }
    }
}

template <typename WT, int D, int CH>
__global__ void __launch_bounds__(PS_WG_THREADS) attn_kernel(const StepParams P) {
    extern __shared__ __attribute__((aligned(256))) char smem[];
    attn_phase<WT, D, CH>(P, blockIdx.x, gridDim.x, smem);
}

template <typename WT, int D> struct AttnCfg {
    static constexpr int CH = Traits<WT>::BF ? 128 : (D == 64 ? 128 : 64);
    static constexpr int LDS = 256 + PS_MAX_ROWS * D * 4 + PS_MAX_ROWS * CH * 4 + 2 * CH * (D * Traits<WT>::ESZ + 16);
};

// ------------------------------------------------------------------------------------------
// LM-head merge: one wavefront per output row combines the workgroups' partial statistics
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64) lm_merge_kernel(const StepParams P) {
    const int m = blockIdx.x, lane = threadIdx.x;
    const int nparts = P.plan[PH_LMHEAD].nwg;
    const int topk = P.topk, stride = 2 + 2 * topk;
    const float* base = P.lm_part + (size_t)m * stride;
    const size_t pstride = (size_t)P.Rtot * stride;
    float mx = -INFINITY;
    for (int g = lane; g < nparts; g += 64) mx = fmaxf(mx, base[g * pstride]);
    mx = wave_max(mx);
    float se = 0.f;
    for (int g = lane; g < nparts; g += 64) {
        const float pm = base[g * pstride];
        if (pm > -INFINITY) se += base[g * pstride + 1] * expf(pm - mx);
    }
    se = wave_sum(se);
    const float lse = mx + logf(se);
    if (lane == 0) P.lse[m] = lse;
    float pv = INFINITY; int pid = -1;
    const int ncand = nparts * topk;
    for (int t = 0; t < topk; ++t) {
        float bv = -INFINITY; int bid = 0x7FFFFFFF;
        for (int x = lane; x < ncand; x += 64) {
            const int g = x / topk, tt = x - g * topk;
            const float v = base[g * pstride + 2 + tt];
            const int id = reinterpret_cast<const int*>(base + g * pstride)[2 + topk + tt];
            const bool after_prev = v < pv || (v == pv && id > pid);
            if (v > -INFINITY && after_prev && cand_better(v, id, bv, bid)) { bv = v; bid = id; }
        }
        wave_best(bv, bid);
        if (lane == 0) {
            P.top_ids[(size_t)m * topk + t] = bid;
            P.top_p[(size_t)m * topk + t] = expf(bv - lse);
        }
        pv = bv; pid = bid;
    }
}

__global__ void __launch_bounds__(256) probs_kernel(const StepParams P) {
    const int m = blockIdx.y;
    const float lse = P.lse[m];
    for (int n = blockIdx.x * 256 + threadIdx.x; n < P.V; n += gridDim.x * 256)
        P.probs[(size_t)m * P.V + n] = expf(P.logits_store[(size_t)m * P.V + n] - lse);
}

// ------------------------------------------------------------------------------------------
// host side: instantiation tables and launch sequence
// ------------------------------------------------------------------------------------------
typedef void (*kernel_fn)(const StepParams);

template <typename WT, int PH> static kernel_fn gemm_fn(int mt) {
    switch (mt) {
        case 1: return gemm_kernel<WT, 1, PH>;
        case 2: return gemm_kernel<WT, 2, PH>;
        case 3: return gemm_kernel<WT, 3, PH>;
        default: return gemm_kernel<WT, 4, PH>;
    }
}
template <typename WT> static kernel_fn gemm_fn_ph(int ph, int mt) {
    switch (ph) {
        case PH_QKV: return gemm_fn<WT, PH_QKV>(mt);
        case PH_OPROJ: return gemm_fn<WT, PH_OPROJ>(mt);
        case PH_GATEUP: return gemm_fn<WT, PH_GATEUP>(mt);
        case PH_DOWN: return gemm_fn<WT, PH_DOWN>(mt);
        default: return gemm_fn<WT, PH_LMHEAD>(mt);
    }
}
static kernel_fn gemm_fn_any(int dtype, int ph, int mt) {
    return dtype == PS_BF16 ? gemm_fn_ph<bf16_t>(ph, mt) : gemm_fn_ph<float>(ph, mt);
}
static kernel_fn attn_fn_any(int dtype, int d, int* lds) {
    if (dtype == PS_BF16) {
        if (d == 64) { *lds = AttnCfg<bf16_t, 64>::LDS; return attn_kernel<bf16_t, 64, AttnCfg<bf16_t, 64>::CH>; }
        *lds = AttnCfg<bf16_t, 128>::LDS; return attn_kernel<bf16_t, 128, AttnCfg<bf16_t, 128>::CH>;
    }
    if (d == 64) { *lds = AttnCfg<float, 64>::LDS; return attn_kernel<float, 64, AttnCfg<float, 64>::CH>; }
    *lds = AttnCfg<float, 128>::LDS; return attn_kernel<float, 128, AttnCfg<float, 128>::CH>;
}

int ps_attn_chunk(int dtype, int d) {
    if (dtype == PS_BF16) return d == 64 ? AttnCfg<bf16_t, 64>::CH : AttnCfg<bf16_t, 128>::CH;
    return d == 64 ? AttnCfg<float, 64>::CH : AttnCfg<float, 128>::CH;
}

hipError_t ps_kernels_prepare(int lds_limit) {
    for (int dtype = 0; dtype < 2; ++dtype) {
        for (int ph = 0; ph < PH_COUNT; ++ph)
            for (int mt = 1; mt <= 4; ++mt) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_fn_any(dtype, ph, mt)),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds_limit);
                if (e != hipSuccess) return e;
            }
        for (int d = 64; d <= 128; d += 64) {
            int lds = 0;
            kernel_fn f = attn_fn_any(dtype, d, &lds);
            if (lds > lds_limit) return hipErrorInvalidValue;
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(f),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

hipError_t ps_launch_step(const StepParams& P, int dtype, hipStream_t stream, hipEvent_t* events) {
    const int mt_all = (P.Mtot + 15) / 16, mt_lm = (P.Rtot + 15) / 16;
    int n_ev = 0;
    auto mark = [&]() -> hipError_t { return events ? hipEventRecord(events[n_ev++], stream) : hipSuccess; };
    auto gemm = [&](int ph, int mt) -> hipError_t {
        const PhasePlan& pl = P.plan[ph];
        hipLaunchKernelGGL(gemm_fn_any(dtype, ph, mt), dim3(pl.nwg), dim3(PS_WG_THREADS), pl.lds_bytes, stream, P);
        hipError_t le = hipGetLastError();
        return le != hipSuccess ? le : mark();
    };
    hipError_t e;
    if ((e = mark()) != hipSuccess) return e;
    if ((e = gemm(PH_QKV, mt_all)) != hipSuccess) return e;
    {
        int lds = 0;
        kernel_fn f = attn_fn_any(dtype, P.d, &lds);
        hipLaunchKernelGGL(f, dim3(P.attn_nwg), dim3(PS_WG_THREADS), lds, stream, P);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if ((e = mark()) != hipSuccess) return e;
    }
    if ((e = gemm(PH_OPROJ, mt_all)) != hipSuccess) return e;
    if ((e = gemm(PH_GATEUP, mt_all)) != hipSuccess) return e;
    if ((e = gemm(PH_DOWN, mt_all)) != hipSuccess) return e;
    if ((e = gemm(PH_LMHEAD, mt_lm)) != hipSuccess) return e;
    hipLaunchKernelGGL(lm_merge_kernel, dim3(P.Rtot), dim3(64), 0, stream, P);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (P.probs) {
        hipLaunchKernelGGL(probs_kernel, dim3((P.V + 255) / 256 < 256 ? (P.V + 255) / 256 : 256, P.Rtot), dim3(256), 0,
                           stream, P);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return mark();
}
