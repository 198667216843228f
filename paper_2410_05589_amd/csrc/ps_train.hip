// Attention of group-wise parallel training (see include/ps_train.h; Section 4.1).
//
// Three kernels per call: the rotary table (cos, sin of position * base^(-2j/d) in double precision), the
// rotation of q (to float32) and k (to the storage type, rounded as the inference path caches keys), and the
// attention itself.
//
// The attention kernel never touches a key the mask hides.  A query tile is a whole number of parallel groups
// (as many as fit into 16 rows); what its rows may see are (a) real tokens of groups up to their own - these
// are gathered with a stride of k + 1 rows, 16 per key tile - and (b) [MASK] tokens of their own group, which
// all lie inside the query tile's own 16 rows: one more key tile.  The wavefronts of a workgroup take the key
// tiles in turn, each with its own running maximum, sum and output (online softmax); their results meet in LDS
// at the end.  Scores are one MFMA tile per key tile (the keys' rows are the 16-row operand, straight from
// memory; the 16 query rows, split into bf16 high and low parts, the 16-column operand in LDS).  P.V for bf16
// values is MFMA work too: the score tile comes out of the matrix core with a lane holding four consecutive keys of
// one query, which is exactly the 16-row operand layout of v_mfma_f32_16x16x16_bf16 (P, split into high and low
// parts); the other operand needs four consecutive keys of one value column per lane, so the wavefront passes its
// 16 value rows through LDS with the rows of a key pair interleaved (one dword = the same column of two keys).
// A wavefront works on two key tiles at a time (one softmax update per 32 keys, one v_mfma_f32_16x16x32_bf16 per
// part and 16 output columns) and refills the tiles' registers as soon as they are consumed.
// float32 values take plain FMAs, a key tile at a time: a lane owns head_dim / 64 output columns for all 16 rows.
#include "ps_device.h"
#include "ps_train.h"

namespace {

constexpr int GA_THREADS = 256, GA_WAVES = GA_THREADS / 64;

struct GaParams {
    int seqs, T, k, nq, nkv, rows, gpt, ntiles;   // gpt: groups per query tile
    float inv_sqrt_d;
    const void *q, *k_, *v;
    float* out;
    float2* table;      // [T + k][d / 2]
    float* q_rot;       // [seqs][rows][nq][d]
    void* k_rot;        // [seqs][rows][nkv][d] storage type
    double log_base;
};

template <int D>
__global__ void __launch_bounds__(256) ga_table_kernel(const GaParams P) {
    const int n = (P.T + P.k) * (D / 2);
    for (int x = blockIdx.x * 256 + threadIdx.x; x < n; x += gridDim.x * 256) {
        const int pos = x / (D / 2), j = x - pos * (D / 2);
        const double a = (double)pos * exp(-2.0 * j / D * P.log_base);
        P.table[x] = make_float2((float)cos(a), (float)sin(a));
    }
}

// one thread per (row, head, pair of 4 + 4 elements j..j+3, j+d/2..): q heads first, then k heads
template <typename WT, int D>
__global__ void __launch_bounds__(256) ga_rope_kernel(const GaParams P) {
    constexpr int ESZ = Traits<WT>::ESZ, Q4 = D / 8;     // groups of 4 pairs per head
    const long long n = (long long)P.seqs * P.rows * (P.nq + P.nkv) * Q4;
    for (long long x = (long long)blockIdx.x * 256 + threadIdx.x; x < n; x += (long long)gridDim.x * 256) {
        const int g4 = (int)(x % Q4);
        long long y = x / Q4;
        const int h = (int)(y % (P.nq + P.nkv));
        const long long sr = y / (P.nq + P.nkv);           // seq * rows + row
        const int row = (int)(sr % P.rows);
        const int pos = row / (P.k + 1) + row % (P.k + 1);  // group + slot
        const bool isq = h < P.nq;
        const size_t base = isq ? ((size_t)sr * P.nq + h) * D : ((size_t)sr * P.nkv + (h - P.nq)) * D;
        const char* src = (const char*)(isq ? P.q : P.k_);
        const f32x4 a = load4<WT>(src + (base + 4 * g4) * ESZ), b = load4<WT>(src + (base + D / 2 + 4 * g4) * ESZ);
        f32x4 ra, rb;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float2 t = P.table[(size_t)pos * (D / 2) + 4 * g4 + e];
            ra[e] = a[e] * t.x - b[e] * t.y;
            rb[e] = b[e] * t.x + a[e] * t.y;
        }
        if (isq) {
            *reinterpret_cast<f32x4*>(P.q_rot + base + 4 * g4) = ra;
            *reinterpret_cast<f32x4*>(P.q_rot + base + D / 2 + 4 * g4) = rb;
        } else {
            store4<WT>((char*)P.k_rot + (base + 4 * g4) * ESZ, ra);
            store4<WT>((char*)P.k_rot + (base + D / 2 + 4 * g4) * ESZ, rb);
        }
    }
}

template <typename WT, int D>
__global__ void __launch_bounds__(GA_THREADS, Traits<WT>::BF ? 3 : 2) ga_attn_kernel(const GaParams P) {   // workgroups per compute unit
    constexpr bool BF = Traits<WT>::BF;
    constexpr int ESZ = Traits<WT>::ESZ, KSTEP = Traits<WT>::KSTEP, STEPS = D / KSTEP, DPL = D / 64;
    constexpr int OFF_Q = 0;                                // 16 query rows as MFMA operands (hi, lo): 16 * D * 4 bytes
    constexpr int OFF_P = OFF_Q + 16 * D * 4;               // float32 values: [waves][16 rows][16 keys] probabilities
    constexpr int OFF_A = OFF_P + (BF ? 0 : GA_WAVES * 16 * 16 * 4);   // [waves][16] rescale factors of the running output
    constexpr int OFF_ML = OFF_A + GA_WAVES * 16 * 4;       // [waves][16][2] final (max, sum)
    constexpr int VSTR = D + 8;                             // dwords between key pairs of the staged values (no bank conflicts)
    // bf16 values: [waves][2 key tiles][8 key pairs][VSTR] dwords (value of key 2m, value of key 2m+1); a wavefront's
    // final output [16][D] takes the place of its staged values (which it alone uses).  float32: [waves][16][D] outputs
    constexpr int OSTRIDE = BF ? 2 * 8 * VSTR : 16 * D;     // floats between the wavefronts' output areas
    static_assert(!BF || 2 * 8 * VSTR >= 16 * D, "a wavefront's outputs fit its staging area");
    constexpr int OFF_O = OFF_ML + GA_WAVES * 16 * 2 * 4;
    constexpr int OFF_V = OFF_O;
    __shared__ __attribute__((aligned(16))) char smem[OFF_O + GA_WAVES * OSTRIDE * 4];
    typedef typename VRaw<WT, DPL>::type raw_t;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, kb = lane >> 4;
    const int tile = P.ntiles - 1 - (int)blockIdx.x;        // the tiles with the most keys start first
    const int h = blockIdx.y, seq = blockIdx.z, hk = h / (P.nq / P.nkv);
    const int K1 = P.k + 1;
    const int g0 = tile * P.gpt, ng = min(P.gpt, P.T - g0), nrows = ng * K1, r0 = g0 * K1;
    const int g_last = g0 + ng - 1;
    char* sQ = smem + OFF_Q;
    float* sP = reinterpret_cast<float*>(smem + OFF_P) + wave * 256;
    float* sA = reinterpret_cast<float*>(smem + OFF_A) + wave * 16;
    float* sML = reinterpret_cast<float*>(smem + OFF_ML);
    float* sO = reinterpret_cast<float*>(smem + OFF_O);
    unsigned* sV = reinterpret_cast<unsigned*>(smem + OFF_V) + wave * 2 * 8 * VSTR;
    typedef short s16x4 __attribute__((ext_vector_type(4)));

    // ---- the query rows (rotated, float32) into LDS as the 16-column MFMA operand; rows beyond the tile repeat the last
    const float* qbase = P.q_rot + ((size_t)seq * P.rows * P.nq + h) * D;
    for (int t2 = tid; t2 < 16 * (D / 4); t2 += GA_THREADS) {
        const int r = min(t2 / (D / 4), nrows - 1), g4 = t2 % (D / 4);
        const u32x4 x = *reinterpret_cast<const u32x4*>(qbase + (size_t)(r0 + r) * P.nq * D + 4 * g4);
        attn_store_q<WT, D>(sQ, t2, x);
    }
    __syncthreads();
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
    // this lane's query (column c of the score tile): group and slot
    const int qr = min(c, nrows - 1), qg = g0 + qr / K1, qs = qr % K1;
    const bool qlive = c < nrows;

    const char* kbase = (const char*)P.k_rot + ((size_t)seq * P.rows * P.nkv + hk) * D * ESZ;
    const char* vbase = (const char*)P.v + ((size_t)seq * P.rows * P.nkv + hk) * D * ESZ;
    const size_t rstride = (size_t)P.nkv * D * ESZ;        // bytes between layout rows
    const int n_real = (g_last >> 4) + 1;                   // key tiles of real tokens; one more tile: the tile's own [MASK] rows
    float m_run = -INFINITY, l_run = 0.f;                   // of query c (the same in the four lanes that share it)
    float o[BF ? 1 : 16][DPL];                               // float32 values: this lane's columns of all 16 rows
    f32x4 oacc[D / 16];                                     // bf16 values: MFMA tiles, lane (c, kb): column 16 j + c of rows 4 kb .. 4 kb + 3
#pragma unroll
    for (int rr = 0; rr < (BF ? 1 : 16); ++rr)
#pragma unroll
        for (int e = 0; e < DPL; ++e) o[rr][e] = 0.f;
#pragma unroll
    for (int j = 0; j < D / 16; ++j) oacc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // layout row of key j of key tile t (clamped to a row that exists); tile n_real holds the [MASK] rows of the
    // query tile's own groups
    auto key_row = [&](int t, int j) __attribute__((always_inline)) {
        return t >= n_real ? r0 + min(j, nrows - 1) : min(16 * t + j, g_last) * K1;
    };
    constexpr int CBN = D / 16;                             // column blocks of 16
    const int vm = lane / CBN, vcb = lane % CBN;            // bf16 values: this lane's key pair and column block (lanes < 8 CBN)
    // The loads of a key tile: K rows as the MFMA operand (lane (c, kb): bytes [64 t + 16 kb, +16) of key c), and
    // the value rows.  They are requested one tile ahead, while the previous tile is worked on.
    auto load_tile = [&](int t, uint4 (&kreg)[STEPS], uint4 (&va)[2], uint4 (&vb)[2], raw_t (&vraw)[BF ? 1 : 16]) __attribute__((always_inline)) {
        const char* krow = kbase + (size_t)key_row(t, c) * rstride + kb * 16;
#pragma unroll
        for (int st = 0; st < STEPS; ++st) kreg[st] = ld16(krow + st * 64);
        if constexpr (BF) {
            const int mm = min(vm, 7);
            const char* pa_ = vbase + (size_t)key_row(t, 2 * mm) * rstride + vcb * 32;
            const char* pb_ = vbase + (size_t)key_row(t, 2 * mm + 1) * rstride + vcb * 32;
            va[0] = ld16(pa_); va[1] = ld16(pa_ + 16);
            vb[0] = ld16(pb_); vb[1] = ld16(pb_ + 16);
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j)
                vraw[j] = *reinterpret_cast<const raw_t*>(vbase + (size_t)key_row(t, j) * rstride + (size_t)DPL * lane * ESZ);
        }
    };
    const int n_tiles = n_real + (P.k > 0 ? 1 : 0);         // real-token tiles, then the own-[MASK] tile
    if constexpr (BF) {
        // bf16 values: a wavefront works on two key tiles at a time (tiles kt and kt + 4 of the query tile's list),
        // with the K and V rows of the next two requested meanwhile (two sets of registers take turns, every request
        // unconditional: beyond the last tile it repeats it and nobody uses it).  Scores in units of ln 2 (the
        // exponentials are single v_exp_f32); the maxima and sums of the four lanes that share a query row are
        // exchanged with row swaps; the 32 keys of the two tiles feed one v_mfma_f32_16x16x32_bf16 per part (P high,
        // P low) and 16 output columns; the running output is rescaled only when a maximum moved.
        constexpr float LOG2E = 1.4426950408889634f;
        const float scale2 = P.inv_sqrt_d * LOG2E;
        struct KvT { uint4 k[STEPS]; uint4 va[2], vb[2]; };
        const int vmm = min(vm, 7);
        // (requests beyond the last tile repeat it: nobody uses them)
        auto load_k = [&](int t, KvT& r) __attribute__((always_inline)) {
            const char* krow = kbase + (size_t)key_row(min(t, n_tiles - 1), c) * rstride + kb * 16;
#pragma unroll
            for (int st = 0; st < STEPS; ++st) r.k[st] = ld16(krow + st * 64);
        };
        auto load_v = [&](int t, KvT& r) __attribute__((always_inline)) {
            const int tc = min(t, n_tiles - 1);
            const char* pa_ = vbase + (size_t)key_row(tc, 2 * vmm) * rstride + vcb * 32;
            const char* pb_ = vbase + (size_t)key_row(tc, 2 * vmm + 1) * rstride + vcb * 32;
            r.va[0] = ld16(pa_); r.va[1] = ld16(pa_ + 16);
            r.vb[0] = ld16(pb_); r.vb[1] = ld16(pb_ + 16);
        };
        // is key j of tile t visible to this lane's query?
        auto visible = [&](int t, int j) __attribute__((always_inline)) {
            if (t < n_real) return 16 * t + j <= qg;                          // the real token of a group up to the query's own
            if (t >= n_tiles) return false;
            const int kg = g0 + j / K1, ks = j % K1;                          // a [MASK] token of the query's own group, not after it
            return j < nrows && ks > 0 && kg == qg && ks <= qs;
        };
        // the pair of tiles (t0, t0 + 4); its registers are refilled with the pair (t0 + 8, t0 + 12) as soon as they are
        // consumed: the K rows after the score MFMAs, the V rows once they are staged in LDS
        auto process2 = [&](KvT (&r)[2], int t0) __attribute__((always_inline)) {
            f32x4 acc[2][1];
#pragma unroll
            for (int g = 0; g < 2; ++g) acc[g][0] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < STEPS; ++t) {
                BRegs<WT, 1> bqt;                            // the query rows (read per step: registers are scarce)
                bqt.h[0] = ld16(sQ + (2 * t * 64 + lane) * 16);
                bqt.l[0] = ld16(sQ + ((2 * t + 1) * 64 + lane) * 16);
#pragma unroll
                for (int g = 0; g < 2; ++g) mma_step<WT, 1>(r[g].k[t], bqt, acc[g]);
            }
            load_k(t0 + 2 * GA_WAVES, r[0]); load_k(t0 + 3 * GA_WAVES, r[1]);
            float sc[2][4], mt = -INFINITY;
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    sc[g][e] = (qlive && visible(t0 + GA_WAVES * g, 4 * kb + e)) ? acc[g][0][e] * scale2 : -INFINITY;
                    mt = fmaxf(mt, sc[g][e]);
                }
            mt = quad_rows_max(mt);
            const float m_new = fmaxf(m_run, mt);
            const float alpha = m_new > -INFINITY ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.f;
            const float m_use = m_new > -INFINITY ? m_new : 0.f;
            f32x4 pr[2];
            float ls = 0.f;
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    pr[g][e] = __builtin_amdgcn_exp2f(sc[g][e] - m_use);
                    ls += pr[g][e];
                }
            ls = quad_rows_sum(ls);
            l_run = l_run * alpha + ls;
            m_run = m_new;
            if (kb == 0) sA[c] = alpha;
            if (vm < 8) {                                   // the value rows into LDS, the two keys of a pair interleaved
#pragma unroll
                for (int g = 0; g < 2; ++g) {
                    unsigned ov[16];
#pragma unroll
                    for (int w = 0; w < 8; ++w) {
                        const unsigned a2 = w < 4 ? (&r[g].va[0].x)[w] : (&r[g].va[1].x)[w - 4], b2 = w < 4 ? (&r[g].vb[0].x)[w] : (&r[g].vb[1].x)[w - 4];
                        ov[2 * w] = __builtin_amdgcn_perm(b2, a2, 0x05040100u);
                        ov[2 * w + 1] = __builtin_amdgcn_perm(b2, a2, 0x07060302u);
                    }
                    uint4* dst = reinterpret_cast<uint4*>(sV + (g * 8 + vm) * VSTR + 16 * vcb);
#pragma unroll
                    for (int w = 0; w < 4; ++w) dst[w] = make_uint4(ov[4 * w], ov[4 * w + 1], ov[4 * w + 2], ov[4 * w + 3]);
                }
            }
            load_v(t0 + 2 * GA_WAVES, r[0]); load_v(t0 + 3 * GA_WAVES, r[1]);
            lds_sync_wave();
            __builtin_amdgcn_wave_barrier();
            const f32x4 al = *reinterpret_cast<const f32x4*>(sA + 4 * kb);
            if (__any(alpha != 1.f)) {
#pragma unroll
                for (int j = 0; j < D / 16; ++j) oacc[j] *= al;
            }
            unsigned ph2[2][2], pl2[2][2];
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                ph2[g][0] = pack_bf16x2(pr[g][0], pr[g][1]); ph2[g][1] = pack_bf16x2(pr[g][2], pr[g][3]);
                pl2[g][0] = pack_bf16x2(pr[g][0] - __uint_as_float(ph2[g][0] << 16), pr[g][1] - __uint_as_float(ph2[g][0] & 0xFFFF0000u));
                pl2[g][1] = pack_bf16x2(pr[g][2] - __uint_as_float(ph2[g][1] << 16), pr[g][3] - __uint_as_float(ph2[g][1] & 0xFFFF0000u));
            }
            const bf16x8 pa = __builtin_bit_cast(bf16x8, make_uint4(ph2[0][0], ph2[0][1], ph2[1][0], ph2[1][1]));
            const bf16x8 pb = __builtin_bit_cast(bf16x8, make_uint4(pl2[0][0], pl2[0][1], pl2[1][0], pl2[1][1]));
#pragma unroll
            for (int j = 0; j < D / 16; ++j) {
                const bf16x8 vv = __builtin_bit_cast(bf16x8, make_uint4(sV[(2 * kb) * VSTR + 16 * j + c], sV[(2 * kb + 1) * VSTR + 16 * j + c],
                                                                        sV[(8 + 2 * kb) * VSTR + 16 * j + c], sV[(8 + 2 * kb + 1) * VSTR + 16 * j + c]));
                const f32x4 t = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, vv, oacc[j], 0, 0, 0);
                oacc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pb, vv, t, 0, 0, 0);
            }
            lds_sync_wave();
            __builtin_amdgcn_wave_barrier();
        };
        KvT ra[2];
        load_k(wave, ra[0]); load_k(wave + GA_WAVES, ra[1]);
        load_v(wave, ra[0]); load_v(wave + GA_WAVES, ra[1]);
        for (int kt = wave; kt < n_tiles; kt += 2 * GA_WAVES) process2(ra, kt);
    } else {
    uint4 kreg[STEPS], va[2], vb[2], kreg_n[STEPS], va_n[2], vb_n[2];
    raw_t vraw[BF ? 1 : 16], vraw_n[BF ? 1 : 16];
    load_tile(min(wave, n_tiles - 1), kreg, va, vb, vraw);
    for (int kt = wave; kt < n_tiles; kt += GA_WAVES) {
        const bool own = kt == n_real;                      // the [MASK] tokens of the tile's own groups
        load_tile(min(kt + GA_WAVES, n_tiles - 1), kreg_n, va_n, vb_n, vraw_n);   // (beyond the last: a repeat nobody uses)
        f32x4 acc[1] = {f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int t = 0; t < STEPS; ++t) mma_step<WT, 1>(kreg[t], bq[t], acc);
        // scores of keys 4 kb .. 4 kb + 3 for query c, masked
        float sc[4], mt = -INFINITY;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int j = 4 * kb + r;
            bool vis;
            if (own) {
                const int kg = g0 + j / K1, ks = j % K1;
                vis = j < nrows && ks > 0 && kg == qg && ks <= qs;       // a [MASK] token of the query's own group, not after it
            } else {
                vis = 16 * kt + j <= qg;                                  // the real token of a group up to the query's own
            }
            sc[r] = (vis && qlive) ? acc[0][r] * P.inv_sqrt_d : -INFINITY;
            mt = fmaxf(mt, sc[r]);
        }
        mt = fmaxf(mt, __shfl_xor(mt, 16, 64));
        mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
        const float m_new = fmaxf(m_run, mt);
        const float alpha = m_new > -INFINITY ? expf(m_run - m_new) : 1.f;   // exp(-inf) = 0 when nothing was seen before
        f32x4 pr;
        float ls = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            pr[r] = sc[r] > -INFINITY ? expf(sc[r] - m_new) : 0.f;
            ls += pr[r];
        }
        ls += __shfl_xor(ls, 16, 64);
        ls += __shfl_xor(ls, 32, 64);
        l_run = l_run * alpha + ls;
        m_run = m_new;
        *reinterpret_cast<f32x4*>(sP + c * 16 + 4 * kb) = pr;
        if (kb == 0) sA[c] = alpha;
        lds_sync_wave();                                    // written and read by this wavefront only
        __builtin_amdgcn_wave_barrier();
        if constexpr (BF) {
            // the value rows into LDS, the two keys of a pair interleaved column by column
            if (vm < 8) {
                unsigned ov[16];
#pragma unroll
                for (int w = 0; w < 8; ++w) {
                    const unsigned a2 = w < 4 ? (&va[0].x)[w] : (&va[1].x)[w - 4], b2 = w < 4 ? (&vb[0].x)[w] : (&vb[1].x)[w - 4];
                    ov[2 * w] = (a2 & 0xFFFFu) | (b2 << 16);
                    ov[2 * w + 1] = (a2 >> 16) | (b2 & 0xFFFF0000u);
                }
                uint4* dst = reinterpret_cast<uint4*>(sV + vm * VSTR + 16 * vcb);
#pragma unroll
                for (int w = 0; w < 4; ++w) dst[w] = make_uint4(ov[4 * w], ov[4 * w + 1], ov[4 * w + 2], ov[4 * w + 3]);
            }
            lds_sync_wave();
            __builtin_amdgcn_wave_barrier();
            // P (query c, keys 4 kb .. 4 kb + 3) as the 16-row operand, split into bf16 high and low parts
            const unsigned h01 = pack_bf16x2(pr[0], pr[1]), h23 = pack_bf16x2(pr[2], pr[3]);
            const unsigned l01 = pack_bf16x2(pr[0] - __uint_as_float(h01 << 16), pr[1] - __uint_as_float(h01 & 0xFFFF0000u));
            const unsigned l23 = pack_bf16x2(pr[2] - __uint_as_float(h23 << 16), pr[3] - __uint_as_float(h23 & 0xFFFF0000u));
            const s16x4 ph_ = __builtin_bit_cast(s16x4, make_uint2(h01, h23)), pl_ = __builtin_bit_cast(s16x4, make_uint2(l01, l23));
            const f32x4 al = *reinterpret_cast<const f32x4*>(sA + 4 * kb);   // rescale factors of rows 4 kb .. 4 kb + 3
#pragma unroll
            for (int j = 0; j < D / 16; ++j) {
                // values of keys 4 kb .. 4 kb + 3, column 16 j + c: the key pairs 2 kb and 2 kb + 1
                const unsigned w0 = sV[(2 * kb) * VSTR + 16 * j + c], w1 = sV[(2 * kb + 1) * VSTR + 16 * j + c];
                const s16x4 vv = __builtin_bit_cast(s16x4, make_uint2(w0, w1));
                f32x4 t = oacc[j] * al;
                t = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ph_, vv, t, 0, 0, 0);
                oacc[j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pl_, vv, t, 0, 0, 0);
            }
        } else {
            float v[16][DPL];
    #pragma unroll
            for (int j = 0; j < 16; ++j) widen_v(vraw[j], v[j]);
    #pragma unroll
            for (int rr = 0; rr < 16; ++rr) {
                if (rr < nrows) {                               // wavefront-uniform
                    const float a = sA[rr];
                    const f32x4* prow = reinterpret_cast<const f32x4*>(sP + rr * 16);
    #pragma unroll
                    for (int e = 0; e < DPL; ++e) o[rr][e] *= a;
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
        lds_sync_wave();
        __builtin_amdgcn_wave_barrier();                    // the next tile overwrites the probabilities
#pragma unroll
        for (int st = 0; st < STEPS; ++st) kreg[st] = kreg_n[st];
        va[0] = va_n[0]; va[1] = va_n[1]; vb[0] = vb_n[0]; vb[1] = vb_n[1];
#pragma unroll
        for (int j = 0; j < (BF ? 1 : 16); ++j) vraw[j] = vraw_n[j];
    }
    }
    // ---- the wavefronts' results meet in LDS
    if (kb == 0) { sML[(wave * 16 + c) * 2] = m_run; sML[(wave * 16 + c) * 2 + 1] = l_run; }
    if constexpr (BF) {
#pragma unroll
        for (int j = 0; j < D / 16; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) sO[wave * OSTRIDE + (4 * kb + r) * D + 16 * j + c] = oacc[j][r];
    } else {
#pragma unroll
        for (int rr = 0; rr < 16; ++rr)
#pragma unroll
            for (int e = 0; e < DPL; ++e) sO[wave * OSTRIDE + rr * D + DPL * lane + e] = o[rr][e];
    }
    __syncthreads();
    float* obase = P.out + ((size_t)seq * P.rows * P.nq + h) * D;
    for (int x = tid; x < nrows * D; x += GA_THREADS) {
        const int rr = x / D, dd = x - rr * D;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < GA_WAVES; ++w) M = fmaxf(M, sML[(w * 16 + rr) * 2]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < GA_WAVES; ++w) {
            const float mw = sML[(w * 16 + rr) * 2];
            const float f = mw > -INFINITY ? (BF ? __builtin_amdgcn_exp2f(mw - M) : expf(mw - M)) : 0.f;
            num += sO[w * OSTRIDE + rr * D + dd] * f;
            den += sML[(w * 16 + rr) * 2 + 1] * f;
        }
        obase[(size_t)(r0 + rr) * P.nq * D + dd] = num / den;   // (every row sees at least its own real token: den > 0)
    }
}

size_t a256(size_t v) { return (v + 255) & ~(size_t)255; }

int check(const ps_group_attn_args* a) {
    if (!a) return PS_ERR_NULL;
    if (a->seqs < 1 || a->tokens < 1 || a->k < 0 || a->n_heads < 1 || a->n_kv_heads < 1 || a->head_dim < 1) return PS_ERR_SHAPE;
    if (a->dtype != PS_F32 && a->dtype != PS_BF16) return PS_ERR_SHAPE;
    if (a->n_heads % a->n_kv_heads != 0 || !(a->rope_base > 0.f)) return PS_ERR_SHAPE;
    if (a->head_dim != 64 && a->head_dim != 128) return PS_ERR_UNSUPPORTED;
    if (a->k > 15 || (long long)a->tokens + a->k > (1 << 20)) return PS_ERR_UNSUPPORTED;
    if (a->n_heads > 65535 || a->seqs > 65535) return PS_ERR_UNSUPPORTED;
    return PS_OK;
}

struct GaLayout { size_t table, q_rot, k_rot, total; };
GaLayout layout(const ps_group_attn_args* a) {
    GaLayout L;
    const size_t rows = (size_t)a->tokens * (a->k + 1), esz = a->dtype == PS_BF16 ? 2 : 4;
    L.table = 0;
    L.q_rot = a256((size_t)(a->tokens + a->k) * (a->head_dim / 2) * sizeof(float2));
    L.k_rot = L.q_rot + a256((size_t)a->seqs * rows * a->n_heads * a->head_dim * 4);
    L.total = L.k_rot + a256((size_t)a->seqs * rows * a->n_kv_heads * a->head_dim * esz);
    return L;
}

template <typename WT, int D>
int launch(const GaParams& P, hipStream_t s) {
    const long long nrope = (long long)P.seqs * P.rows * (P.nq + P.nkv) * (D / 8);
    hipLaunchKernelGGL((ga_table_kernel<D>), dim3(min(1024, ((P.T + P.k) * (D / 2) + 255) / 256)), dim3(256), 0, s, P);
    hipLaunchKernelGGL((ga_rope_kernel<WT, D>), dim3((unsigned)min(65535LL, (nrope + 255) / 256)), dim3(256), 0, s, P);
    hipLaunchKernelGGL((ga_attn_kernel<WT, D>), dim3(P.ntiles, P.nq, P.seqs), dim3(GA_THREADS), 0, s, P);
    return hipGetLastError() == hipSuccess ? PS_OK : PS_ERR_DEVICE;
}

}   // namespace

extern "C" size_t ps_group_attention_workspace_bytes(const ps_group_attn_args* a) {
    return check(a) == PS_OK ? layout(a).total : 0;
}

extern "C" int ps_group_attention(const ps_group_attn_args* a, void* stream) {
    const int st = check(a);
    if (st != PS_OK) return st;
    if (!a->q || !a->k_ || !a->v || !a->out || !a->workspace) return PS_ERR_NULL;
    const GaLayout L = layout(a);
    if (a->workspace_bytes < L.total || ((uintptr_t)a->workspace & 255)) return PS_ERR_WORKSPACE;
    GaParams P;
    P.seqs = a->seqs; P.T = a->tokens; P.k = a->k; P.nq = a->n_heads; P.nkv = a->n_kv_heads;
    P.rows = a->tokens * (a->k + 1);
    P.gpt = 16 / (a->k + 1);
    P.ntiles = (a->tokens + P.gpt - 1) / P.gpt;
    P.inv_sqrt_d = (float)(1.0 / sqrt((double)a->head_dim));
    P.q = a->q; P.k_ = a->k_; P.v = a->v; P.out = a->out;
    char* ws = (char*)a->workspace;
    P.table = (float2*)(ws + L.table); P.q_rot = (float*)(ws + L.q_rot); P.k_rot = ws + L.k_rot;
    P.log_base = log((double)a->rope_base);
    hipStream_t s = (hipStream_t)stream;
    if (a->dtype == PS_BF16) return a->head_dim == 128 ? launch<bf16_t, 128>(P, s) : launch<bf16_t, 64>(P, s);
    return a->head_dim == 128 ? launch<float, 128>(P, s) : launch<float, 64>(P, s);
}
