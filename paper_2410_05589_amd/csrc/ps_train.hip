// Attention of group-wise parallel training (see include/ps_train.h; Section 4.1).
//
// Three kernels per call: the rotary table (cos, sin of position * base^(-2j/d) in double precision), the
// rotation of k (to the storage type, rounded as the inference path caches keys), and the attention itself,
// which rotates its 16 query rows (in float32) while it stages them.
//
// The attention kernel never touches a key the mask hides.  A query tile is a whole number of parallel groups
// (as many as fit into 16 rows); what its rows may see are (a) real tokens of groups up to their own - these
// are gathered with a stride of k + 1 rows, 16 per key tile - and (b) [MASK] tokens of their own group, which
// all lie inside the query tile's own 16 rows: one more key tile.  The wavefronts of a workgroup take the key
// tiles in turn, each with its own running maximum, sum and output (online softmax); their results meet in LDS
// at the end.  Scores are one MFMA tile per key tile (the keys' rows are the 16-row operand; the 16 query rows, split
// into bf16 high and low parts, the 16-column operand in LDS).  P.V for bf16 values is MFMA work too: the score tile
// comes out of the matrix core with a lane holding four consecutive keys of one query, which is exactly the 16-row
// operand layout (P, split into high and low parts); the other operand needs consecutive keys of one value column
// per lane, so the value rows pass through LDS, transposed in units of key pairs.  A wavefront works on two key tiles
// at a time (one softmax update per 32 keys, one v_mfma_f32_16x16x32_bf16 per part and 16 output columns) and refills
// the tiles' registers as soon as they are consumed.  The K and V rows are loaded 64 adjacent bytes per four lanes and
// change to the operand order in LDS (see the bf16 branch of the kernel).
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

// rotary embedding of the keys: one thread per (row, kv head, pair of 4 + 4 elements j..j+3, j+d/2..)
template <typename WT, int D>
__global__ void __launch_bounds__(256) ga_rope_kernel(const GaParams P) {
    constexpr int ESZ = Traits<WT>::ESZ, Q4 = D / 8;     // groups of 4 pairs per head
    const long long n = (long long)P.seqs * P.rows * P.nkv * Q4;
    for (long long x = (long long)blockIdx.x * 256 + threadIdx.x; x < n; x += (long long)gridDim.x * 256) {
        const int g4 = (int)(x % Q4);
        const long long y = x / Q4;                        // (seq * rows + row) * nkv + head
        const int row = (int)((y / P.nkv) % P.rows);
        const int pos = row / (P.k + 1) + row % (P.k + 1);  // group + slot
        const size_t base = (size_t)y * D;
        const char* src = (const char*)P.k_;
        const f32x4 a = load4<WT>(src + (base + 4 * g4) * ESZ), b = load4<WT>(src + (base + D / 2 + 4 * g4) * ESZ);
        f32x4 ra, rb;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float2 t = P.table[(size_t)pos * (D / 2) + 4 * g4 + e];
            ra[e] = a[e] * t.x - b[e] * t.y;
            rb[e] = b[e] * t.x + a[e] * t.y;
        }
        store4<WT>((char*)P.k_rot + (base + 4 * g4) * ESZ, ra);
        store4<WT>((char*)P.k_rot + (base + D / 2 + 4 * g4) * ESZ, rb);
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
    // bf16 values, per wavefront, [4 blocks of 4 keys][RSTR] dwords: a column of a block holds four dwords, the values of
    // keys (4 kb, 4 kb + 1) and (4 kb + 2, 4 kb + 3) of the first key tile, then those of the second; every 8 columns
    // 4 dwords are left out and every block 4 more, which keeps writers and readers off each other's LDS banks.  The
    // same area first takes the K rows of the two tiles on their way from the order they are loaded in to the order
    // the matrix core wants (16 keys x 2 D bytes per tile), and in the end the wavefront's output [16][D].
    // float32: [waves][16][D] outputs
    constexpr int RSTR = (D / 8) * 36 + 4;
    constexpr int OSTRIDE = BF ? 4 * RSTR : 16 * D;         // floats between the wavefronts' areas
    static_assert(!BF || (OSTRIDE >= 16 * D && OSTRIDE * 4 >= 2 * 16 * D * 2), "a wavefront's outputs and its staged K rows fit its area");
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
    unsigned* sV = reinterpret_cast<unsigned*>(smem + OFF_V) + wave * OSTRIDE;
    typedef short s16x4 __attribute__((ext_vector_type(4)));

    // ---- the query rows, rotated in float32 (bf16 values: and scaled by log2(e) / sqrt(d), so the scores come out in
    // units of ln 2), into LDS as the 16-column MFMA operand; rows beyond the tile repeat the last
    const char* qsrc = (const char*)P.q + ((size_t)seq * P.rows * P.nq + h) * D * ESZ;
    const float qscale = BF ? P.inv_sqrt_d * 1.4426950408889634f : 1.f;
    for (int t2 = tid; t2 < 16 * (D / 8); t2 += GA_THREADS) {
        const int r = min(t2 / (D / 8), nrows - 1), g4 = t2 % (D / 8);
        const int row = r0 + r, pos = row / K1 + row % K1;                      // group + slot
        const char* qrow = qsrc + (size_t)row * P.nq * D * ESZ;
        const f32x4 a = load4<WT>(qrow + 4 * g4 * ESZ), b = load4<WT>(qrow + (D / 2 + 4 * g4) * ESZ);
        u32x4 ra, rb;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float2 t = P.table[(size_t)pos * (D / 2) + 4 * g4 + e];
            ra[e] = __float_as_uint((a[e] * t.x - b[e] * t.y) * qscale);
            rb[e] = __float_as_uint((b[e] * t.x + a[e] * t.y) * qscale);
        }
        const int ts = (t2 / (D / 8)) * (D / 4) + g4;                           // (row, group of 4 elements) as attn_store_q counts
        attn_store_q<WT, D>(sQ, ts, ra);
        attn_store_q<WT, D>(sQ, ts + D / 8, rb);
    }
    __syncthreads();
    BRegs<WT, 1> bq[STEPS];                                 // float32: the query rows stay in registers (bf16: read per step)
    if constexpr (!BF) {
#pragma unroll
        for (int t = 0; t < STEPS; ++t) bq[t].h[0] = ld16(sQ + (t * 64 + lane) * 16);
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
    const int n_tiles = n_real + (P.k > 0 ? 1 : 0);         // real-token tiles, then the own-[MASK] tile
    if constexpr (BF) {
        // bf16 values: a wavefront works on two key tiles at a time (tiles kt and kt + 4 of the query tile's list) and
        // refills the tiles' registers as soon as they are consumed (every request unconditional: beyond the last tile
        // it repeats it and nobody uses it).
        //
        // Loads: four adjacent lanes read 64 adjacent bytes (the texture unit handles a load in units of four lanes; a
        // lane that fetched its own MFMA operand directly would make every lane of such a unit touch another row).
        // K: lane (key = lane / 4, j = lane % 4) reads bytes [64 t + 16 j, +16) of its key in request t; the rows pass
        // through LDS, where lane (c, kb) picks up bytes [64 t + 16 kb, +16) of key c, its operand of MFMA step t (the
        // 16-byte pieces of a row are placed at (t ^ key % 4, j ^ key / 4 % 4), which keeps writers and readers off
        // each other's banks).  V: lane (kbw = lane / (D/8), cc = lane % (D/8)) reads 16 bytes (columns 8 cc .. 8 cc + 7)
        // of keys 4 kbw .. 4 kbw + 3 of both tiles and stores, per column, the dwords (key 4 kbw, 4 kbw + 1) and
        // (4 kbw + 2, 4 kbw + 3) of the first tile and of the second side by side: lane (c, kb) then reads, per 16 output
        // columns, one 16-byte piece = its 8 keys of the 32-key contraction (index 8 kb + e = key 4 kb + e of the first
        // tile, 4 kb + e - 4 of the second).
        //
        // Scores in units of ln 2 (the exponentials are single v_exp_f32); the maxima and sums of the four lanes that
        // share a query row are exchanged with row swaps; the running output is rescaled only when a maximum moved.
        constexpr int NCH = D / 8;                          // 16-byte pieces of a K or V row
        constexpr int KT = 16 * D * 2;                      // bytes of a staged K tile
        struct KvT { uint4 k[STEPS]; uint4 v[4]; };
        const unsigned rs32 = (unsigned)rstride;
        // K: the lane's key and piece as a loader, and its offsets into the staged tile as a writer (request 0) and as a
        // reader (step 0); request / step t flips bits 6.. of the offset
        const int kkey = lane >> 2, kj = lane & 3;
        constexpr int TM = STEPS - 1, TL = STEPS == 4 ? 2 : 1;   // the row's 64-byte segments: mask and log2
        auto k_lds = [&](int key, int j) __attribute__((always_inline)) {
            return key * (2 * D) + (((key & TM)) << 6) + ((j ^ ((key >> TL) & 3)) << 4);
        };
        char* const sK = reinterpret_cast<char*>(sV);
        const int kw_rel = k_lds(kkey, kj), kr_rel = k_lds(c, kb);
        // Addresses: a wavefront-uniform base (the tile's first row) plus a 32-bit offset per lane.  For a tile of real
        // tokens that lies inside the sequence the offset is the same every time; the last such tile (rows clamped to the
        // last group) and the tile of the own [MASK] rows compute theirs.
        const unsigned K1rs = (unsigned)K1 * rs32;                      // bytes between real tokens
        const size_t tileb = (size_t)16 * K1rs;                         // ... between key tiles of real tokens
        const char* const kown = kbase + (size_t)r0 * rs32;
        const char* const vown = vbase + (size_t)r0 * rs32;
        const unsigned koff_real = (unsigned)kkey * K1rs + kj * 16, koff_own = (unsigned)min(kkey, nrows - 1) * rs32 + kj * 16;
        // V: the lane's block of four keys and its piece of their rows (lanes beyond 4 NCH repeat the last block and store nothing)
        const int kbw = min(lane / NCH, 3), cc = lane % NCH;
        const bool vlane = lane < 4 * NCH;
        const unsigned voff_real = (unsigned)(4 * kbw) * K1rs + cc * 16;
        unsigned* const sVw = sV + kbw * RSTR + cc * 36;
        const unsigned* const sVr = sV + kb * RSTR + (c >> 3) * 36 + (c & 7) * 4;
        // (requests beyond the last tile repeat it: nobody uses them)
        auto load_k = [&](int t, KvT& r) __attribute__((always_inline)) {
            const int tc = min(t, n_tiles - 1);
            const char* sb = kown;
            unsigned off = koff_own;
            if (tc < n_real) {
                sb = kbase + (size_t)tc * tileb;
                off = 16 * tc + 15 <= g_last ? koff_real : (unsigned)min(kkey, g_last - 16 * tc) * K1rs + kj * 16;
            }
#pragma unroll
            for (int st = 0; st < STEPS; ++st) r.k[st] = ld16(sb + off + st * 64);
        };
        auto load_v = [&](int t, KvT& r) __attribute__((always_inline)) {
            const int tc = min(t, n_tiles - 1);
            if (tc < n_real && 16 * tc + 15 <= g_last) {
                const char* sb = vbase + (size_t)tc * tileb;
#pragma unroll
                for (int i = 0; i < 4; ++i) r.v[i] = ld16(sb + (size_t)i * K1rs + voff_real);
            } else {
                const bool real = tc < n_real;
                const char* sb = real ? vbase + (size_t)tc * tileb : vown;
                const unsigned step = real ? K1rs : rs32;
                const int last = real ? g_last - 16 * tc : nrows - 1;
#pragma unroll
                for (int i = 0; i < 4; ++i) r.v[i] = ld16(sb + (unsigned)min(4 * kbw + i, last) * step + cc * 16);
            }
        };
        // which keys 4 kb + e of a tile this lane's query sees: e in [lo, hi].  Real tokens: those of groups up to the
        // query's own; the tile's own [MASK] rows: those of the query's group, up to its slot
        const int real_hi0 = qlive ? qg - 4 * kb : -(1 << 20);
        const int own_lo = qr - qs + 1 - 4 * kb, own_hi = qlive ? qr - 4 * kb : -(1 << 20);
        // the pair of tiles (t0, t0 + 4); its registers are refilled with the pair (t0 + 8, t0 + 12) as soon as they are
        // consumed: the K rows once they are in LDS, the V rows once they are staged
        auto process2 = [&](KvT (&r)[2], int t0) __attribute__((always_inline)) {
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int t = 0; t < STEPS; ++t)
                    *reinterpret_cast<uint4*>(sK + g * KT + (kw_rel ^ (t << 6))) = r[g].k[t];
            load_k(t0 + 2 * GA_WAVES, r[0]); load_k(t0 + 3 * GA_WAVES, r[1]);
            lds_sync_wave();
            __builtin_amdgcn_wave_barrier();
            f32x4 acc[2][1];
#pragma unroll
            for (int g = 0; g < 2; ++g) acc[g][0] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < STEPS; ++t) {
                BRegs<WT, 1> bqt;                            // the query rows (read per step: registers are scarce)
                bqt.h[0] = ld16(sQ + (2 * t * 64 + lane) * 16);
                bqt.l[0] = ld16(sQ + ((2 * t + 1) * 64 + lane) * 16);
#pragma unroll
                for (int g = 0; g < 2; ++g)
                    mma_step<WT, 1>(ld16(sK + g * KT + (kr_rel ^ (t << 6))), bqt, acc[g]);
            }
            float sc[2][4], mt = -INFINITY;
            const int t1 = t0 + GA_WAVES;
            if (t1 < n_real && 16 * t1 + 15 <= g0) {        // every key of both tiles is visible to every query of the tile
#pragma unroll
                for (int g = 0; g < 2; ++g)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        sc[g][e] = acc[g][0][e];
                        mt = fmaxf(mt, sc[g][e]);
                    }
            } else {
#pragma unroll
                for (int g = 0; g < 2; ++g) {
                    const int t = t0 + GA_WAVES * g;
                    const int lo = t < n_real ? 0 : own_lo;
                    const int hi = t < n_real ? real_hi0 - 16 * t : (t < n_tiles ? own_hi : -(1 << 20));
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        sc[g][e] = (e >= lo && e <= hi) ? acc[g][0][e] : -INFINITY;
                        mt = fmaxf(mt, sc[g][e]);
                    }
                }
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
            if (vlane) {                                    // the value rows into LDS (after the last read of the K rows there)
#pragma unroll
                for (int w = 0; w < 4; ++w) {               // dword w of the lane's 16 bytes: columns 2 w and 2 w + 1
                    unsigned lo[4], hi[4];
#pragma unroll
                    for (int g = 0; g < 2; ++g) {
                        const unsigned k0 = (&r[g].v[0].x)[w], k1 = (&r[g].v[1].x)[w], k2 = (&r[g].v[2].x)[w], k3 = (&r[g].v[3].x)[w];
                        lo[2 * g] = __builtin_amdgcn_perm(k1, k0, 0x05040100u); lo[2 * g + 1] = __builtin_amdgcn_perm(k3, k2, 0x05040100u);
                        hi[2 * g] = __builtin_amdgcn_perm(k1, k0, 0x07060302u); hi[2 * g + 1] = __builtin_amdgcn_perm(k3, k2, 0x07060302u);
                    }
                    *reinterpret_cast<uint4*>(sVw + 8 * w) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
                    *reinterpret_cast<uint4*>(sVw + 8 * w + 4) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
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
            // four blocks of 16 output columns at a time: the MFMAs with P's high parts, then those with its low parts
            // (an MFMA that follows the one it depends on directly would wait for it)
#pragma unroll
            for (int j0 = 0; j0 < D / 16; j0 += 4) {
                bf16x8 vv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) vv[u] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(sVr + 72 * (j0 + u)));
#pragma unroll
                for (int u = 0; u < 4; ++u) oacc[j0 + u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, vv[u], oacc[j0 + u], 0, 0, 0);
#pragma unroll
                for (int u = 0; u < 4; ++u) oacc[j0 + u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pb, vv[u], oacc[j0 + u], 0, 0, 0);
            }
            lds_sync_wave();
            __builtin_amdgcn_wave_barrier();
        };
        KvT ra[2];
        load_k(wave, ra[0]); load_k(wave + GA_WAVES, ra[1]);
        load_v(wave, ra[0]); load_v(wave + GA_WAVES, ra[1]);
        for (int kt = wave; kt < n_tiles; kt += 2 * GA_WAVES) process2(ra, kt);
    } else {
        // float32 values: a key tile at a time; the K rows (lane (c, kb): bytes [64 t + 16 kb, +16) of key c, its MFMA
        // operand) and the value rows (a lane owns D / 64 columns of all 16 keys) are requested one tile ahead
        auto load_tile = [&](int t, uint4 (&kreg)[STEPS], raw_t (&vraw)[16]) __attribute__((always_inline)) {
            const char* krow = kbase + (size_t)key_row(t, c) * rstride + kb * 16;
#pragma unroll
            for (int st = 0; st < STEPS; ++st) kreg[st] = ld16(krow + st * 64);
#pragma unroll
            for (int j = 0; j < 16; ++j)
                vraw[j] = *reinterpret_cast<const raw_t*>(vbase + (size_t)key_row(t, j) * rstride + (size_t)DPL * lane * ESZ);
        };
        uint4 kreg[STEPS], kreg_n[STEPS];
        raw_t vraw[16], vraw_n[16];
        load_tile(min(wave, n_tiles - 1), kreg, vraw);
        for (int kt = wave; kt < n_tiles; kt += GA_WAVES) {
            const bool own = kt == n_real;                      // the [MASK] tokens of the tile's own groups
            load_tile(min(kt + GA_WAVES, n_tiles - 1), kreg_n, vraw_n);   // (beyond the last: a repeat nobody uses)
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
            lds_sync_wave();
            __builtin_amdgcn_wave_barrier();                    // the next tile overwrites the probabilities
#pragma unroll
            for (int st = 0; st < STEPS; ++st) kreg[st] = kreg_n[st];
#pragma unroll
            for (int j = 0; j < 16; ++j) vraw[j] = vraw_n[j];
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
    if ((long long)(a->k + 1) * a->n_kv_heads * a->head_dim * 4 > (1LL << 27)) return PS_ERR_UNSUPPORTED;   // 32-bit offsets inside a key tile
    return PS_OK;
}

struct GaLayout { size_t table, k_rot, total; };
GaLayout layout(const ps_group_attn_args* a) {
    GaLayout L;
    const size_t rows = (size_t)a->tokens * (a->k + 1), esz = a->dtype == PS_BF16 ? 2 : 4;
    L.table = 0;
    L.k_rot = a256((size_t)(a->tokens + a->k) * (a->head_dim / 2) * sizeof(float2));
    L.total = L.k_rot + a256((size_t)a->seqs * rows * a->n_kv_heads * a->head_dim * esz);
    return L;
}

template <typename WT, int D>
int launch(const GaParams& P, hipStream_t s) {
    const long long nrope = (long long)P.seqs * P.rows * P.nkv * (D / 8);
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
    P.table = (float2*)(ws + L.table); P.k_rot = ws + L.k_rot;
    P.log_base = log((double)a->rope_base);
    hipStream_t s = (hipStream_t)stream;
    if (a->dtype == PS_BF16) return a->head_dim == 128 ? launch<bf16_t, 128>(P, s) : launch<bf16_t, 64>(P, s);
    return a->head_dim == 128 ? launch<float, 128>(P, s) : launch<float, 64>(P, s);
}
