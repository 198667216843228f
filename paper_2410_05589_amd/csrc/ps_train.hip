// Attention of group-wise parallel training (see include/ps_train.h; Section 4.1).
//
// Three kernels per call: the rotary table (cos, sin of position * base^(-2j/d) in double precision), the
// rotation of k (to the storage type, rounded as the inference path caches keys), and the attention itself,
// which rotates its 16 query rows (in float32) while it stages them.
//
// The attention kernels never touch a key the mask hides.  A query tile is a whole number of parallel groups
// (as many as fit into 16 rows); what its rows may see are (a) real tokens of groups up to their own - these
// are gathered with a stride of k + 1 rows, 16 per key tile - and (b) [MASK] tokens of their own group, which
// all lie inside the query tile's own 16 rows: one more key tile.  Online softmax over the key tiles; scores are
// MFMA tiles (the keys' rows are the 16-row operand, the 16 query rows the 16-column operand).  There is one kernel
// per storage type (ga_attn_bf16_kernel, ga_attn_f32_kernel); each describes its own scheme.
#include "ps_device.h"
#include "ps_train.h"

namespace {

constexpr int GA_THREADS = 256, GA_WAVES = GA_THREADS / 64;
constexpr float GA_LAZY = 8.f;

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

// ------------------------------------------------------------------------------------------
// float32 values.  A workgroup takes one query tile; its four wavefronts take the key tiles in turn, each with
// its own running maximum, sum and output, and their results meet in LDS at the end.  Scores are MFMA tiles (the K
// rows, lane (c, kb): bytes [64 t + 16 kb, +16) of key c, straight from memory as the 16-row operand; the query
// rows, rotated while they are staged, the 16-column operand in registers); P.V is plain FMA work: a lane owns
// head_dim / 64 output columns of all 16 rows and reads the probabilities as LDS broadcasts.
// ------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(GA_THREADS, 2) ga_attn_f32_kernel(const GaParams P) {   // workgroups per compute unit
    typedef float WT;
    constexpr int ESZ = 4, STEPS = D / Traits<WT>::KSTEP, DPL = D / 64;
    constexpr int OFF_Q = 0;                                // 16 query rows as MFMA operands: 16 * D * 4 bytes
    constexpr int OFF_P = OFF_Q + 16 * D * 4;               // [waves][16 rows][16 keys] probabilities
    constexpr int OFF_A = OFF_P + GA_WAVES * 16 * 16 * 4;   // [waves][16] rescale factors of the running output
    constexpr int OFF_ML = OFF_A + GA_WAVES * 16 * 4;       // [waves][16][2] final (max, sum)
    constexpr int OFF_O = OFF_ML + GA_WAVES * 16 * 2 * 4;   // [waves][16][D] outputs
    __shared__ __attribute__((aligned(16))) char smem[OFF_O + GA_WAVES * 16 * D * 4];
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

    // ---- the query rows, rotated, into LDS as the 16-column MFMA operand; rows beyond the tile repeat the last
    const char* qsrc = (const char*)P.q + ((size_t)seq * P.rows * P.nq + h) * D * ESZ;
    for (int t2 = tid; t2 < 16 * (D / 8); t2 += GA_THREADS) {
        const int r = min(t2 / (D / 8), nrows - 1), g4 = t2 % (D / 8);
        const int row = r0 + r, pos = row / K1 + row % K1;                      // group + slot
        const char* qrow = qsrc + (size_t)row * P.nq * D * ESZ;
        const f32x4 a = load4<WT>(qrow + 4 * g4 * ESZ), b = load4<WT>(qrow + (D / 2 + 4 * g4) * ESZ);
        u32x4 ra, rb;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float2 t = P.table[(size_t)pos * (D / 2) + 4 * g4 + e];
            ra[e] = __float_as_uint(a[e] * t.x - b[e] * t.y);
            rb[e] = __float_as_uint(b[e] * t.x + a[e] * t.y);
        }
        const int ts = (t2 / (D / 8)) * (D / 4) + g4;                           // (row, group of 4 elements) as attn_store_q counts
        attn_store_q<WT, D>(sQ, ts, ra);
        attn_store_q<WT, D>(sQ, ts + D / 8, rb);
    }
    __syncthreads();
    BRegs<WT, 1> bq[STEPS];
#pragma unroll
    for (int t = 0; t < STEPS; ++t) bq[t].h[0] = ld16(sQ + (t * 64 + lane) * 16);
    // this lane's query (column c of the score tile): group and slot
    const int qr = min(c, nrows - 1), qg = g0 + qr / K1, qs = qr % K1;
    const bool qlive = c < nrows;

    const char* kbase = (const char*)P.k_rot + ((size_t)seq * P.rows * P.nkv + hk) * D * ESZ;
    const char* vbase = (const char*)P.v + ((size_t)seq * P.rows * P.nkv + hk) * D * ESZ;
    const size_t rstride = (size_t)P.nkv * D * ESZ;        // bytes between layout rows
    const int n_real = (g_last >> 4) + 1;                   // key tiles of real tokens; one more tile: the tile's own [MASK] rows
    const int n_tiles = n_real + (P.k > 0 ? 1 : 0);
    float m_run = -INFINITY, l_run = 0.f;                   // of query c (the same in the four lanes that share it)
    float o[16][DPL];                                       // this lane's columns of all 16 rows
#pragma unroll
    for (int rr = 0; rr < 16; ++rr)
#pragma unroll
        for (int e = 0; e < DPL; ++e) o[rr][e] = 0.f;
    // layout row of key j of key tile t (clamped to a row that exists); tile n_real holds the [MASK] rows of the
    // query tile's own groups
    auto key_row = [&](int t, int j) __attribute__((always_inline)) {
        return t >= n_real ? r0 + min(j, nrows - 1) : min(16 * t + j, g_last) * K1;
    };
    {
    // a key tile at a time; its K rows and value rows are requested one tile ahead
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
#pragma unroll
    for (int rr = 0; rr < 16; ++rr)
#pragma unroll
        for (int e = 0; e < DPL; ++e) sO[(wave * 16 + rr) * D + DPL * lane + e] = o[rr][e];
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
            const float f = mw > -INFINITY ? expf(mw - M) : 0.f;
            num += sO[(w * 16 + rr) * D + dd] * f;
            den += sML[(w * 16 + rr) * 2 + 1] * f;
        }
        obase[(size_t)(r0 + rr) * P.nq * D + dd] = num / den;   // (every row sees at least its own real token: den > 0)
    }
}

// ------------------------------------------------------------------------------------------
// bf16 values.  A workgroup takes four adjacent query tiles, one per wavefront, and walks the key tiles of real
// tokens two at a time; the pair's K and V rows are brought in once for all four wavefronts.
//
// Loads are laid out for the texture unit, which handles a load in units of four lanes: four adjacent lanes read
// adjacent bytes of one row (a lane that fetched its own MFMA operand directly would make every lane of such a unit
// touch another row).  K: wavefront w brings in half of tile w / 2's rows; lane (key = lane / 4, j = lane % 4) reads
// bytes [64 t + 16 j, +16) of its key and puts them into LDS at (t ^ key % 4, j ^ key / 4 % 4) of the key's row,
// where lane (c, kb) of every wavefront picks up bytes [64 t + 16 kb, +16) of key c, its operand of MFMA step t (the
// placement keeps writers and readers off each other's banks).  V: wavefront w brings in keys 4 w .. 4 w + 3 of both
// tiles; a lane reads 4 bytes (two columns) of each and stores, per column, the dwords (key 4 w, 4 w + 1) and
// (4 w + 2, 4 w + 3) of the first tile and of the second side by side: lane (c, kb) then reads, per 16 output columns,
// one 16-byte piece = its 8 keys of the 32-key contraction (index 8 kb + e = key 4 kb + e of the first tile,
// 4 kb + e - 4 of the second); 4 dwords are left out every 8 columns and 4 more per block of 4 keys (banks again).
// Two such buffers take turns: while a pair is worked on, the next one is written (from registers that were
// requested an iteration earlier) and the one after it is requested; one barrier per pair.
//
// The tile of a query tile's own [MASK] rows comes last: the four wavefronts' own tiles are staged like two more
// pairs, and a wavefront works on the one that holds its tile with the other tile masked.
//
// Per wavefront: the 16 query rows, rotated in float32, scaled by log2(e) / sqrt(d) (scores in units of ln 2: the
// exponentials are single v_exp_f32) and split into bf16 high and low parts, stay in registers as the 16-column
// operand; online softmax per pair of tiles (the maxima and sums of the four lanes that share a query row are
// exchanged with row swaps; the running output is rescaled only when a maximum moved); P, split into high and low
// parts, is the 16-row operand of P.V straight from the score registers.  A wavefront owns its rows: no merge.
// ------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(GA_THREADS, 4) ga_attn_bf16_kernel(const GaParams P) {
    typedef bf16_t WT;
    constexpr int STEPS = D / 32, NCH = D / 8;
    constexpr int KT = 16 * D * 2;                          // bytes of a staged K tile
    constexpr int RSTR = (D / 8) * 36 + 4;                  // dwords per block of 4 keys of the staged V pair
    constexpr int BUF = 2 * KT + 4 * RSTR * 4;              // bytes of a buffer: two K tiles, the V pair
    constexpr int OFF_A = 2 * BUF;                          // [waves][16] rescale factors, later the rows' sums
    constexpr int QAREA = 16 * D * 4;                       // a wavefront's query rows on their way into registers, later its output
    static_assert(GA_WAVES * QAREA <= 2 * BUF, "the wavefronts' query and output areas fit the buffers");
    __shared__ __attribute__((aligned(16))) char smem[OFF_A + GA_WAVES * 16 * 4];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, kb = lane >> 4;
    const int K1 = P.k + 1;
    const int nblk = (P.ntiles + GA_WAVES - 1) / GA_WAVES;
    const int blk = nblk - 1 - (int)blockIdx.x;             // the tiles with the most keys start first
    const int h = blockIdx.y, seq = blockIdx.z, hk = h / (P.nq / P.nkv);
    // this wavefront's query tile (a wavefront beyond the last tile keeps the last one's numbers and only helps to stage)
    const int qt = GA_WAVES * blk + wave;
    const bool active = qt < P.ntiles;
    const int g0 = min(qt, P.ntiles - 1) * P.gpt, ng = min(P.gpt, P.T - g0), nrows = ng * K1, r0 = g0 * K1, g_last = g0 + ng - 1;
    // the workgroup's key tiles of real tokens, in pairs, then two pairs with the four own-[MASK] tiles
    const int g_last_wg = min((min(GA_WAVES * blk + GA_WAVES - 1, P.ntiles - 1) + 1) * P.gpt, P.T) - 1;
    const int real_pairs = ((g_last_wg >> 4) + 2) >> 1;
    const int n_pairs = real_pairs + (P.k > 0 ? 2 : 0);

    float* sA = reinterpret_cast<float*>(smem + OFF_A) + wave * 16;
    char* const sQ = smem + wave * QAREA;
    const unsigned rs32 = (unsigned)(P.nkv * D * 2);       // bytes between layout rows
    const unsigned K1rs = (unsigned)K1 * rs32;              // ... between real tokens
    const char* kbase = (const char*)P.k_rot + ((size_t)seq * P.rows * P.nkv + hk) * D * 2;
    const char* vbase = (const char*)P.v + ((size_t)seq * P.rows * P.nkv + hk) * D * 2;

    // ---- the query rows into registers, by way of LDS
    {
        const char* qsrc = (const char*)P.q + ((size_t)seq * P.rows * P.nq + h) * D * 2;
        const float qscale = P.inv_sqrt_d * 1.4426950408889634f;
        for (int t2 = lane; t2 < 16 * (D / 8); t2 += 64) {
            const int r = min(t2 / (D / 8), nrows - 1), g4 = t2 % (D / 8);
            const int row = r0 + r, pos = row / K1 + row % K1;                  // group + slot
            const char* qrow = qsrc + (size_t)row * P.nq * D * 2;
            const f32x4 a = load4<WT>(qrow + 4 * g4 * 2), b = load4<WT>(qrow + (D / 2 + 4 * g4) * 2);
            u32x4 ra, rb;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float2 t = P.table[(size_t)pos * (D / 2) + 4 * g4 + e];
                ra[e] = __float_as_uint((a[e] * t.x - b[e] * t.y) * qscale);
                rb[e] = __float_as_uint((b[e] * t.x + a[e] * t.y) * qscale);
            }
            const int ts = (t2 / (D / 8)) * (D / 4) + g4;                       // (row, group of 4 elements) as attn_store_q counts
            attn_store_q<WT, D>(sQ, ts, ra);
            attn_store_q<WT, D>(sQ, ts + D / 8, rb);
        }
    }
    lds_sync_wave();
    __builtin_amdgcn_wave_barrier();
    BRegs<WT, 1> bq[STEPS];
#pragma unroll
    for (int t = 0; t < STEPS; ++t) {
        bq[t].h[0] = ld16(sQ + (2 * t * 64 + lane) * 16);
        bq[t].l[0] = ld16(sQ + ((2 * t + 1) * 64 + lane) * 16);
    }
    __syncthreads();                                        // the buffers take K and V rows from here on

    // ---- staging: this lane's share of a pair
    // K: tile kg of the pair, requests t = kt0 .. kt0 + STEPS / 2 - 1 of (key kkey, piece kj)
    constexpr int KL = STEPS / 2;                           // K requests per lane
    constexpr int TM = STEPS - 1, TL = STEPS == 4 ? 2 : 1;  // the row's 64-byte segments: mask and log2
    const int kg = wave >> 1, kt0 = (wave & 1) * KL, kkey = lane >> 2, kj = lane & 3;
    auto k_lds = [&](int key, int j) __attribute__((always_inline)) {
        return key * (2 * D) + ((key & TM) << 6) + ((j ^ ((key >> TL) & 3)) << 4);
    };
    const int kw_rel = kg * KT + k_lds(kkey, kj), kr_rel = k_lds(c, kb);
    // V: keys 4 wave .. 4 wave + 3 of both tiles, columns 2 vc, 2 vc + 1 (lanes beyond D / 2 columns repeat the last and store nothing)
    const int vc = min(lane, D / 2 - 1);
    const bool vlane = lane < D / 2;
    const int vw_rel = 2 * KT + (wave * RSTR + (vc >> 2) * 36 + (vc & 3) * 8) * 4;
    const int vr_rel = 2 * KT + (kb * RSTR + (c >> 3) * 36 + (c & 7) * 4) * 4;
    struct Stage { uint4 k[KL]; unsigned v[2][4]; };
    // layout row of key j of tile g of pair p: real tokens up to the workgroup's last group, then the own rows of query
    // tile 4 blk + 2 (p - real_pairs) + g (clamped to rows that exist)
    auto stage_load = [&](int p, Stage& s) __attribute__((always_inline)) {
        size_t voff[2][4];                                  // bytes from vbase to the V rows (wavefront-uniform)
        unsigned krow, kmul;                                // the lane's K row: index and bytes per index
        if (p < real_pairs) {
            krow = (unsigned)min(16 * (2 * p + kg) + kkey, g_last_wg);
            kmul = K1rs;
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int i = 0; i < 4; ++i) voff[g][i] = (size_t)(unsigned)min(16 * (2 * p + g) + 4 * wave + i, g_last_wg) * K1rs;
        } else {
            const int o = p - real_pairs;
            int first[2], last[2];                          // the own rows of the pair's two query tiles
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const int go = min(GA_WAVES * blk + 2 * o + g, P.ntiles - 1) * P.gpt;
                first[g] = go * K1;
                last[g] = min(P.gpt, P.T - go) * K1 - 1;
            }
            krow = (unsigned)(first[kg] + min(kkey, last[kg]));
            kmul = rs32;
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int i = 0; i < 4; ++i) voff[g][i] = (size_t)(unsigned)(first[g] + min(4 * wave + i, last[g])) * rs32;
        }
        const char* kp = kbase + (size_t)krow * kmul + kj * 16;
#pragma unroll
        for (int u = 0; u < KL; ++u) s.k[u] = ld16(kp + (kt0 + u) * 64);
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int i = 0; i < 4; ++i)                      // (descriptor at the pair's first row, scalar offset per row: no vector address arithmetic)
                s.v[g][i] = __builtin_amdgcn_raw_buffer_load_b32(make_rsrc(vbase + voff[0][0]), (unsigned)(vc * 4), (unsigned)(voff[g][i] - voff[0][0]), 0);
    };
    auto stage_store = [&](char* buf, const Stage& s) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < KL; ++u) *reinterpret_cast<uint4*>(buf + (kw_rel ^ ((kt0 + u) << 6))) = s.k[u];
        if (vlane) {
            unsigned lo[4], hi[4];
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                lo[2 * g] = __builtin_amdgcn_perm(s.v[g][1], s.v[g][0], 0x05040100u); lo[2 * g + 1] = __builtin_amdgcn_perm(s.v[g][3], s.v[g][2], 0x05040100u);
                hi[2 * g] = __builtin_amdgcn_perm(s.v[g][1], s.v[g][0], 0x07060302u); hi[2 * g + 1] = __builtin_amdgcn_perm(s.v[g][3], s.v[g][2], 0x07060302u);
            }
            *reinterpret_cast<uint4*>(buf + vw_rel) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
            *reinterpret_cast<uint4*>(buf + vw_rel + 16) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
        }
    };

    // ---- this lane's query (column c of the score tile): group, slot, and which keys 4 kb + e of a tile it sees
    const int qr = min(c, nrows - 1), qg = g0 + qr / K1, qs = qr % K1;
    const bool qlive = active && c < nrows;
    const int real_hi0 = qlive ? qg - 4 * kb : -(1 << 20);   // real tokens of tile t: e <= real_hi0 - 16 t
    const int own_lo = qr - qs + 1 - 4 * kb, own_hi = qlive ? qr - 4 * kb : -(1 << 20);   // own [MASK] rows: those of the query's group, up to its slot
    float m_run = -INFINITY, l_run = 0.f;                   // of query c (the same in the four lanes that share it)
    f32x4 oacc[D / 16];                                     // MFMA tiles, lane (c, kb): column 16 j + c of rows 4 kb .. 4 kb + 3
#pragma unroll
    for (int j = 0; j < D / 16; ++j) oacc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // one pair of tiles: lo[g] <= e <= hi[g] are the keys 4 kb + e of tile g the lane's query sees (unmasked: all of them)
    auto work = [&](const char* buf, bool unmasked, int lo0, int hi0, int lo1, int hi1) __attribute__((always_inline)) {
        f32x4 acc[2][1];
#pragma unroll
        for (int g = 0; g < 2; ++g) acc[g][0] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < STEPS; ++t)
#pragma unroll
            for (int g = 0; g < 2; ++g) mma_step<WT, 1>(ld16(buf + g * KT + (kr_rel ^ (t << 6))), bq[t], acc[g]);
        float sc[2][4], mt = -INFINITY;
        if (unmasked) {
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
                const int lo = g ? lo1 : lo0, hi = g ? hi1 : hi0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    sc[g][e] = (e >= lo && e <= hi) ? acc[g][0][e] : -INFINITY;
                    mt = fmaxf(mt, sc[g][e]);
                }
            }
        }
        mt = quad_rows_max(mt);
        // The reference m_run the exponentials are taken against follows the row's maximum only when that has moved
        // up by more than GA_LAZY (in units of ln 2): sums and outputs are relative to the same reference, so the
        // quotient is the same, the probabilities stay below 2^GA_LAZY, and most pairs need no rescaling
        const bool moved = mt > m_run + GA_LAZY;            // (also the first keys a row sees: m_run = -inf)
        const float m_new = moved ? mt : m_run;
        const float alpha = moved ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.f;   // exp2(-inf) = 0 when nothing was seen before
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
        if (__any(moved)) {                                 // rows 4 kb .. 4 kb + 3 of the running output: their factors by way of LDS
            if (kb == 0) sA[c] = alpha;
            lds_sync_wave();
            __builtin_amdgcn_wave_barrier();
            const f32x4 al = *reinterpret_cast<const f32x4*>(sA + 4 * kb);
#pragma unroll
            for (int j = 0; j < D / 16; ++j) oacc[j] *= al;
            lds_sync_wave();
            __builtin_amdgcn_wave_barrier();
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
            for (int u = 0; u < 4; ++u) vv[u] = __builtin_bit_cast(bf16x8, ld16(buf + vr_rel + 72 * 4 * (j0 + u)));
#pragma unroll
            for (int u = 0; u < 4; ++u) oacc[j0 + u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, vv[u], oacc[j0 + u], 0, 0, 0);
#pragma unroll
            for (int u = 0; u < 4; ++u) oacc[j0 + u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pb, vv[u], oacc[j0 + u], 0, 0, 0);
        }
    };

    // ---- the pairs
    Stage st;
    stage_load(0, st);
    stage_store(smem, st);
    if (n_pairs > 1) stage_load(1, st);
    __syncthreads();
    for (int p = 0; p < n_pairs; ++p) {
        const char* buf = smem + (p & 1) * BUF;
        if (p + 1 < n_pairs) stage_store(smem + ((p + 1) & 1) * BUF, st);
        if (p + 2 < n_pairs) stage_load(p + 2, st);
        // what this wavefront's queries see of the pair.  Real tokens: nothing if every key of the pair lies after the
        // tile's last group, everything if every key lies before its first.  The own-[MASK] pairs: the pair
        // p - real_pairs = wave / 2 holds this wavefront's tile, as its tile wave % 2; the other tile is masked
        const bool real = p < real_pairs, mine = (wave >> 1) == p - real_pairs, first = (wave & 1) == 0;
        const bool busy = active && (real ? 32 * p <= g_last : mine);
        const bool unmasked = real && 32 * p + 31 <= g0;
        const int lo = real ? 0 : own_lo;
        const int hi0 = real ? real_hi0 - 32 * p : (first ? own_hi : -(1 << 20));
        const int hi1 = real ? real_hi0 - 32 * p - 16 : (first ? -(1 << 20) : own_hi);
        if (busy) work(buf, unmasked, lo, hi0, lo, hi1);
        __syncthreads();
    }

    // ---- output: rows by way of the wavefront's LDS area (the buffers are free now), divided by their sums
    if (kb == 0) sA[c] = l_run;
    float* sO = reinterpret_cast<float*>(sQ);
#pragma unroll
    for (int j = 0; j < D / 16; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) sO[(4 * kb + r) * D + 16 * j + c] = oacc[j][r];
    lds_sync_wave();
    __builtin_amdgcn_wave_barrier();
    if (active) {
        float* obase = P.out + ((size_t)seq * P.rows * P.nq + h) * D;
        for (int x = lane; x < nrows * D; x += 64) {
            const int rr = x / D, dd = x - rr * D;
            obase[(size_t)(r0 + rr) * P.nq * D + dd] = sO[x] / sA[rr];   // (every row sees at least its own real token: the sum is > 0)
        }
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
    if constexpr (Traits<WT>::BF)
        hipLaunchKernelGGL((ga_attn_bf16_kernel<D>), dim3((P.ntiles + GA_WAVES - 1) / GA_WAVES, P.nq, P.seqs), dim3(GA_THREADS), 0, s, P);
    else
        hipLaunchKernelGGL((ga_attn_f32_kernel<D>), dim3(P.ntiles, P.nq, P.seqs), dim3(GA_THREADS), 0, s, P);
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
