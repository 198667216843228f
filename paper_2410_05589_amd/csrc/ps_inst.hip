// One instantiation unit of the device code: compiled once per (storage type, head_dim) with
// -DPS_INST_BF16=0/1 -DPS_INST_D=64/128; exports a table of launchers the host dispatcher uses.
#include "ps_device.h"

#if PS_INST_BF16
typedef bf16_t WT_;
#else
typedef float WT_;
#endif
constexpr int D_ = PS_INST_D;

typedef void (*kernel_fn)(const StepParams);

template <int PH> static kernel_fn gemm_fn(int mt) {
    switch (mt) {
        case 1: return gemm_kernel<WT_, 1, PH>;
        case 2: return gemm_kernel<WT_, 2, PH>;
        case 3: return gemm_kernel<WT_, 3, PH>;
        default: return gemm_kernel<WT_, 4, PH>;
    }
}
static kernel_fn gemm_fn_ph(int ph, int mt) {
    switch (ph) {
        case PH_QKV: return gemm_fn<PH_QKV>(mt);
        case PH_OPROJ: return gemm_fn<PH_OPROJ>(mt);
        case PH_GATEUP: return gemm_fn<PH_GATEUP>(mt);
        case PH_DOWN: return gemm_fn<PH_DOWN>(mt);
        case PH_FC: return gemm_fn<PH_FC>(mt);
        default: return gemm_fn<PH_LMHEAD>(mt);
    }
}
static kernel_fn fused_fn(int mt) {
    switch (mt) {
        case 1: return fused_kernel<WT_, D_, 1>;
        case 2: return fused_kernel<WT_, D_, 2>;
        case 3: return fused_kernel<WT_, D_, 3>;
        default: return fused_kernel<WT_, D_, 4>;
    }
}

static kernel_fn attn_fn(int nk, int single) {
#if PS_INST_BF16
    return attn2_kernel<WT_, D_>;
#endif
    switch (2 * nk + (single ? 1 : 0)) {
        case 2: return attn_kernel<WT_, D_, 1, false>;
        case 3: return attn_kernel<WT_, D_, 1, true>;
        default: return attn_kernel<WT_, D_, 2, true>;   // (host: two key groups only with a single pass)
    }
}

// dynamic LDS of the attention kernel (bf16 storage: one variant, see attn_phase2)
static int attn_lds(int nk) { return PS_INST_BF16 ? ps_attn2_lds_bytes(D_) : ps_attn_lds_bytes(D_, nk); }

static hipError_t prepare(int lds_limit) {
    hipError_t e;
    for (int mt = 1; mt <= 4; ++mt) {
        for (int ph = 0; ph < PH_COUNT; ++ph) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_fn_ph(ph, mt)),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds_limit);
            if (e != hipSuccess) return e;
        }
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(fused_fn(mt)),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds_limit);
        if (e != hipSuccess) return e;
    }
    if (attn_lds(2) > lds_limit) return hipErrorInvalidValue;
    for (int v = 2; v < 6; ++v) {
        if (v == 4) continue;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_fn(v >> 1, v & 1)), hipFuncAttributeMaxDynamicSharedMemorySize,
                                attn_lds(v >> 1));
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// one kernel per phase; events: NULL or PS_PROFILE_EVENTS events recorded around the kernels
static hipError_t launch_multi(const StepParams& P, hipStream_t stream, hipEvent_t* events) {
    const int mt_all = (P.Mtot + 15) / 16, mt_lm = (P.Rtot + 15) / 16;
    int n_ev = 0;
    auto mark = [&]() -> hipError_t { return events ? hipEventRecord(events[n_ev++], stream) : hipSuccess; };
    auto gemm = [&](int ph, int mt) -> hipError_t {
        const PhaseDesc& pl = P.ph[ph];
        hipLaunchKernelGGL(gemm_fn_ph(ph, mt), dim3(pl.nwg), dim3(PS_WG_THREADS), pl.lds_bytes, stream, P);
        hipError_t le = hipGetLastError();
        return le != hipSuccess ? le : mark();
    };
    hipError_t e;
    if ((e = mark()) != hipSuccess) return e;
    if ((e = gemm(PH_QKV, mt_all)) != hipSuccess) return e;
    hipLaunchKernelGGL(attn_fn(P.attn_nk, P.attn_single), dim3(P.attn_nwg), dim3(PS_WG_THREADS), attn_lds(P.attn_nk), stream, P);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = mark()) != hipSuccess) return e;
    if ((e = gemm(PH_OPROJ, mt_all)) != hipSuccess) return e;
    if ((e = gemm(PH_GATEUP, mt_all)) != hipSuccess) return e;
    if ((e = gemm(PH_DOWN, mt_all)) != hipSuccess) return e;
    if ((e = gemm(PH_LMHEAD, mt_lm)) != hipSuccess) return e;
    hipLaunchKernelGGL(lm_merge_kernel, dim3(P.Rtot), dim3(PS_WG_THREADS), PS_MERGE_BYTES + PS_LDS_BASE, stream, P);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    return mark();
}

// The whole step as one launch of the persistent kernel.  Its workgroups wait for each other's
// data, so all of them must get a compute unit: the grid is one workgroup per CU and a workgroup
// (512 threads x up to 256 VGPRs, more than half of the LDS) fills a CU by itself, so they all become
// resident as soon as CUs are free; kernels that still occupy CUs end on their own.  Every wait
// in the kernel is bounded, so even a machine that withholds CUs cannot hang it.  (A cooperative
// launch would assert the same residency but costs ~17 us per launch on this runtime.)
static hipError_t launch_fused(const StepParams& P, hipStream_t stream) {
    const int mt = (P.Mtot + 15) / 16;
    hipLaunchKernelGGL(fused_fn(mt), dim3(P.fused_nwg), dim3(PS_WG_THREADS), (unsigned)P.fused_lds, stream, P);
    return hipGetLastError();
}

// the input projection of the feature-fusion input mode: a kernel of its own in front of the step
static hipError_t launch_fc(const StepParams& P, hipStream_t stream) {
    const PhaseDesc& pl = P.ph[PH_FC];
    hipLaunchKernelGGL(gemm_fn_ph(PH_FC, (pl.rows + 15) / 16), dim3(pl.nwg), dim3(PS_WG_THREADS), pl.lds_bytes, stream, P);
    return hipGetLastError();
}

static hipError_t fused_resident(int mt, int lds, int* per_cu) {
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(per_cu, reinterpret_cast<const void*>(fused_fn(mt)), PS_WG_THREADS, (size_t)lds);
}

static hipError_t launch_probs(const StepParams& P, hipStream_t stream) {
    hipLaunchKernelGGL(probs_kernel, dim3((P.V + 255) / 256 < 256 ? (P.V + 255) / 256 : 256, P.Rtot), dim3(256), 0,
                       stream, P);
    return hipGetLastError();
}

typedef void (*pack_fn)(const StepParams, int, int, int, char*);
static hipError_t pack(const StepParams& P, int ph, int T, int Kt, int Kreal, char* dst, hipStream_t stream) {
    pack_fn f;
    switch (ph) {
        case PH_QKV: f = pack_kernel<WT_, PH_QKV>; break;
        case PH_OPROJ: f = pack_kernel<WT_, PH_OPROJ>; break;
        case PH_GATEUP: f = pack_kernel<WT_, PH_GATEUP>; break;
        case PH_DOWN: f = pack_kernel<WT_, PH_DOWN>; break;
        case PH_FC: f = pack_kernel<WT_, PH_FC>; break;
        default: f = pack_kernel<WT_, PH_LMHEAD>; break;
    }
    const size_t units = (size_t)T * Kt;
    const int grid = (int)((units + 3) / 4 < 65536 ? (units + 3) / 4 : 65536);
    hipLaunchKernelGGL(f, dim3(grid), dim3(256), 0, stream, P, T, Kt, Kreal, dst);
    return hipGetLastError();
}

#define PS_CAT2(a, b) a##b
#define PS_CAT(a, b) PS_CAT2(a, b)
const PsInstance* PS_CAT(ps_instance_, PS_INST_NAME)() {
    static const PsInstance inst = {
        PS_INST_BF16 ? PS_BF16 : PS_F32, PS_INST_D,
        prepare, launch_multi, launch_fused, launch_probs, launch_fc, fused_resident, pack,
    };
    return &inst;
}
