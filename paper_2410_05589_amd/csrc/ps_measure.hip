// Reference kernels for the benchmark (see ps_draft_debug.h): a plain streaming read with the access
// pattern of the draft step's weight streams, and a plain copy of known size.  No part of the method.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ps_draft_debug.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int MEASURE_THREADS = 512, MEASURE_U = 8;

// Every wavefront reads a contiguous range of `per_wave` KiB (the last one what is left), one KiB per load
// instruction, MEASURE_U loads in flight per lane; the values are folded into one word that is stored only
// if it has a value it cannot have, so the loads cannot be dropped.
__global__ void __launch_bounds__(MEASURE_THREADS) stream_read_kernel(const char* __restrict__ src, size_t kib, size_t per_wave,
                                                                      unsigned* sink) {
    const int lane = threadIdx.x & 63;
    const size_t wave = (size_t)blockIdx.x * (MEASURE_THREADS / 64) + (threadIdx.x >> 6);
    const size_t lo = wave * per_wave;
    if (lo >= kib) return;
    const size_t n = per_wave < kib - lo ? per_wave : kib - lo;
    const char* p = src + lo * 1024 + lane * 16;
    u32x4 acc = {0u, 0u, 0u, 0u}, buf[MEASURE_U];
#pragma unroll
    for (int u = 0; u < MEASURE_U; ++u) buf[u] = __builtin_nontemporal_load((const u32x4*)(p + (size_t)(u < n ? u : n - 1) * 1024));
    for (size_t t0 = 0; t0 < n; t0 += MEASURE_U) {
#pragma unroll
        for (int u = 0; u < MEASURE_U; ++u) {
            acc ^= buf[u];
            const size_t t = t0 + u + MEASURE_U;
            buf[u] = __builtin_nontemporal_load((const u32x4*)(p + (t < n ? t : n - 1) * 1024));
        }
    }
    const unsigned r = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    if (r == 0x9E3779B9u && sink) *sink = r;
}

__global__ void __launch_bounds__(256) copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

}   // namespace

extern "C" int ps_measure_stream_read(const void* src, size_t bytes, void* stream) {
    if (!src) return PS_ERR_NULL;
    if (bytes == 0 || bytes % 1024 != 0 || ((uintptr_t)src & 15)) return PS_ERR_SHAPE;
    int dev = 0, n_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
        return PS_ERR_DEVICE;
    const size_t kib = bytes / 1024, waves = (size_t)n_cu * (MEASURE_THREADS / 64);
    const size_t per_wave = (kib + waves - 1) / waves;
    hipLaunchKernelGGL(stream_read_kernel, dim3(n_cu), dim3(MEASURE_THREADS), 0, (hipStream_t)stream, (const char*)src, kib, per_wave,
                       (unsigned*)nullptr);
    return hipGetLastError() == hipSuccess ? PS_OK : PS_ERR_DEVICE;
}

extern "C" int ps_measure_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src) return PS_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0 || (((uintptr_t)dst | (uintptr_t)src) & 15)) return PS_ERR_SHAPE;
    hipLaunchKernelGGL(copy_kernel, dim3(4096), dim3(256), 0, (hipStream_t)stream, (u32x4*)dst, (const u32x4*)src, bytes / 16);
    return hipGetLastError() == hipSuccess ? PS_OK : PS_ERR_DEVICE;
}
