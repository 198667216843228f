/*
 * ps_draft_debug.h - testing, tuning and measurement aids of libps_draft.so.
 *
 * None of this is part of the method or of the product interface (ps_draft.h, ps_verify.h):
 * the entries here let the tests look at the launch plan and force the give-up paths from the
 * host, let a -DPS_TIMELINE build hand out its clock stamps, and give the benchmark two
 * reference kernels (a plain streaming read and a plain copy) to calibrate its HBM figures.
 * Same conventions: extern "C", plain pointers, int ps_status results.
 */
#ifndef PS_DRAFT_DEBUG_H
#define PS_DRAFT_DEBUG_H
#include <stddef.h>
#include <stdint.h>
#include "ps_draft.h"
#ifdef __cplusplus
extern "C" {
#endif

/*
 * Host only.  For a configuration and the shape of a step, how ps_draft_step would cut up the
 * five GEMM phases on a device with n_cu compute units and lds_limit bytes of LDS per workgroup
 * (persistent-kernel mode): per phase PS_PLAN_FIELDS ints {T, Kt, K, rows, kw_log, s_log, Gs,
 * per_round, rounds, piece_groups, npieces, lds_bytes} into out[5 * PS_PLAN_FIELDS].
 */
#define PS_PLAN_FIELDS 12
PS_API int ps_draft_debug_plan(const ps_draft_config* config, int batch, int n_new, int k, int all_rows, int n_cu,
                        int lds_limit, int* out);

/*
 * Host only.  How ps_draft_step would cut up the attention of a step over bf16 caches (PS_ERR_UNSUPPORTED for
 * float32) for sequences of kv_len[0 .. batch) valid positions on a device with n_cu compute units: out[4] =
 * {NK: groups of 16 keys per wavefront and block (blocks of 128 NK cache keys), work units (blocks x passes of 16
 * query rows), blocks, merge items (0: every sequence is a single block and hands its rows on directly)}.
 */
PS_API int ps_draft_debug_attn_plan(const ps_draft_config* config, int batch, const int32_t* kv_len, int n_new, int k,
                             int n_cu, int* out);

/*
 * The following steps of ctx give up a wait for data of another workgroup after `spins` polls
 * (<= 0: the default, about a second).  With 1 every wait whose data is not there at the first
 * look is given up at once: the kernel still ends normally, the step's outputs are marked
 * (top_ids -1, lse NaN) and ps_draft_last_status reports PS_ERR_TIMEOUT.
 */
PS_API int ps_draft_debug_spin_limit(ps_draft_ctx* ctx, int spins);

/*
 * Builds with -DPS_TIMELINE only: DEVICE buffer of 64 x 1024 uint64 that receives per-workgroup
 * clock stamps of the following steps (NULL = off).
 */
PS_API int ps_draft_debug_timeline(ps_draft_ctx* ctx, void* buf);

/*
 * The following multi-workgroup acceptance walks give up a wait after `spins` polls (<= 0: the
 * default) and wait for `ghosts` (0 or 1) workgroups per sequence that do not exist, so the
 * give-up path runs while every kernel still ends normally.
 */
PS_API void ps_verify_debug_exchange(int spins, int ghosts);

/*
 * Reference kernels for the benchmark.  ps_measure_stream_read reads `bytes` (a multiple of 1024)
 * of DEVICE memory at src once, with the access pattern of the weight streams (every wavefront a
 * contiguous range, 16-byte non-temporal loads, 8 in flight per lane) and nothing else: the HBM
 * read rate an implementation of the draft step can hope for on this machine.  ps_measure_copy
 * copies `bytes` from src to dst (DEVICE, 16-byte aligned, not overlapping): exactly `bytes` read
 * and `bytes` written, to scale the profiler's FETCH_SIZE / WRITE_SIZE counters.  Asynchronous on
 * stream.  Errors: PS_ERR_NULL, PS_ERR_SHAPE (bytes not a positive multiple of 1024 resp. 16, or a misaligned pointer), PS_ERR_DEVICE.
 */
PS_API int ps_measure_stream_read(const void* src, size_t bytes, void* stream);
PS_API int ps_measure_copy(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PS_DRAFT_DEBUG_H */
