/*
 * lsm_bench.h -- benchmark aids of the gfx950 LSM library.  Nothing here is part of the method (the
 * paper's Eq. 5 / Algorithm 2 path is declared in lsm.h); these calls exist so that a benchmark can time
 * the library's kernels one by one, measure the arithmetic rate of the intra-chunk phase apart from HBM,
 * and calibrate the two rooflines (a streaming copy, a loop of nothing but MFMAs) in the same run.
 * Same conventions as lsm.h: device pointers, 16-byte aligned, work enqueued on `stream`, lsm_status
 * returns, argument checks before the first HIP call.
 */
#ifndef LSM_BENCH_H
#define LSM_BENCH_H

#include "lsm.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Optional per-kernel timing for benchmarks (not part of the method).  After lsm_profile_start()
 * every kernel the library enqueues is bracketed by a pair of HIP events on the call's stream;
 * lsm_profile_stop() waits for them, writes up to `capacity` (kernel id, elapsed ms) pairs in launch
 * order, returns how many it wrote, and switches timing off again.  Process-wide state: do not use
 * from concurrent threads while other calls are in flight.  lsm_kernel_name() names an id.
 */
int lsm_profile_start(void);
int lsm_profile_stop(int* kernel_ids, float* milliseconds, int capacity);
const char* lsm_kernel_name(int kernel_id);

/*
 * Benchmark aid (not part of the method): the intra-chunk phase of the forward (masked decayed scores
 * times V plus Q times the chunk state; Algorithm 2, O_intra + O_inter) as a kernel of its own, one
 * chunk per workgroup, with its compute phase repeated `repeats` times on the tiles resident in LDS,
 * so that the arithmetic rate of that phase can be measured apart from the HBM traffic that bounds
 * the streamed path.  Only for parameter sets with lsm_kernel_path() == 1, a decay kind other than
 * LSM_DECAY_VECTOR and no packed input (else LSM_ERR_UNSUPPORTED).  The call first materialises one
 * chunk state per chunk in `workspace` (at least lsm_bench_intra_chunk_workspace_bytes(p), 0 if
 * unsupported), from a zero initial state; `o` receives lsm_chunk_fwd's output for init_state = NULL
 * (to rounding).
 */
size_t lsm_bench_intra_chunk_workspace_bytes(const lsm_params* p);
int lsm_bench_intra_chunk(const lsm_params* p, const void* q, const void* k, const void* v,
                          const float* log_decay, void* o, void* workspace, size_t workspace_bytes,
                          int repeats, void* stream);

/*
 * Calibration.  lsm_calib_copy: dst[0..bytes) = src[0..bytes) by a plain grid-stride kernel (bytes a
 * multiple of 16): bytes read + bytes written over its duration is the HBM rate a streaming kernel
 * reaches on this GPU.  lsm_calib_mfma: `workgroups` workgroups of four waves, every wave issuing
 * 4 * iters independent v_mfma_f32_32x32x16_bf16 on register operands; `out` receives
 * workgroups * 256 floats (only there to keep the results alive).  lsm_calib_mfma_flops gives the flop
 * count of such a launch (host-only); over the launch's duration it is the bf16 MFMA rate the chip
 * sustains at the clock it holds under that load.
 */
int lsm_calib_copy(void* dst, const void* src, size_t bytes, void* stream);
int lsm_calib_mfma(float* out, int workgroups, int iters, void* stream);
double lsm_calib_mfma_flops(int workgroups, int iters);

#ifdef __cplusplus
}
#endif
#endif /* LSM_BENCH_H */
