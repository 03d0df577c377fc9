/*
 * Measurement aids of libkdloss.  Not part of the method and not needed to use the library:
 * bench.py uses them to time single kernel families with HIP events, to read the shader clock a
 * kernel ran at, and to measure what the matrix pipe sustains with nothing else going on.
 * They are the only entry points that keep state (a per-thread hook, cleared by the caller).
 */
#ifndef KDLOSS_BENCH_H
#define KDLOSS_BENCH_H

#include "kdloss.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Benchmark aid (not part of the method): per-kernel timing without a profiler.
 * While a hook is set on the calling thread, every launch of the selected kernel
 * family made by kd_loss_fwd / kd_loss_fwd_bwd on that thread is bracketed by
 * hipEventRecord(events[2i]) before and hipEventRecord(events[2i+1]) after it, on the
 * call's stream, i counting launches since the hook was set, while 2i+1 < n_events.
 * `events` is a host array of hipEvent_t owned by the caller, which must outlive the
 * hook.  which < 0 clears the hook.  Host only; touches no device memory. */
typedef enum {
  KD_PROF_STATS = 0,        /* logit tiles + online log-sum-exp (one launch per teacher) */
  KD_PROF_ROWS = 1,         /* row pass of JSD / TVD / skewed KL (one launch per teacher) */
  KD_PROF_GRAD = 2,         /* logit tiles + dL/dz_s epilogue (one launch per chunk and teacher) */
  KD_PROF_GEMM_GRAD_W = 3,  /* grad_W_s product (one launch per chunk)                  */
  KD_PROF_GEMM_GRAD_H = 4   /* grad_h_s product (one launch per chunk)                  */
} kd_prof_kernel;
kd_status kd_loss_profile_hook(int which, void** events, int n_events);
/* Pairs recorded since the hook was set. */
int kd_loss_profile_count(void);

/* Benchmark aid: while set (per host thread; NULL clears it), workgroup 0 of the statistics kernel of
 * kd_loss_fwd / kd_loss_fwd_bwd and of kd_probe_mfma_rate stores into the two int64 at this device
 * address the shader-clock cycles and the 100 MHz reference ticks that its main loop took: their ratio
 * is the shader clock the GPU held under that kernel's load (it is set by the power limit, far below the
 * nominal 2.4 GHz for these kernels).  Host only. */
kd_status kd_loss_profile_clock(void* two_int64_device);

/* Benchmark aid, not part of the method: what the bf16 matrix pipe sustains on this GPU with nothing
 * else going on.  One launch of 256 workgroups x 8 waves (the occupancy of the logit kernels), each wave
 * issuing `iters` x 8 independent MFMA 32x32x16 on operands taken from `operands` (device, 128 KiB of
 * bf16 values; the shader clock under this load depends on them, so pass values like real data).
 * Executes KD_PROBE_FLOP_PER_ITER * iters flop.  `sink` (device, 256 * 512 floats) receives sums that
 * only keep the work alive.  Time the launch with events on `hip_stream`. */
/* Compile-time configuration of the loaded library as text (tile shapes, ablation switch), and the ablation
 * switch alone: 0 for the product; anything else is a measurement build (-DKD_ABLATE=n, see the top of
 * kd_kernels.hip) whose results are wrong by design. */
const char* kd_build_info(void);
int kd_build_ablation(void);

#define KD_PROBE_FLOP_PER_ITER (256.0 * 8 * 8 * 2 * 32 * 32 * 16)
kd_status kd_probe_mfma_rate(const void* operands, int iters, float* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* KDLOSS_BENCH_H */
