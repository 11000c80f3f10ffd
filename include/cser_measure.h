/*
 * cser_measure.h -- MEASUREMENT ONLY.  Entry points the benchmark and the tests use to time the kernels,
 * to pick a launch shape for an experiment and to read what a launch got.  Nothing here changes a result:
 * every kernel computes the same bits.  Not part of the optimizer interface (cser.h).
 */
#ifndef CSER_MEASURE_H
#define CSER_MEASURE_H

#include "cser.h"

#ifdef __cplusplus
extern "C" {
#endif
#if defined(__GNUC__)
#pragma GCC visibility push(default) /* the library is built with hidden visibility: only these entry points are exported */
#endif

/*
 * Per-kernel timing.  When enabled, every launch of the fused-step kernel (which = 0) and of the
 * reset kernel (which = 1) is bracketed by HIP events on the launch stream; cser_profile_read
 * waits for the recorded events, adds their elapsed times and launch counts to running totals,
 * returns the totals and recycles the events.  At most 4096 launches per kind are held between
 * reads; later ones go untimed.
 */
int cser_profile_enable(cser_ctx* ctx, int on);
int cser_profile_read(cser_ctx* ctx, int which, double* total_ms, uint64_t* launches);
int cser_profile_clear(cser_ctx* ctx);

typedef enum cser_tuning_key {
  CSER_TUNE_KERNEL = 0,            /* 0 (default) automatic; 1 one-wavefront workgroups, a worker's row each (W <= 64);
                                      2 W-wavefront workgroups, worker sums staged in LDS (W <= 16); 3 a lane walks all
                                      workers (any W); 4 a pair of launches, 1 on the blocks neither compressor chose and
                                      2 (beyond 16 workers: 3) on the others.  A kernel that does not take the context's W falls back to 0. */
  CSER_TUNE_NONTEMPORAL = 1,       /* -1 (default) non-temporal accesses unless all state fits 256 MiB; 0 never; 1 always */
  CSER_TUNE_FUSE_RESET = 2,        /* 1 (default) on iterations with t mod H = 0 the error reset runs inside the fused-step
                                      kernel (x and e of its blocks make one trip instead of two); 0 separate reset kernel */
  CSER_TUNE_TILE_WAVES_PER_CU = 3, /* kernel 1: most resident wavefronts per CU; -1 (default) 12 / 18 / no cap for 4 / 3 / 2
                                      load streams per wavefront; 0 no cap */
  CSER_TUNE_SHARED_GROUPS_PER_CU = 4 /* kernel 2 and the reset kernel: most resident workgroups per CU; -1 (default)
                                      max(2, 24 / W); 0 no cap */
} cser_tuning_key;
int cser_set_tuning(cser_ctx* ctx, int key, int64_t value);

/* What has been enqueued through this context so far. */
typedef struct cser_counters {
  uint64_t steps;             /* iterations carried out                                                  */
  uint64_t window_draws;      /* times the masks of the next iterations were drawn (selector launches)   */
  uint64_t resets_fused;      /* error resets carried out inside the fused-step kernel                   */
  uint64_t resets_separate;   /* error resets carried out by the reset kernel                            */
  uint64_t launches_tile;     /* fused steps by kernel choice (1, 2, 3, 4 of CSER_TUNE_KERNEL)           */
  uint64_t launches_shared;
  uint64_t launches_general;
  uint64_t launches_split;
} cser_counters;
int cser_measure_counters(const cser_ctx* ctx, cser_counters* out);

/*
 * Which fused-step kernel (1 .. 4 of CSER_TUNE_KERNEL) a configuration's iterations take by default: ordinary
 * iterations (reset_iteration = 0) and iterations that carry the error reset as well (reset_iteration = 1).  Host
 * arithmetic only, no device needed.
 */
int cser_measure_kernel_choice(const cser_config* cfg, int reset_iteration, int* kernel);

/*
 * Residency the launches of this context get: dynamic LDS bytes requested per workgroup and the number of
 * workgroups the runtime's occupancy calculator fits on a CU with that request (tile kernel: one wavefront
 * per workgroup; shared kernels: W wavefronts per workgroup).  0 where a kernel does not take the context's W.
 */
typedef struct cser_residency {
  uint32_t tile_lds, tile_groups_per_cu;
  uint32_t shared_lds, shared_groups_per_cu;
  uint32_t shared_reset_lds, shared_reset_groups_per_cu;
  uint32_t reset_lds, reset_groups_per_cu;
} cser_residency;
int cser_measure_residency(const cser_ctx* ctx, cser_residency* out);

/*
 * Practical bandwidth ceiling: a plain copy kernel dst[i] = src[i] over n_bytes (device pointers,
 * 16-byte aligned, n_bytes a multiple of 16), enqueued on hip_stream.  Also the known-size kernel the
 * HBM traffic counters are calibrated on.
 */
int cser_copy_probe(void* dst, const void* src, uint64_t n_bytes, void* hip_stream);

#if defined(__GNUC__)
#pragma GCC visibility pop
#endif
#ifdef __cplusplus
}
#endif
#endif /* CSER_MEASURE_H */
