/* Benchmark instrumentation of the LASER-KV library: per-kernel event timing and single-kernel replays.
 * Not part of the method's interface (include/laserkv.h); nothing here is needed to use the library, and
 * laserkv_profile_isolate makes a context skip kernels, so its outputs are not valid while it is active. */
#ifndef LASERKV_PROFILE_H
#define LASERKV_PROFILE_H

#include "laserkv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-kernel timing for benchmarks.  Between laserkv_profile_begin and laserkv_profile_end every
 * kernel the context launches is bracketed by a pair of HIP events on the call's stream (which adds
 * a little time between kernels, so whole-path timings belong outside such a bracket).
 * laserkv_profile_end synchronises on those events and returns, per kernel kind (laserkv_kernel_id),
 * the summed elapsed milliseconds and the number of launches; both arrays are HOST pointers with
 * LKV_N_KERNELS entries.  At most LKV_PROFILE_MAX_LAUNCHES launches are recorded per bracket;
 * later ones run untimed.  Errors: LKV_EINVAL (null / not begun), LKV_EHIP. */
typedef enum {
  LKV_KERN_SWEEP1 = 0, /* exact score sweep 1 (row maxima and sums) + SimHash codes of keys and window queries
                          + histograms of the query codes */
  LKV_KERN_SWEEP2 = 1, /* exact score sweep 2 (pooled probabilities) + collision counts by histogram lookup */
  LKV_KERN_COUNT = 2,  /* collision counts as a kernel of their own (codes wider than 12 bits) */
  LKV_KERN_SELECT = 3, /* two-stage TopK and compaction (with the gather in laserkv_compress_block); also the
                          accumulation kernel of laserkv_score_block */
  LKV_KERN_APPEND = 4, /* gather-append as a kernel of its own */
  LKV_KERN_ATTEND = 5, /* attention over the compacted cache (both of its kernels) */
  LKV_KERN_SINGLE = 6, /* the one sweep of a block whose rows come with their complete log-sum-exp: SimHash codes,
                          pooled probabilities and collision counts from one read of the keys */
  LKV_N_KERNELS = 7
} laserkv_kernel_id;
#define LKV_PROFILE_MAX_LAUNCHES 8192

int laserkv_profile_begin(laserkv_ctx* ctx);
int laserkv_profile_end(laserkv_ctx* ctx, double* ms_per_kernel, int64_t* launches);

/* For benchmarks that time one kernel kind without event pairs between kernels: while kernel_id names a
 * laserkv_kernel_id, every call on the context launches only kernels of that kind (all checks still run,
 * outputs are NOT valid); a negative kernel_id restores normal operation.  The workspace keeps the
 * intermediates of the last complete call, so an isolated kernel runs on valid inputs of the same shape.
 * Errors: LKV_EINVAL (null context, kernel_id >= LKV_N_KERNELS). */
int laserkv_profile_isolate(laserkv_ctx* ctx, int32_t kernel_id);

#ifdef __cplusplus
}
#endif
#endif /* LASERKV_PROFILE_H */
