/*
 * eagle3_measure.h — measurement hooks of the eagle3 library.  NOT part of the product interface (include/eagle3.h):
 * bench.py uses them to time individual kernel launches on the stream they run on.
 */
#ifndef EAGLE3_MEASURE_H
#define EAGLE3_MEASURE_H

#include "eagle3.h"

#ifdef __cplusplus
extern "C" {
#endif

/* While profiling is on, every weight-streaming GEMM launch of the step calls carries a start/stop pair of HIP
 * events attached to the dispatch itself on the caller's stream, i.e. the kernel's own begin and end timestamps (the
 * launches no longer overlap their neighbours: do not time whole steps with it on).  eagle3_profile_read
 * synchronises, then reports the summed kernel duration, the number of launches and the weight bytes those launches
 * read, for one kind of launch:
 *   EAGLE3_GEMM_FEW_ROWS   at most 32 activation rows (the draft's GEMMs, feature fusion)
 *   EAGLE3_GEMM_TILE64     33..64 rows, 64-weight-row workgroups with split-K (q/k/v, o, down at verification width)
 *   EAGLE3_GEMM_TILE128    33..64 rows, 128-weight-row workgroups (gate/up, LM head at verification width)
 *   EAGLE3_GEMM_MANY_ROWS  more than 64 rows (batched verification)
 * The counters are reset by eagle3_profile_begin. */
enum { EAGLE3_GEMM_FEW_ROWS = 0, EAGLE3_GEMM_TILE64 = 1, EAGLE3_GEMM_TILE128 = 2, EAGLE3_GEMM_MANY_ROWS = 3 };
int eagle3_profile_begin(eagle3_ctx* ctx);
int eagle3_profile_read(eagle3_ctx* ctx, int kind, double* ms_total, int64_t* launches, double* weight_bytes);
int eagle3_profile_end(eagle3_ctx* ctx);


#ifdef __cplusplus
}
#endif
#endif /* EAGLE3_MEASURE_H */
