/*
 * hps_measure.h -- measurement aids of the HBM-PS pull/push library.  Nothing here is part of
 *                  the path: a benchmark uses these calls to time the path's stages and to
 *                  learn the rate at which the GPU returns random rows, which bounds the
 *                  pooling and push stages.  Conventions as in hps.h.
 */
#ifndef HPS_MEASURE_H_
#define HPS_MEASURE_H_

#include "hps.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Reads random rows of d_rows (n_rows rows of row_bytes bytes each, device, 16-byte aligned;
 * row_bytes = 64 or 256: the rows of a dim-16 and of a dim-64 float32 table) with the pooling
 * kernel's access shape and grid -- row_bytes / 16 lanes per row, eight rows in flight per lane
 * group -- about n_accesses of them, and writes one float per lane to d_sink (room for 262144
 * floats).  A benchmark times it to learn the rate at which this GPU returns such rows.
 * Errors: HPS_EINVAL. */
hps_status hps_probe_random_rows(const void* d_rows, uint64_t n_rows, uint32_t row_bytes,
                                 uint64_t n_accesses, float* d_sink, void* stream);

/* Stage timing.  Stages of one step: */
enum {
  HPS_STAGE_SORT = 0,    /* pull: order the key occurrences                        */
  HPS_STAGE_UNIQUE = 1,  /* pull: unique keys, inverse, grouping                   */
  HPS_STAGE_LOOKUP = 2,  /* pull: find or insert every unique key                  */
  HPS_STAGE_POOL = 3,    /* pull: row gather + bag sums                            */
  HPS_STAGE_PUSH = 4,    /* push: reduce by key + optimizer update                 */
  HPS_N_STAGES = 5
};

/* While bit s of stage_mask is set, every pull/push brackets stage s with a pair
 * of HIP events recorded on the call's stream (at most 4096 pairs per stage are
 * kept between two hps_stage_times calls; later ones are dropped).  Setting the
 * mask discards pairs recorded so far. */
hps_status hps_set_stage_timing(hps_table* t, uint32_t stage_mask);

/* Waits for the recorded events and adds up, per stage, the elapsed milliseconds
 * (h_ms_sum[HPS_N_STAGES]) and the number of pairs (h_count[HPS_N_STAGES]); the
 * recorded pairs are then discarded.  Host arrays. */
hps_status hps_stage_times(hps_table* t, double* h_ms_sum, uint32_t* h_count);

#ifdef __cplusplus
}
#endif
#endif /* HPS_MEASURE_H_ */
