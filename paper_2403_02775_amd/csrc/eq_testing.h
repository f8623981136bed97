/*
 * eq_testing.h -- hooks of libeasyquant.so for its own tests and measurements.
 *
 * These symbols are exported by the library but are NOT part of its C ABI (include/easyquant.h):
 * they may change with the kernels.  Nothing here changes a result: the overrides only change
 * which of several equivalent kernels serves a matrix or how the rows are cut into work items
 * (the two that concern the sorted evaluation also change what eq_workspace_bytes() returns: size
 * the workspace under the setting the call will run with).
 */
#ifndef EQ_TESTING_H_
#define EQ_TESTING_H_

#include "easyquant.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Kernel-selection overrides, process-wide, 0 = the library's own choice (the default). */
enum {
  EQ_OVR_UNITS_PER_ITEM = 0, /* n > 0: units a workgroup walks through (how the work is cut up) */
  EQ_OVR_FORCE_GENERAL = 1,  /* 1: every matrix goes to the general kernel */
  EQ_OVR_RTN_THREADS = 2,    /* 128 | 256 | 512: workgroup size of the kernel without optimisation steps
                                (128 only for rows of up to 8192 columns, 512 only for longer ones) */
  EQ_OVR_CHANNEL_KERNEL = 3, /* 128: per-channel rows stay on the kernel with 128-element segments
                                where another one would serve them */
  EQ_OVR_MATVEC_ARITHMETIC = 4, /* 1: eq_dequant_matvec takes the plain arithmetic for grouped 4-bit
                                   codes instead of the per-group tables (same weights either way) */
  EQ_OVR_MATVEC_LOOKUP = 5,  /* eq_dequant_matvec, 4-bit codes with one range per row: 1 = half of the pairs of
                                weights from the table of pairs and half from the table of single values,
                                2 = all from the table of single values (default: all from the table of pairs) */
  EQ_OVR_SORTED_ROWS = 6,    /* rows with one range each and at most 4 bits: 1 = always optimised element by element
                                (the per-channel lane kernels), 2 = from their sorted values whatever the number of
                                steps (default: when steps x (columns - 960) >= 57 x columns) */
  EQ_OVR_SORT_CHUNK_ROWS = 7, /* n > 0: at most n rows (rounded down to a multiple of 4) per chunk of the sorted
                                 evaluation, instead of as many as 2 GiB of records hold */
  EQ_OVR_CLASS_STREAMS = 8,  /* the row-length classes of a batch alternate between the caller's stream and the
                                library's second one, so that their main kernels run side by side: 1 = never,
                                2 = whenever the batch has two classes (default: without optimisation steps) */
  EQ_OVR_COUNT = 9
};
EQ_API int eq_test_set_override(int which, int64_t value);   /* EQ_OK or EQ_E_PARAM */

/* The launch plan of eq_quantize_batch for these shapes (host only, no GPU): writes up to
 * max_items work items, five numbers each, into `items` and returns the number of items of the
 * plan (which may exceed max_items), or a negative EQ_E_* code.  An item is (matrix, first row,
 * rows, stride, step): the workgroup takes rows [first, first + rows) of the matrix, all of them
 * when stride == 0, else the `step` rows at first, first + stride, first + 2 stride, ...
 * Matrices that the general kernel serves (one workgroup per row) have no items.
 * `launch_of_item`, if not NULL, receives for each written item the index of the launch
 * (row-length class) it belongs to. */
EQ_API int64_t eq_test_plan_items(int32_t n, const int64_t* rows, const int64_t* cols, const int64_t* out_capacity,
                                  const eq_params* p, int32_t* items, int32_t* launch_of_item, int64_t max_items);

/* The chunks of the sorted evaluation of rows with one range each for these shapes (host only):
 * writes up to max_segs segments, seven numbers each, into `segs` and returns the number of
 * segments of the plan, or a negative EQ_E_* code.  A segment is (chunk, matrix, first row, rows,
 * index of its first group of 4 rows in the chunk, index of its first row in the chunk, byte offset
 * of its first record in the chunk's region of the workspace): a run of rows of one matrix whose
 * records lie one after the other.  `record_region_bytes`, if not NULL, receives the size of that
 * region (the largest chunk). */
EQ_API int64_t eq_test_plan_sort_segments(int32_t n, const int64_t* rows, const int64_t* cols, const int64_t* out_capacity,
                                          const eq_params* p, int64_t* segs, int64_t max_segs, int64_t* record_region_bytes);

/* The library divides by values whose correctly rounded reciprocal it knows (Adam's bias
 * corrections, the level count D) with a short multiply-add sequence instead of a hardware
 * division.  These run that same sequence on the host so that a test can confirm it returns the
 * IEEE quotient a / b bit for bit. */
EQ_API double eq_test_div_f64(double a, double b);
EQ_API float eq_test_div_f32(float a, float b);

#ifdef __cplusplus
}
#endif
#endif /* EQ_TESTING_H_ */
