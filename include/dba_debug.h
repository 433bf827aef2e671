/*
 * libdba - diagnostics.  Not part of the decoding boundary (include/dba.h): these calls run pieces of
 * the device code in isolation so that tests and benchmarks can check or time them.
 */
#ifndef DBA_DEBUG_H
#define DBA_DEBUG_H

#include "dba.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Diagnostic: runs the device-side bank allocation of Sec. 3.2 alone, on one
 * wavefront, for n_cases independent problems (adjust = 0: without the adjustment, Sec. 5).
 *   k_host [n_cases], C_host [n_cases] (0..64), cnt_host [n_cases][65] candidates per bank,
 *   alloc_host [n_cases][65] receives the slots per bank.  All host pointers; the call
 * stages them through `scratch_dev` (device, >= n_cases*132*4 bytes) on `hip_stream`
 * and synchronises.
 */
DBA_API int dba_debug_allocate(int n_cases, int adjust, const int32_t *k_host, const int32_t *C_host,
                       const int32_t *cnt_host, int32_t *alloc_host, void *scratch_dev,
                       size_t scratch_bytes, void *hip_stream);

/*
 * Diagnostic: runs the wavefront selection primitives the stream phase is built from
 * (64-lane sort, merge of two sorted lists, single insert) on caller data, one
 * wavefront per case, so that they can be checked against a host sort.
 *   keys_host [n_cases][128] distinct non-zero 64-bit keys, vals_host [n_cases][64] floats,
 *   out_host [n_cases][256]: sorted keys[0:64] | top 64 of all 128, sorted | sorted keys[0:64]
 *   after inserting keys[64..71] | low word: the 64 greatest of the 128 high words (merged as
 *   32-bit keys, equal ones allowed), high word: the greatest high word that was left out;
 *   fout_host [n_cases][64]: vals sorted.  All decreasing.
 * Host pointers; staged through scratch_dev (device, >= n_cases*3584 bytes); synchronises.
 */
DBA_API int dba_debug_wave_select(int n_cases, const uint64_t *keys_host, const float *vals_host,
                                  uint64_t *out_host, float *fout_host, void *scratch_dev,
                                  size_t scratch_bytes, void *hip_stream);

/*
 * Diagnostic: the reference read.  out_max_dev[r] = largest of the V floats of row r of
 * src_dev [rows, V] (device, 16-byte aligned, V a multiple of 4), one workgroup per row,
 * with the loads and the tile order of the step's streaming phase and no other work.  The
 * step of Alg. 2 has to read its [B,k,V] scores once (Sec. 3.1: the k x V matrix is the
 * input); this kernel's duration is what the device needs for that read alone, so a
 * benchmark can state the step's time as a multiple of it.  Asynchronous on hip_stream;
 * out_max_dev is device memory of `rows` floats owned by the caller.
 */
DBA_API int dba_debug_row_max(const float *src_dev, int rows, int V, float *out_max_dev,
                              void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DBA_DEBUG_H */
