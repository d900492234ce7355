/*
 * Measurement aids of the CSB-RNN library (csbrnn.h).  NOT operations of the method and not
 * part of the stable interface: bench.py and the tests use them to produce the load-balance and
 * bandwidth figures that are reported next to the kernels' timings.  Same conventions as
 * csbrnn.h (device pointers, 0 on success, csb_last_error()).
 */
#ifndef CSBRNN_DEBUG_H
#define CSBRNN_DEBUG_H

#include "csbrnn.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * csb_spmv with clock stamps, for load-balance evidence: same result, and every wavefront also
 * writes stamps to d_stamps (device, csb_debug_stamp_count(m) values of 64 bits).
 * Row-owned layout: per workgroup and wavefront 8 values of the 100 MHz wall clock: start, input
 * vector staged (after the barrier), first segment unit in LDS (twice), products done, after
 * the last barrier, end, one unused.  Tile-based layout: per workgroup 8 phase stamps of the
 * shader clock (start, loads issued, staged in LDS, mat-vec done, tile sums written, end, 2
 * unused), then three for each of its 16 wavefronts: begin of its share, its kernel values
 * arrived, end of the share.  d_ws as for csb_spmv.
 */
size_t csb_debug_stamp_count(const csb_matrix *m);
int csb_debug_spmv_stamps(const csb_matrix *m, const float *d_x, float *d_y, void *d_ws,
                          unsigned long long *d_stamps, void *stream);

/*
 * A plain streaming read of d_buf (device, 16-byte aligned, `bytes` a multiple of 16) whose
 * timing gives the read bandwidth this GPU reaches in practice for a launch of that size.
 * Every thread writes its partial sum to d_out (device, csb_debug_stream_read_out_floats()
 * floats).  Asynchronous on `stream`.
 */
size_t csb_debug_stream_read_out_floats(void);
int csb_debug_stream_read(const void *d_buf, size_t bytes, float *d_out, void *stream);

#ifdef __cplusplus
}
#endif

#endif
