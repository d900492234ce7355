// Internal entry points between the translation units of the library.
#pragma once

#include <hip/hip_runtime.h>

#include "csb_internal.hpp"

namespace csb {

// y = A [x0[0..n0) ; x1[0..cols-n0)] on `stream`; y has the image's rows_out entries.
int spmv_segments(const csb_matrix *m, const float *d_x0, uint32_t n0, const float *d_x1, float *d_y,
                  void *d_ws, void *stream, unsigned long long *d_stamps = nullptr);

// Y = A Z for `batch` right-hand sides.  Element (column j, right-hand side n) of Z is
// p0[j*sj0 + n*sn0] for j < n0 and p1[(j-n0)*sj1 + n*sn1] otherwise; Y is [rows_out][ldy].
int spmm_strided(const csb_matrix *mat, const float *p0, uint32_t n0, int64_t sj0, int64_t sn0, const float *p1,
                 int64_t sj1, int64_t sn1, float *d_Y, int64_t ldy, int32_t batch, void *stream);

// Raises a kernel's limit of dynamic LDS on the current device to `bytes` if it is below it.
// (The limit sticks to the kernel; setting it is a runtime call of its own, too slow to repeat
// before every launch of a path that launches a kernel per timestep.)
hipError_t ensure_dynamic_lds(const void *kernel, size_t bytes);

}  // namespace csb
