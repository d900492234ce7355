// Internal entry points between the translation units of the library.
#pragma once

#include "csb_internal.hpp"

namespace csb {

// y = A [x0[0..n0) ; x1[0..cols-n0)] on `stream`; y has the image's rows_out entries.
int spmv_segments(const csb_matrix *m, const float *d_x0, uint32_t n0, const float *d_x1, float *d_y,
                  void *d_ws, void *stream, unsigned long long *d_stamps = nullptr);

}  // namespace csb
