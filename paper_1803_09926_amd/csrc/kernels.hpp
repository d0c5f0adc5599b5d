// Host-side launch entry points of every kernel family.  Each returns hipGetLastError() after
// the launch.  All pointers are device pointers; T-typed tensors are passed as void*.
#pragma once
#include "common.hpp"

namespace dwc {

enum { LAYOUT_NCHW = 0, LAYOUT_NHWC = 1 };
enum { DT_F32 = 0, DT_BF16 = 1 };

// ---- generic fallback: any K, stride, pad, multiplier (generic.hip) -------------------------
hipError_t generic_fwd(const Geom &g, int layout, int dtype, const void *x, const void *w, void *y,
                       hipStream_t st);
hipError_t generic_bwd_data(const Geom &g, int layout, int dtype, const void *dy, const void *w, void *dx,
                            hipStream_t st);
int generic_bwd_filter_parts(const Geom &g);
hipError_t generic_bwd_filter(const Geom &g, int layout, int dtype, const void *x, const void *dy,
                              float *ws, int parts, hipStream_t st);

// ---- second stage of the filter-gradient reduction (generic.hip) ----------------------------
// dw[j] = sum_{p < parts} ws[p*J + j], j < J, added in a fixed order.
hipError_t reduce_partials(const float *ws, int parts, int J, float *dw, hipStream_t st);

}  // namespace dwc
