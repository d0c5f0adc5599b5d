// Kernel-variant selection.  A Plan is computed on the host from the geometry alone, so the
// workspace query and the launch always agree.
#pragma once
#include "../../include/dwconv.h"
#include "kernels.hpp"

namespace dwc {

enum Variant {
    V_GENERIC = 0,
    V_NHWC_S1,          // a = V, b = TH
    V_NHWC_K3S2,        // a = V, b = TH
    V_NHWC_BWD_FILTER,  // a = V, b = TH, c = NI
    V_NCHW_FWD,         // b = TR (forward, or backward-data with the filter rotated)
    V_NCHW_BWD_DATA_K3S2,  // b = TR
    V_NCHW_BWD_FILTER,  // b = TR, c = NI
    V_NCHWD_S1,         // a = V, b = TH
    V_NCHWD_K3S2,       // a = V, b = TH
    V_NCHWD_BWD_FILTER, // a = V, b = TH
    V_NCHWS_FWD,        // small planes: forward / backward-data stride 1 (rotated filter)
    V_NCHWS_BWD_DATA_S2,
    V_NCHWS_BWD_FILTER, // a = U, c = NI
    V_NHWC_BWD_FUSED,   // a = V, b = TH, c = NI (input gradient and filter gradient in one kernel)
    V_NCHWD_BWD_FUSED,  // a = V, b = TH
    V_NCHWS_BWD_FUSED,  // a = U, c = NI
};

struct Plan {
    int variant;
    int parts;         // bwd_filter: number of partial sums per dw element in the workspace
    int a, b, c;       // variant-specific launch parameters
    const char *name;
};

// Checks a descriptor on the host (no HIP call) and fills the geometry; returns a dwconv_status.
int validate_desc(const dwconv_desc *d, Geom *g);

Plan plan_fwd(const Geom &g, int layout, int dtype);
Plan plan_bwd_data(const Geom &g, int layout, int dtype);
Plan plan_bwd_filter(const Geom &g, int layout, int dtype);
// Whole backward pass (dx and dw).  V_GENERIC here means: no fused kernel, run the two passes one after the other.
Plan plan_bwd(const Geom &g, int layout, int dtype);

hipError_t launch_fwd(const Plan &pl, const Geom &g, int layout, int dtype, const void *x, const void *w, void *y,
                      hipStream_t st);
hipError_t launch_bwd_data(const Plan &pl, const Geom &g, int layout, int dtype, const void *dy, const void *w,
                           void *dx, hipStream_t st);
hipError_t launch_bwd_filter(const Plan &pl, const Geom &g, int layout, int dtype, const void *x, const void *dy,
                             float *ws, hipStream_t st);
hipError_t launch_bwd_fused(const Plan &pl, const Geom &g, int layout, int dtype, const void *x, const void *dy,
                            const void *w, void *dx, float *ws, hipStream_t st);

}  // namespace dwc
