#include "gconv.hpp"
namespace dwc {
bool gconv_nhwc_supported(const GGeom &) { return false; }
hipError_t gconv_nhwc_s1(const GGeom &, int, const void *, const void *, void *, bool, hipStream_t) { return hipErrorInvalidValue; }
int gconv_nhwc_bwd_filter_parts(const GGeom &) { return 0; }
hipError_t gconv_nhwc_bwd_filter(const GGeom &, int, const void *, const void *, float *, int, hipStream_t) { return hipErrorInvalidValue; }
}
