// Group convolution (more than one channel per group): geometry and host-side launch entry points.
#pragma once
#include "kernels.hpp"

namespace dwc {

struct GGeom {
    int N, C, H, W;     // input dims
    int K, s, p;        // filter size, stride, pad
    int G, O;           // groups, output channels
    int Cg, Og;         // input / output channels per group
    int Ho, Wo;
};

enum GVariant { GV_GENERIC = 0, GV_NCHW_K3S1, GV_NHWC_K3S1, GV_NCHWS_K3S1, GV_NHWC_MFMA_S2, GV_NHWC_BWD_FILTER_S2, GV_NCHWS_MFMA_BWD_FILTER, GV_NCHWS_MFMA_FWD, GV_NHWC_LDS_MFMA_BWD_FILTER, GV_NHWC_TR_BWD_FILTER };

struct GPlan {
    int variant;
    int parts;          // bwd_filter: partial sums per weight entry
    int a, b, c;        // variant-specific tiling
    const char *name;
};

// ---- generic kernels: any K, stride, pad, group size, both layouts (gconv.hip) ---------------------
hipError_t gconv_generic_fwd(const GGeom &g, int layout, int dtype, const void *x, const void *w, void *y, hipStream_t st);
hipError_t gconv_generic_bwd_data(const GGeom &g, int layout, int dtype, const void *dy, const void *w, void *dx,
                                  hipStream_t st);
int gconv_generic_bwd_filter_parts(const GGeom &g);
hipError_t gconv_generic_bwd_filter(const GGeom &g, int layout, int dtype, const void *x, const void *dy, float *ws,
                                    int parts, hipStream_t st);

// ---- NCHW row-walk kernels, 3x3 stride 1 pad 1, 2, 4 or 8 channels per group on both sides (gconv_nchw.hip)
bool gconv_nchw_supported(const GGeom &g);
// flip = false: forward (in = x, out = y); flip = true: backward-data (in = dy, out = dx)
hipError_t gconv_nchw_s1(const GGeom &g, int dtype, const void *in, const void *w, void *out, bool flip, hipStream_t st);
int gconv_nchw_bwd_filter_parts(const GGeom &g);
hipError_t gconv_nchw_bwd_filter(const GGeom &g, int dtype, const void *x, const void *dy, float *ws, int parts,
                                 hipStream_t st);

// ---- NCHW filter gradient on the matrix cores: 3x3 stride 1 pad 1, 4 or 8 channels per group on both sides, 28x28
// or 56x56 planes (gconv_nchw_mfma.hip); nhwc: the same kernel fed from NHWC tensors (28x28 and 56x56), the channels
// scattered to planes on their way into LDS
bool gconv_nchws_mfma_bwd_filter_supported(const GGeom &g, int dtype, bool nhwc);
int gconv_nchws_mfma_bwd_filter_parts(const GGeom &g, int dtype);
hipError_t gconv_nchws_mfma_bwd_filter(const GGeom &g, int dtype, bool nhwc, const void *x, const void *dy, float *ws, int parts,
                                       hipStream_t st);
// forward (flip = false) and backward-data (flip = true) of the same shapes (gconv_nchw_mfma_fwd.hip)
bool gconv_nchws_mfma_fwd_supported(const GGeom &g);
hipError_t gconv_nchws_mfma_fwd(const GGeom &g, int dtype, const void *in, const void *w, void *out, bool flip, hipStream_t st);

// ---- NHWC row-walk kernels, same shapes (gconv_nhwc.hip) ----------------------------------------------
bool gconv_nhwc_supported(const GGeom &g);
hipError_t gconv_nhwc_s1(const GGeom &g, int dtype, const void *in, const void *w, void *out, bool flip, hipStream_t st);
int gconv_nhwc_bwd_filter_parts(const GGeom &g, int dtype);
hipError_t gconv_nhwc_bwd_filter(const GGeom &g, int dtype, const void *x, const void *dy, float *ws, int parts,
                                 hipStream_t st);

// ---- NHWC lane-exchange walk: 4 or 8 channels per group on both sides (gconv_nhwc_xchg.hip); gconv_nhwc_s1
// forwards to it where it applies
bool gconv_nhwc_xchg_supported(const GGeom &g);
hipError_t gconv_nhwc_xchg_s1(const GGeom &g, int dtype, const void *in, const void *w, void *out, bool flip, hipStream_t st);
// filter gradient, stage 1: the tiling comes from gconv_nhwc_bwd_filter (one channel per lane)
hipError_t gconv_nhwc_xchg_bwd_filter(const GGeom &g, int dtype, const void *x, const void *dy, float *ws, int CT, int nctiles,
                                      int nowtiles, int TH, int nstrips, int NI, unsigned nblocks, int J, hipStream_t st);

// ---- NHWC on the matrix cores: 4 or 8 channels per group on both sides, channels a multiple of 64 (bf16: 128)
// (gconv_nhwc_mfma.hip); gconv_nhwc_s1 forwards to it where it applies
bool gconv_nhwc_mfma_supported(const GGeom &g, int dtype);
hipError_t gconv_nhwc_mfma_s1(const GGeom &g, int dtype, const void *in, const void *w, void *out, bool flip, hipStream_t st);

// ---- NHWC filter gradient on the matrix cores, 4x4 tiles transposed in registers: 3x3 stride 1 pad 1, groups of 4 or 8
// on both sides, channels a multiple of 64 (bf16: 128) (gconv_nhwc_tr.hip)
bool gconv_nhwc_tr_bwd_filter_supported(const GGeom &g, int dtype);
int gconv_nhwc_tr_bwd_filter_parts(const GGeom &g, int dtype);
hipError_t gconv_nhwc_tr_bwd_filter(const GGeom &g, int dtype, const void *x, const void *dy, float *ws, int parts, hipStream_t st);

// ---- NHWC 3x3 stride 2 pad 1 on the matrix cores, same group sizes and channel counts: forward (pass 0) and
// backward-data (pass 1, even H and W) (gconv_nhwc_mfma_s2.hip)
// filter gradient at stride 2, groups of 4 or 8 on both sides, any channel count (gconv_nhwc_xchg.hip)
bool gconv_nhwc_bwd_filter_s2_supported(const GGeom &g);
int gconv_nhwc_bwd_filter_s2_parts(const GGeom &g);
hipError_t gconv_nhwc_bwd_filter_s2(const GGeom &g, int dtype, const void *x, const void *dy, float *ws, int parts, hipStream_t st);
bool gconv_nhwc_mfma_s2_supported(const GGeom &g, int dtype, int pass);
hipError_t gconv_nhwc_mfma_s2(const GGeom &g, int dtype, const void *in, const void *w, void *out, bool bwd, hipStream_t st);

}  // namespace dwc
