// Host-side launch entry points of every kernel family.  Each returns hipGetLastError() after
// the launch.  All pointers are device pointers; T-typed tensors are passed as void*.
#pragma once
#include "common.hpp"
#include "tune.hpp"
#include <stdio.h>
#include <stdlib.h>

namespace dwc {

enum { LAYOUT_NCHW = 0, LAYOUT_NHWC = 1 };

// Whether a kernel family writes its output with non-temporal stores.  `dflt_min_bytes` is the
// smallest output for which it does (negative: never).  In a tuning snapshot DWCONV_TUNE_NT=0/1
// overrides every family and DWCONV_TUNE_NT_<family>=0/1 one of them.
inline int stream_stores(const char *family, long long out_bytes, long long dflt_min_bytes = 64ll << 20)
{
    if (tune_active()) {
        char name[64];
        snprintf(name, sizeof name, "DWCONV_TUNE_NT_%s", family);
        const char *e = tune_env(name);
        if (e) return atoi(e) != 0;
        e = tune_env("DWCONV_TUNE_NT");
        if (e) return atoi(e) != 0;
    }
    return dflt_min_bytes >= 0 && out_bytes >= dflt_min_bytes;
}
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

// ---- NHWC row-walk kernels, multiplier 1 (nhwc.hip) ------------------------------------------
// V = channels per lane (4 for fp32; 8 or 4 for bf16), TH = rows per strip.
// stride 1, K in {3,5}, pad (K-1)/2; flip = true gives backward-data.
// PF = rows loaded ahead of the row being consumed.
hipError_t nhwc_s1(const Geom &g, int dtype, int V, const void *x, const void *w, void *y, bool flip, int TH, int PF,
                   hipStream_t st);
// 3x3 stride 2 pad 1; bwd = false: forward (in = x, out = y); bwd = true: backward-data (in = dy, out = dx).
hipError_t nhwc_k3s2(const Geom &g, int dtype, int V, const void *in, const void *w, void *out, bool bwd, int TH,
                     hipStream_t st);
// filter gradient stage 1; NI = images per block.
void nhwc_bwd_filter_tiling(const Geom &g, int V, int TH, int NI, int *CT, int *nctiles, int *nowtiles, int *nstrips,
                            int *ngroups);
// fused backward (input gradient + stage 1 of the filter gradient), 3x3 stride 1 (nhwc_fused.hip); tiling as nhwc_bwd_filter
bool nhwc_bwd_fused_supported(const Geom &g, int dtype, int V);
hipError_t nhwc_bwd_fused(const Geom &g, int dtype, int V, const void *x, const void *dy, const void *w, void *dx,
                          float *ws, int TH, int NI, hipStream_t st);
hipError_t nhwc_bwd_filter(const Geom &g, int dtype, int V, const void *x, const void *dy, float *ws, int TH, int NI,
                           hipStream_t st);
// bf16 stage 1 with packed two-row dot products (nhwc_dot2.hip); mapping and tiling of nhwc_bwd_filter
bool nhwc_bwd_filter_dot2_supported(const Geom &g, int V);
hipError_t nhwc_bwd_filter_dot2(const Geom &g, int V, const void *x, const void *dy, float *ws, int CT, int nctiles,
                                int nowtiles, int TH, int nstrips, int NI, unsigned nblocks, hipStream_t st);

// ---- NCHW LDS-tile kernels (nchw.hip) ----------------------------------------------------------
// TR = rows per unit.  K in {3,5}, stride in {1,2}, any pad, any multiplier for forward and the
// filter gradient; flip = true gives backward-data for stride 1, "same" padding, multiplier 1.
bool nchw_fwd_supported(const Geom &g, int TR);
hipError_t nchw_fwd(const Geom &g, int dtype, const void *x, const void *w, void *y, bool flip, int TR, hipStream_t st);
bool nchw_bwd_data_k3s2_supported(const Geom &g, int TR);
hipError_t nchw_bwd_data_k3s2(const Geom &g, int dtype, const void *dy, const void *w, void *dx, int TR, hipStream_t st);
int nchw_bwd_filter_parts(const Geom &g, int TR, int NI);   // 0 = unsupported
hipError_t nchw_bwd_filter(const Geom &g, int dtype, const void *x, const void *dy, float *ws, int TR, int NI,
                           hipStream_t st);

// ---- NCHW row-walk kernels for rows that are whole 16-byte vectors (nchw_direct.hip) -----------
// pass: 0 fwd, 1 bwd_data, 2 bwd_filter.  Returns the columns per lane, 0 if not applicable.
int nchwd_vec(const Geom &g, int dtype, int pass);
hipError_t nchwd_s1(const Geom &g, int dtype, int V, const void *x, const void *w, void *y, bool flip, int TH,
                    hipStream_t st);
hipError_t nchwd_k3s2(const Geom &g, int dtype, int V, const void *in, const void *w, void *out, bool bwd, int TH,
                      hipStream_t st);
void nchwd_bwd_filter_tiling(const Geom &g, int V, int TH, int *items_per_round, int *nstrips, int *rounds, int *parts);
// fused backward, 3x3 stride 1 fp32 (input gradient + stage 1 of the filter gradient); returns the row group (0: not applicable)
int nchwd_bwd_fused_rs(const Geom &g, int dtype, int V);
hipError_t nchwd_bwd_fused(const Geom &g, int dtype, int V, const void *x, const void *dy, const void *w, void *dx,
                           float *ws, int TH, hipStream_t st);
hipError_t nchwd_bwd_filter(const Geom &g, int dtype, int V, const void *x, const void *dy, float *ws, int TH,
                            hipStream_t st);

// ---- NCHW small-plane kernels: rows of 7, 14 or 28 elements, 3x3 pad 1, multiplier 1 (nchw_small.hip)
bool nchws_supported(const Geom &g, int pass);
hipError_t nchws_fwd(const Geom &g, int dtype, const void *x, const void *w, void *y, bool flip, hipStream_t st);
hipError_t nchws_bwd_data_s2(const Geom &g, int dtype, const void *dy, const void *w, void *dx, hipStream_t st);
// group convolution with cg channels per group on both sides through the same forward kernel (filter [O][cg][3][3])
bool nchws_group_supported(const Geom &g, int cg);
hipError_t nchws_group_fwd(const Geom &g, int cg, int dtype, const void *x, const void *w, void *y, bool flip, hipStream_t st);
hipError_t nchws_group_bwd_data_s2(const Geom &g, int cg, int dtype, const void *dy, const void *w, void *dx, hipStream_t st);
void nchws_bwd_filter_tiling(const Geom &g, int dtype, int *U, int *NI, int *parts, int cg = 1);
hipError_t nchws_group_bwd_filter(const Geom &g, int cg, int dtype, const void *x, const void *dy, float *ws, int U, int NI,
                                  hipStream_t st);
// fused backward on small planes (3x3 stride 1): x and dy staged in LDS once for both gradients
bool nchws_bwd_fused_supported(const Geom &g);
void nchws_bwd_fused_tiling(const Geom &g, int dtype, int *U, int *NI, int *parts);
hipError_t nchws_bwd_fused(const Geom &g, int dtype, const void *x, const void *dy, const void *w, void *dx, float *ws,
                           int U, int NI, hipStream_t st);
hipError_t nchws_bwd_filter(const Geom &g, int dtype, const void *x, const void *dy, float *ws, int U, int NI,
                            hipStream_t st);

}  // namespace dwc
