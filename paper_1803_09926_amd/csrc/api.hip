// C ABI of the library: argument validation (host only, before any HIP call), kernel-variant
// selection, launches.  See include/dwconv.h for the contract.
#include "../../include/dwconv.h"
#include "kernels.hpp"
#include "plan.hpp"

using namespace dwc;

namespace dwc {
int validate_desc(const dwconv_desc *d, Geom *g)
{
    if (!d) return DWCONV_ERR_NULL;
    if (d->layout != DWCONV_NCHW && d->layout != DWCONV_NHWC) return DWCONV_ERR_BAD_ENUM;
    if (d->dtype != DWCONV_F32 && d->dtype != DWCONV_BF16) return DWCONV_ERR_BAD_ENUM;
    if (d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->K < 1 || d->stride < 1 || d->pad < 0 || d->mult < 1)
        return DWCONV_ERR_BAD_DIM;
    if (d->K > DWCONV_MAX_K) return DWCONV_ERR_UNSUPPORTED;
    const long long sh = (long long)d->H + 2ll * d->pad - d->K, sw = (long long)d->W + 2ll * d->pad - d->K;
    if (sh < 0 || sw < 0) return DWCONV_ERR_BAD_DIM;
    const long long Ho = sh / d->stride + 1, Wo = sw / d->stride + 1;
    const long long O = (long long)d->C * d->mult;
    const long long lim = 1ll << 31;
    // 32-bit indexing: every tensor, and the padded extents the kernels form, must stay below 2^31
    if (O >= lim || (long long)d->pad >= (1 << 20) ||
        (long long)d->N * d->C * d->H * d->W >= lim || (long long)d->N * O * Ho * Wo >= lim ||
        O * d->K * d->K >= lim)
        return DWCONV_ERR_TOO_LARGE;
    if (g) {
        g->N = d->N; g->C = d->C; g->H = d->H; g->W = d->W;
        g->K = d->K; g->s = d->stride; g->p = d->pad; g->m = d->mult;
        g->O = (int)O; g->Ho = (int)Ho; g->Wo = (int)Wo;
    }
    return DWCONV_OK;
}
}  // namespace dwc

static inline int validate(const dwconv_desc *d, Geom *g) { return validate_desc(d, g); }

static inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

extern "C" {

int dwconv_out_dims(const dwconv_desc *desc, int32_t *Ho, int32_t *Wo)
{
    Geom g;
    int rc = validate(desc, &g);
    if (rc != DWCONV_OK) return rc;
    if (Ho) *Ho = g.Ho;
    if (Wo) *Wo = g.Wo;
    return DWCONV_OK;
}

size_t dwconv_bwd_filter_workspace_bytes(const dwconv_desc *desc)
{
    Geom g;
    if (validate(desc, &g) != DWCONV_OK) return 0;
    Plan pl = plan_bwd_filter(g, desc->layout, desc->dtype);
    return (size_t)pl.parts * (size_t)g.O * g.K * g.K * sizeof(float);
}

int dwconv_fwd(const dwconv_desc *desc, const void *x, const void *w, void *y, void *stream)
{
    Geom g;
    int rc = validate(desc, &g);
    if (rc != DWCONV_OK) return rc;
    if (!x || !w || !y) return DWCONV_ERR_NULL;
    if (misaligned(x) || misaligned(w) || misaligned(y)) return DWCONV_ERR_ALIGN;
    Plan pl = plan_fwd(g, desc->layout, desc->dtype);
    hipError_t e = launch_fwd(pl, g, desc->layout, desc->dtype, x, w, y, (hipStream_t)stream);
    return e == hipSuccess ? DWCONV_OK : DWCONV_ERR_LAUNCH;
}

int dwconv_bwd_data(const dwconv_desc *desc, const void *dy, const void *w, void *dx, void *stream)
{
    Geom g;
    int rc = validate(desc, &g);
    if (rc != DWCONV_OK) return rc;
    if (!dy || !w || !dx) return DWCONV_ERR_NULL;
    if (misaligned(dy) || misaligned(w) || misaligned(dx)) return DWCONV_ERR_ALIGN;
    Plan pl = plan_bwd_data(g, desc->layout, desc->dtype);
    hipError_t e = launch_bwd_data(pl, g, desc->layout, desc->dtype, dy, w, dx, (hipStream_t)stream);
    return e == hipSuccess ? DWCONV_OK : DWCONV_ERR_LAUNCH;
}

int dwconv_bwd_filter(const dwconv_desc *desc, const void *x, const void *dy, void *dw, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    Geom g;
    int rc = validate(desc, &g);
    if (rc != DWCONV_OK) return rc;
    if (!x || !dy || !dw) return DWCONV_ERR_NULL;
    if (misaligned(x) || misaligned(dy) || misaligned(dw)) return DWCONV_ERR_ALIGN;
    Plan pl = plan_bwd_filter(g, desc->layout, desc->dtype);
    const size_t need = (size_t)pl.parts * (size_t)g.O * g.K * g.K * sizeof(float);
    if (!workspace || workspace_bytes < need) return DWCONV_ERR_WORKSPACE;
    if (misaligned(workspace)) return DWCONV_ERR_ALIGN;
    hipError_t e = launch_bwd_filter(pl, g, desc->layout, desc->dtype, x, dy, (float *)workspace, (hipStream_t)stream);
    if (e != hipSuccess) return DWCONV_ERR_LAUNCH;
    e = reduce_partials((const float *)workspace, pl.parts, g.O * g.K * g.K, (float *)dw, (hipStream_t)stream);
    return e == hipSuccess ? DWCONV_OK : DWCONV_ERR_LAUNCH;
}

const char *dwconv_status_string(int status)
{
    switch (status) {
    case DWCONV_OK: return "ok";
    case DWCONV_ERR_NULL: return "null pointer";
    case DWCONV_ERR_BAD_DIM: return "bad dimension (N,C,H,W,K,stride,mult must be >= 1, pad >= 0, output non-empty)";
    case DWCONV_ERR_BAD_ENUM: return "bad layout or dtype";
    case DWCONV_ERR_WORKSPACE: return "bwd_filter workspace missing or too small";
    case DWCONV_ERR_ALIGN: return "pointer not 16-byte aligned";
    case DWCONV_ERR_UNSUPPORTED: return "unsupported (K larger than DWCONV_MAX_K)";
    case DWCONV_ERR_LAUNCH: return "HIP kernel launch failed";
    case DWCONV_ERR_TOO_LARGE: return "tensor has 2^31 or more elements";
    case DWCONV_ERR_SCRATCH: return "shape needs more scratch than the library's static buffer holds (use dwconv_bwd_filter with a workspace)";
    default: return "unknown status";
    }
}

size_t dwconv_bwd_workspace_bytes(const dwconv_desc *desc)
{
    Geom g;
    if (validate(desc, &g) != DWCONV_OK) return 0;
    Plan pl = plan_bwd(g, desc->layout, desc->dtype);
    if (pl.variant == V_GENERIC) pl = plan_bwd_filter(g, desc->layout, desc->dtype);
    return (size_t)pl.parts * (size_t)g.O * g.K * g.K * sizeof(float);
}

int dwconv_bwd(const dwconv_desc *desc, const void *x, const void *dy, const void *w, void *dx, void *dw,
               void *workspace, size_t workspace_bytes, void *stream)
{
    Geom g;
    int rc = validate(desc, &g);
    if (rc != DWCONV_OK) return rc;
    if (!x || !dy || !w || !dx || !dw) return DWCONV_ERR_NULL;
    if (misaligned(x) || misaligned(dy) || misaligned(w) || misaligned(dx) || misaligned(dw)) return DWCONV_ERR_ALIGN;
    const Plan pl = plan_bwd(g, desc->layout, desc->dtype);
    if (pl.variant == V_GENERIC) {
        // no fused kernel for this shape: the two passes, filter gradient first (the input gradient
        // then finds dy in cache)
        rc = dwconv_bwd_filter(desc, x, dy, dw, workspace, workspace_bytes, stream);
        if (rc != DWCONV_OK) return rc;
        return dwconv_bwd_data(desc, dy, w, dx, stream);
    }
    const size_t need = (size_t)pl.parts * (size_t)g.O * g.K * g.K * sizeof(float);
    if (!workspace || workspace_bytes < need) return DWCONV_ERR_WORKSPACE;
    if (misaligned(workspace)) return DWCONV_ERR_ALIGN;
    hipError_t e = launch_bwd_fused(pl, g, desc->layout, desc->dtype, x, dy, w, dx, (float *)workspace, (hipStream_t)stream);
    if (e != hipSuccess) return DWCONV_ERR_LAUNCH;
    e = reduce_partials((const float *)workspace, pl.parts, g.O * g.K * g.K, (float *)dw, (hipStream_t)stream);
    return e == hipSuccess ? DWCONV_OK : DWCONV_ERR_LAUNCH;
}

int dwconv_tuning_reload(void) { return tune_reload(); }

const char *dwconv_variant_name(const dwconv_desc *desc, int pass)
{
    Geom g;
    if (validate(desc, &g) != DWCONV_OK || pass < 0 || pass > 3) return "invalid";
    Plan pl = pass == 0 ? plan_fwd(g, desc->layout, desc->dtype)
            : pass == 1 ? plan_bwd_data(g, desc->layout, desc->dtype)
            : pass == 2 ? plan_bwd_filter(g, desc->layout, desc->dtype)
                        : plan_bwd(g, desc->layout, desc->dtype);
    return pl.name;
}

}  // extern "C"
