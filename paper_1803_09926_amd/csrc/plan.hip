// Variant selection and launch dispatch.
#include "plan.hpp"

namespace dwc {

Plan plan_fwd(const Geom &g, int layout, int dtype)
{
    Plan pl = {V_GENERIC, 0, 0, 0, 0, "generic"};
    return pl;
}

Plan plan_bwd_data(const Geom &g, int layout, int dtype)
{
    Plan pl = {V_GENERIC, 0, 0, 0, 0, "generic"};
    return pl;
}

Plan plan_bwd_filter(const Geom &g, int layout, int dtype)
{
    Plan pl = {V_GENERIC, generic_bwd_filter_parts(g), 0, 0, 0, "generic"};
    return pl;
}

hipError_t launch_fwd(const Plan &pl, const Geom &g, int layout, int dtype, const void *x, const void *w, void *y,
                      hipStream_t st)
{
    switch (pl.variant) {
    default: return generic_fwd(g, layout, dtype, x, w, y, st);
    }
}

hipError_t launch_bwd_data(const Plan &pl, const Geom &g, int layout, int dtype, const void *dy, const void *w,
                           void *dx, hipStream_t st)
{
    switch (pl.variant) {
    default: return generic_bwd_data(g, layout, dtype, dy, w, dx, st);
    }
}

hipError_t launch_bwd_filter(const Plan &pl, const Geom &g, int layout, int dtype, const void *x, const void *dy,
                             float *ws, hipStream_t st)
{
    switch (pl.variant) {
    default: return generic_bwd_filter(g, layout, dtype, x, dy, ws, pl.parts, st);
    }
}

}  // namespace dwc
