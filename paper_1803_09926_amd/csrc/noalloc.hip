// Filter gradient for callers that cannot allocate device memory (code under HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc): the partial sums of the two-stage
// reduction live in a file-scope device array instead of a caller-supplied workspace.
#include "plan.hpp"
#include <mutex>

using namespace dwc;

// The array every call on a GPU shares.  Each GPU the library runs on holds its own copy, at its own
// address, until the process ends.  In host code the name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[DWCONV_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_lock;
void *g_scratch_ptr[MAX_DEVICES];   // device address of `scratch` on each device, looked up once per device

// Device address of the current device's copy of `scratch`; DWCONV_OK or DWCONV_ERR_LAUNCH.
int scratch_address(float **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return DWCONV_ERR_LAUNCH;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DWCONV_ERR_LAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *out = (float *)g_scratch_ptr[dev];
    return DWCONV_OK;
}

}  // namespace

extern "C" int dwconv_bwd_filter_noalloc(const dwconv_desc *desc, const void *x, const void *dy, void *dw, void *stream)
{
    Geom g;
    const int rc = validate_desc(desc, &g);
    if (rc != DWCONV_OK) return rc;
    if (!x || !dy || !dw) return DWCONV_ERR_NULL;
    if (((uintptr_t)x | (uintptr_t)dy | (uintptr_t)dw) & 15u) return DWCONV_ERR_ALIGN;
    const Plan pl = plan_bwd_filter(g, desc->layout, desc->dtype);
    const size_t need = (size_t)pl.parts * (size_t)g.O * g.K * g.K * sizeof(float);
    if (need > (size_t)DWCONV_NOALLOC_SCRATCH_BYTES) return DWCONV_ERR_SCRATCH;
    float *ws = nullptr;
    const int ra = scratch_address(&ws);
    if (ra != DWCONV_OK) return ra;
    // stage 1 writes every partial that stage 2 reads, so what an earlier call left in the array is never seen
    hipError_t e = launch_bwd_filter(pl, g, desc->layout, desc->dtype, x, dy, ws, (hipStream_t)stream);
    if (e != hipSuccess) return DWCONV_ERR_LAUNCH;
    e = reduce_partials(ws, pl.parts, g.O * g.K * g.K, (float *)dw, (hipStream_t)stream);
    return e == hipSuccess ? DWCONV_OK : DWCONV_ERR_LAUNCH;
}
