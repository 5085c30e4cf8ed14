// Kernel selection: specialised kernels where one exists for the shape, generic kernels otherwise.
#include "bq_internal.h"

namespace bq {

hipError_t launch_transform(Mode mode, const void *in, void *out, const PlanView &pv, const Shape &s,
                            const QuantArgs *q, hipStream_t stream)
{
    if (k12_supported(mode, in, out, s, q)) return launch_k12(mode, in, out, pv, s, q, stream);
    if (small_supported(mode, in, out, s, q)) return launch_small(mode, in, out, pv, s, q, stream);
    return launch_generic(mode, in, out, pv, s, q, stream);
}

size_t bwd_workspace_bytes(const Shape &s) { return bwd_workspace_bytes_generic(s); }

hipError_t launch_bwd(const void *x, const void *dy, const PlanView &pv, void *dx, float *dtheta, void *ws,
                      const Shape &s, hipStream_t stream)
{
    return launch_generic_bwd(x, dy, pv, dx, dtheta, ws, s, stream);
}

}  // namespace bq
