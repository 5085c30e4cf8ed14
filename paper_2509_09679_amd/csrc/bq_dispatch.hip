// Kernel selection: specialised kernels where one exists for the shape, generic kernels otherwise.
#include "bq_internal.h"

namespace bq {

hipError_t launch_transform(Mode mode, const void *in, void *out, const PlanView &pv, const Shape &s,
                            const QuantArgs *q, hipStream_t stream)
{
    if (k12_supported(mode, in, out, s, q)) {
        hipError_t e = launch_k12(mode, in, out, pv, s, q, stream);
        const int64_t done = (s.rows / k12_block_rows(s)) * k12_block_rows(s);
        if (e != hipSuccess || done == s.rows) return e;
        // rows that do not fill a block of the kernel: the generic kernel (rows are independent)
        const size_t isz = s.dtype == BQ_F32 ? 4 : 2;
        Shape t = s;
        t.rows = s.rows - done;
        const void *in_t = (const char *)in + (size_t)done * s.ld_x * isz;
        void *out_t = out ? (char *)out + (size_t)done * s.ld_y * isz : nullptr;
        QuantArgs qt;
        if (q) {
            qt = *q;
            if (q->codes) qt.codes = q->codes + (size_t)done * s.n * s.heads * q->bits / 8;
            if (q->scales) qt.scales = (char *)q->scales + (size_t)done * (s.n * s.heads / q->group) * (q->scale_f16 ? 2 : 4);
        }
        return launch_generic(mode, in_t, out_t, pv, t, q ? &qt : nullptr, stream);
    }
    if (small_supported(mode, in, out, s, q)) return launch_small(mode, in, out, pv, s, q, stream);
    return launch_generic(mode, in, out, pv, s, q, stream);
}

size_t bwd_workspace_bytes(const Shape &s)
{
    size_t need = bwd_workspace_bytes_generic(s);
    if (s.k >= 8 && s.k <= 13 && s.rows > 0 && (s.heads == 1 || (s.k < 12 && (int64_t)s.n * s.heads <= 4096))) {
        const size_t fast = bwd_fast_workspace_bytes(s);
        if (fast > need) need = fast;
    }
    if (s.k >= 3 && s.k <= 7 && s.rows > 0) {
        const size_t small = small_bwd_workspace_bytes(s);
        if (small > need) need = small;
    }
    return need;
}

hipError_t launch_bwd(const void *x, const void *dy, const PlanView &pv, void *dx, float *dtheta, void *ws,
                      const Shape &s, hipStream_t stream)
{
    if (!dtheta) {  // dx alone is the transposed transform of dy
        Shape t = s;
        return launch_transform(kInv, dy, dx, pv, t, nullptr, stream);
    }
    if (bwd_fast_supported(x, dy, dx, dtheta, s)) {
        hipError_t e = launch_bwd_fast(x, dy, pv, dx, dtheta, ws, s, stream);
        if (e != hipSuccess) return e;
        return launch_generic_bwd(x, dy, pv, dx, dtheta, ws, s, stream, /*only_if_bad=*/true);
    }
    if (small_bwd_supported(x, dy, dx, dtheta, s)) {
        hipError_t e = launch_small_bwd(x, dy, pv, dx, dtheta, ws, s, stream);
        if (e != hipSuccess) return e;
        return launch_generic_bwd(x, dy, pv, dx, dtheta, ws, s, stream, /*only_if_bad=*/true);
    }
    return launch_generic_bwd(x, dy, pv, dx, dtheta, ws, s, stream);
}

}  // namespace bq
