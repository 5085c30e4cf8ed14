// C ABI of libbq: argument validation and dispatch.  No transform kernels here; the only device objects of
// this file are the fixed scratch array of bq_butterfly_bwd_static and a fill kernel.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "bq_internal.h"

namespace {

thread_local char g_err[512] = "";

bq_status fail(bq_status s, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return s;
}

bq_status ok()
{
    g_err[0] = '\0';
    return BQ_OK;
}

int itemsize(int dtype) { return dtype == BQ_F32 ? 4 : 2; }

bool misaligned(const void *p, size_t a) { return ((uintptr_t)p % a) != 0; }

// Validates a bq_rows descriptor and converts it.
bq_status check_rows(const bq_rows *r, bq::Shape *s, const char *who)
{
    if (!r) return fail(BQ_ERR_NULL, "%s: rows descriptor is NULL", who);
    if (r->dtype != BQ_F32 && r->dtype != BQ_F16 && r->dtype != BQ_BF16)
        return fail(BQ_ERR_DTYPE, "%s: unknown dtype %d", who, (int)r->dtype);
    int k = bq::ilog2_exact(r->n);
    if (k < 0 || r->n > 16384) return fail(BQ_ERR_SHAPE, "%s: n=%d is not a power of two in [2, 16384]", who, r->n);
    if (r->heads < 1) return fail(BQ_ERR_SHAPE, "%s: heads=%d < 1", who, r->heads);
    if (r->rows < 0) return fail(BQ_ERR_SHAPE, "%s: rows=%lld < 0", who, (long long)r->rows);
    int64_t w = (int64_t)r->n * r->heads;
    if (w > (int64_t)1 << 24) return fail(BQ_ERR_SHAPE, "%s: row width %lld too large", who, (long long)w);
    if (r->ld_x < w || r->ld_y < w)
        return fail(BQ_ERR_SHAPE, "%s: leading dimensions (%lld, %lld) smaller than the row width %lld", who,
                    (long long)r->ld_x, (long long)r->ld_y, (long long)w);
    if (r->rows > 0 && r->rows > ((int64_t)1 << 40) / w) return fail(BQ_ERR_SHAPE, "%s: batch too large", who);
    const int64_t ld_max = r->ld_x > r->ld_y ? r->ld_x : r->ld_y;  // byte offsets of the last row must fit 64 bits
    if (r->rows > 0 && ld_max > ((int64_t)1 << 44) / r->rows)
        return fail(BQ_ERR_SHAPE, "%s: rows * leading dimension exceeds 2^44 elements", who);
    s->rows = r->rows;
    s->n = r->n;
    s->heads = r->heads;
    s->k = k;
    s->ld_x = r->ld_x;
    s->ld_y = r->ld_y;
    s->dtype = r->dtype;
    return BQ_OK;
}

bq_status check_plan(const void *plan, const char *who)
{
    if (!plan) return fail(BQ_ERR_NULL, "%s: plan is NULL", who);
    if (misaligned(plan, 256)) return fail(BQ_ERR_ALIGN, "%s: plan must be aligned to 256 bytes", who);
    return BQ_OK;
}

bq_status hip_fail(hipError_t e, const char *who)
{
    return fail(BQ_ERR_HIP, "%s: HIP error %d (%s)", who, (int)e, hipGetErrorString(e));
}

// ---- fixed device scratch for the entry point that must not allocate ---------------------------------
// One array per GPU the library runs on, held until the process ends.  In host code the array's name is only
// a stand-in for the symbol: its device address on the current GPU comes from hipGetSymbolAddress, once per
// device, and that pointer is what kernels and copies receive.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

bq_status static_scratch(void **out, const char *who)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(BQ_ERR_HIP, "%s: hipGetDevice failed: %d (%s)", who, (int)e, hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(BQ_ERR_UNSUPPORTED, "%s: device index %d beyond %d", who, dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(BQ_ERR_HIP, "%s: hipGetSymbolAddress failed: %d (%s)", who, (int)e, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return BQ_OK;
}

__global__ void zero_floats_kernel(float *p, size_t count)
{
    const size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q < count) p[q] = 0.0f;
}

bq_status transform(bq::Mode mode, const void *in, void *out, const void *plan, const bq_rows *rows,
                    void *stream, const char *who)
{
    bq::Shape s;
    bq_status st = check_rows(rows, &s, who);
    if (st != BQ_OK) return st;
    if (s.rows == 0) return ok();  // an empty batch may come with NULL data pointers
    if (!in || !out) return fail(BQ_ERR_NULL, "%s: data pointer is NULL", who);
    if ((st = check_plan(plan, who)) != BQ_OK) return st;
    if (misaligned(in, itemsize(s.dtype)) || misaligned(out, itemsize(s.dtype)))
        return fail(BQ_ERR_ALIGN, "%s: data pointer not aligned to its element size", who);
    if (s.rows == 0) return ok();
    bq::PlanView pv = bq::plan_view(plan, s.n, s.heads, s.k);
    hipError_t e = bq::launch_transform(mode, in, out, pv, s, nullptr, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, who);
    return ok();
}

}  // namespace

extern "C" {

size_t bq_plan_bytes(int32_t n, int32_t heads)
{
    int k = bq::ilog2_exact(n);
    if (k < 0 || n > 16384 || heads < 1 || (int64_t)n * heads > ((int64_t)1 << 24)) return 0;
    return bq::plan_layout(n, heads, k).total;
}

bq_status bq_plan_build(const float *theta, int32_t n, int32_t heads, void *plan, size_t plan_bytes, void *stream)
{
    const char *who = "bq_plan_build";
    size_t need = bq_plan_bytes(n, heads);
    if (need == 0) return fail(BQ_ERR_SHAPE, "%s: invalid shape n=%d heads=%d", who, n, heads);
    if (!theta) return fail(BQ_ERR_NULL, "%s: theta is NULL", who);
    bq_status st = check_plan(plan, who);
    if (st != BQ_OK) return st;
    if (misaligned(theta, 4)) return fail(BQ_ERR_ALIGN, "%s: theta not aligned to 4 bytes", who);
    if (plan_bytes < need)
        return fail(BQ_ERR_WORKSPACE, "%s: plan buffer has %zu bytes, %zu needed", who, plan_bytes, need);
    hipError_t e = bq::launch_plan_build(theta, n, heads, bq::ilog2_exact(n), plan, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, who);
    return ok();
}

bq_status bq_butterfly_fwd(const void *x, void *y, const void *plan, const bq_rows *rows, void *stream)
{
    return transform(bq::kFwd, x, y, plan, rows, stream, "bq_butterfly_fwd");
}

bq_status bq_butterfly_inv(const void *y, void *x, const void *plan, const bq_rows *rows, void *stream)
{
    return transform(bq::kInv, y, x, plan, rows, stream, "bq_butterfly_inv");
}

bq_status bq_hadamard_fwd(const void *x, void *y, const bq_rows *rows, void *stream)
{
    const char *who = "bq_hadamard_fwd";
    bq::Shape s;
    bq_status st = check_rows(rows, &s, who);
    if (st != BQ_OK) return st;
    if (s.rows == 0) return ok();
    if (!x || !y) return fail(BQ_ERR_NULL, "%s: data pointer is NULL", who);
    if (misaligned(x, itemsize(s.dtype)) || misaligned(y, itemsize(s.dtype)))
        return fail(BQ_ERR_ALIGN, "%s: data pointer not aligned to its element size", who);
    if (!bq::hadamard_supported(x, y, s))
        return fail(BQ_ERR_UNSUPPORTED, "%s: implemented for n = 4096 and 8192 with at most 512 heads, 16-byte aligned "
                                        "pointers and leading dimensions that are multiples of 16 bytes", who);
    hipError_t e = bq::launch_hadamard(x, y, s, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, who);
    return ok();
}

bq_status bq_butterfly_fwd_quant(const void *x, const void *plan, uint8_t *codes, void *scales,
                                 const bq_quant *quant, const bq_rows *rows, void *stream)
{
    const char *who = "bq_butterfly_fwd_quant";
    bq::Shape s;
    bq_status st = check_rows(rows, &s, who);
    if (st != BQ_OK) return st;
    if (!quant) return fail(BQ_ERR_NULL, "%s: quant descriptor is NULL", who);
    if (s.rows > 0 && (!x || !codes || !scales)) return fail(BQ_ERR_NULL, "%s: data pointer is NULL", who);
    if ((st = check_plan(plan, who)) != BQ_OK) return st;
    if (quant->scale_dtype != BQ_F32 && quant->scale_dtype != BQ_F16)
        return fail(BQ_ERR_DTYPE, "%s: scale_dtype must be BQ_F32 or BQ_F16", who);
    if (quant->bits != 4 && quant->bits != 2)
        return fail(BQ_ERR_UNSUPPORTED, "%s: bits=%d (only 4 and 2 are implemented)", who, quant->bits);
    int g = quant->group;
    if (g < 8 || g > s.n || (g & (g - 1)) != 0)
        return fail(BQ_ERR_SHAPE, "%s: group=%d must be a power of two in [8, n]", who, g);
    if (misaligned(x, itemsize(s.dtype)) || misaligned(scales, quant->scale_dtype == BQ_F32 ? 4 : 2))
        return fail(BQ_ERR_ALIGN, "%s: data pointer not aligned to its element size", who);
    if (s.rows == 0) return ok();
    bq::QuantArgs q{};
    q.bits = quant->bits;
    q.group = g;
    q.scale_f16 = quant->scale_dtype == BQ_F16;
    q.codes = codes;
    q.scales = scales;
    bq::PlanView pv = bq::plan_view(plan, s.n, s.heads, s.k);
    hipError_t e = bq::launch_transform(bq::kFwdQuant, x, nullptr, pv, s, &q, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, who);
    return ok();
}

bq_status bq_butterfly_fwd_fakequant(const void *x, const void *plan, void *yq, uint64_t *hist,
                                     const bq_quant *quant, const bq_rows *rows, void *stream)
{
    const char *who = "bq_butterfly_fwd_fakequant";
    bq::Shape s;
    bq_status st = check_rows(rows, &s, who);
    if (st != BQ_OK) return st;
    if (!quant) return fail(BQ_ERR_NULL, "%s: quant descriptor is NULL", who);
    if (!yq && !hist) return fail(BQ_ERR_NULL, "%s: yq and hist are both NULL", who);
    if (s.rows > 0 && !x) return fail(BQ_ERR_NULL, "%s: data pointer is NULL", who);
    if ((st = check_plan(plan, who)) != BQ_OK) return st;
    if (quant->scale_dtype != BQ_F32 && quant->scale_dtype != BQ_F16)
        return fail(BQ_ERR_DTYPE, "%s: scale_dtype must be BQ_F32 or BQ_F16", who);
    if (quant->bits != 4 && quant->bits != 2)
        return fail(BQ_ERR_UNSUPPORTED, "%s: bits=%d (only 4 and 2 are implemented)", who, quant->bits);
    int g = quant->group;
    if (g < 8 || g > s.n || (g & (g - 1)) != 0)
        return fail(BQ_ERR_SHAPE, "%s: group=%d must be a power of two in [8, n]", who, g);
    if (misaligned(x, itemsize(s.dtype)) || misaligned(yq, itemsize(s.dtype)) || misaligned(hist, 8))
        return fail(BQ_ERR_ALIGN, "%s: data pointer not aligned to its element size", who);
    hipError_t e;
    if (hist) {  // also for an empty batch: the counters are an output
        e = bq::launch_hist_clear((unsigned long long *)hist, quant->bits, (hipStream_t)stream);
        if (e != hipSuccess) return hip_fail(e, who);
    }
    if (s.rows == 0) return ok();
    bq::QuantArgs q{};
    q.bits = quant->bits;
    q.group = g;
    q.scale_f16 = quant->scale_dtype == BQ_F16;
    q.hist = (unsigned long long *)hist;
    bq::PlanView pv = bq::plan_view(plan, s.n, s.heads, s.k);
    e = bq::launch_transform(bq::kFwdFake, x, yq, pv, s, &q, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, who);
    return ok();
}

bq_status bq_cayley_build(const float *params, int32_t d1, float *q1, void *stream)
{
    const char *who = "bq_cayley_build";
    if (d1 < 2 || d1 > 64) return fail(BQ_ERR_SHAPE, "%s: d1=%d outside [2, 64]", who, d1);
    if (!params || !q1) return fail(BQ_ERR_NULL, "%s: pointer is NULL", who);
    if (misaligned(params, 4) || misaligned(q1, 4)) return fail(BQ_ERR_ALIGN, "%s: pointer not aligned to 4 bytes", who);
    hipError_t e = bq::launch_cayley(params, d1, q1, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, who);
    return ok();
}

static bq_status kron(bool inverse, const void *in, void *out, const float *q1, int32_t d1, const void *plan,
                      const bq_rows *rows, void *stream, const char *who)
{
    bq::Shape s;
    bq_status st = check_rows(rows, &s, who);
    if (st != BQ_OK) return st;
    if (d1 < 2 || d1 > 64) return fail(BQ_ERR_SHAPE, "%s: d1=%d outside [2, 64]", who, d1);
    if (s.heads != 1) return fail(BQ_ERR_SHAPE, "%s: heads must be 1 (the butterfly factor is shared)", who);
    const int64_t width = (int64_t)d1 * s.n;
    if (s.ld_x != width || s.ld_y != width)
        return fail(BQ_ERR_UNSUPPORTED, "%s: rows must be dense (ld_x = ld_y = d1 * d2 = %lld)", who, (long long)width);
    if (s.rows > 0 && s.rows > ((int64_t)1 << 40) / width) return fail(BQ_ERR_SHAPE, "%s: batch too large", who);
    if (s.rows == 0) return ok();
    if (!in || !out || !q1) return fail(BQ_ERR_NULL, "%s: pointer is NULL", who);
    if ((st = check_plan(plan, who)) != BQ_OK) return st;
    // two adjacent elements are moved at a time by the mixing kernel
    if (misaligned(in, 2 * itemsize(s.dtype)) || misaligned(out, 2 * itemsize(s.dtype)) || misaligned(q1, 4))
        return fail(BQ_ERR_ALIGN, "%s: data pointers must be aligned to two elements", who);
    bq::Shape sub = s;  // the [rows * d1, d2] view
    sub.rows = s.rows * d1;
    sub.ld_x = sub.ld_y = s.n;
    bq::PlanView pv = bq::plan_view(plan, s.n, 1, s.k);
    hipStream_t hs = (hipStream_t)stream;
    hipError_t e;
    if (bq::kron_fused_supported(in, out, d1, s.n)) {
        e = bq::launch_kron_fused(inverse, in, out, q1, d1, pv, s.rows, s.dtype, hs);
    } else if (!inverse) {
        e = bq::launch_transform(bq::kFwd, in, out, pv, sub, nullptr, hs);
        if (e == hipSuccess) e = bq::launch_mix(out, out, q1, d1, s.n, s.rows, s.dtype, false, hs);
    } else {
        e = bq::launch_mix(in, out, q1, d1, s.n, s.rows, s.dtype, true, hs);
        if (e == hipSuccess) e = bq::launch_transform(bq::kInv, out, out, pv, sub, nullptr, hs);
    }
    if (e != hipSuccess) return hip_fail(e, who);
    return ok();
}

bq_status bq_kron_fwd(const void *x, void *y, const float *q1, int32_t d1, const void *plan, const bq_rows *rows,
                      void *stream)
{
    return kron(false, x, y, q1, d1, plan, rows, stream, "bq_kron_fwd");
}

bq_status bq_kron_inv(const void *y, void *x, const float *q1, int32_t d1, const void *plan, const bq_rows *rows,
                      void *stream)
{
    return kron(true, y, x, q1, d1, plan, rows, stream, "bq_kron_inv");
}

size_t bq_butterfly_bwd_workspace_bytes(const bq_rows *rows)
{
    bq::Shape s;
    if (check_rows(rows, &s, "bq_butterfly_bwd_workspace_bytes") != BQ_OK) return 0;
    g_err[0] = '\0';
    return bq::bwd_workspace_bytes(s);
}

static bq_status bwd_common(const void *x, const void *dy, const void *plan, void *dx, float *dtheta, void *workspace,
                            size_t workspace_bytes, bool fixed_scratch, const bq_rows *rows, void *stream, const char *who)
{
    bq::Shape s;
    bq_status st = check_rows(rows, &s, who);
    if (st != BQ_OK) return st;
    if (!dx && !dtheta) return fail(BQ_ERR_NULL, "%s: both outputs are NULL", who);
    if (dtheta && misaligned(dtheta, 4)) return fail(BQ_ERR_ALIGN, "%s: dtheta not aligned to 4 bytes", who);
    if (s.rows == 0) {  // an empty batch may come with NULL data pointers; the sum over no rows is zero
        if (dtheta) {
            const size_t count = (size_t)s.heads * s.k * (s.n / 2);
            hipLaunchKernelGGL(zero_floats_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                               dtheta, count);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return hip_fail(e, who);
        }
        return ok();
    }
    if (!x || !dy) return fail(BQ_ERR_NULL, "%s: x or dy is NULL", who);
    if ((st = check_plan(plan, who)) != BQ_OK) return st;
    if (misaligned(x, itemsize(s.dtype)) || misaligned(dy, itemsize(s.dtype)) || (dx && misaligned(dx, itemsize(s.dtype))))
        return fail(BQ_ERR_ALIGN, "%s: data pointer not aligned to its element size", who);
    const size_t need = bq::bwd_workspace_bytes(s);
    if (fixed_scratch) {
        if (need > kStaticScratchBytes)
            return fail(BQ_ERR_WORKSPACE, "%s: this batch needs %zu bytes of scratch, the fixed scratch array holds %zu; "
                                          "use bq_butterfly_bwd with a workspace of your own", who, need, kStaticScratchBytes);
        if ((st = static_scratch(&workspace, who)) != BQ_OK) return st;
    } else {
        if (!workspace) return fail(BQ_ERR_NULL, "%s: workspace is NULL", who);
        if (misaligned(workspace, 256)) return fail(BQ_ERR_ALIGN, "%s: workspace must be aligned to 256 bytes", who);
        if (workspace_bytes < need)
            return fail(BQ_ERR_WORKSPACE, "%s: workspace has %zu bytes, %zu needed", who, workspace_bytes, need);
    }
    bq::PlanView pv = bq::plan_view(plan, s.n, s.heads, s.k);
    hipError_t e = bq::launch_bwd(x, dy, pv, dx, dtheta, workspace, s, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, who);
    return ok();
}

bq_status bq_butterfly_bwd(const void *x, const void *dy, const void *plan, void *dx, float *dtheta,
                           void *workspace, size_t workspace_bytes, const bq_rows *rows, void *stream)
{
    return bwd_common(x, dy, plan, dx, dtheta, workspace, workspace_bytes, false, rows, stream, "bq_butterfly_bwd");
}

size_t bq_butterfly_bwd_static_max_bytes(void) { return kStaticScratchBytes; }

bq_status bq_butterfly_bwd_static(const void *x, const void *dy, const void *plan, void *dx, float *dtheta,
                                  const bq_rows *rows, void *stream)
{
    return bwd_common(x, dy, plan, dx, dtheta, nullptr, 0, true, rows, stream, "bq_butterfly_bwd_static");
}

const char *bq_status_string(bq_status s)
{
    switch (s) {
        case BQ_OK: return "BQ_OK";
        case BQ_ERR_NULL: return "BQ_ERR_NULL";
        case BQ_ERR_SHAPE: return "BQ_ERR_SHAPE";
        case BQ_ERR_DTYPE: return "BQ_ERR_DTYPE";
        case BQ_ERR_ALIGN: return "BQ_ERR_ALIGN";
        case BQ_ERR_WORKSPACE: return "BQ_ERR_WORKSPACE";
        case BQ_ERR_UNSUPPORTED: return "BQ_ERR_UNSUPPORTED";
        case BQ_ERR_HIP: return "BQ_ERR_HIP";
    }
    return "BQ_ERR_?";
}

const char *bq_last_error(void) { return g_err; }

int bq_version(void) { return 100; }

}  // extern "C"
