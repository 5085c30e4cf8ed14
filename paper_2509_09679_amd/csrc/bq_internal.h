// Internal declarations shared by the translation units of libbq (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hip/hip_bf16.h>
#include <stddef.h>
#include <stdint.h>

#include "bq.h"

namespace bq {

// ---------------------------------------------------------------------------------------------
// Plan: everything derived from theta.  Device memory, laid out as
//   [PlanHeader (256 B)]
//   [cs      : float2 (cos, sin)  [heads][k][n/2]]            plain twiddles, pair order
//   [fg_fwd  : float  [heads][k][n]]   scale-deferred ("fast Givens") forward coefficients
//   [fd_fwd  : float  [heads][n]]      forward output scales
//   [fm_fwd  : float  [heads][n]]      scale of the forward state before the last layer, divided by that
//                                      layer's cosine: turns it into the transposed cascade's deferred units
//                                      after its first layer (the n = 8192 backward pass starts there)
//   [fg_inv  : float  [heads][k][n]]   the same for the transposed cascade
//   [fd_inv  : float  [heads][n]]
//   [fw_inv  : float  [heads][k][n]]   scale D of every element just BEFORE transposed layer i is applied
//                                      (row i-1); the backward kernels turn sums accumulated in deferred
//                                      units into dtheta with the factor D[a] * D[b] of the pair
//
// Scale-deferred form.  A rotation  ya = c xa - s xb, yb = s xa + c xb  with t = s / c is
//   ya = c (xa - t xb),  yb = c (xb + t xa).
// Carrying every element as x = D * u with a per-element scale D that depends on theta only,
// one layer becomes  u[e] += coef[e] * u[partner(e)]  (one FMA per element) with
//   coef[a] = -t * D[b] / D[a],  coef[b] = +t * D[a] / D[b],  D'[e] = c * D[e],
// and the output is y[e] = D_k[e] * u_k[e].  coef and D_k are evaluated in double at plan build and
// rounded once to float.  If any |log2 |D|| or |log2 |coef|| leaves a safe range (a cosine very
// close to zero), the header's fast_ok flag is cleared and kernels use (cos, sin) instead.
// ---------------------------------------------------------------------------------------------

constexpr uint32_t kPlanMagic = 0x42515031u;  // "BQP1"

struct PlanHeader {
    uint32_t magic;
    int32_t n, heads, k;
    int32_t fast_bad_fwd;  // != 0: forward scale-deferred tables unusable
    int32_t fast_bad_inv;  // != 0: inverse scale-deferred tables unusable
    int32_t pad[58];
};
static_assert(sizeof(PlanHeader) == 256, "header is 256 bytes");

struct PlanLayout {
    size_t cs, fg_fwd, fd_fwd, fm_fwd, fg_inv, fd_inv, fw_inv, total;
};

inline size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

inline PlanLayout plan_layout(int n, int heads, int k)
{
    PlanLayout L;
    size_t H = (size_t)heads, N = (size_t)n, K = (size_t)k;
    size_t off = sizeof(PlanHeader);
    L.cs = off;      off = align256(off + H * K * (N / 2) * sizeof(float2));
    L.fg_fwd = off;  off = align256(off + H * K * N * sizeof(float));
    L.fd_fwd = off;  off = align256(off + H * N * sizeof(float));
    L.fm_fwd = off;  off = align256(off + H * N * sizeof(float));
    L.fg_inv = off;  off = align256(off + H * K * N * sizeof(float));
    L.fd_inv = off;  off = align256(off + H * N * sizeof(float));
    L.fw_inv = off;  off = align256(off + H * K * N * sizeof(float));
    L.total = off;
    return L;
}

inline int ilog2_exact(int n)
{
    if (n < 2) return -1;
    int k = 0;
    while ((1 << k) < n) ++k;
    return ((1 << k) == n) ? k : -1;
}

// What a kernel needs to tell whether the plan it was handed is one that bq_plan_build wrote for the
// shape of this call.  Every kernel that reads plan tables tests plan_matches() before its first table
// access and returns without writing anything when the test fails: a buffer that was never built, or
// built for another (n, heads), then leaves the outputs as they were instead of being read past its end.
struct PlanRef {
    const PlanHeader *hdr;
    int32_t n, heads;
};

__device__ __forceinline__ bool plan_matches(const PlanRef &p)
{
    return p.hdr->magic == kPlanMagic && p.hdr->n == p.n && p.hdr->heads == p.heads;
}

// the plan is of this shape and both of its scale-deferred table sets (forward, transposed) are usable
__device__ __forceinline__ bool plan_fast_both(const PlanRef &p)
{
    return plan_matches(p) && (p.hdr->fast_bad_fwd | p.hdr->fast_bad_inv) == 0;
}

struct PlanView {  // device pointers into a plan
    const PlanHeader *hdr;
    PlanRef ref;
    const float2 *cs;
    const float *fg_fwd, *fd_fwd, *fm_fwd, *fg_inv, *fd_inv, *fw_inv;
};

inline PlanView plan_view(const void *plan, int n, int heads, int k)
{
    PlanLayout L = plan_layout(n, heads, k);
    const char *p = (const char *)plan;
    PlanView v;
    v.hdr = (const PlanHeader *)p;
    v.ref = PlanRef{v.hdr, n, heads};
    v.cs = (const float2 *)(p + L.cs);
    v.fg_fwd = (const float *)(p + L.fg_fwd);
    v.fd_fwd = (const float *)(p + L.fd_fwd);
    v.fm_fwd = (const float *)(p + L.fm_fwd);
    v.fg_inv = (const float *)(p + L.fg_inv);
    v.fd_inv = (const float *)(p + L.fd_inv);
    v.fw_inv = (const float *)(p + L.fw_inv);
    return v;
}

// ---------------------------------------------------------------------------------------------
// Shapes as the launchers see them (already validated)
// ---------------------------------------------------------------------------------------------
struct Shape {
    int64_t rows;
    int n, heads, k;
    int64_t ld_x, ld_y;
    int dtype;
};

struct QuantArgs {
    int bits, group, scale_f16;
    uint8_t *codes;
    void *scales;
    unsigned long long *hist;  // kFwdFake: 2^bits counters, may be NULL
};

// kFwdFake: forward + quantise + dequantise (`out` receives s * q, may be NULL) + code-bin histogram
// kHadamard: the fixed Walsh-Hadamard transform H_n / sqrt(n) (additions and subtractions only; no plan)
enum Mode { kFwd = 0, kInv = 1, kFwdQuant = 2, kFwdFake = 3, kHadamard = 4 };

// generic (any n) kernels: bq_generic.hip
hipError_t launch_generic(Mode mode, const void *in, void *out, const PlanView &pv, const Shape &s,
                          const QuantArgs *q, hipStream_t stream);
size_t bwd_workspace_bytes_generic(const Shape &s);
// only_if_bad: run only when the plan flags its scale-deferred tables as unusable (the specialised
// backward kernels, launched before, then did nothing)
hipError_t launch_generic_bwd(const void *x, const void *dy, const PlanView &pv, void *dx, float *dtheta,
                              void *ws, const Shape &s, hipStream_t stream, bool only_if_bad = false);

int small_span(int64_t width);  // bq_small.hip: elements per workgroup of the small-transform kernels, 0 = unsupported
// backward for n = 8 .. 128 (bq_bwd_small.hip)
bool small_bwd_supported(const void *x, const void *dy, const void *dx, const float *dtheta, const Shape &s);
size_t small_bwd_workspace_bytes(const Shape &s);
hipError_t launch_small_bwd(const void *x, const void *dy, const PlanView &pv, void *dx, float *dtheta, void *ws,
                            const Shape &s, hipStream_t stream);
// n = 256 .. 8192 backward: bq_bwd.hip
bool bwd_fast_supported(const void *x, const void *dy, const void *dx, const float *dtheta, const Shape &s);
size_t bwd_fast_workspace_bytes(const Shape &s);
hipError_t launch_bwd_fast(const void *x, const void *dy, const PlanView &pv, void *dx, float *dtheta, void *ws,
                           const Shape &s, hipStream_t stream);

// n = 4096 specialised kernels (also blocks of 4096 / n rows for n = 256 .. 2048): bq_k12.hip
bool k12_supported(Mode mode, const void *in, const void *out, const Shape &s, const QuantArgs *q);
int k12_block_rows(const Shape &s);  // launch_k12 processes floor(rows / this) * this rows, from the first
hipError_t launch_k12(Mode mode, const void *in, void *out, const PlanView &pv, const Shape &s,
                      const QuantArgs *q, hipStream_t stream);

// y = H_n x / sqrt(n) for n = 4096 and 8192 (bq_k12.hip); false if the shape or alignment is not covered
bool hadamard_supported(const void *in, const void *out, const Shape &s);
hipError_t launch_hadamard(const void *in, void *out, const Shape &s, hipStream_t stream);

// Raises a kernel's dynamic shared-memory limit once per device instead of on every launch (the call costs
// host time, which the small-batch calls feel).  One object per kernel instantiation.
struct LdsLimitOnce {
    bool done[64] = {};
    hipError_t set(const void *kernel, size_t bytes)
    {
        int dev = -1;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64 && done[dev]) return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e == hipSuccess && dev >= 0 && dev < 64) done[dev] = true;  // (a race between first calls repeats the same setting)
        return e;
    }
};

// n = 8..128 specialised kernels: bq_small.hip
bool small_supported(Mode mode, const void *in, const void *out, const Shape &s, const QuantArgs *q);
hipError_t launch_small(Mode mode, const void *in, void *out, const PlanView &pv, const Shape &s,
                        const QuantArgs *q, hipStream_t stream);

// dispatch between specialised and generic kernels: bq_dispatch.hip
hipError_t launch_transform(Mode mode, const void *in, void *out, const PlanView &pv, const Shape &s,
                            const QuantArgs *q, hipStream_t stream);
size_t bwd_workspace_bytes(const Shape &s);
hipError_t launch_bwd(const void *x, const void *dy, const PlanView &pv, void *dx, float *dtheta, void *ws,
                      const Shape &s, hipStream_t stream);

// clears the 2^bits counters of a histogram (a fill kernel: safe inside a captured graph)
hipError_t launch_hist_clear(unsigned long long *hist, int bits, hipStream_t stream);

// composite transform for widths d1 * d2: bq_kron.hip
hipError_t launch_cayley(const float *params, int d1, float *q, hipStream_t stream);
hipError_t launch_mix(const void *in, void *out, const float *q, int d1, int d2, int64_t rows, int dtype,
                      bool transpose, hipStream_t stream);
bool kron_fused_supported(const void *in, const void *out, int d1, int d2);
hipError_t launch_kron_fused(bool inverse, const void *in, void *out, const float *q, int d1, const PlanView &pv,
                             int64_t rows, int dtype, hipStream_t stream);

// plan build: bq_plan.hip
hipError_t launch_plan_build(const float *theta, int n, int heads, int k, void *plan, hipStream_t stream);

}  // namespace bq
