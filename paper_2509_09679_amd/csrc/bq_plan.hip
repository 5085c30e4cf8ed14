// Plan build: cos/sin twiddles and the scale-deferred coefficient tables, all derived from theta.
// (Paper: "pre-computed cos/sin twiddle factors stored in a lookup table", section "Inference
// Efficiency"; kept in float32 here, evaluated in double and rounded once.)
#include "bq_internal.h"

namespace bq {

__global__ void plan_cs_kernel(const float *__restrict__ theta, float2 *__restrict__ cs, size_t count,
                               PlanHeader *hdr, int n, int heads, int k)
{
    size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q == 0) {
        hdr->magic = kPlanMagic;
        hdr->n = n;
        hdr->heads = heads;
        hdr->k = k;
        hdr->fast_bad_fwd = 0;
        hdr->fast_bad_inv = 0;
    }
    if (q < count) {
        double t = (double)theta[q];
        cs[q] = make_float2((float)cos(t), (float)sin(t));
    }
}

// Layers are processed in cascade order with workgroup barriers between them.
constexpr int kPlanThreads = 1024;
constexpr int kPlanMaxPerThread = 16;  // n <= 16384

// One workgroup per (head, direction): blockIdx.y = 0 builds the forward tables, 1 those of the transposed
// cascade.  The running scales D (double) live in LDS.
struct PlanFastArgs {
    const float *theta;
    int n, k;
    float *fg[2], *fd[2];
    float *fw;  // transposed cascade only
    float *fm;  // forward cascade only
    int *bad[2];
};

__global__ __launch_bounds__(kPlanThreads) void plan_fast_kernel(PlanFastArgs A)
{
    extern __shared__ double D[];  // [n]
    const int head = blockIdx.x, inverse = blockIdx.y;
    const int tid = threadIdx.x, n = A.n, k = A.k;
    const float *th = A.theta + (size_t)head * k * (n / 2);
    float *fgh = A.fg[inverse] + (size_t)head * k * n;
    float *fw = inverse ? A.fw : nullptr, *fm = inverse ? nullptr : A.fm;
    for (int e = tid; e < n; e += kPlanThreads) D[e] = 1.0;
    __syncthreads();
    int bad = 0;
    const double lo_d = 0x1p-60, hi_d = 0x1p60, lo_c = 0x1p-100, hi_c = 0x1p100;
    for (int step = 0; step < k; ++step) {
        const int i = inverse ? (k - step) : (step + 1);
        const int h = 1 << (i - 1);
        double newD[kPlanMaxPerThread];
        int j = 0;
        for (int e = tid; e < n; e += kPlanThreads, ++j) {
            const int a = e & ~h;
            const int p = ((a >> i) << (i - 1)) | (a & (h - 1));
            const double t = (double)th[(size_t)(i - 1) * (n / 2) + p];
            const double c = cos(t), s = sin(t);
            double tt = s / c;
            if (inverse) tt = -tt;
            const double Dself = D[e], Dpart = D[e ^ h];
            // lower element: u_a -= t (D_b / D_a) u_b ; upper element: u_b += t (D_a / D_b) u_a
            double coef = tt * Dpart / Dself;
            if (!(e & h)) coef = -coef;
            const double nd = c * Dself;
            newD[j] = nd;
            fgh[(size_t)(i - 1) * n + e] = (float)coef;
            if (fw) fw[((size_t)head * k + (i - 1)) * n + e] = (float)Dself;  // scale before this layer
            if (fm && step == k - 1) {
                const double m = Dself / c;
                fm[(size_t)head * n + e] = (float)m;
                if (!(fabs(m) > lo_d && fabs(m) < hi_d)) bad = 1;
            }
            const double ac = fabs(coef), ad = fabs(nd);
            if (!(ad > lo_d && ad < hi_d)) bad = 1;
            if (!(ac == 0.0 || (ac > lo_c && ac < hi_c))) bad = 1;
        }
        __syncthreads();
        j = 0;
        for (int e = tid; e < n; e += kPlanThreads, ++j) D[e] = newD[j];
        __syncthreads();
    }
    for (int e = tid; e < n; e += kPlanThreads) A.fd[inverse][(size_t)head * n + e] = (float)D[e];
    if (bad) atomicOr(A.bad[inverse], 1);
}

hipError_t launch_plan_build(const float *theta, int n, int heads, int k, void *plan, hipStream_t stream)
{
    PlanLayout L = plan_layout(n, heads, k);
    char *p = (char *)plan;
    PlanHeader *hdr = (PlanHeader *)p;
    size_t count = (size_t)heads * k * (n / 2);
    unsigned blocks = (unsigned)((count + 255) / 256);
    hipLaunchKernelGGL(plan_cs_kernel, dim3(blocks), dim3(256), 0, stream, theta, (float2 *)(p + L.cs), count,
                       hdr, n, heads, k);
    PlanFastArgs F{};
    F.theta = theta;
    F.n = n;
    F.k = k;
    F.fg[0] = (float *)(p + L.fg_fwd);
    F.fg[1] = (float *)(p + L.fg_inv);
    F.fd[0] = (float *)(p + L.fd_fwd);
    F.fd[1] = (float *)(p + L.fd_inv);
    F.fw = (float *)(p + L.fw_inv);
    F.fm = (float *)(p + L.fm_fwd);
    F.bad[0] = &hdr->fast_bad_fwd;
    F.bad[1] = &hdr->fast_bad_inv;
    const size_t lds = (size_t)n * sizeof(double);
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)plan_fast_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(plan_fast_kernel, dim3(heads, 2), dim3(kPlanThreads), lds, stream, F);
    return hipGetLastError();
}

}  // namespace bq
