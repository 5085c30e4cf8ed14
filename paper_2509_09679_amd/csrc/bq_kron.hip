// Composite transform for widths d = d1 * d2 that are not powers of two (paper, "Composite Butterfly
// Transforms for Non-Power-of-2 Dimensions"):  Q = Q1 (x) B(theta),  Q1 a d1 x d1 orthogonal matrix from
// the Cayley parameterisation,  B(theta) the butterfly of size d2 = 2^k.  With a row viewed as the d1 x d2
// matrix X (element (i, j) at i * d2 + j),  Q x = Q1 X B^T: the butterfly runs over the d1 sub-rows of
// every row (the ordinary transform kernels on the [rows * d1, d2] view), and the kernel here mixes the
// sub-rows:  Y[i][j] = sum_k Q1[i][k] Z[k][j].
//
// The mix is a small dense product (d1^2 * d2 multiply-adds per row, 40 per element for d1 = 40).  A
// thread owns two adjacent columns j of one row and all d1 outputs of them: it reads its 2 * d1 inputs
// (4- or 8-byte loads, contiguous across lanes, eight sub-rows ahead), keeps 2 * d1 sums in registers and
// takes Q1 from LDS, where the workgroup put it transposed and zero-padded: every lane reads the same four
// coefficients with one 16-byte LDS read (a broadcast), then does eight FMAs.  In place is safe: a thread
// reads all its inputs before it writes, and no other thread touches its columns.
#include "bq_cascade.h"

namespace bq {

// ---- Q1 = (I - A)(I + A)^-1 ------------------------------------------------------------------------------
// One workgroup, Gauss-Jordan with partial pivoting on [I + A | I - A] in double (I + A is never singular:
// its eigenvalues are 1 + i*lambda).  d1 <= 64.
constexpr int kCayleyMax = 64;
constexpr int kCayleyThreads = 256;

__global__ __launch_bounds__(kCayleyThreads) void cayley_kernel(const float *__restrict__ params, int d1,
                                                                float *__restrict__ q)
{
    extern __shared__ double aug[];  // [d1][2 * d1]
    __shared__ int pivot_row;
    const int w = 2 * d1;
    for (int e = threadIdx.x; e < d1 * w; e += kCayleyThreads) {
        const int i = e / w, j = e % w;
        const int c = j % d1;  // column inside its half
        double a = 0.0;        // A[i][c]
        if (i < c)
            a = (double)params[(size_t)i * d1 - (size_t)i * (i + 1) / 2 + (c - i - 1)];
        else if (i > c)
            a = -(double)params[(size_t)c * d1 - (size_t)c * (c + 1) / 2 + (i - c - 1)];
        const double id = (i == c) ? 1.0 : 0.0;
        aug[e] = (j < d1) ? id + a : id - a;
    }
    __syncthreads();
    for (int col = 0; col < d1; ++col) {
        if (threadIdx.x == 0) {
            int best = col;
            double bv = fabs(aug[col * w + col]);
            for (int r = col + 1; r < d1; ++r) {
                const double v = fabs(aug[r * w + col]);
                if (v > bv) {
                    bv = v;
                    best = r;
                }
            }
            pivot_row = best;
        }
        __syncthreads();
        const int pr = pivot_row;
        if (pr != col) {
            for (int j = threadIdx.x; j < w; j += kCayleyThreads) {
                const double t = aug[col * w + j];
                aug[col * w + j] = aug[pr * w + j];
                aug[pr * w + j] = t;
            }
        }
        __syncthreads();
        const double inv = 1.0 / aug[col * w + col];
        __syncthreads();
        for (int j = threadIdx.x; j < w; j += kCayleyThreads) aug[col * w + j] *= inv;
        __syncthreads();
        // eliminate the column from every other row; element (r, j) is owned by one thread
        for (int e = threadIdx.x; e < d1 * w; e += kCayleyThreads) {
            const int r = e / w, j = e % w;
            if (r != col && j != col) aug[e] -= aug[r * w + col] * aug[col * w + j];
        }
        __syncthreads();
        for (int r = threadIdx.x; r < d1; r += kCayleyThreads)
            if (r != col) aug[r * w + col] = 0.0;
        __syncthreads();
    }
    for (int e = threadIdx.x; e < d1 * d1; e += kCayleyThreads) q[e] = (float)aug[(e / d1) * w + d1 + (e % d1)];
}

hipError_t launch_cayley(const float *params, int d1, float *q, hipStream_t stream)
{
    const size_t lds = (size_t)d1 * 2 * d1 * sizeof(double);
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)cayley_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(cayley_kernel, dim3(1), dim3(kCayleyThreads), lds, stream, params, d1, q);
    return hipGetLastError();
}

// ---- the mix ---------------------------------------------------------------------------------------------
constexpr int kMixThreads = 256;

struct MixArgs {
    const void *in;
    void *out;
    const float *q;  // [d1][d1] row-major
    int64_t rows;    // rows of d1 * d2 elements, dense
    int d1, d2;
    int transpose;   // != 0: apply Q1^T
};

template <typename T>
struct Pair;  // two adjacent elements as one load / store
template <>
struct Pair<float> {
    typedef float2 raw;
    static __device__ __forceinline__ void unpack(raw v, float &a, float &b) { a = v.x; b = v.y; }
    static __device__ __forceinline__ raw pack(float a, float b) { return make_float2(a, b); }
};
template <>
struct Pair<__half> {
    typedef uint32_t raw;
    static __device__ __forceinline__ void unpack(raw v, float &a, float &b)
    {
        const __half2 h = *(const __half2 *)&v;
        a = __low2float(h);
        b = __high2float(h);
    }
    static __device__ __forceinline__ raw pack(float a, float b)
    {
        const __half2 h = __halves2half2(__float2half_rn(a), __float2half_rn(b));
        return *(const uint32_t *)&h;
    }
};
template <>
struct Pair<bf16_t> {
    typedef uint32_t raw;
    static __device__ __forceinline__ void unpack(raw v, float &a, float &b)
    {
        a = __uint_as_float(v << 16);
        b = __uint_as_float(v & 0xFFFF0000u);
    }
    static __device__ __forceinline__ raw pack(float a, float b) { return f32x2_to_bf16x2_bits(a, b); }
};

// D1: d1 rounded up to a multiple of 8.  qs[k * D1 + i] is the weight of input sub-row k in output sub-row i
// (zero for i >= d1, so the padded sums stay zero and are never stored).
// kExact: d1 == D1 (no bounds to test on loads and stores).
template <typename T, int D1, bool kExact>
__global__ __launch_bounds__(kMixThreads) void mix_kernel(MixArgs A)
{
    typedef typename Pair<T>::raw raw_t;
    __shared__ __align__(16) float qs[D1 * D1];
    const int d1 = kExact ? D1 : A.d1, d2 = A.d2;
    for (int e = threadIdx.x; e < D1 * D1; e += kMixThreads) {
        const int k = e / D1, i = e % D1;
        float c = 0.0f;
        if (k < d1 && i < d1) c = A.transpose ? A.q[k * d1 + i] : A.q[i * d1 + k];
        qs[e] = c;
    }
    __syncthreads();
    const int pairs = d2 >> 1;             // threads per row
    const int64_t units = A.rows * pairs;  // one unit = two columns of one row
    const int64_t stride = (int64_t)gridDim.x * kMixThreads;
    for (int64_t u = (int64_t)blockIdx.x * kMixThreads + threadIdx.x; u < units; u += stride) {
        const int64_t row = u / pairs;
        const int col = (int)(u - row * pairs) * 2;
        const raw_t *src = (const raw_t *)((const T *)A.in + row * ((int64_t)d1 * d2) + col);
        raw_t *dst = (raw_t *)((T *)A.out + row * ((int64_t)d1 * d2) + col);
        float acc0[D1], acc1[D1];
#pragma unroll
        for (int i = 0; i < D1; ++i) acc0[i] = acc1[i] = 0.0f;
        raw_t z[8], zn[8];
        auto fetch = [&](int k0, raw_t(&dstz)[8]) {
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const int k = (kExact || k0 + kk < d1) ? k0 + kk : d1 - 1;  // past the end: any valid sub-row (weight zero)
                dstz[kk] = src[(size_t)k * pairs];              // sub-rows are d2 elements = `pairs` pairs apart
            }
        };
        fetch(0, z);
#pragma unroll 1
        for (int k0 = 0; k0 < D1; k0 += 8) {
            if (k0 + 8 < D1) fetch(k0 + 8, zn);
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                float z0, z1;
                Pair<T>::unpack(z[kk], z0, z1);
                const float4 *c4 = (const float4 *)&qs[(k0 + kk) * D1];
#pragma unroll
                for (int i4 = 0; i4 < D1 / 4; ++i4) {
                    const float4 c = c4[i4];
                    acc0[4 * i4 + 0] = __builtin_fmaf(c.x, z0, acc0[4 * i4 + 0]);
                    acc1[4 * i4 + 0] = __builtin_fmaf(c.x, z1, acc1[4 * i4 + 0]);
                    acc0[4 * i4 + 1] = __builtin_fmaf(c.y, z0, acc0[4 * i4 + 1]);
                    acc1[4 * i4 + 1] = __builtin_fmaf(c.y, z1, acc1[4 * i4 + 1]);
                    acc0[4 * i4 + 2] = __builtin_fmaf(c.z, z0, acc0[4 * i4 + 2]);
                    acc1[4 * i4 + 2] = __builtin_fmaf(c.z, z1, acc1[4 * i4 + 2]);
                    acc0[4 * i4 + 3] = __builtin_fmaf(c.w, z0, acc0[4 * i4 + 3]);
                    acc1[4 * i4 + 3] = __builtin_fmaf(c.w, z1, acc1[4 * i4 + 3]);
                }
            }
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) z[kk] = zn[kk];
        }
#pragma unroll
        for (int i = 0; i < D1; ++i)
            if (kExact || i < d1) dst[(size_t)i * pairs] = Pair<T>::pack(acc0[i], acc1[i]);
    }
}

template <typename T>
static hipError_t launch_mix_t(const MixArgs &A, hipStream_t stream)
{
    void (*kern)(MixArgs) = nullptr;
    const bool exact = (A.d1 % 8) == 0;
#define BQ_MIX_CASE(D) kern = exact ? mix_kernel<T, D, true> : mix_kernel<T, D, false>
    switch ((A.d1 + 7) / 8) {
        case 1: BQ_MIX_CASE(8); break;
        case 2: BQ_MIX_CASE(16); break;
        case 3: BQ_MIX_CASE(24); break;
        case 4: BQ_MIX_CASE(32); break;
        case 5: BQ_MIX_CASE(40); break;
        case 6: BQ_MIX_CASE(48); break;
        case 7: BQ_MIX_CASE(56); break;
        default: BQ_MIX_CASE(64); break;
    }
#undef BQ_MIX_CASE
    const int64_t units = A.rows * (A.d2 / 2);
    int64_t blocks = (units + kMixThreads - 1) / kMixThreads;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(kMixThreads), 0, stream, A);
    return hipGetLastError();
}

// ---- fused composite transform for d2 = 128 --------------------------------------------------------------
// One workgroup per row at a time, 16 lanes per sub-row (8 consecutive elements per lane): the butterfly of
// every sub-row runs in registers (as in the small-transform kernels), the float32 results go to an LDS tile,
// and after a barrier wave w mixes: its lane c owns columns 2c, 2c+1 and outputs 4w .. 4w+3, reading column
// values (8-byte LDS reads, consecutive lanes on consecutive banks) and four coefficients (one 16-byte
// broadcast read) per input sub-row.  The two factors act on different indices and commute, so the inverse
// runs the transposed butterfly first and then mixes with Q1^T: same structure.  One rounding to the row type
// at the end; the tile is double-buffered so that one barrier per row suffices.
// d1 is padded to D1P = a multiple of 4 (waves = D1P / 4); sub-rows past d1 are idle in the first phase.
constexpr int kFusedD2 = 128;
constexpr int kTileRow = kFusedD2 + 4;  // floats; the pad keeps 16-byte alignment of the lanes' 32-byte writes

struct FusedArgs {
    const void *in;
    void *out;
    const float *q;  // [d1][d1]
    const float *fg, *fd;
    const float2 *cs;
    const int *fast_bad;
    int64_t rows;
    int d1;
};

// kBound: the largest workgroup the instantiation is launched with (640 covers d1 <= 40 and leaves each
// thread more registers than the 1024-thread variant gets).
template <typename T, bool kInverse, int kBound>
__global__ __launch_bounds__(kBound) void kron128_kernel(FusedArgs A)
{
    typedef typename Pair<T>::raw raw_t;
    extern __shared__ __align__(16) float lds[];
    const int d1 = A.d1;
    const int d1p = (d1 + 3) & ~3;
    float *qs = lds;                       // [d1][d1p]: weight of input sub-row k in output i, zero padded
    float *tile = lds + d1 * d1p;          // 2 x [d1][kTileRow]
    const int tid = threadIdx.x, sub = tid >> 4, l16 = tid & 15;
    const int wave = tid >> 6, lane = tid & 63;
    for (int e = tid; e < d1 * d1p; e += blockDim.x) {
        const int k = e / d1p, i = e % d1p;
        qs[e] = (i < d1) ? (kInverse ? A.q[k * d1 + i] : A.q[i * d1 + k]) : 0.0f;
    }
    const int idx = lane_chunk(l16) * 8;  // first column of the thread's 8 elements
    const bool fast = (*A.fast_bad == 0);
    float c[7][8], d[8];
#pragma unroll
    for (int j = 0; j < 7; ++j)
#pragma unroll
        for (int r = 0; r < 8; ++r) c[j][r] = A.fg[j * kFusedD2 + idx + r];
#pragma unroll
    for (int r = 0; r < 8; ++r) d[r] = A.fd[idx + r];
    const bool loader = sub < d1;
    const T *in = (const T *)A.in + (size_t)sub * kFusedD2 + idx;
    const int64_t width = (int64_t)d1 * kFusedD2;
    int64_t row = blockIdx.x;
    Raw8 raw = {};
    if (loader && row < A.rows) raw = load8(in + row * width);
    int par = 0;
    for (; row < A.rows; row += gridDim.x) {
        float *t = tile + par * d1 * kTileRow;
        par ^= 1;
        if (loader) {
            float u[8];
            unpack8(raw, u, (const T *)nullptr);
            const int64_t next = row + gridDim.x;
            if (next < A.rows) raw = load8(in + next * width);
            if (fast)
                fast_small<7, kInverse>(u, c, d);
            else
                slow_small<7, kInverse>(u, A.cs, idx);
            float4 *dst = (float4 *)&t[sub * kTileRow + idx];
            dst[0] = make_float4(u[0], u[1], u[2], u[3]);
            dst[1] = make_float4(u[4], u[5], u[6], u[7]);
        }
        __syncthreads();  // also orders this row's tile reads before the writes two rows later
        float a0[4] = {0, 0, 0, 0}, a1[4] = {0, 0, 0, 0};
        const float *zc = t + 2 * lane;
        const float *qc = qs + 4 * wave;
#pragma unroll 8
        for (int k = 0; k < d1; ++k) {
            const float2 z = *(const float2 *)&zc[k * kTileRow];
            const float4 w = *(const float4 *)&qc[k * d1p];
            a0[0] = __builtin_fmaf(w.x, z.x, a0[0]);
            a1[0] = __builtin_fmaf(w.x, z.y, a1[0]);
            a0[1] = __builtin_fmaf(w.y, z.x, a0[1]);
            a1[1] = __builtin_fmaf(w.y, z.y, a1[1]);
            a0[2] = __builtin_fmaf(w.z, z.x, a0[2]);
            a1[2] = __builtin_fmaf(w.z, z.y, a1[2]);
            a0[3] = __builtin_fmaf(w.w, z.x, a0[3]);
            a1[3] = __builtin_fmaf(w.w, z.y, a1[3]);
        }
        raw_t *out = (raw_t *)((T *)A.out + row * width) + lane;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (4 * wave + j < d1) out[(size_t)(4 * wave + j) * (kFusedD2 / 2)] = Pair<T>::pack(a0[j], a1[j]);
    }
}

bool kron_fused_supported(const void *in, const void *out, int d1, int d2)
{
    return d2 == kFusedD2 && d1 >= 2 && d1 <= 64 && !((uintptr_t)in & 15) && !((uintptr_t)out & 3);
}

template <typename T>
static hipError_t launch_kron_fused_t(bool inverse, FusedArgs &A, hipStream_t stream)
{
    const int d1p = (A.d1 + 3) & ~3;
    const int threads = d1p * 16;  // a multiple of 64
    const size_t lds = ((size_t)A.d1 * d1p + 2 * (size_t)A.d1 * kTileRow) * sizeof(float);
    void (*kern)(FusedArgs);
    if (threads <= 640)
        kern = inverse ? kron128_kernel<T, true, 640> : kron128_kernel<T, false, 640>;
    else
        kern = inverse ? kron128_kernel<T, true, 1024> : kron128_kernel<T, false, 1024>;
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    int64_t grid = 256 * 2;
    if (grid > A.rows) grid = A.rows;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(threads), lds, stream, A);
    return hipGetLastError();
}

hipError_t launch_kron_fused(bool inverse, const void *in, void *out, const float *q, int d1, const PlanView &pv,
                             int64_t rows, int dtype, hipStream_t stream)
{
    FusedArgs A{};
    A.in = in;
    A.out = out;
    A.q = q;
    A.fg = inverse ? pv.fg_inv : pv.fg_fwd;
    A.fd = inverse ? pv.fd_inv : pv.fd_fwd;
    A.cs = pv.cs;
    A.fast_bad = inverse ? &pv.hdr->fast_bad_inv : &pv.hdr->fast_bad_fwd;
    A.rows = rows;
    A.d1 = d1;
    switch (dtype) {
        case BQ_F32: return launch_kron_fused_t<float>(inverse, A, stream);
        case BQ_F16: return launch_kron_fused_t<__half>(inverse, A, stream);
        default: return launch_kron_fused_t<bf16_t>(inverse, A, stream);
    }
}

hipError_t launch_mix(const void *in, void *out, const float *q, int d1, int d2, int64_t rows, int dtype,
                      bool transpose, hipStream_t stream)
{
    MixArgs A{};
    A.in = in;
    A.out = out;
    A.q = q;
    A.rows = rows;
    A.d1 = d1;
    A.d2 = d2;
    A.transpose = transpose ? 1 : 0;
    switch (dtype) {
        case BQ_F32: return launch_mix_t<float>(A, stream);
        case BQ_F16: return launch_mix_t<__half>(A, stream);
        default: return launch_mix_t<bf16_t>(A, stream);
    }
}

}  // namespace bq
