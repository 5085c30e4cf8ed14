// Composite transform for widths d = d1 * d2 that are not powers of two (paper, "Composite Butterfly
// Transforms for Non-Power-of-2 Dimensions"):  Q = Q1 (x) B(theta),  Q1 a d1 x d1 orthogonal matrix from
// the Cayley parameterisation,  B(theta) the butterfly of size d2 = 2^k.  With a row viewed as the d1 x d2
// matrix X (element (i, j) at i * d2 + j),  Q x = Q1 X B^T: the butterfly runs over the d1 sub-rows of
// every row (the ordinary transform kernels on the [rows * d1, d2] view), and the kernel here mixes the
// sub-rows:  Y[i][j] = sum_k Q1[i][k] Z[k][j].
//
// The mix is the one dense contraction of the method (d1^2 * d2 multiply-adds per row, 40 per element for
// d1 = 40).  Two kernels here:
//   * kron128_kernel (d2 = 128, d1 <= 40): butterflies and mix in one pass over the row.  Three wave groups
//     pipeline a row through LDS tiles: 16 lanes per sub-row run the 128-point butterflies in registers; four
//     waves mix the sub-rows on the matrix cores (Q1 zero-padded and resident in registers as A operands;
//     float32 MFMA for float32 and bfloat16 rows, bfloat16 MFMA on two-way splits of both factors for
//     binary16 rows); two waves store the result with one rounding.
//   * mix_kernel (any other shape, after or before the ordinary transform kernels on the [rows * d1, d2] view):
//     plain FMAs.  A thread owns two adjacent columns j of one row and all d1 outputs of them: it reads its
//     2 * d1 inputs (4- or 8-byte loads, contiguous across lanes, eight sub-rows ahead), keeps 2 * d1 sums in
//     registers and takes Q1 from LDS, where the workgroup put it transposed and zero-padded: every lane reads
//     the same four coefficients with one 16-byte LDS read (a broadcast), then does eight FMAs.  In place is
//     safe: a thread reads all its inputs before it writes, and no other thread touches its columns.
#include <type_traits>

#include "bq_cascade.h"

namespace bq {

// ---- Q1 = (I - A)(I + A)^-1 ------------------------------------------------------------------------------
// One workgroup, Gauss-Jordan with partial pivoting on [I + A | I - A] in double (I + A is never singular:
// its eigenvalues are 1 + i*lambda).  d1 <= 64.
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
        return f32x2_to_f16x2_bits(a, b);
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
// One workgroup per pair of rows at a time, three groups of waves working on different pairs, one barrier per step
// (per pair of rows; the text below says row t for the rows of step t):
//   * the butterfly group (16 lanes per sub-row, 8 consecutive elements per lane) transforms row t at step t:
//     the butterfly of every sub-row runs in registers (as in the small-transform kernels) and the float32
//     results go to an LDS tile Z[d1][128];
//   * the store group (two waves) stores row t-2: 16-byte pieces read back from that row's tile, one rounding
//     to the row type;
//   * the mix group (four waves, one per SIMD) takes row t-1: Y = Q1 Z is a dense product, done on the matrix
//     cores.  float32 rows: in float32 (v_mfma_f32_16x16x4_f32: no rounding of Z or Q1, float32 accumulation),
//     as described next.  binary16 rows: as three bfloat16 products of two-way splits of both factors with
//     float32 accumulation (v_mfma_f32_16x16x32_bf16; the tile then holds each value of Z as a (hi, lo) pair of
//     bfloat16 in one word), which keeps the error far under the bound for such rows at less than half
//     the matrix cycles: 65536 rows of 5120 went from 0.49 to 0.36 ms.  A wave owns two
//     blocks of 16 columns; per step of four input sub-rows it reads one B operand per block from the tile
//     (lane l: sub-row 4 s + l / 16, column l % 16 of the block) and issues one MFMA per block of 16 output
//     sub-rows; Q1 (zero-padded) stays in registers as the A operands (lane l: output 16 i + l % 16, input
//     4 s + l / 16).  Results (lane l, register r: output 16 i + 4 (l / 16) + r, column l % 16) overwrite
//     the wave's own columns of the tile.
// Three sets of tiles rotate.  (Measured with timing-only builds: the matrix instructions' time adds to the vector
// work of the waves on the same SIMD instead of hiding behind it, so a row costs about the sum of the two.)  The two factors
// act on different indices and commute, so the inverse runs the transposed butterfly first and then mixes
// with Q1^T: same structure.
constexpr int kFusedD2 = 128;
constexpr int kTileRow = kFusedD2 + 16;  // floats: sub-rows 16 banks apart, so a B-operand read (4 sub-rows x 16
                                         // columns) touches every bank twice, the minimum for 256 bytes
constexpr int kFusedMaxD1 = 40;  // 40 sub-rows x 16 lanes + six more waves = 1024 threads
constexpr int kStepRows = 2;  // rows between two barriers (per group); 3 * kStepRows tiles rotate
constexpr int kMixWaves = 4;
constexpr int kStoreWaves = 2;
constexpr int kFusedMaxThreads = kFusedMaxD1 * 16 + (kMixWaves + kStoreWaves) * 64;

// Rows of binary16 mix on the bfloat16 matrix instruction (two-way splits, three products): the error this adds, up
// to 3 * 2^-16 of sum_k |Q[i][k] z[k][j]|, is a tenth of such a row's own rounding step (2^-11 of the value).  For
// bfloat16 rows, whose rounding step (2^-8 of the value) already uses up their 2e-3 bound, nothing is to spare, and for
// float32 rows it is far too much: both keep the float32 matrix instruction.
template <typename T>
constexpr bool kSplitMix = std::is_same<T, __half>::value;

struct FusedArgs {
    const void *in;
    void *out;
    const float *q;  // [d1][d1]
    const float *fg, *fd;
    const float2 *cs;
    const int *fast_bad;
    PlanRef plan;
    int64_t rows;
    int d1;
    int bfly_threads;  // threads of the butterfly group (whole waves); the mix group follows
};

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8b __attribute__((ext_vector_type(8)));

// Two-way bfloat16 split of float32 values for the matrix cores: v = hi + lo + e with hi = v rounded to
// bfloat16 (8 significant bits), lo = (v - hi) rounded to bfloat16 (the difference is exact), |e| <= 2^-16 |v|.
// bfloat16 has float32's exponent range, so no scaling is needed.  Eight values make one operand of
// v_mfma_f32_16x16x32_bf16 (four registers).
__device__ __forceinline__ uint32_t bf16_bits_of(float v) { return (__float_as_uint(v) + 0x8000u) & 0xFFFF0000u; }
__device__ __forceinline__ void split8_bf16(const float (&v)[8], v8b *hi, v8b *lo)
{
    uint32_t h[8], l[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        h[j] = bf16_bits_of(v[j]);
        l[j] = bf16_bits_of(v[j] - __uint_as_float(h[j]));
    }
    *hi = __builtin_bit_cast(v8b, make_uint4((h[0] >> 16) | h[1], (h[2] >> 16) | h[3], (h[4] >> 16) | h[5], (h[6] >> 16) | h[7]));
    *lo = __builtin_bit_cast(v8b, make_uint4((l[0] >> 16) | l[1], (l[2] >> 16) | l[3], (l[4] >> 16) | l[5], (l[6] >> 16) | l[7]));
}

// KS: steps of four input sub-rows (d1 <= 4 KS; inputs past d1 carry zero weights and re-read the last
// sub-row), IT = ceil(KS / 4) blocks of 16 output sub-rows.  kSlow: the variant for plans whose scale-deferred tables
// are flagged unusable (plain rotations); both variants are launched and the one that does not apply exits at
// once, which keeps the out-of-line rotation code, and the stack traffic it brings, out of the fast variant.
template <typename T, bool kInverse, int KS, bool kSlow>
__global__ __launch_bounds__(kFusedMaxThreads) void kron128_kernel(FusedArgs A)
{
    constexpr int IT = (KS + 3) / 4;
    extern __shared__ __align__(16) float tile[];  // 3 kStepRows x [d1][kTileRow]
    if (!plan_matches(A.plan) || (*A.fast_bad != 0) != kSlow) return;
    const int d1 = A.d1;
    const int tile_floats = d1 * kTileRow;
    const int tid = threadIdx.x, lane = tid & 63;
    const int64_t mine = A.rows > (int64_t)blockIdx.x ? (A.rows - blockIdx.x + gridDim.x - 1) / gridDim.x : 0;
    const int64_t width = (int64_t)d1 * kFusedD2;
    // Step s: the butterfly group transforms rows kStepRows * s .. + kStepRows - 1 into the tiles of slot s % 3, the mix
    // group takes the rows of step s - 1 and the store group those of step s - 2; one barrier per step.
    const int64_t steps = (mine + kStepRows - 1) / kStepRows + 2;
    auto tile_of = [&](int64_t step, int r) { return tile + ((int)(step % 3) * kStepRows + r) * tile_floats; };
    if (tid < A.bfly_threads) {
        // ---- butterfly group ---------------------------------------------------------------------------------
        const int sub = tid >> 4, l16 = tid & 15;
        const int idx = lane_chunk(l16) * 8;  // first column of the thread's 8 elements
        const bool live = sub < d1;
        float c[7][8], d[8];
#pragma unroll
        for (int j = 0; j < 7; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r) c[j][r] = A.fg[j * kFusedD2 + idx + r];
#pragma unroll
        for (int r = 0; r < 8; ++r) d[r] = A.fd[idx + r];
        const T *in = (const T *)A.in + (size_t)sub * kFusedD2 + idx;
        // kAhead rows are in flight from memory: a compute unit runs one workgroup, and a row is only 256 bytes
        // per sub-row, so it takes several to cover the latency (four instead of two: d1 = 8 and 16 run 20 % and
        // 16 % faster; d1 = 40, which is bound by arithmetic, is unchanged; six measured slower again).
        // This group only loads; the rows are stored by the store group: memory operations of a wave retire
        // in order, so a wave that both stores and prefetches ends up waiting for its stores to be
        // acknowledged before it may use a prefetched row.
        constexpr int kAhead = 4;
        Raw8 raw[kAhead] = {};
#pragma unroll
        for (int a = 0; a < kAhead; ++a)
            if (live && mine > a) raw[a] = load8(in + ((int64_t)blockIdx.x + a * (int64_t)gridDim.x) * width);
        // one step: row `it` out of `slot`, which is then refilled with row it + kAhead (the loop below is unrolled
        // over the slots, so that no row moves between registers)
        auto row_step = [&](int64_t it, Raw8 &slot, float *z_tile) {
            if (live && it < mine) {  // transform row it
                float u[8];
                unpack8(slot, u, (const T *)nullptr);
                if (it + kAhead < mine) slot = load8(in + (blockIdx.x + (it + kAhead) * gridDim.x) * width);
                if (!kSlow)
                    fast_small<7, kInverse>(u, c, d);
                else
                    slow_small<7, kInverse>(u, A.cs, idx);
                if (kSplitMix<T>) {
                    // binary16 rows: the tile takes each value as its two-way bfloat16 split, hi (rounded) in the upper
                    // half of the word and lo (truncated: |v - hi - lo| < 2^-16 |v| either way) in the lower, ready
                    // to be packed into matrix operands by the mix group
#pragma unroll
                    for (int r = 0; r < 8; ++r) {
                        const uint32_t h = bf16_bits_of(u[r]);
                        const float rest = u[r] - __uint_as_float(h);
                        u[r] = __uint_as_float(__builtin_amdgcn_perm(h, __float_as_uint(rest), 0x07060302u));
                    }
                }
                float4 *dst = (float4 *)&z_tile[sub * kTileRow + idx];
                dst[0] = make_float4(u[0], u[1], u[2], u[3]);
                dst[1] = make_float4(u[4], u[5], u[6], u[7]);
            }
        };
        static_assert(kAhead % kStepRows == 0, "whole steps per turn of the prefetch slots");
        for (int64_t st = 0; st < steps; st += kAhead / kStepRows) {
#pragma unroll
            for (int h = 0; h < kAhead / kStepRows; ++h)
                if (st + h < steps) {
#pragma unroll
                    for (int r = 0; r < kStepRows; ++r)
                        row_step((st + h) * kStepRows + r, raw[h * kStepRows + r], tile_of(st + h, r));
                    __syncthreads();
                }
        }
    } else if (tid >= A.bfly_threads + kMixWaves * 64) {
        // ---- store group: row it-2, 16-byte pieces of 8 consecutive elements, one rounding to the row type ------
        const int stid = tid - A.bfly_threads - kMixWaves * 64;
        // pieces per lane (d1 <= 4 KS sub-rows of 16 pieces over the group's lanes): all of a row's tile reads are
        // issued before the first conversion, so their latency is paid once per row
        constexpr int kPieces = (4 * KS * 16 + kStoreWaves * 64 - 1) / (kStoreWaves * 64);
        for (int64_t st = 0; st < steps; ++st) {
            for (int r = 0; r < kStepRows; ++r) {
                const int64_t row = (st - 2) * kStepRows + r;
                if (st < 2 || row >= mine) continue;
                const float *y_tile = tile_of(st - 2, r);
                T *out_row = (T *)A.out + (blockIdx.x + row * gridDim.x) * width;
                float4 a[kPieces], b[kPieces];
#pragma unroll
                for (int p = 0; p < kPieces; ++p) {
                    const int piece = stid + p * kStoreWaves * 64;
                    if (piece < d1 * 16) {
                        const float4 *src = (const float4 *)&y_tile[(piece >> 4) * kTileRow + (piece & 15) * 8];
                        a[p] = src[0];
                        b[p] = src[1];
                    }
                }
#pragma unroll
                for (int p = 0; p < kPieces; ++p) {
                    const int piece = stid + p * kStoreWaves * 64;
                    if (piece < d1 * 16) {
                        const float y[8] = {a[p].x, a[p].y, a[p].z, a[p].w, b[p].x, b[p].y, b[p].z, b[p].w};
                        store8(out_row + (piece >> 4) * kFusedD2 + (piece & 15) * 8, y);
                    }
                }
            }
            __syncthreads();
        }
    } else {
        // ---- mix group ---------------------------------------------------------------------------------------
        const int mw = (tid - A.bfly_threads) >> 6;  // 0 .. kMixWaves-1: column blocks 2 mw and 2 mw + 1
        if constexpr (kSplitMix<T>) {
            // binary16 rows: the product runs on the bfloat16 matrix instruction with two-way splits of both
            // factors, Y = Q_hi Z_hi + Q_hi Z_lo + Q_lo Z_hi accumulated in float32 (relative error of a term
            // below 3 * 2^-16 = 4.6e-5, a tenth of such a row's rounding step), because the float32 matrix
            // instruction does not overlap the other groups' vector work and costs four times the cycles.
            // Contraction index of lane l, element j of an operand, step s: k = 32 s + l / 16 + 4 j (the same
            // map in both operands; consecutive k over the lane groups keeps the tile reads two per bank).
            constexpr int SK = (4 * KS + 31) / 32;  // steps of 32 input sub-rows
            v8b qh[IT][SK], ql[IT][SK];
#pragma unroll
            for (int t = 0; t < IT; ++t)
#pragma unroll
                for (int s2 = 0; s2 < SK; ++s2) {
                    float w[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const int i = 16 * t + (lane & 15), k = 32 * s2 + (lane >> 4) + 4 * j;
                        w[j] = (i < d1 && k < d1) ? (kInverse ? A.q[k * d1 + i] : A.q[i * d1 + k]) : 0.0f;
                    }
                    split8_bf16(w, &qh[t][s2], &ql[t][s2]);
                }
            for (int64_t st = 0; st < steps; ++st) {
                for (int r2 = 0; r2 < kStepRows; ++r2) {  // mix the rows of step st-1 in place
                    if (st < 1 || (st - 1) * kStepRows + r2 >= mine) continue;
                    float *t = tile_of(st - 1, r2) + 32 * mw + (lane & 15);
                    v4f acc[2][IT];
#pragma unroll
                    for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                        for (int i = 0; i < IT; ++i) acc[jb][i] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                    for (int s2 = 0; s2 < SK; ++s2) {
                        uint32_t z[2][8];  // operand words (hi | lo)
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            int k = 32 * s2 + (lane >> 4) + 4 * j;
                            k = k < d1 ? k : d1 - 1;  // weight zero
                            z[0][j] = __float_as_uint(t[k * kTileRow]);
                            z[1][j] = __float_as_uint(t[k * kTileRow + 16]);
                        }
                        v8b zh[2], zl[2];
#pragma unroll
                        for (int jb = 0; jb < 2; ++jb) {
                            const uint32_t *w = z[jb];
                            zh[jb] = __builtin_bit_cast(v8b, make_uint4(__builtin_amdgcn_perm(w[1], w[0], 0x07060302u),
                                                                        __builtin_amdgcn_perm(w[3], w[2], 0x07060302u),
                                                                        __builtin_amdgcn_perm(w[5], w[4], 0x07060302u),
                                                                        __builtin_amdgcn_perm(w[7], w[6], 0x07060302u)));
                            zl[jb] = __builtin_bit_cast(v8b, make_uint4(__builtin_amdgcn_perm(w[1], w[0], 0x05040100u),
                                                                        __builtin_amdgcn_perm(w[3], w[2], 0x05040100u),
                                                                        __builtin_amdgcn_perm(w[5], w[4], 0x05040100u),
                                                                        __builtin_amdgcn_perm(w[7], w[6], 0x05040100u)));
                        }
                        // the small products first; 2 IT independent accumulators between two uses of the same one
#pragma unroll
                        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                            for (int i = 0; i < IT; ++i)
                                acc[jb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ql[i][s2], zh[jb], acc[jb][i], 0, 0, 0);
#pragma unroll
                        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                            for (int i = 0; i < IT; ++i)
                                acc[jb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qh[i][s2], zl[jb], acc[jb][i], 0, 0, 0);
#pragma unroll
                        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                            for (int i = 0; i < IT; ++i)
                                acc[jb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qh[i][s2], zh[jb], acc[jb][i], 0, 0, 0);
                    }
#pragma unroll
                    for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                        for (int i = 0; i < IT; ++i)
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const int o = 16 * i + 4 * (lane >> 4) + r;
                                if (o < d1) t[o * kTileRow + 16 * jb] = acc[jb][i][r];
                            }
                }
                __syncthreads();
            }
            return;
        }
        // A operands: the weight of input sub-row k in output sub-row i is Q1[i][k] (forward) or Q1[k][i]
        float qa[IT][KS];
#pragma unroll
        for (int t = 0; t < IT; ++t)
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const int i = 16 * t + (lane & 15), k = 4 * s + (lane >> 4);
                qa[t][s] = (i < d1 && k < d1) ? (kInverse ? A.q[k * d1 + i] : A.q[i * d1 + k]) : 0.0f;
            }
        for (int64_t st = 0; st < steps; ++st) {
            for (int r2 = 0; r2 < kStepRows; ++r2) {  // mix the rows of step st-1 in place
                if (st < 1 || (st - 1) * kStepRows + r2 >= mine) continue;
                float *t = tile_of(st - 1, r2) + 32 * mw + (lane & 15);
                v4f acc[2][IT];
#pragma unroll
                for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                    for (int i = 0; i < IT; ++i) acc[jb][i] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
                // all B operands of the row first (branch-free, so the reads overlap the matrix instructions)
                float b0[KS], b1[KS];
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    int k = 4 * s + (lane >> 4);
                    k = k < d1 ? k : d1 - 1;
                    b0[s] = t[k * kTileRow];
                    b1[s] = t[k * kTileRow + 16];
                }
#pragma unroll
                for (int s = 0; s < KS; ++s)
#pragma unroll
                    for (int i = 0; i < IT; ++i) {
                        acc[0][i] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[i][s], b0[s], acc[0][i], 0, 0, 0);
                        acc[1][i] = __builtin_amdgcn_mfma_f32_16x16x4f32(qa[i][s], b1[s], acc[1][i], 0, 0, 0);
                    }
#pragma unroll
                for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                    for (int i = 0; i < IT; ++i)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int o = 16 * i + 4 * (lane >> 4) + r;
                            if (o < d1) t[o * kTileRow + 16 * jb] = acc[jb][i][r];
                        }
            }
            __syncthreads();
        }
    }
}

bool kron_fused_supported(const void *in, const void *out, int d1, int d2)
{
    return d2 == kFusedD2 && d1 >= 2 && d1 <= kFusedMaxD1 && !((uintptr_t)in & 15) && !((uintptr_t)out & 15);
}

template <typename T, bool kInverse>
static hipError_t launch_kron_fused_t(FusedArgs &A, hipStream_t stream)
{
    A.bfly_threads = ((A.d1 * 16 + 63) / 64) * 64;  // 16 lanes per sub-row, whole waves
    const int threads = A.bfly_threads + (kMixWaves + kStoreWaves) * 64;
    const size_t lds = 3 * kStepRows * (size_t)A.d1 * kTileRow * sizeof(float);
    void (*kern)(FusedArgs), (*kern_slow)(FusedArgs);
    if (A.d1 <= 16) {
        kern = kron128_kernel<T, kInverse, 4, false>;
        kern_slow = kron128_kernel<T, kInverse, 4, true>;
    } else if (A.d1 <= 32) {
        kern = kron128_kernel<T, kInverse, 8, false>;
        kern_slow = kron128_kernel<T, kInverse, 8, true>;
    } else {
        kern = kron128_kernel<T, kInverse, 10, false>;
        kern_slow = kron128_kernel<T, kInverse, 10, true>;
    }
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)kern_slow, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    // one workgroup per compute unit; two for d1 <= 8 (8 waves each), which a single one leaves latency-bound
    // (d1 = 8: 0.81 -> 0.54 ms for 327680 rows; at d1 = 16 two fit as well but measured no faster)
    int64_t grid = A.d1 <= 8 ? 512 : 256;
    if (grid > A.rows) grid = A.rows;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(threads), lds, stream, A);
    hipLaunchKernelGGL(kern_slow, dim3((unsigned)grid), dim3(threads), lds, stream, A);
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
    A.plan = pv.ref;
    A.rows = rows;
    A.d1 = d1;
    if (inverse) {
        switch (dtype) {
            case BQ_F32: return launch_kron_fused_t<float, true>(A, stream);
            case BQ_F16: return launch_kron_fused_t<__half, true>(A, stream);
            default: return launch_kron_fused_t<bf16_t, true>(A, stream);
        }
    }
    switch (dtype) {
        case BQ_F32: return launch_kron_fused_t<float, false>(A, stream);
        case BQ_F16: return launch_kron_fused_t<__half, false>(A, stream);
        default: return launch_kron_fused_t<bf16_t, false>(A, stream);
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
