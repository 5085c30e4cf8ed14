// Generic kernels: any power-of-two n up to 16384, any head count, any row type.  One tile of rows
// lives in LDS as float32; every layer is one sweep over the tile's index pairs with (cos, sin)
// read from the plan.  These kernels are the library's fallback for shapes without a specialised
// kernel; they favour simplicity over speed.
//
// Layer i (1-based) pairs a = ((p >> (i-1)) << i) | (p & (2^(i-1) - 1)) with b = a + 2^(i-1) for the
// pair index p = 0..n/2-1, i.e. the p-th pair in increasing order of a (paper, appendix "Concrete
// Example: Butterfly Matrix Structure for n=8").
#include "bq_device.h"

namespace bq {

constexpr int kGenThreads = 256;
constexpr int kGenTileMin = 2048;  // elements per tile for small n (several transforms per tile)
constexpr int kBwdTileMin = 1024;

struct GenArgs {
    const void *in;
    void *out;
    const float2 *cs;
    PlanRef plan;
    int64_t rows, ld_in, ld_out;
    int n, heads, k;
    int tile_elems;  // U * n
    int64_t n_tiles;
    // quantiser
    uint8_t *codes;
    void *scales;
    unsigned long long *hist;
    int bits, group, scale_f16;
};

template <bool kInverse>
__device__ __forceinline__ void rotate_pair(float &va, float &vb, float c, float s)
{
    const float xa = va, xb = vb;
    if (!kInverse) {  // G(theta):  [c -s; s c]
        va = __builtin_fmaf(c, xa, -(s * xb));
        vb = __builtin_fmaf(s, xa, c * xb);
    } else {  // G(theta)^T: [c s; -s c]
        va = __builtin_fmaf(c, xa, s * xb);
        vb = __builtin_fmaf(c, xb, -(s * xa));
    }
}

// One layer over a whole tile held in LDS.  Units of a tile are consecutive (row, head) pairs.
template <bool kInverse>
__device__ __forceinline__ void tile_layer(float *buf, const float2 *__restrict__ cs, int i, int n, int k,
                                           int heads, int64_t unit0, int tile_elems)
{
    const int h = 1 << (i - 1);
    const int half_mask = (n >> 1) - 1;
    for (int q = threadIdx.x; q < (tile_elems >> 1); q += kGenThreads) {
        const int ul = q >> (k - 1);
        const int p = q & half_mask;
        const int head = (int)((unit0 + ul) % heads);
        const float2 w = cs[((size_t)head * k + (i - 1)) * (size_t)(n >> 1) + p];
        const int a = (ul << k) + (((p >> (i - 1)) << i) | (p & (h - 1)));
        rotate_pair<kInverse>(buf[a], buf[a + h], w.x, w.y);
    }
}

template <typename T, int kMode>
__global__ __launch_bounds__(kGenThreads) void generic_kernel(GenArgs A)
{
    extern __shared__ float lds[];
    if (!plan_matches(A.plan)) return;
    float *buf = lds;
    float *inv_lds = lds + A.tile_elems;  // one reciprocal scale per group of the tile
    float *s_lds = inv_lds + A.tile_elems / (A.group > 0 ? A.group : 1);  // kFwdFake: the scales themselves
    __shared__ unsigned hist_lds[16];
    const T *__restrict__ in = (const T *)A.in;
    T *__restrict__ out = (T *)A.out;
    const int n = A.n, k = A.k, heads = A.heads;
    const int units_per_tile = A.tile_elems >> k;
    const int64_t total_units = A.rows * heads;

    for (int64_t tile = blockIdx.x; tile < A.n_tiles; tile += gridDim.x) {
        const int64_t unit0 = tile * units_per_tile;
        for (int e = threadIdx.x; e < A.tile_elems; e += kGenThreads) {
            const int64_t unit = unit0 + (e >> k);
            float v = 0.0f;
            if (unit < total_units) {
                const int64_t row = unit / heads;
                const int head = (int)(unit - row * heads);
                v = to_float(in[row * A.ld_in + (int64_t)head * n + (e & (n - 1))]);
            }
            buf[e] = v;
        }
        __syncthreads();
        if (kMode == kInv) {
            for (int i = k; i >= 1; --i) {
                tile_layer<true>(buf, A.cs, i, n, k, heads, unit0, A.tile_elems);
                __syncthreads();
            }
        } else {
            for (int i = 1; i <= k; ++i) {
                tile_layer<false>(buf, A.cs, i, n, k, heads, unit0, A.tile_elems);
                __syncthreads();
            }
        }
        if (kMode == kFwd || kMode == kInv) {
            for (int e = threadIdx.x; e < A.tile_elems; e += kGenThreads) {
                const int64_t unit = unit0 + (e >> k);
                if (unit < total_units) {
                    const int64_t row = unit / heads;
                    const int head = (int)(unit - row * heads);
                    out[row * A.ld_out + (int64_t)head * n + (e & (n - 1))] = from_float<T>(buf[e]);
                }
            }
        } else {
            const int group = A.group;
            const int groups_per_unit = n / group;
            const int n_groups = A.tile_elems / group;
            const float qmax = (float)((1 << (A.bits - 1)) - 1);
            const float qmin = -(float)(1 << (A.bits - 1));
            for (int g = threadIdx.x; g < n_groups; g += kGenThreads) {
                const float *v = buf + (size_t)g * group;
                float amax = 0.0f;
                for (int j = 0; j < group; ++j) amax = fmaxf(amax, fabsf(v[j]));
                float inv;
                const float s = group_scale(amax, qmax, A.scale_f16 != 0, &inv);
                inv_lds[g] = inv;
                if (kMode == kFwdFake) s_lds[g] = s;
                const int64_t unit = unit0 + g / groups_per_unit;
                if (kMode == kFwdQuant && unit < total_units) {
                    const int64_t sidx = unit * groups_per_unit + (g % groups_per_unit);
                    if (A.scale_f16)
                        ((__half *)A.scales)[sidx] = __float2half_rn(s);
                    else
                        ((float *)A.scales)[sidx] = s;
                }
            }
            if (kMode == kFwdFake && threadIdx.x < 16) hist_lds[threadIdx.x] = 0;
            __syncthreads();
            if (kMode == kFwdFake) {
                // Dequant(Quant(v)) = s * q, one float32 multiplication, then one rounding to the row type;
                // bin occupancy through LDS counters, added to the caller's once per tile
                const int off = 1 << (A.bits - 1);
                for (int e = threadIdx.x; e < A.tile_elems; e += kGenThreads) {
                    const int64_t unit = unit0 + (e >> k);
                    if (unit >= total_units) continue;
                    const int g = e / group;
                    const int q = quant_code(buf[e], inv_lds[g], qmin, qmax);
                    if (out) {
                        const int64_t row = unit / heads;
                        const int head = (int)(unit - row * heads);
                        float p = s_lds[g] * (float)q;
                        asm volatile("" : "+v"(p));  // a float32 product: not merged with the conversion below
                        out[row * A.ld_out + (int64_t)head * n + (e & (n - 1))] = from_float<T>(p);
                    }
                    if (A.hist) atomicAdd(&hist_lds[q + off], 1u);
                }
                __syncthreads();
                if (A.hist && threadIdx.x < (1 << A.bits) && hist_lds[threadIdx.x] != 0)
                    atomicAdd(&A.hist[threadIdx.x], (unsigned long long)hist_lds[threadIdx.x]);
                __syncthreads();
                continue;
            }
            const int per = 8 / A.bits;
            const int tile_bytes = A.tile_elems / per;
            const int64_t unit_bytes = n / per;
            const unsigned mask = (1u << A.bits) - 1u;
            for (int b = threadIdx.x; b < tile_bytes; b += kGenThreads) {
                const int e0 = b * per;
                const float inv = inv_lds[e0 / group];
                unsigned byte = 0;
                for (int j = 0; j < per; ++j)
                    byte |= ((unsigned)quant_code(buf[e0 + j], inv, qmin, qmax) & mask) << (j * A.bits);
                const int64_t unit = unit0 + (e0 >> k);
                if (unit < total_units) A.codes[unit0 * unit_bytes + b] = (uint8_t)byte;
            }
        }
        __syncthreads();
    }
}

template <typename T>
static hipError_t launch_generic_t(Mode mode, GenArgs &A, size_t lds_bytes, unsigned grid, hipStream_t stream)
{
    void (*kern)(GenArgs) = nullptr;
    switch (mode) {
        case kFwd: kern = generic_kernel<T, kFwd>; break;
        case kInv: kern = generic_kernel<T, kInv>; break;
        case kFwdQuant: kern = generic_kernel<T, kFwdQuant>; break;
        case kFwdFake: kern = generic_kernel<T, kFwdFake>; break;
    }
    if (lds_bytes > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_bytes);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kGenThreads), lds_bytes, stream, A);
    return hipGetLastError();
}

hipError_t launch_generic(Mode mode, const void *in, void *out, const PlanView &pv, const Shape &s,
                          const QuantArgs *q, hipStream_t stream)
{
    GenArgs A{};
    A.in = in;
    A.out = out;
    A.cs = pv.cs;
    A.plan = pv.ref;
    A.rows = s.rows;
    A.ld_in = s.ld_x;
    A.ld_out = s.ld_y;
    A.n = s.n;
    A.heads = s.heads;
    A.k = s.k;
    A.tile_elems = s.n > kGenTileMin ? s.n : kGenTileMin;
    const int units_per_tile = A.tile_elems / s.n;
    const int64_t total_units = s.rows * s.heads;
    A.n_tiles = (total_units + units_per_tile - 1) / units_per_tile;
    if (q) {
        A.codes = q->codes;
        A.scales = q->scales;
        A.hist = q->hist;
        A.bits = q->bits;
        A.group = q->group;
        A.scale_f16 = q->scale_f16;
    }
    size_t lds_bytes = (size_t)A.tile_elems * sizeof(float);
    if (mode == kFwdQuant) lds_bytes += (size_t)(A.tile_elems / q->group) * sizeof(float);
    if (mode == kFwdFake) lds_bytes += 2 * (size_t)(A.tile_elems / q->group) * sizeof(float);
    unsigned grid = (unsigned)(A.n_tiles < 4096 ? A.n_tiles : 4096);
    switch (s.dtype) {
        case BQ_F32: return launch_generic_t<float>(mode, A, lds_bytes, grid, stream);
        case BQ_F16: return launch_generic_t<__half>(mode, A, lds_bytes, grid, stream);
        default: return launch_generic_t<bf16_t>(mode, A, lds_bytes, grid, stream);
    }
}

__global__ void hist_clear_kernel(unsigned long long *hist, int count)
{
    if ((int)threadIdx.x < count) hist[threadIdx.x] = 0ull;
}

hipError_t launch_hist_clear(unsigned long long *hist, int bits, hipStream_t stream)
{
    hipLaunchKernelGGL(hist_clear_kernel, dim3(1), dim3(64), 0, stream, hist, 1 << bits);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Backward.  A tile is U consecutive rows of ONE head, so that the thread owning pair p of a layer
// owns it for every row of the tile and for every tile its workgroup processes: the per-workgroup
// partial sums in `partial` are read-modify-written by one thread only, in a fixed order.
// dtheta_{i,p} += g_i[b] x_i[a] - g_i[a] x_i[b], evaluated on the layer's outputs (which follows from
// dG/dtheta = [[-s,-c],[c,-s]]: d y_a / d theta = -y_b, d y_b / d theta = y_a); then both x_i and g_i
// are taken back through the transposed layer (orthogonality makes stored activations unnecessary).
// ---------------------------------------------------------------------------------------------
struct BwdArgs {
    const void *x, *dy;
    void *dx;
    const float2 *cs;
    float *partial;  // [grid][heads*k*n/2]
    int64_t rows, ld_in, ld_out;
    int n, heads, k, rows_per_tile;
    int64_t n_tiles;
    PlanRef plan;
    int only_if_bad;  // != 0: run only when one of the plan's table sets is flagged unusable
};

template <typename T>
__global__ __launch_bounds__(kGenThreads) void generic_bwd_kernel(BwdArgs A)
{
    extern __shared__ float lds[];
    if (!plan_matches(A.plan) || (A.only_if_bad && plan_fast_both(A.plan))) return;
    const int n = A.n, k = A.k, heads = A.heads, U = A.rows_per_tile;
    float *xb = lds;
    float *gb = lds + (size_t)U * n;
    const T *__restrict__ x = (const T *)A.x;
    const T *__restrict__ dy = (const T *)A.dy;
    T *__restrict__ dx = (T *)A.dx;
    const size_t n_angles = (size_t)heads * k * (n >> 1);
    float *__restrict__ part = A.partial + (size_t)blockIdx.x * n_angles;
    for (size_t q = threadIdx.x; q < n_angles; q += kGenThreads) part[q] = 0.0f;

    for (int64_t tile = blockIdx.x; tile < A.n_tiles; tile += gridDim.x) {
        const int head = (int)(tile % heads);
        const int64_t row0 = (tile / heads) * U;
        for (int e = threadIdx.x; e < U * n; e += kGenThreads) {
            const int64_t row = row0 + (e >> k);
            float vx = 0.0f, vg = 0.0f;
            if (row < A.rows) {
                const int64_t off = row * A.ld_in + (int64_t)head * n + (e & (n - 1));
                vx = to_float(x[off]);
                vg = to_float(dy[off]);
            }
            xb[e] = vx;
            gb[e] = vg;
        }
        __syncthreads();
        const float2 *__restrict__ csh = A.cs + (size_t)head * k * (n >> 1);
        for (int i = 1; i <= k; ++i) {  // recompute the layer outputs x_1 .. x_k
            const int h = 1 << (i - 1);
            for (int q = threadIdx.x; q < ((U * n) >> 1); q += kGenThreads) {
                const int ul = q >> (k - 1);
                const int p = q & ((n >> 1) - 1);
                const float2 w = csh[(size_t)(i - 1) * (n >> 1) + p];
                const int a = (ul << k) + (((p >> (i - 1)) << i) | (p & (h - 1)));
                rotate_pair<false>(xb[a], xb[a + h], w.x, w.y);
            }
            __syncthreads();
        }
        for (int i = k; i >= 1; --i) {
            const int h = 1 << (i - 1);
            for (int p = threadIdx.x; p < (n >> 1); p += kGenThreads) {
                const float2 w = csh[(size_t)(i - 1) * (n >> 1) + p];
                const int a0 = ((p >> (i - 1)) << i) | (p & (h - 1));
                float acc = 0.0f;
                for (int ul = 0; ul < U; ++ul) {
                    const int a = (ul << k) + a0;
                    float xa = xb[a], xv = xb[a + h], ga = gb[a], gv = gb[a + h];
                    acc += gv * xa - ga * xv;
                    rotate_pair<true>(xa, xv, w.x, w.y);
                    rotate_pair<true>(ga, gv, w.x, w.y);
                    xb[a] = xa;
                    xb[a + h] = xv;
                    gb[a] = ga;
                    gb[a + h] = gv;
                }
                part[((size_t)head * k + (i - 1)) * (size_t)(n >> 1) + p] += acc;
            }
            __syncthreads();
        }
        if (dx) {
            for (int e = threadIdx.x; e < U * n; e += kGenThreads) {
                const int64_t row = row0 + (e >> k);
                if (row < A.rows)
                    dx[row * A.ld_out + (int64_t)head * n + (e & (n - 1))] = from_float<T>(gb[e]);
            }
        }
        __syncthreads();
    }
}

// dtheta[q] = sum over workgroups of partial[w][q], accumulated in double in workgroup order.
__global__ void reduce_partials_kernel(const float *__restrict__ partial, float *__restrict__ dtheta,
                                       size_t n_angles, int n_parts, PlanRef plan, int only_if_bad)
{
    if (!plan_matches(plan) || (only_if_bad && plan_fast_both(plan))) return;
    size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= n_angles) return;
    double acc = 0.0;
    for (int w = 0; w < n_parts; ++w) acc += (double)partial[(size_t)w * n_angles + q];
    dtheta[q] = (float)acc;
}

static void bwd_geometry(const Shape &s, int *rows_per_tile, int64_t *n_tiles, unsigned *grid)
{
    int U = s.n >= kBwdTileMin ? 1 : kBwdTileMin / s.n;
    int64_t chunks = (s.rows + U - 1) / U;
    int64_t tiles = chunks * s.heads;
    // the grid must be a multiple of heads so that a workgroup always sees the same head sequence;
    // any grid works for correctness, this one keeps partial slices dense
    int64_t g = tiles < 512 ? tiles : 512;
    // ... and the partial slices (one per workgroup) within 32 MiB where 8 workgroups or more still fit
    const int64_t slice_bytes = (int64_t)s.heads * s.k * (s.n / 2) * (int64_t)sizeof(float);
    int64_t cap = ((int64_t)32 << 20) / slice_bytes;
    cap -= cap % s.heads;
    if (cap < 8 * (int64_t)s.heads) cap = 8 * (int64_t)s.heads;
    if (g > cap) g = cap;
    if (g < 1) g = 1;
    *rows_per_tile = U;
    *n_tiles = tiles;
    *grid = (unsigned)g;
}

size_t bwd_workspace_bytes_generic(const Shape &s)
{
    int U;
    int64_t tiles;
    unsigned grid;
    bwd_geometry(s, &U, &tiles, &grid);
    size_t n_angles = (size_t)s.heads * s.k * (s.n / 2);
    return align256((size_t)grid * n_angles * sizeof(float));
}

hipError_t launch_generic_bwd(const void *x, const void *dy, const PlanView &pv, void *dx, float *dtheta,
                              void *ws, const Shape &s, hipStream_t stream, bool only_if_bad)
{
    BwdArgs A{};
    unsigned grid;
    bwd_geometry(s, &A.rows_per_tile, &A.n_tiles, &grid);
    A.x = x;
    A.dy = dy;
    A.dx = dx;
    A.cs = pv.cs;
    A.partial = (float *)ws;
    A.rows = s.rows;
    A.ld_in = s.ld_x;
    A.ld_out = s.ld_y;
    A.n = s.n;
    A.heads = s.heads;
    A.k = s.k;
    A.plan = pv.ref;
    A.only_if_bad = only_if_bad ? 1 : 0;
    size_t lds_bytes = (size_t)2 * A.rows_per_tile * s.n * sizeof(float);
    void (*kern)(BwdArgs) = s.dtype == BQ_F32   ? generic_bwd_kernel<float>
                            : s.dtype == BQ_F16 ? generic_bwd_kernel<__half>
                                                : generic_bwd_kernel<bf16_t>;
    if (lds_bytes > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_bytes);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kGenThreads), lds_bytes, stream, A);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (dtheta) {
        size_t n_angles = (size_t)s.heads * s.k * (s.n / 2);
        unsigned blocks = (unsigned)((n_angles + 255) / 256);
        hipLaunchKernelGGL(reduce_partials_kernel, dim3(blocks), dim3(256), 0, stream, (const float *)ws, dtheta,
                           n_angles, (int)grid, A.plan, A.only_if_bad);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace bq
