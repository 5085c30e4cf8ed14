// Backward pass for small transforms, n = 8 .. 128 (k = 3 .. 7), for the row widths the small forward kernels
// take: dx = B^T dy and dtheta (paper, "Gradient Flow Through Butterfly Layers").
//
// Geometry of the small forward kernels (bq_small.hip): a transform occupies n/8 consecutive lanes, 8
// consecutive elements per lane, no LDS and no barrier; a workgroup of 256 threads covers 2048 consecutive
// elements (a slice of a wide row or several narrow rows) and loops over the batch.  Per row a thread
// recomputes the forward state of its 8 elements (layers 1..k), then runs the transposed cascade on the
// state and the gradient together with the deferred sums of bq_bwd_blocks.h.  Everything a thread needs
// for that (both directions' coefficients, 44 sums) stays in registers: about 230 of them, so two waves
// share a SIMD; the loop has no dependence on LDS or barriers to hide.
//
// Partial sums: every (workgroup, row position inside its span) pair owns one slot of `partial` holding all
// angles; an entry is written by exactly one thread.  A second kernel adds the slots in double in a fixed
// order: no atomics, the result does not depend on scheduling.
//
// The kernels exit at once when the plan flags the scale-deferred tables as unusable; the generic backward
// kernel, launched behind them with the opposite condition, then does the work.
#include "bq_bwd_blocks.h"
#include "bq_internal.h"

namespace bq {

constexpr int kSbThreads = 256;
constexpr int kSbMaxSlots = 4096;  // (8192 measured no faster for narrow rows and slower where the reduction grows)

struct SmallBwdArgs {
    const void *x, *dy;
    void *dx;
    float *partial;  // [slots][n_angles]
    const float *fg_fwd, *fd_fwd, *fg_inv, *fd_inv, *fw_inv;
    const int *bad_fwd, *bad_inv;
    PlanRef plan;
    int64_t rows, ld_in, ld_out;
    int heads, width;    // width = heads * n
    int span;            // elements covered by a workgroup: 2048, or the largest power of two below it that
                         // divides a wider row (the workgroup then has span / 8 threads)
    int rows_per_block;  // span / width if width < span, else 1
    int slices;          // width / span if width >= span, else 1
    int64_t n_groups;    // row groups = ceil(rows / rows_per_block)
    int64_t n_angles;    // heads * k * n / 2
};

template <typename T, int K, bool kDx>
__global__ __launch_bounds__(kSbThreads) void small_bwd_kernel(SmallBwdArgs A)
{
    constexpr int n = 1 << K;
    if (!plan_matches(A.plan) || (*A.bad_fwd | *A.bad_inv) != 0) return;
    const int tid = threadIdx.x;
    const int chunk = (tid & ~15) | lane_chunk(tid & 15);  // chunk of 8 elements inside the workgroup's span
    const int e0 = chunk * 8;
    int row_in_block, col;
    int64_t grp_first, grp_step, slot;
    if (A.slices > 1) {
        row_in_block = 0;
        col = (int)(blockIdx.x % A.slices) * A.span + e0;
        grp_first = blockIdx.x / A.slices;
        grp_step = gridDim.x / A.slices;
        slot = grp_first;
    } else {
        row_in_block = e0 / A.width;
        col = e0 - row_in_block * A.width;
        grp_first = blockIdx.x;
        grp_step = gridDim.x;
        slot = (int64_t)blockIdx.x * A.rows_per_block + row_in_block;
    }
    const int head = col >> K;
    const int idx = col & (n - 1);
    const uint32_t col_bytes = (uint32_t)col * (uint32_t)sizeof(T);

    float cf[7][8], df[8], di[8];
    CoefRegs ci;
    {
        const float *ff = A.fg_fwd + (size_t)head * K * n, *fi = A.fg_inv + (size_t)head * K * n;
#pragma unroll
        for (int j = 0; j < 7; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r) {  // layers above k do not exist: weight zero leaves the element as it is
                cf[j][r] = (j < K) ? ff[j * n + idx + r] : 0.0f;
                ci.c[j][r] = (j < K) ? fi[j * n + idx + r] : 0.0f;
            }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            df[r] = A.fd_fwd[(size_t)head * n + idx + r];
            di[r] = A.fd_inv[(size_t)head * n + idx + r];
        }
    }
    NAcc acc;
    acc.clear();

    auto row_of = [&](int64_t g) { return g * A.rows_per_block + row_in_block; };
    auto load_row = [&](const void *base, int64_t g) {
        int64_t row = row_of(g);
        if (row >= A.rows) row = A.rows - 1;  // clamp (in bounds); such a row gets a zero gradient below
        uint32_t off = col_bytes;
        asm volatile("" : "+v"(off));
        return load8((const T *)((const char *)((const T *)base + row * A.ld_in) + off));
    };
    if (grp_first < A.n_groups) {
        Raw8 rx = load_row(A.x, grp_first), rg = load_row(A.dy, grp_first);
        for (int64_t g = grp_first; g < A.n_groups; g += grp_step) {
            float vx[8], vg[8];
            unpack8(rx, vx, (const T *)nullptr);
            unpack8(rg, vg, (const T *)nullptr);
            const int64_t nxt = g + grp_step < A.n_groups ? g + grp_step : g;
            rx = load_row(A.x, nxt);
            rg = load_row(A.dy, nxt);
            const int64_t row = row_of(g);
            const bool live = row < A.rows;  // lanes of a wave may hold different rows
            if (!live) {
#pragma unroll
                for (int r = 0; r < 8; ++r) vg[r] = 0.0f;
            }
            fast_small<K, false>(vx, cf, df);  // x_k
            n_phase(vx, vg, ci, acc);
            if (kDx && live) {
#pragma unroll
                for (int r = 0; r < 8; ++r) vg[r] *= di[r];
                uint32_t off = col_bytes;
                asm volatile("" : "+v"(off));
                store8((T *)((char *)((T *)A.dx + row * A.ld_out) + off), vg);
            }
        }
    }
    // deferred sums -> this slot's entries (workgroups without rows write zeros)
    float *part = A.partial + slot * A.n_angles + (size_t)head * K * (n / 2);
    const float *fw_head = A.fw_inv + (size_t)head * K * n;
#pragma unroll
    for (int J = 0; J < 3; ++J) {  // layers 1..3: pairs of registers
        const int i = J + 1;
        const float *fw = fw_head + (size_t)(i - 1) * n;
        int q = 0;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            if (!(r & (1 << J))) {
                const int a = idx + r, b = idx + (r | (1 << J));
                part[(i - 1) * (n / 2) + pair_index(a, i)] = acc.r[J][q] * (fw[a] * fw[b]);
                ++q;
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {  // layers 4..7: pairs of lanes (masks 1, 2, 7, 8)
        const int i = 4 + j;
        if (i > K) continue;
        const float *fw = fw_head + (size_t)(i - 1) * n;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const float mine = acc.d[j][r];
            const float other = lane_partner(mine, j);
            const int e = idx + r;
            if (!(e & (1 << (i - 1)))) {  // the lane holding the lower element writes
                const int b = e | (1 << (i - 1));
                part[(i - 1) * (n / 2) + pair_index(e, i)] = (mine - other) * (fw[e] * fw[b]);
            }
        }
    }
}

// dtheta[q] = sum over slots of partial[slot][q], in double: a workgroup takes 32 angles, its 8 groups of 32
// threads take every eighth slot each and their sums are added in group order.
__global__ __launch_bounds__(256) void small_bwd_reduce_kernel(const float *__restrict__ partial, float *__restrict__ dtheta,
                                                               int64_t n_angles, int64_t slots, PlanRef plan)
{
    if (!plan_fast_both(plan)) return;
    __shared__ double sums[8][32];
    const int lane = threadIdx.x & 31, grp = threadIdx.x >> 5;
    const int64_t q = (int64_t)blockIdx.x * 32 + lane;
    double acc = 0.0;
    if (q < n_angles)
        for (int64_t s = grp; s < slots; s += 8) acc += (double)partial[s * n_angles + q];
    sums[grp][lane] = acc;
    __syncthreads();
    if (grp == 0 && q < n_angles) {
        double t = sums[0][lane];
#pragma unroll
        for (int g = 1; g < 8; ++g) t += sums[g][lane];
        dtheta[q] = (float)t;
    }
}

// ---- host side -----------------------------------------------------------------------------------
struct SmallBwdGrid {
    int span, rows_per_block, slices;
    int64_t n_groups, slots;
    unsigned grid;
};

static SmallBwdGrid small_bwd_grid(const Shape &s)
{
    SmallBwdGrid g;
    const int64_t width = (int64_t)s.n * s.heads;
    g.span = small_span(width);
    g.rows_per_block = width < g.span ? (int)(g.span / width) : 1;
    g.slices = width >= g.span ? (int)(width / g.span) : 1;
    g.n_groups = (s.rows + g.rows_per_block - 1) / g.rows_per_block;
    // 2048 waves, eight per compute unit (all that fit with these kernels' registers), whatever the workgroup width;
    // the slot count (partial sums to write and to add) stays bounded
    const int64_t wgs = 2048 / (g.span / 512);
    int64_t per_slice = wgs / g.slices > 0 ? wgs / g.slices : 1;
    if (per_slice * g.rows_per_block > kSbMaxSlots) per_slice = kSbMaxSlots / g.rows_per_block;
    if (per_slice > g.n_groups) per_slice = g.n_groups;
    g.grid = (unsigned)(per_slice * g.slices);
    g.slots = per_slice * g.rows_per_block;
    return g;
}

bool small_bwd_supported(const void *x, const void *dy, const void *dx, const float *dtheta, const Shape &s)
{
    if (s.k < 3 || s.k > 7 || dtheta == nullptr || s.rows == 0) return false;
    const int64_t width = (int64_t)s.n * s.heads;
    if (small_span(width) == 0 || width / small_span(width) > 512) return false;
    const int vec = s.dtype == BQ_F32 ? 4 : 8;
    if (((uintptr_t)x & 15) || ((uintptr_t)dy & 15) || (dx && ((uintptr_t)dx & 15))) return false;
    if ((s.ld_x % vec) || (s.ld_y % vec)) return false;
    return true;
}

size_t small_bwd_workspace_bytes(const Shape &s)
{
    if (small_span((int64_t)s.n * s.heads) == 0) return 0;  // not a shape of these kernels
    const SmallBwdGrid g = small_bwd_grid(s);
    return align256((size_t)g.slots * s.heads * s.k * (s.n / 2) * sizeof(float));
}

template <typename T, int K>
static void launch_small_bwd_k(const SmallBwdArgs &A, unsigned grid, hipStream_t stream)
{
    if (A.dx)
        hipLaunchKernelGGL((small_bwd_kernel<T, K, true>), dim3(grid), dim3(A.span / 8), 0, stream, A);
    else
        hipLaunchKernelGGL((small_bwd_kernel<T, K, false>), dim3(grid), dim3(A.span / 8), 0, stream, A);
}

template <typename T>
static void launch_small_bwd_t(const SmallBwdArgs &A, int k, unsigned grid, hipStream_t stream)
{
    switch (k) {
        case 3: return launch_small_bwd_k<T, 3>(A, grid, stream);
        case 4: return launch_small_bwd_k<T, 4>(A, grid, stream);
        case 5: return launch_small_bwd_k<T, 5>(A, grid, stream);
        case 6: return launch_small_bwd_k<T, 6>(A, grid, stream);
        default: return launch_small_bwd_k<T, 7>(A, grid, stream);
    }
}

hipError_t launch_small_bwd(const void *x, const void *dy, const PlanView &pv, void *dx, float *dtheta, void *ws,
                            const Shape &s, hipStream_t stream)
{
    const SmallBwdGrid g = small_bwd_grid(s);
    SmallBwdArgs A{};
    A.x = x;
    A.dy = dy;
    A.dx = dx;
    A.partial = (float *)ws;
    A.fg_fwd = pv.fg_fwd;
    A.fd_fwd = pv.fd_fwd;
    A.fg_inv = pv.fg_inv;
    A.fd_inv = pv.fd_inv;
    A.fw_inv = pv.fw_inv;
    A.bad_fwd = &pv.hdr->fast_bad_fwd;
    A.bad_inv = &pv.hdr->fast_bad_inv;
    A.plan = pv.ref;
    A.rows = s.rows;
    A.ld_in = s.ld_x;
    A.ld_out = s.ld_y;
    A.heads = s.heads;
    A.width = s.n * s.heads;
    A.span = g.span;
    A.rows_per_block = g.rows_per_block;
    A.slices = g.slices;
    A.n_groups = g.n_groups;
    A.n_angles = (int64_t)s.heads * s.k * (s.n / 2);
    switch (s.dtype) {
        case BQ_F32: launch_small_bwd_t<float>(A, s.k, g.grid, stream); break;
        case BQ_F16: launch_small_bwd_t<__half>(A, s.k, g.grid, stream); break;
        default: launch_small_bwd_t<bf16_t>(A, s.k, g.grid, stream); break;
    }
    const unsigned blocks = (unsigned)((A.n_angles + 31) / 32);
    hipLaunchKernelGGL(small_bwd_reduce_kernel, dim3(blocks), dim3(256), 0, stream, (const float *)ws, dtheta, A.n_angles,
                       g.slots, A.plan);
    return hipGetLastError();
}

}  // namespace bq
