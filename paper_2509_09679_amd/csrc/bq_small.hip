// Specialised kernels for small transforms, n = 8 .. 128 (k = 3 .. 7): forward, inverse and fused forward +
// quantisation, for any number of heads whose row width divides 2048 or is a multiple of 512 (rows that are
// not a multiple of 2048 elements wide are covered by narrower workgroups: 1024 or 512 elements, 128 or 64
// threads).
//
// A transform of n elements occupies n/8 consecutive lanes (at most one 16-lane row), 8 consecutive
// elements per lane, and never touches LDS: layers 1-3 pair registers, layers 4..k pair lanes through
// DPP (bq_cascade.h).  All k*8 scale-deferred coefficients and the 8 output scales of a thread stay
// in registers; a workgroup of 256 threads covers 2048 consecutive elements — a slice of a wide row
// (e.g. 32 heads x 128) or several narrow rows (e.g. 16 rows of 128) — and loops over the batch with
// the same coefficients.  Two independent row groups are processed per iteration and the next two are
// prefetched meanwhile, so that four 16-byte loads per lane are in flight.
//
// If the plan flags the scale-deferred tables as unusable, rows go through plain (cos, sin) rotations
// with the twiddles re-read from the plan (slow, rare).
#include "bq_cascade.h"

namespace bq {

constexpr int kSmallThreads = 256;
constexpr int kSmallSpan = kSmallThreads * 8;  // elements covered by a workgroup

struct SmallArgs {
    const void *in;
    void *out;
    const float *fg, *fd;
    const float2 *cs;
    const int *fast_bad;
    PlanRef plan;
    int64_t rows, ld_in, ld_out;
    int heads, width;    // width = heads * n
    int span;            // elements covered by a workgroup: kSmallSpan, or the largest power of two below it that
                         // divides a wider row (the workgroup then has span / 8 threads)
    int rows_per_block;  // span / width if width < span, else 1
    int slices;          // width / span if width >= span, else 1
    int64_t n_groups;    // row groups = ceil(rows / rows_per_block)
    uint8_t *codes;
    void *scales;
    unsigned long long *hist;  // kFwdFake: 2^bits counters or NULL
    int group, scale_f16;
};

template <typename T, int K, int kMode, int kBits>
__global__ __launch_bounds__(kSmallThreads) void small_kernel(SmallArgs A)
{
    constexpr int n = 1 << K;
    constexpr bool kInverse = (kMode == kInv);
    if (!plan_matches(A.plan)) return;
    const int tid = threadIdx.x;
    __shared__ unsigned long long wg_bins[16];  // kFwdFake: this workgroup's bin counts
    BinCount<kBits> bins;
    bins.clear();
    if (kMode == kFwdFake) {
        if (tid < 16) wg_bins[tid] = 0;
        __syncthreads();
    }
    auto flush_bins = [&]() {  // every thread gets here
        if (kMode == kFwdFake && A.hist) {
            bins.drain(wg_bins);
            __syncthreads();
            if (tid < (1 << kBits) && wg_bins[tid]) atomicAdd(&A.hist[tid], wg_bins[tid]);
        }
    };
    const int chunk = (tid & ~15) | lane_chunk(tid & 15);  // chunk of 8 elements inside the workgroup's span
    const int e0 = chunk * 8;
    int row_in_block, col;
    int64_t grp_first, grp_step;
    if (A.slices > 1) {
        row_in_block = 0;
        col = (int)(blockIdx.x % A.slices) * A.span + e0;
        grp_first = blockIdx.x / A.slices;
        grp_step = gridDim.x / A.slices;
    } else {
        row_in_block = e0 / A.width;
        col = e0 - row_in_block * A.width;
        grp_first = blockIdx.x;
        grp_step = gridDim.x;
    }
    const int head = col >> K;
    const int idx = col & (n - 1);
    const bool fast = (*A.fast_bad == 0);

    const float2 *cs_head = A.cs + (size_t)head * K * (n >> 1);
    const T *in = (const T *)A.in;
    const uint32_t col_bytes = (uint32_t)col * (uint32_t)sizeof(T);

    auto row_of = [&](int64_t g) { return g * A.rows_per_block + row_in_block; };
    auto load_row = [&](int64_t g) {
        int64_t row = row_of(g);
        if (row >= A.rows) row = A.rows - 1;  // clamp: the value is not used
        uint32_t off = col_bytes;
        asm volatile("" : "+v"(off));
        return load8((const T *)((const char *)(in + row * A.ld_in) + off));
    };
    auto finish = [&](const float (&y)[8], int64_t g) {
        const int64_t row = row_of(g);
        if (kMode == kFwdFake) {
            const bool live = row < A.rows;  // lanes of a wave may hold different rows
            float f[8], s;
            bool ordinary;
            rounded8<kBits>(y, A.group >> 3, A.scale_f16 != 0, f, &s, &ordinary);
            if (A.hist) {
                if (live)
                    count8<kBits>(bins, f, ordinary);
                else
                    bins.skip();
                if (bins.full()) bins.drain(wg_bins);
            }
            if (A.out && live) {
                float yq[8];
                dequant8(f, s, yq);
                uint32_t off = col_bytes;
                asm volatile("" : "+v"(off));
                store8((T *)((char *)((T *)A.out + row * A.ld_out) + off), yq);
            }
            return;
        }
        if (row >= A.rows) return;
        if (kMode != kFwdQuant) {
            uint32_t off = col_bytes;
            asm volatile("" : "+v"(off));
            store8((T *)((char *)((T *)A.out + row * A.ld_out) + off), y);
        } else {
            const int lanes = A.group >> 3;
            float s;
            const uint32_t packed = quant8<kBits>(y, lanes, A.scale_f16 != 0, &s);
            uint8_t *codes_row = A.codes + row * (int64_t)(A.width * kBits / 8);
            const uint32_t coff = (uint32_t)col * kBits / 8;
            if (kBits == 2)
                *(uint16_t *)(codes_row + coff) = (uint16_t)packed;
            else
                *(uint32_t *)(codes_row + coff) = packed;
            const int64_t sidx = row * (int64_t)(A.width / A.group) + (uint32_t)col / (uint32_t)A.group;
            if (A.scale_f16)
                ((__half *)A.scales)[sidx] = __float2half_rn(s);
            else
                ((float *)A.scales)[sidx] = s;
        }
    };

    if (grp_first >= A.n_groups) return;
    if (!fast) {  // rare
        for (int64_t g = grp_first; g < A.n_groups; g += grp_step) {
            float u[8];
            unpack8(load_row(g), u, (const T *)nullptr);
            slow_small<K, kInverse>(u, cs_head, idx);
            finish(u, g);
        }
        flush_bins();
        return;
    }
    float c[7][8], d[8];
    {
        const float *fg = A.fg + (size_t)head * K * n;
#pragma unroll
        for (int j = 0; j < 7; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r) c[j][r] = (j < K) ? fg[j * n + idx + r] : 0.0f;
#pragma unroll
        for (int r = 0; r < 8; ++r) d[r] = A.fd[(size_t)head * n + idx + r];
    }
    Raw8 raw0 = load_row(grp_first);
    Raw8 raw1 = load_row(grp_first + grp_step);
    for (int64_t g = grp_first; g < A.n_groups; g += 2 * grp_step) {
        float u0[8], u1[8];
        unpack8(raw0, u0, (const T *)nullptr);
        unpack8(raw1, u1, (const T *)nullptr);
        raw0 = load_row(g + 2 * grp_step);
        raw1 = load_row(g + 3 * grp_step);
        fast_small<K, kInverse>(u0, c, d);
        fast_small<K, kInverse>(u1, c, d);
        finish(u0, g);
        if (g + grp_step < A.n_groups) finish(u1, g + grp_step);
    }
    flush_bins();
}

template <typename T, int K>
static void (*pick_small(Mode mode, int bits))(SmallArgs)
{
    if (mode == kFwd) return small_kernel<T, K, kFwd, 4>;
    if (mode == kInv) return small_kernel<T, K, kInv, 4>;
    if (mode == kFwdFake) return bits == 2 ? small_kernel<T, K, kFwdFake, 2> : small_kernel<T, K, kFwdFake, 4>;
    return bits == 2 ? small_kernel<T, K, kFwdQuant, 2> : small_kernel<T, K, kFwdQuant, 4>;
}

template <typename T>
static void (*pick_small_k(int k, Mode mode, int bits))(SmallArgs)
{
    switch (k) {
        case 3: return pick_small<T, 3>(mode, bits);
        case 4: return pick_small<T, 4>(mode, bits);
        case 5: return pick_small<T, 5>(mode, bits);
        case 6: return pick_small<T, 6>(mode, bits);
        default: return pick_small<T, 7>(mode, bits);
    }
}

// Elements per workgroup for rows of `width` elements: 2048 where rows tile it or it tiles rows, else the
// largest power of two that divides the row, down to one wave (512); 0 if there is none.
int small_span(int64_t width)
{
    if (width < kSmallSpan && kSmallSpan % width == 0) return kSmallSpan;  // several whole rows per workgroup
    const int64_t low = width & -width;
    const int span = (int)(low < kSmallSpan ? low : kSmallSpan);
    return span >= 512 ? span : 0;
}

bool small_supported(Mode mode, const void *in, const void *out, const Shape &s, const QuantArgs *q)
{
    if (s.k < 3 || s.k > 7) return false;
    const int64_t width = (int64_t)s.n * s.heads;
    if (small_span(width) == 0) return false;
    const int isz = s.dtype == BQ_F32 ? 4 : 2;
    const int vec = 16 / isz;
    if (((uintptr_t)in & 15) || (s.ld_x % vec)) return false;
    if (mode != kFwdQuant && out && (((uintptr_t)out & 15) || (s.ld_y % vec))) return false;
    if (mode == kFwdQuant || mode == kFwdFake) {
        if (q->group > s.n) return false;
        if (mode == kFwdQuant && ((uintptr_t)q->codes & 3)) return false;
    }
    return true;
}

hipError_t launch_small(Mode mode, const void *in, void *out, const PlanView &pv, const Shape &s,
                        const QuantArgs *q, hipStream_t stream)
{
    SmallArgs A{};
    A.in = in;
    A.out = out;
    A.fg = mode == kInv ? pv.fg_inv : pv.fg_fwd;
    A.fd = mode == kInv ? pv.fd_inv : pv.fd_fwd;
    A.cs = pv.cs;
    A.fast_bad = mode == kInv ? &pv.hdr->fast_bad_inv : &pv.hdr->fast_bad_fwd;
    A.plan = pv.ref;
    A.rows = s.rows;
    A.ld_in = s.ld_x;
    A.ld_out = s.ld_y;
    A.heads = s.heads;
    A.width = s.n * s.heads;
    A.span = small_span(A.width);
    // the plain transforms of 16-bit rows stream fastest from single-wave workgroups (measured: up to 20 % over
    // four-wave ones at the same number of waves; float32 rows and the quantisers prefer the wider ones)
    if ((mode == kFwd || mode == kInv) && s.dtype != BQ_F32 && (A.width % 512 == 0 || 512 % A.width == 0)) A.span = 512;
    A.rows_per_block = A.width < A.span ? A.span / A.width : 1;
    A.slices = A.width >= A.span ? A.width / A.span : 1;
    A.n_groups = (s.rows + A.rows_per_block - 1) / A.rows_per_block;
    int bits = 4;
    if (q) {
        A.codes = q->codes;
        A.scales = q->scales;
        A.hist = q->hist;
        A.group = q->group;
        A.scale_f16 = q->scale_f16;
        bits = q->bits;
    }
    // Persistent workgroups, a multiple of the slice count.  How many waves stream best was measured per mode
    // (262144 rows of 32 x 128): the plain transforms and everything on float32 rows with 2048 waves (8 per
    // compute unit: 5.5 TB/s against 4.4 TB/s with four times as many), the 16-bit quantisers, which need the
    // occupancy to hide their arithmetic, with 8192.
    const bool few = mode == kFwd || mode == kInv || s.dtype == BQ_F32;
    const int64_t wgs = (few ? 2048 : 8192) / (A.span / 512);
    int64_t per_slice = wgs / A.slices > 0 ? wgs / A.slices : 1;
    if (per_slice > A.n_groups) per_slice = A.n_groups;
    const unsigned grid = (unsigned)(per_slice * A.slices);
    void (*kern)(SmallArgs) = s.dtype == BQ_F32   ? pick_small_k<float>(s.k, mode, bits)
                              : s.dtype == BQ_F16 ? pick_small_k<__half>(s.k, mode, bits)
                                                  : pick_small_k<bf16_t>(s.k, mode, bits);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(A.span / 8), 0, stream, A);
    return hipGetLastError();
}

}  // namespace bq
