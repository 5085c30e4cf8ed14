// Backward pass for n = 4096 and n = 8192 (k = 12, 13), one head: dx = B^T dy and
// dtheta[i][p] = sum over rows of  g_i[b] x_i[a] - g_i[a] x_i[b]   (x_i, g_i at the output of layer i;
// paper, "Gradient Flow Through Butterfly Layers": d y_a / d theta = -y_b, d y_b / d theta = y_a).
//
// Orthogonality makes stored activations unnecessary: x_{i-1} = B_i^T x_i.  The forward state is
// recomputed once, then the transposed cascade runs on x and g together.  Both start it with scale 1, so
// they share the scale-deferred coefficients and, before layer i, the scales D_i[e] (plan table fw_inv).
// Sums are accumulated in deferred units,
//   acc += v_g[b] v_x[a] - v_g[a] v_x[b],   dtheta = D_i[a] D_i[b] acc,
// the factor being applied once per workgroup at the end.  For a layer that pairs lanes each lane keeps
// the partial sum of its own element (one v_fmac_f32 with a DPP operand per element); the two lanes'
// sums are combined at the end.
//
// All kernels work on 4096 points with 8 points per thread.  Registers cannot hold the coefficients of
// all layers in both directions plus the sums, so the pass is two kernels, and the second one splits
// its work over two groups of waves:
//
//   F:  x -> forward cascade of layers 1..12, float32 result into the workspace
//   PN: waves 0..7  (phase P): layers 12..8 transposed on (x, g), sums of those layers
//       waves 8..15 (phase N): layers 7..1 transposed on the row that phase P finished one step
//                              earlier (handed over through LDS), sums of those layers, dx out
//
// n = 8192: layers 1..12 act inside each half of a row, only layer 13 couples the halves.  A workgroup
// takes one half of its rows.  F stops before layer 13 and writes the state in the units the transposed
// cascade has after its first layer (plan table fm_fwd); phase P reads both halves of dy, forms its own
// half of g_12 and, for the sum of layer 13, the other half as well:
//   dtheta_13[p] = sum over rows of  g_12[b] x_12[a] - g_12[a] x_12[b]
// (the same expression one layer further down: rotating both vectors of a pair leaves it unchanged),
// the lower-half workgroup contributing the first term and the upper-half one the second.
//
// Every workgroup owns one slice of `partial`; a slice entry is written by exactly one thread, chunks
// of rows add to it in stream order, and a last kernel sums the slices in double in a fixed order: no
// atomics, the result does not depend on scheduling.
//
// All kernels exit at once when the plan flags the scale-deferred tables as unusable; the generic
// backward kernel, launched behind them with the opposite condition, then does the work.
#include "bq_bwd_blocks.h"

namespace bq {

template <int K>
struct Geo {
    static constexpr int n = 1 << K;
    static constexpr int threads = n / 8;
    static constexpr int kStepR1 = (1 << (K - 2)) + 2 * (1 << (K - 7)) + 2 * (1 << (K - 11));
    static constexpr int kStepR2 = 2 * kStepR1;
    static constexpr int kRowFloats = ((n - 1) + 2 * ((n - 1) >> 5) + 2 * ((n - 1) >> 9) + 1 + 3) & ~3;
};

__device__ __forceinline__ int lds_addr2(int idx) { return idx + 2 * (idx >> 5) + 2 * (idx >> 9); }

// base index of a thread in layout P: idx bits 7.. are the chunk bits of the low lane bits (DPP
// masks 1, 2, 7), idx bit 0 and the two top bits are register bits, the rest lanes 3..5 / waves.
template <int K>
__device__ __forceinline__ int base_p2(int wave, int lane)
{
    static_assert(K == 12, "4096-point geometry");
    const int c3 = lane_chunk(lane & 15) & 7;
    return (c3 << 7) | (((lane >> 3) & 1) << 2) | (((lane >> 4) & 1) << 1) | (((lane >> 5) & 1) << 3) | (wave << 4);
}
template <int K>
__device__ __forceinline__ int p_reg_idx2(int r)
{
    return (r & 1) + ((r >> 1) & 1) * (1 << (K - 2)) + (r >> 2) * (1 << (K - 1));
}

template <int K>
__device__ __forceinline__ void lds_write_p2(float *buf, int ap, const float (&u)[8])
{
#pragma unroll
    for (int j = 0; j < 4; ++j)
        *(float2 *)&buf[ap + (j & 1) * Geo<K>::kStepR1 + (j >> 1) * Geo<K>::kStepR2] = make_float2(u[2 * j], u[2 * j + 1]);
}
template <int K>
__device__ __forceinline__ void lds_read_p2(const float *buf, int ap, float (&u)[8])
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float2 v = *(const float2 *)&buf[ap + (j & 1) * Geo<K>::kStepR1 + (j >> 1) * Geo<K>::kStepR2];
        u[2 * j] = v.x;
        u[2 * j + 1] = v.y;
    }
}
__device__ __forceinline__ void lds_write_n2(float *buf, int an, const float (&u)[8])
{
#pragma unroll
    for (int j = 0; j < 4; ++j) *(float2 *)&buf[an + 2 * j] = make_float2(u[2 * j], u[2 * j + 1]);
}
__device__ __forceinline__ void lds_read_n2(const float *buf, int an, float (&u)[8])
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float2 v = *(const float2 *)&buf[an + 2 * j];
        u[2 * j] = v.x;
        u[2 * j + 1] = v.y;
    }
}

struct BwdFastArgs {
    const void *x, *dy;
    void *dx;
    float *xk;       // chunk intermediate, [chunk_rows][n] float32
    float *partial;  // [slices][slice_floats]
    const float *fg_fwd, *fd_fwd, *fm_fwd, *fg_inv, *fd_inv, *fw_inv;
    const int *bad_fwd, *bad_inv;
    int64_t row0, rows;  // this chunk: rows [row0, row0 + rows) of the batch
    int64_t ld_in, ld_out;
    int64_t slice_floats;
    int first_chunk;  // != 0: slices are overwritten, else added to
    // n = 2^n_log < 4096 (kVirt): a row of the kernels is a block of 4096 / n consecutive rows of the caller;
    // row0, rows, ld_in, ld_out then count and stride blocks, sub_ld_* are the caller's strides and total_rows
    // its row count (the last block may be short: its missing rows are given dy = 0 and are not stored)
    // Several heads (row width heads * n <= 4096): a block is 4096 / width whole rows, row_log = log2 of the width,
    // and every 2^n_log-element piece of a row has its own tables.
    int n, n_log, row_log, heads;
    int64_t sub_ld_in, sub_ld_out, total_rows;
};

__device__ __forceinline__ bool plan_is_bad(const BwdFastArgs &A) { return (*A.bad_fwd | *A.bad_inv) != 0; }

constexpr int K = 12;  // layers inside one 4096-point block
using G = Geo<K>;

// Which rows and which part of them a workgroup takes, and how it indexes the plan's tables.
// kHalf (n = 8192): blocks 16 j + 8 h + c take half h of the rows of slot 8 j + c, so that the two workgroups
// of a slot, which read the same dy rows at about the same time, sit on the same die (blocks go round the
// eight dies) and share its L2.  kVirt (n < 4096): see BwdFastArgs.
template <bool kHalf, bool kVirt>
struct Part {
    int half, slot, nslots, c0;
    int ts;     // row length of the plan's tables (n)
    int tmask;  // an element e of the 4096-point block uses table column (c0 + e) & tmask
    int n_log;
    int row_log, rmask;  // kVirt: log2 of the caller's row width and width - 1 (else 0, 0)
    // Row counters are 32-bit: a launch covers at most 2^18 kernel rows, and 64-bit comparisons of uniform values
    // would run on the vector unit.
    int tail_row;  // kVirt: the kernel row (counted from this launch's first) that is the short last block, or -1
    int tail;          // ... and the number of rows it has
    static constexpr int xs = kHalf ? 2 * G::n : G::n;  // row length of x_k; a slice holds xs / 2 sums per layer
    __device__ __forceinline__ Part(const BwdFastArgs &A)
    {
        half = kHalf ? (blockIdx.x >> 3) & 1 : 0;
        slot = kHalf ? (int)((blockIdx.x & 7) | ((blockIdx.x >> 4) << 3)) : (int)blockIdx.x;
        nslots = kHalf ? (int)(gridDim.x >> 1) : (int)gridDim.x;
        c0 = half * G::n;
        ts = kVirt ? A.n : xs;
        tmask = ts - 1;
        n_log = kVirt ? A.n_log : (kHalf ? K + 1 : K);
        row_log = kVirt ? A.row_log : 0;
        rmask = kVirt ? (1 << A.row_log) - 1 : 0;
        const int64_t tr = kVirt ? (A.total_rows >> (K - A.row_log)) - A.row0 : -1;
        tail_row = (tr >= 0 && tr < A.rows) ? (int)tr : -1;
        tail = kVirt ? (int)(A.total_rows & ((G::n >> A.row_log) - 1)) : 0;
    }
    __device__ __forceinline__ int col(int e) const { return (c0 + e) & tmask; }
    // the head (transform of the caller's row) of block element e; 0 unless kVirt with several heads
    __device__ __forceinline__ int head(int e) const { return kVirt ? (e & rmask) >> n_log : 0; }
    // offset into a [head][layer][n] table of the row of layer `layer` (0-based) for block element e
    __device__ __forceinline__ size_t trow(int e, int layer) const { return ((size_t)head(e) * n_log + layer) * ts; }
    // element offset of block element e (a multiple of 8) from the start of this workgroup's part of a kernel row
    __device__ __forceinline__ uint32_t off(int e, int64_t sub_ld) const
    {
        return kVirt ? (uint32_t)((e >> row_log) * (int)sub_ld + (e & rmask)) : (uint32_t)e;
    }
    // kVirt: is the row of element e missing from the short last block?
    __device__ __forceinline__ bool in_tail_gap(int e) const { return kVirt && (e >> row_log) >= tail; }
};

// ---- F: forward cascade of layers 1..12 to float32 ------------------------------------------------------
template <typename T, bool kHalf, bool kVirt>
__global__ __launch_bounds__(G::threads) __attribute__((amdgpu_waves_per_eu(4))) void bwd_f_kernel(BwdFastArgs A)
{
    extern __shared__ float lds[];  // [row buffer][output scales]
    if (plan_is_bad(A)) return;
    const Part<kHalf, kVirt> part(A);
    const int ts = part.ts;
    constexpr int xs = Part<kHalf, kVirt>::xs;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int idx_n = (wave * 64 + lane_chunk(lane)) * 8;
    const int idx_p = base_p2<K>(wave, lane);
    const int an = lds_addr2(idx_n), ap = lds_addr2(idx_p);
    float *buf = lds, *dtab = lds + G::kRowFloats;
    const float *fg = A.fg_fwd;
    float cn[7][8], cp[K - 7][8];
#pragma unroll
    for (int j = 0; j < 7; ++j)
#pragma unroll
        for (int r = 0; r < 8; ++r) cn[j][r] = fg[part.trow(idx_n, j) + part.col(idx_n) + r];
#pragma unroll
    for (int j = 0; j < K - 7; ++j)
#pragma unroll
        for (int r = 0; r < 8; ++r)  // layers above log2 n do not exist: weight zero leaves the element as it is
            cp[j][r] = (!kVirt || 8 + j <= part.n_log)
                           ? fg[part.trow(idx_p + p_reg_idx2<K>(r), 7 + j) + part.col(idx_p + p_reg_idx2<K>(r))]
                           : 0.0f;
    {
        const float *scale = kHalf ? A.fm_fwd : A.fd_fwd;
        float d[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) d[r] = scale[(size_t)part.head(idx_n) * ts + part.col(idx_n) + r];
        lds_write_n2(dtab, an, d);
    }
    const T *x = (const T *)A.x + A.row0 * A.ld_in + part.c0;
    // kVirt: a sub-row missing from the last block reads the block's first row instead (its dy will be zero)
    const uint32_t off_x = part.off(idx_n, A.sub_ld_in), off_x0 = part.off(idx_n & part.tmask, A.sub_ld_in);
    const bool gap = part.in_tail_gap(idx_n);
    auto load_row = [&](int r) { return load8(x + r * A.ld_in + ((gap && r == part.tail_row) ? off_x0 : off_x)); };
    float *xk = A.xk + part.c0 + idx_n;
    const int n_rows = (int)A.rows;
    int row = part.slot;
    if (row >= n_rows) return;
    Raw8 raw = load_row(row);
    for (; row < n_rows; row += part.nslots) {
        float u[8];
        unpack8(raw, u, (const T *)nullptr);
        const int next = row + part.nslots;
        if (next < n_rows) raw = load_row(next);
        reg_layer_first<0>(u, cn[0]);
        reg_layer<1>(u, cn[1]);
        reg_layer<2>(u, cn[2]);
        dpp_layer_xor1(u, cn[3]);
        dpp_layer_xor2(u, cn[4]);
        dpp_layer_xor7(u, cn[5]);
        dpp_layer_xor8(u, cn[6]);
        __syncthreads();  // the previous row's reads of buf are complete
        lds_write_n2(buf, an, u);
        __syncthreads();
        lds_read_p2<K>(buf, ap, u);
        dpp_layer_xor1(u, cp[0]);
        dpp_layer_xor2(u, cp[1]);
        dpp_layer_xor7(u, cp[2]);
        reg_layer<1>(u, cp[3]);
        reg_layer<2>(u, cp[4]);
        lds_write_p2<K>(buf, ap, u);
        __syncthreads();
        lds_read_n2(buf, an, u);
        float d[8];
        lds_read_n2(dtab, an, d);
#pragma unroll
        for (int r = 0; r < 8; ++r) u[r] *= d[r];
        store8(xk + (size_t)row * xs, u);
    }
}

// ---- building blocks of PN ------------------------------------------------------------------------------
struct PAcc {  // deferred sums of phase P: lane layers 8..10, register layers 11 and 12
    float d[3][8], r1[4], r2[4];
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int j = 0; j < 3; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r) d[j][r] = 0.0f;
#pragma unroll
        for (int q = 0; q < 4; ++q) r1[q] = r2[q] = 0.0f;
    }
};
// layers 12..8 transposed on (vx, vg) held in layout P; cp[j] = coefficients of layer 8 + j.  kFirst: layer
// 12 is the first layer of the transposed cascade (scales still 1).
template <bool kFirst>
__device__ __forceinline__ void p_phase(float (&vx)[8], float (&vg)[8], const float (&cp)[5][8], PAcc &acc)
{
    reg_acc<2>(acc.r2, vg, vx);  // layer 12 (register bit 2)
    if (kFirst) {
        reg_layer_first<2>(vx, cp[4]);
        reg_layer_first<2>(vg, cp[4]);
    } else {
        reg_layer<2>(vx, cp[4]);
        reg_layer<2>(vg, cp[4]);
    }
    reg_acc<1>(acc.r1, vg, vx);  // layer 11 (register bit 1)
    reg_layer<1>(vx, cp[3]);
    reg_layer<1>(vg, cp[3]);
    dpp_acc_xor7(acc.d[2], vg, vx);  // layer 10
    dpp_layer_xor7(vx, cp[2]);
    dpp_layer_xor7(vg, cp[2]);
    dpp_acc_xor2(acc.d[1], vg, vx);  // layer 9
    dpp_layer_xor2(vx, cp[1]);
    dpp_layer_xor2(vg, cp[1]);
    dpp_acc_xor1(acc.d[0], vg, vx);  // layer 8
    dpp_layer_xor1(vx, cp[0]);
    dpp_layer_xor1(vg, cp[0]);
}

// Coefficients of layers 1..7 for the eight points a thread holds in layout N: the first kLds layers in
// LDS (written and read by the same thread), the others in registers.
template <int kLds>
struct CoefSplit {
    float c[7 - kLds][8];
    const float4 *tab;  // float4 index (2 j + half) * kSlots + slot: consecutive lanes, consecutive banks
    int first;
    static constexpr int kSlots = 512;
    __device__ __forceinline__ void load(const float *fg, int stride, int idx, float *lds_tab, int slot)
    {
        tab = (const float4 *)lds_tab;
        first = slot;
        float4 *t = (float4 *)lds_tab + first;
#pragma unroll
        for (int j = 0; j < kLds; ++j) {
            t[(2 * j) * kSlots] = *(const float4 *)(fg + j * stride + idx);
            t[(2 * j + 1) * kSlots] = *(const float4 *)(fg + j * stride + idx + 4);
        }
#pragma unroll
        for (int j = kLds; j < 7; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r) c[j - kLds][r] = fg[j * stride + idx + r];
    }
    template <int J>
    __device__ __forceinline__ void get(float (&o)[8]) const
    {
        if (J < kLds) {
            int f = first;
            asm volatile("" : "+v"(f));  // keeps the reads inside the row loop (hoisted, they would spill)
            const float4 a = tab[f + 2 * J * kSlots], b = tab[f + (2 * J + 1) * kSlots];
            o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
        } else {
#pragma unroll
            for (int r = 0; r < 8; ++r) o[r] = c[(J < kLds ? kLds : J) - kLds][r];
        }
    }
};

// fw_inv entry (scale before transposed layer i) of block element e; rmask != 0: the tables of e's own head
__device__ __forceinline__ float fw_at(const float *fw_inv, int stride, int tmask, int n_log, int rmask, int c0, int e, int i)
{
    const int hd = (e & rmask) >> n_log;
    return fw_inv[((size_t)hd * n_log + (i - 1)) * stride + ((c0 + e) & tmask)];
}

// Deferred sums -> dtheta partials of this workgroup.  part: its slice, `pairs` sums per layer, indexed by the
// pair's position in the whole kernel row (c0 + element); fw_inv: the plan table, rows `stride` apart, column
// (c0 + element) & tmask.
__device__ __forceinline__ void finalize_p(float *part, const PAcc &acc, int idx_p, const float *fw_inv, int stride, int tmask,
                                           int pairs, int c0, int n_log, int rmask, int first)
{
#pragma unroll
    for (int J = 1; J <= 2; ++J) {  // register layers
        const int i = (J == 2) ? K : K - 1;
        if (i > n_log) continue;  // a layer the transform does not have: no table row, nothing to write
        int q = 0;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            if (!(r & (1 << J))) {
                const int a = idx_p + p_reg_idx2<K>(r), b = idx_p + p_reg_idx2<K>(r | (1 << J));
                const float v = (J == 2 ? acc.r2[q] : acc.r1[q]) * (fw_at(fw_inv, stride, tmask, n_log, rmask, c0, a, i) * fw_at(fw_inv, stride, tmask, n_log, rmask, c0, b, i));
                put_partial(part + (size_t)(i - 1) * pairs + pair_index(c0 + a, i), v, first);
                ++q;
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 3; ++j) {  // lane layers: layer 8 + j, lane masks 1, 2, 7
        const int i = 8 + j;
        if (i > n_log) continue;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const float mine = acc.d[j][r];
            const float other = lane_partner(mine, j);
            const int e = idx_p + p_reg_idx2<K>(r);
            if (!(e & (1 << (i - 1)))) {  // the lane holding the lower element writes
                const int b = e | (1 << (i - 1));
                put_partial(part + (size_t)(i - 1) * pairs + pair_index(c0 + e, i), (mine - other) * (fw_at(fw_inv, stride, tmask, n_log, rmask, c0, e, i) * fw_at(fw_inv, stride, tmask, n_log, rmask, c0, b, i)), first);
            }
        }
    }
}

__device__ __forceinline__ void finalize_n(float *part, const NAcc &acc, int idx, const float *fw_inv, int stride, int tmask,
                                           int pairs, int c0, int n_log, int rmask, int first)
{
#pragma unroll
    for (int J = 0; J < 3; ++J) {  // layers 1..3
        const int i = J + 1;
        int q = 0;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            if (!(r & (1 << J))) {
                const int a = idx + r, b = idx + (r | (1 << J));
                put_partial(part + (size_t)(i - 1) * pairs + pair_index(c0 + a, i), acc.r[J][q] * (fw_at(fw_inv, stride, tmask, n_log, rmask, c0, a, i) * fw_at(fw_inv, stride, tmask, n_log, rmask, c0, b, i)), first);
                ++q;
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {  // layers 4..7, lane masks 1, 2, 7, 8
        const int i = 4 + j;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const float mine = acc.d[j][r];
            const float other = lane_partner(mine, j);
            const int e = idx + r;
            if (!(e & (1 << (i - 1)))) {
                const int b = e | (1 << (i - 1));
                put_partial(part + (size_t)(i - 1) * pairs + pair_index(c0 + e, i), (mine - other) * (fw_at(fw_inv, stride, tmask, n_log, rmask, c0, e, i) * fw_at(fw_inv, stride, tmask, n_log, rmask, c0, b, i)), first);
            }
        }
    }
}

// store8 through a raw buffer descriptor: the hardware drops every access that reaches past `bytes` from
// `base`, which masks lanes without a branch.  off: byte offset of the lane's 8 elements.
typedef int bwd_v4i __attribute__((ext_vector_type(4)));
template <typename T>
__device__ __forceinline__ void store8_bounded(T *base, uint32_t bytes, uint32_t off, const float (&y)[8])
{
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)bytes, 0x00020000);
    if constexpr (sizeof(T) == 4) {
        bwd_v4i a = {(int)__float_as_uint(y[0]), (int)__float_as_uint(y[1]), (int)__float_as_uint(y[2]), (int)__float_as_uint(y[3])};
        bwd_v4i b = {(int)__float_as_uint(y[4]), (int)__float_as_uint(y[5]), (int)__float_as_uint(y[6]), (int)__float_as_uint(y[7])};
        __builtin_amdgcn_raw_buffer_store_b128(a, rs, (int)off, 0, 0);
        __builtin_amdgcn_raw_buffer_store_b128(b, rs, (int)off + 16, 0, 0);
    } else {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if constexpr (std::is_same<T, __half>::value) {
                const __half2 h = __halves2half2(__float2half_rn(y[2 * i]), __float2half_rn(y[2 * i + 1]));
                w[i] = *(const uint32_t *)&h;
            } else {
                w[i] = f32x2_to_bf16x2_bits(y[2 * i], y[2 * i + 1]);
            }
        }
        bwd_v4i a = {(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
        __builtin_amdgcn_raw_buffer_store_b128(a, rs, (int)off, 0, 0);
    }
}

__device__ __forceinline__ void load8_f32(const float *p, float (&v)[8])
{
    const float4 a = *(const float4 *)p;
    const float4 b = *((const float4 *)p + 1);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

// ---- PN: the transposed cascade, split over two groups of eight waves -----------------------------------
// Waves 0..7 run phase P on row t while waves 8..15 run phase N on row t-1; a row changes hands through an
// LDS area in layout N.  Each group keeps only its own coefficients and sums in registers (the second
// group also parks the coefficients of its first kPnLdsLayers layers in LDS), which is what lets 1024
// threads fit the 128-register budget.  Both groups execute the same number of workgroup barriers:
//   P, row t:   write area A (layout N) | B1 | read A (layout P), layers 12..8, write area H | B2
//   N, row t-1: read H                  | B1 | layers 7..1, store dx                        | B2
// A slice of `partial` holds k n / 2 sums in dtheta order; for n = 8192 another 4096 follow, the
// upper-half workgroup's (negative) share of layer 13.
constexpr int kPnThreads = 1024;
constexpr int kPnLdsLayers = 4;
constexpr size_t kPnLdsFloats = 4 * (size_t)G::kRowFloats + (1 + kPnLdsLayers) * (size_t)G::n;

template <typename T, bool kDx, bool kHalf, bool kVirt>
__global__ __launch_bounds__(kPnThreads) void bwd_pn_kernel(BwdFastArgs A)
{
    extern __shared__ float lds[];
    if (plan_is_bad(A)) return;
    const Part<kHalf, kVirt> pt(A);
    const int ts = pt.ts;
    constexpr int xs = Part<kHalf, kVirt>::xs;
    const int role = threadIdx.x >> 9;  // uniform per wave
    const int tid = threadIdx.x & 511, wave = tid >> 6, lane = tid & 63;
    const int idx_n = (wave * 64 + lane_chunk(lane)) * 8;
    const int an = lds_addr2(idx_n);
    float *hand = lds + 2 * G::kRowFloats;
    const int mine = A.rows > (int64_t)pt.slot ? (int)((A.rows - pt.slot + pt.nslots - 1) / pt.nslots) : 0;
    float *part = A.partial + (size_t)pt.slot * A.slice_floats;
    const float *fg = A.fg_inv, *fw = A.fw_inv;
    if (role == 0) {
        const int idx_p = base_p2<K>(wave, lane);
        const int ap = lds_addr2(idx_p);
        float cp[5][8];
#pragma unroll
        for (int j = 0; j < 5; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r)
                cp[j][r] = (!kVirt || 8 + j <= pt.n_log)
                               ? fg[pt.trow(idx_p + p_reg_idx2<K>(r), 7 + j) + pt.col(idx_p + p_reg_idx2<K>(r))]
                               : 0.0f;
        float c13[8], acc13[8];  // kHalf only: layer 13 in layout N (it pairs column e with e + 4096)
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            c13[r] = kHalf ? fg[12 * ts + pt.col(idx_n) + r] : 0.0f;
            acc13[r] = 0.0f;
        }
        PAcc acc;
        acc.clear();
        // uniform row pointers + 32-bit per-thread byte offsets: the loads take their base from scalar
        // registers and no 64-bit per-thread pointer stays live across the loop
        const T *dy = (const T *)A.dy + A.row0 * A.ld_in + pt.c0;
        const T *dyo = (const T *)A.dy + A.row0 * A.ld_in + (pt.c0 ^ G::n);  // the other half (kHalf)
        const float *xk = A.xk + pt.c0;
        // kVirt: a sub-row missing from the last block reads the block's first row; its gradient is zeroed below
        const uint32_t off_g = pt.off(idx_n, A.sub_ld_in) * (uint32_t)sizeof(T);
        const uint32_t off_g0 = pt.off(idx_n & pt.tmask, A.sub_ld_in) * (uint32_t)sizeof(T);
        const bool gap = pt.in_tail_gap(idx_n);
        auto fetch = [&](int r, float(&ox)[8], Raw8 &og, Raw8 &ogo) {
            uint32_t offx = (uint32_t)idx_n * 4u, offg = (gap && r == pt.tail_row) ? off_g0 : off_g;
            asm volatile("" : "+v"(offx), "+v"(offg));
            load8_f32((const float *)((const char *)(xk + (size_t)r * xs) + offx), ox);
            og = load8((const T *)((const char *)(dy + r * A.ld_in) + offg));
            if (kHalf) ogo = load8((const T *)((const char *)(dyo + r * A.ld_in) + offg));
        };
        float nx[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        Raw8 ng = {}, ngo = {};
        int row = pt.slot;
        if (mine > 0) fetch(row, nx, ng, ngo);
        for (int it = 0; it < mine; ++it, row += pt.nslots) {
            float vx[8], vg[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) vx[r] = nx[r];
            unpack8(ng, vg, (const T *)nullptr);
            if (gap && row == pt.tail_row) {
#pragma unroll
                for (int r = 0; r < 8; ++r) vg[r] = 0.0f;
            }
            if (kHalf) {
                // transposed layer 13 on g: own half kept, the other half only feeds the layer's sum
                // (its coefficient is the negative of this half's: both scales are still 1)
                float go[8];
                unpack8(ngo, go, (const T *)nullptr);
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    const float other12 = __builtin_fmaf(-c13[r], vg[r], go[r]);
                    acc13[r] = __builtin_fmaf(other12, vx[r], acc13[r]);
                    vg[r] = __builtin_fmaf(c13[r], go[r], vg[r]);
                }
            }
            const int next = it + 1 < mine ? row + pt.nslots : row;  // the last one reads its own row again
            fetch(next, nx, ng, ngo);
            lds_write_n2(lds, an, vx);
            lds_write_n2(lds + G::kRowFloats, an, vg);
            __syncthreads();  // B1
            lds_read_p2<K>(lds, ap, vx);
            lds_read_p2<K>(lds + G::kRowFloats, ap, vg);
            p_phase<!kHalf>(vx, vg, cp, acc);
            lds_write_p2<K>(hand, ap, vx);
            lds_write_p2<K>(hand + G::kRowFloats, ap, vg);
            __syncthreads();  // B2
        }
        __syncthreads();  // the other group's last row
        __syncthreads();
        finalize_p(part, acc, idx_p, fw, ts, pt.tmask, xs / 2, pt.c0, pt.n_log, kVirt ? pt.rmask : 0, A.first_chunk);
        if (kHalf) {
            // sum of layer 13 = (scale after the layer)^2 * deferred sum; the lower half's share goes to the
            // layer's place in the slice, the upper half's, negated, behind the slice's regular part
            float *dst = part + (size_t)(pt.half ? 13 : 12) * G::n + idx_n;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const float d = fw[11 * ts + pt.col(idx_n) + r];
                const float v = acc13[r] * (d * d);
                put_partial(dst + r, pt.half ? -v : v, A.first_chunk);
            }
        }
    } else {
        float *dtab = lds + 4 * G::kRowFloats;  // tables written and read by the same thread
        CoefSplit<kPnLdsLayers> cn;
        cn.load(fg + pt.trow(idx_n, 0), ts, pt.col(idx_n), dtab + G::n, tid);
        const float *fdi = A.fd_inv + (size_t)pt.head(idx_n) * ts + pt.col(idx_n);
        ((float4 *)dtab)[tid] = *(const float4 *)fdi;
        ((float4 *)dtab)[512 + tid] = *(const float4 *)(fdi + 4);
        NAcc acc;
        acc.clear();
        T *dx = (T *)A.dx + A.row0 * A.ld_out + pt.c0;  // used only if kDx
        const uint32_t off_dx = pt.off(idx_n, A.sub_ld_out) * (uint32_t)sizeof(T);
        const uint32_t block_bytes = (uint32_t)(((G::n >> pt.row_log) - 1) * A.sub_ld_out + pt.rmask + 1) * (uint32_t)sizeof(T);
        const uint32_t tail_bytes = pt.tail > 0 ? (uint32_t)((pt.tail - 1) * A.sub_ld_out + pt.rmask + 1) * (uint32_t)sizeof(T) : 0u;
        __syncthreads();  // the other group's first row
        __syncthreads();
        int row = pt.slot;
        for (int it = 0; it < mine; ++it, row += pt.nslots) {
            float vx[8], vg[8];
            lds_read_n2(hand, an, vx);
            lds_read_n2(hand + G::kRowFloats, an, vg);
            __syncthreads();  // B1: the reads above are complete before the other group refills the area
            n_phase(vx, vg, cn, acc);
            if (kDx) {
                const float4 da = ((const float4 *)dtab)[tid], db = ((const float4 *)dtab)[512 + tid];
                vg[0] *= da.x; vg[1] *= da.y; vg[2] *= da.z; vg[3] *= da.w;
                vg[4] *= db.x; vg[5] *= db.y; vg[6] *= db.z; vg[7] *= db.w;
                uint32_t off = off_dx;
                asm volatile("" : "+v"(off));
                if (kVirt)  // the short last block stores only the rows it has
                    store8_bounded(dx + row * A.ld_out, row == pt.tail_row ? tail_bytes : block_bytes, off, vg);
                else
                    store8((T *)((char *)(dx + row * A.ld_out) + off), vg);
            }
            __syncthreads();  // B2
        }
        finalize_n(part, acc, idx_n, fw, ts, pt.tmask, xs / 2, pt.c0, pt.n_log, kVirt ? pt.rmask : 0, A.first_chunk);
    }
}

// out[q] = sum over slices of partial[s][q] (+ the upper-half share of the last layer where a slice has
// one), in double, slice order; skipped for flagged plans
template <typename Out>
__global__ void bwd_reduce_kernel(const float *__restrict__ partial, Out *__restrict__ out, size_t n_angles,
                                  size_t slice_floats, size_t last_layer_at, int n_parts, const int *bad_fwd,
                                  const int *bad_inv)
{
    if ((*bad_fwd | *bad_inv) != 0) return;
    const size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= n_angles) return;
    const size_t extra = slice_floats - n_angles;  // 0, or the number of angles of the last layer
    double acc = 0.0;
    for (int w = 0; w < n_parts; ++w) {
        const float *s = partial + (size_t)w * slice_floats;
        acc += (double)s[q];
        if (extra && q >= last_layer_at) acc += (double)s[q + extra];
    }
    out[q] = (Out)acc;
}

// n < 4096: the sums of a 4096-point block hold, per layer, the block's rows side by side, each with its `heads`
// transforms; dtheta[h][i][p] = sum over the rows, in row order
__global__ void bwd_fold_kernel(const double *__restrict__ sums, float *__restrict__ dtheta, int n_log, int heads,
                                const int *bad_fwd, const int *bad_inv)
{
    if ((*bad_fwd | *bad_inv) != 0) return;
    const int half = 1 << (n_log - 1);
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= heads * n_log * half) return;
    const int p = q & (half - 1), hl = q >> (n_log - 1);
    const int layer = hl % n_log, h = hl / n_log;
    const int block_rows = (G::n >> n_log) / heads;
    double acc = 0.0;
    for (int row = 0; row < block_rows; ++row) acc += sums[layer * (G::n / 2) + (row * heads + h) * half + p];
    dtheta[q] = (float)acc;
}

// ---- host side -----------------------------------------------------------------------------------
// Slices = row slots of the PN kernel, which runs one workgroup per compute unit (n = 8192: two per slot).
static int bwd_fast_slices(int k) { return k == 13 ? 128 : 256; }
static constexpr int kBwdFGrid = 512;
// Kernel rows (of 4096 or 8192 elements) per chunk bound the float32 intermediate in the workspace (2^30
// elements, 4 GiB).  Small chunks that would stay in the last-level cache measured slower: every launch
// re-reads the coefficients and rewrites the partial slices, which only amortises over many rows per workgroup.
static int64_t bwd_fast_chunk_rows(int k) { return (int64_t)1 << (k == 13 ? 17 : 18); }
static size_t bwd_fast_slice_floats(int k) { return k == 13 ? (size_t)13 * 4096 + 4096 : (size_t)K * (G::n / 2); }
static int64_t bwd_fast_block_rows(const Shape &s) { return s.k < K ? (int64_t)G::n / ((int64_t)s.n * s.heads) : 1; }
static int64_t bwd_fast_kernel_rows(const Shape &s)
{
    const int64_t r = bwd_fast_block_rows(s);
    return (s.rows + r - 1) / r;
}

bool bwd_fast_supported(const void *x, const void *dy, const void *dx, const float *dtheta, const Shape &s)
{
    if (s.k < 8 || s.k > 13 || dtheta == nullptr || s.rows == 0) return false;
    // several heads: n < 4096 with rows of at most 4096 elements that tile a 4096-element block
    if (s.heads != 1 && (s.k >= K || (int64_t)s.n * s.heads > G::n || G::n % (s.n * s.heads) != 0)) return false;
    const int vec = s.dtype == BQ_F32 ? 4 : 8;
    if (((uintptr_t)x & 15) || ((uintptr_t)dy & 15) || (dx && ((uintptr_t)dx & 15))) return false;
    if ((s.ld_x % vec) || (s.ld_y % vec)) return false;
    if (s.k < K) {  // offsets inside a block of 4096 / n rows are 32-bit byte offsets
        const int64_t r = bwd_fast_block_rows(s);
        if (r * s.ld_x * 4 >= ((int64_t)1 << 31) || r * s.ld_y * 4 >= ((int64_t)1 << 31)) return false;
    }
    return true;
}

static size_t bwd_fast_fold_bytes(int k) { return k < K ? align256((size_t)K * (G::n / 2) * sizeof(double)) : 0; }

size_t bwd_fast_workspace_bytes(const Shape &s)
{
    const int64_t kr = bwd_fast_kernel_rows(s);
    const size_t chunk = (size_t)(kr < bwd_fast_chunk_rows(s.k) ? kr : bwd_fast_chunk_rows(s.k));
    return align256((size_t)bwd_fast_slices(s.k) * bwd_fast_slice_floats(s.k) * sizeof(float)) + bwd_fast_fold_bytes(s.k) +
           align256(chunk * (s.k == 13 ? 8192 : 4096) * sizeof(float));
}

template <typename T, bool kHalf, bool kVirt>
static hipError_t launch_bwd_fast_t(BwdFastArgs A, const Shape &s, float *dtheta, char *ws, hipStream_t stream)
{
    const int slices = bwd_fast_slices(s.k);
    const int64_t kernel_rows = bwd_fast_kernel_rows(s);
    const int64_t chunk_rows = kernel_rows < bwd_fast_chunk_rows(s.k) ? kernel_rows : bwd_fast_chunk_rows(s.k);
    A.slice_floats = (int64_t)bwd_fast_slice_floats(s.k);
    A.partial = (float *)ws;
    double *fold = (double *)(ws + align256((size_t)slices * A.slice_floats * sizeof(float)));
    A.xk = (float *)((char *)fold + bwd_fast_fold_bytes(s.k));
    const size_t lds_f = 2 * G::kRowFloats * sizeof(float), lds_pn = kPnLdsFloats * sizeof(float);
    hipError_t e = hipFuncSetAttribute((const void *)bwd_f_kernel<T, kHalf, kVirt>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_f);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)bwd_pn_kernel<T, true, kHalf, kVirt>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_pn);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)bwd_pn_kernel<T, false, kHalf, kVirt>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_pn);
    if (e != hipSuccess) return e;
    const int pn_grid = kHalf ? 2 * slices : slices;  // kHalf: a multiple of 16 (see Part)
    for (int64_t r0 = 0; r0 < kernel_rows; r0 += chunk_rows) {
        A.row0 = r0;
        A.rows = kernel_rows - r0 < chunk_rows ? kernel_rows - r0 : chunk_rows;
        A.first_chunk = (r0 == 0);
        // every slice must be written by the first chunk, so the grids do not shrink with the row count
        hipLaunchKernelGGL((bwd_f_kernel<T, kHalf, kVirt>), dim3(kBwdFGrid), dim3(G::threads), lds_f, stream, A);
        if (A.dx)
            hipLaunchKernelGGL((bwd_pn_kernel<T, true, kHalf, kVirt>), dim3(pn_grid), dim3(kPnThreads), lds_pn, stream, A);
        else
            hipLaunchKernelGGL((bwd_pn_kernel<T, false, kHalf, kVirt>), dim3(pn_grid), dim3(kPnThreads), lds_pn, stream, A);
    }
    if (kVirt) {
        const size_t sums = (size_t)s.k * (G::n / 2);  // the layers the transform has
        hipLaunchKernelGGL(bwd_reduce_kernel<double>, dim3((unsigned)((sums + 255) / 256)), dim3(256), 0, stream,
                           (const float *)ws, fold, sums, (size_t)A.slice_floats, sums, slices, A.bad_fwd, A.bad_inv);
        const unsigned angles = (unsigned)(s.heads * s.k * (s.n / 2));
        hipLaunchKernelGGL(bwd_fold_kernel, dim3((angles + 255) / 256), dim3(256), 0, stream, (const double *)fold, dtheta, s.k,
                           s.heads, A.bad_fwd, A.bad_inv);
    } else {
        const size_t angles = (size_t)s.k * (s.n / 2);
        hipLaunchKernelGGL(bwd_reduce_kernel<float>, dim3((unsigned)((angles + 255) / 256)), dim3(256), 0, stream,
                           (const float *)ws, dtheta, angles, (size_t)A.slice_floats, (size_t)(s.k - 1) * (s.n / 2), slices,
                           A.bad_fwd, A.bad_inv);
    }
    return hipGetLastError();
}

template <bool kHalf, bool kVirt>
static hipError_t launch_bwd_fast_d(const BwdFastArgs &A, const Shape &s, float *dtheta, char *ws, hipStream_t stream)
{
    switch (s.dtype) {
        case BQ_F32: return launch_bwd_fast_t<float, kHalf, kVirt>(A, s, dtheta, ws, stream);
        case BQ_F16: return launch_bwd_fast_t<__half, kHalf, kVirt>(A, s, dtheta, ws, stream);
        default: return launch_bwd_fast_t<bf16_t, kHalf, kVirt>(A, s, dtheta, ws, stream);
    }
}

hipError_t launch_bwd_fast(const void *x, const void *dy, const PlanView &pv, void *dx, float *dtheta, void *ws,
                           const Shape &s, hipStream_t stream)
{
    BwdFastArgs A{};
    A.x = x;
    A.dy = dy;
    A.dx = dx;
    A.fg_fwd = pv.fg_fwd;
    A.fd_fwd = pv.fd_fwd;
    A.fm_fwd = pv.fm_fwd;
    A.fg_inv = pv.fg_inv;
    A.fd_inv = pv.fd_inv;
    A.fw_inv = pv.fw_inv;
    A.bad_fwd = &pv.hdr->fast_bad_fwd;
    A.bad_inv = &pv.hdr->fast_bad_inv;
    A.n = s.n;
    A.n_log = s.k;
    A.heads = s.heads;
    A.row_log = s.k < K ? ilog2_exact(s.n * s.heads) : 0;
    A.total_rows = s.rows;
    A.sub_ld_in = s.ld_x;
    A.sub_ld_out = s.ld_y;
    const int64_t block_rows = bwd_fast_block_rows(s);
    A.ld_in = s.ld_x * block_rows;
    A.ld_out = s.ld_y * block_rows;
    char *w = (char *)ws;
    if (s.k < K) return launch_bwd_fast_d<false, true>(A, s, dtheta, w, stream);
    if (s.k == K) return launch_bwd_fast_d<false, false>(A, s, dtheta, w, stream);
    return launch_bwd_fast_d<true, false>(A, s, dtheta, w, stream);
}

}  // namespace bq
