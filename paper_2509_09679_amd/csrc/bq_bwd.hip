// Backward pass for n = 256 .. 8192, in blocks of 4096 points (k = 12): dx = B^T dy and
// dtheta[i][p] = sum over rows of  g_i[b] x_i[a] - g_i[a] x_i[b]   (x_i, g_i at the output of layer i;
// paper, "Gradient Flow Through Butterfly Layers": d y_a / d theta = -y_b, d y_b / d theta = y_a).
//
// Orthogonality makes stored activations unnecessary: x_{i-1} = B_i^T x_i.  The forward state of a row is
// recomputed in the workgroup that consumes it, then the transposed cascade runs on x and g together.  Both
// start it with scale 1, so they share the scale-deferred coefficients c_i and, before layer i, the scales
// E_i[e] (plan table fw_inv).  Sums are accumulated in deferred units,
//   acc += v_g[b] v_x[a] - v_g[a] v_x[b],   dtheta = E_i[a] E_i[b] acc,
// the factor being applied once per workgroup at the end.  For a layer that pairs lanes each lane keeps
// the partial sum of its own element (one v_fmac_f32 with a DPP operand per element); the two lanes'
// sums are combined at the end.
//
// One kernel, one pass over x, dy and dx, nothing else in memory.  What makes that fit a compute unit's
// registers: the forward recomputation uses the SAME coefficient registers as the transposed cascade (see
// reg_layer_swapped below), so a thread holds one coefficient per element and layer plus the layer's sums,
// and the 12 layers are split over two groups of eight waves by position, not by direction:
//   group N (layout N: 8 consecutive elements per thread, layers 1..3 on registers, 4..6 on DPP lanes)
//   group Q (layout Q: layers 7..10 on DPP lanes, 11 and 12 on registers)
// A row goes  N: layers 1..6 forward -> LDS -> Q: layers 7..12 forward, then 12..7 transposed on (x, g)
// with sums -> LDS -> N: layers 6..1 transposed with sums, dx out;  the groups work on different rows at
// the same time (see bwd_fused_kernel).
//
// n = 8192: layers 1..12 act inside each half of a row, only layer 13 couples the halves.  A workgroup
// takes one half of its rows; group Q reads both halves of dy, forms its own half of g_12 and, for the sum of
// layer 13, the other half as well:
//   dtheta_13[p] = sum over rows of  g_12[b] x_12[a] - g_12[a] x_12[b]
// (the same expression one layer further down: rotating both vectors of a pair leaves it unchanged),
// the lower-half workgroup contributing the first term and the upper-half one the second.
//
// Every workgroup owns one slice of `partial`; a slice entry is written by exactly one thread, chunks
// of rows add to it in stream order, and a last kernel sums the slices in double in a fixed order: no
// atomics, the result does not depend on scheduling.
//
// The kernel exits at once when the plan flags the scale-deferred tables as unusable; the generic
// backward kernel, launched behind it with the opposite condition, then does the work.
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
    float *partial;  // [slices][slice_floats]
    const float *fg_inv, *fd_inv, *fw_inv;  // plan tables of the transposed cascade
    const int *bad_fwd, *bad_inv;
    PlanRef plan;
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

// true: this kernel must not run (tables flagged unusable, or not a plan of this shape at all)
__device__ __forceinline__ bool plan_is_bad(const BwdFastArgs &A)
{
    return !plan_matches(A.plan) || (*A.bad_fwd | *A.bad_inv) != 0;
}

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
    static constexpr int xs = kHalf ? 2 * G::n : G::n;  // kernel row length; a slice holds xs / 2 sums per layer
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

// ---- layout Q and the forward recomputation ---------------------------------------------------------------
// base index of a thread in layout Q: the four bits of its chunk inside the 16-lane row are idx bits 7, 8, 9
// (DPP masks 1, 2, 7: layers 8, 9, 10) and idx bit 6 (row_ror:8: layer 7); idx bit 0 and idx bits 10, 11 are
// register bits (layers 11, 12 pair registers); idx bits 1, 2 are lane bits 4, 5 and idx bits 3..5 the wave.
__device__ __forceinline__ int base_q(int wave, int lane)
{
    const int c4 = lane_chunk(lane & 15);
    return ((c4 & 7) << 7) | ((c4 >> 3) << 6) | (((lane >> 4) & 1) << 1) | (((lane >> 5) & 1) << 2) | (wave << 3);
}

// Forward layer in the transposed cascade's own coefficients.  With E_i[e] the scale of element e before
// transposed layer i (plan table fw_inv; E_0 = fd_inv), carry the forward state as w_i = E_i * x_i.  Then
//   w_i[a] = w_{i-1}[a] + c_i[b] w_{i-1}[b],   w_i[b] = w_{i-1}[b] + c_i[a] w_{i-1}[a]
// with c_i the transposed cascade's coefficients: an element's forward coefficient is its PARTNER's coefficient
// of the transposed layer.  (Forward deferred scale F and transposed scale E of a pair satisfy
// F[b] / F[a] = E[a] / E[b] when F = 1 / E, and E_{i-1} = cos * E_i for both elements of a pair.)  After the
// last layer w = x, which is also where the transposed cascade starts (E = 1): no rescaling at the turn.
template <int J>
__device__ __forceinline__ void reg_layer_swapped(float (&u)[8], const float (&c)[8])
{
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        if (!(r & (1 << J))) {
            const int a = r, b = r | (1 << J);
            const float ua = u[a], ub = u[b];
            u[a] = __builtin_fmaf(c[b], ub, ua);
            u[b] = __builtin_fmaf(c[a], ua, ub);
        }
    }
}
// ... and for a pair in two lanes: both the partner's coefficient and the partner's value sit in the other
// lane, so the product is formed there and fetched with one DPP add.
#define BQ_DPP_ADD8(MOD)                                                                               \
    asm volatile("s_nop 1\n\t"                                                                        \
                 "v_add_f32_dpp %0, %8, %0 " MOD " row_mask:0xf bank_mask:0xf\n\t"                    \
                 "v_add_f32_dpp %1, %9, %1 " MOD " row_mask:0xf bank_mask:0xf\n\t"                    \
                 "v_add_f32_dpp %2, %10, %2 " MOD " row_mask:0xf bank_mask:0xf\n\t"                   \
                 "v_add_f32_dpp %3, %11, %3 " MOD " row_mask:0xf bank_mask:0xf\n\t"                   \
                 "v_add_f32_dpp %4, %12, %4 " MOD " row_mask:0xf bank_mask:0xf\n\t"                   \
                 "v_add_f32_dpp %5, %13, %5 " MOD " row_mask:0xf bank_mask:0xf\n\t"                   \
                 "v_add_f32_dpp %6, %14, %6 " MOD " row_mask:0xf bank_mask:0xf\n\t"                   \
                 "v_add_f32_dpp %7, %15, %7 " MOD " row_mask:0xf bank_mask:0xf"                       \
                 : "+v"(u[0]), "+v"(u[1]), "+v"(u[2]), "+v"(u[3]), "+v"(u[4]), "+v"(u[5]), "+v"(u[6]),  \
                   "+v"(u[7])                                                                          \
                 : "v"(z[0]), "v"(z[1]), "v"(z[2]), "v"(z[3]), "v"(z[4]), "v"(z[5]), "v"(z[6]), "v"(z[7]))

#define BQ_DPP_FWD_LAYER(NAME, MOD)                                                        \
    __device__ __forceinline__ void NAME(float (&u)[8], const float (&c)[8])               \
    {                                                                                      \
        float z[8];                                                                        \
        _Pragma("unroll") for (int r = 0; r < 8; ++r) z[r] = c[r] * u[r];                  \
        BQ_DPP_ADD8(MOD);                                                                  \
    }
BQ_DPP_FWD_LAYER(dpp_fwd_xor1, "quad_perm:[1,0,3,2]")
BQ_DPP_FWD_LAYER(dpp_fwd_xor2, "quad_perm:[2,3,0,1]")
BQ_DPP_FWD_LAYER(dpp_fwd_xor7, "row_half_mirror")
BQ_DPP_FWD_LAYER(dpp_fwd_xor8, "row_ror:8")

// ---- deferred sums and the transposed layers of the two wave groups -----------------------------------------
struct QAcc {  // group Q: lane layers 7 (d[0]), 8, 9, 10 (d[1..3]), register layers 11 (r1) and 12 (r2)
    float d[4][8], r1[4], r2[4];
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r) d[j][r] = 0.0f;
#pragma unroll
        for (int q = 0; q < 4; ++q) r1[q] = r2[q] = 0.0f;
    }
};
struct NAcc6 {  // group N: register layers 1..3 (r[0..2]), lane layers 4..6 (d[0..2])
    float d[3][8], r[3][4];
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int j = 0; j < 3; ++j) {
#pragma unroll
            for (int q = 0; q < 8; ++q) d[j][q] = 0.0f;
#pragma unroll
            for (int q = 0; q < 4; ++q) r[j][q] = 0.0f;
        }
    }
};

// Coefficients of layer 7 for group Q: in registers, or parked in LDS (written and read by the same thread)
// where the registers are short.
template <bool kLds>
struct Coef7 {
    float c[kLds ? 1 : 8];
    const float4 *tab;  // kLds: the workgroup's table area; this thread's float4 slots are first and first + 512
    int first;
    __device__ __forceinline__ void init(const float (&v)[8], float4 *table, int slot)
    {
        if (kLds) {
            table[slot] = make_float4(v[0], v[1], v[2], v[3]);
            table[slot + 512] = make_float4(v[4], v[5], v[6], v[7]);
            tab = table;
            first = slot;
        } else {
#pragma unroll
            for (int r = 0; r < 8; ++r) c[kLds ? 0 : r] = v[r];
        }
    }
    __device__ __forceinline__ void get(float (&o)[8]) const
    {
        if (kLds) {
            int f = first;
            asm volatile("" : "+v"(f));  // keeps the reads inside the row loop (hoisted, they would occupy registers again)
            const float4 a = tab[f], b = tab[f + 512];
            o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
        } else {
#pragma unroll
            for (int r = 0; r < 8; ++r) o[r] = c[kLds ? 0 : r];
        }
    }
};

// layers 12..7 transposed on (vx, vg) held in layout Q; cq[j] = coefficients of layer 8 + j
template <class C7>
__device__ __forceinline__ void q_phase(float (&vx)[8], float (&vg)[8], const C7 &c7, const float (&cq)[5][8], QAcc &acc)
{
    reg_acc<2>(acc.r2, vg, vx);  // layer 12 (register bit 2)
    reg_layer<2>(vx, cq[4]);
    reg_layer<2>(vg, cq[4]);
    reg_acc<1>(acc.r1, vg, vx);  // layer 11 (register bit 1)
    reg_layer<1>(vx, cq[3]);
    reg_layer<1>(vg, cq[3]);
    dpp_acc_xor7(acc.d[3], vg, vx);  // layer 10
    dpp_layer_xor7(vx, cq[2]);
    dpp_layer_xor7(vg, cq[2]);
    dpp_acc_xor2(acc.d[2], vg, vx);  // layer 9
    dpp_layer_xor2(vx, cq[1]);
    dpp_layer_xor2(vg, cq[1]);
    dpp_acc_xor1(acc.d[1], vg, vx);  // layer 8
    dpp_layer_xor1(vx, cq[0]);
    dpp_layer_xor1(vg, cq[0]);
    float c[8];
    c7.get(c);
    dpp_acc_xor8(acc.d[0], vg, vx);  // layer 7
    dpp_layer_xor8(vx, c);
    dpp_layer_xor8(vg, c);
}
// layers 7..12 forward on w held in layout Q
template <class C7>
__device__ __forceinline__ void q_forward(float (&w)[8], const C7 &c7, const float (&cq)[5][8])
{
    {
        float c[8];
        c7.get(c);
        dpp_fwd_xor8(w, c);
    }
    dpp_fwd_xor1(w, cq[0]);
    dpp_fwd_xor2(w, cq[1]);
    dpp_fwd_xor7(w, cq[2]);
    reg_layer_swapped<1>(w, cq[3]);
    reg_layer_swapped<2>(w, cq[4]);
}
// layers 6..1 transposed on (vx, vg) held in layout N; on return vg holds g_0 in deferred units
__device__ __forceinline__ void n_phase6(float (&vx)[8], float (&vg)[8], const float (&cn)[6][8], NAcc6 &acc)
{
    dpp_acc_xor7(acc.d[2], vg, vx);  // layer 6
    dpp_layer_xor7(vx, cn[5]);
    dpp_layer_xor7(vg, cn[5]);
    dpp_acc_xor2(acc.d[1], vg, vx);  // layer 5
    dpp_layer_xor2(vx, cn[4]);
    dpp_layer_xor2(vg, cn[4]);
    dpp_acc_xor1(acc.d[0], vg, vx);  // layer 4
    dpp_layer_xor1(vx, cn[3]);
    dpp_layer_xor1(vg, cn[3]);
    reg_acc<2>(acc.r[2], vg, vx);  // layer 3
    reg_layer<2>(vx, cn[2]);
    reg_layer<2>(vg, cn[2]);
    reg_acc<1>(acc.r[1], vg, vx);  // layer 2
    reg_layer<1>(vx, cn[1]);
    reg_layer<1>(vg, cn[1]);
    reg_acc<0>(acc.r[0], vg, vx);  // layer 1 (x is not needed below it)
    reg_layer<0>(vg, cn[0]);
}
// layers 1..6 forward on w held in layout N.  kParked: the partner lane's coefficients of layers 4..6 come from the
// thread's LDS slots (float4 slots first + 1024 j and first + 1024 j + 512 for layer 4 + j).
template <bool kParked>
__device__ __forceinline__ void n_forward(float (&w)[8], const float (&cn)[6][8], const float4 *tab, int first)
{
    reg_layer_swapped<0>(w, cn[0]);
    reg_layer_swapped<1>(w, cn[1]);
    reg_layer_swapped<2>(w, cn[2]);
    if (!kParked) {
        dpp_fwd_xor1(w, cn[3]);
        dpp_fwd_xor2(w, cn[4]);
        dpp_fwd_xor7(w, cn[5]);
    } else {
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            int f = first + 1024 * j;
            asm volatile("" : "+v"(f));  // keeps the reads inside the row loop (hoisted, they would occupy registers)
            const float4 a = tab[f], b = tab[f + 512];
            const float c[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
            if (j == 0) dpp_layer_xor1(w, c);
            if (j == 1) dpp_layer_xor2(w, c);
            if (j == 2) dpp_layer_xor7(w, c);
        }
    }
}

// fw_inv entry (scale before transposed layer i) of block element e; rmask != 0: the tables of e's own head
__device__ __forceinline__ float fw_at(const float *fw_inv, int stride, int tmask, int n_log, int rmask, int c0, int e, int i)
{
    const int hd = (e & rmask) >> n_log;
    return fw_inv[((size_t)hd * n_log + (i - 1)) * stride + ((c0 + e) & tmask)];
}

// Deferred sums -> dtheta partials of this workgroup.  part: its slice, `pairs` sums per layer, indexed by the
// pair's position in the whole kernel row (c0 + element); fw_inv: the plan table, rows `stride` apart, column
// (c0 + element) & tmask.
struct FinArgs {
    float *part;
    const float *fw_inv;
    int stride, tmask, pairs, c0, n_log, rmask, first;
    __device__ __forceinline__ float scale(int a, int b, int i) const
    {
        return fw_at(fw_inv, stride, tmask, n_log, rmask, c0, a, i) * fw_at(fw_inv, stride, tmask, n_log, rmask, c0, b, i);
    }
    __device__ __forceinline__ float *at(int a, int i) const { return part + (size_t)(i - 1) * pairs + pair_index(c0 + a, i); }
};

// lane layer i whose pairs sit in lanes `mask_j` apart (0..3: masks 1, 2, 7, 8); e[r]: the thread's elements
template <class Idx>
__device__ __forceinline__ void finalize_lane_layer(const FinArgs &F, const float (&acc)[8], int i, int mask_j, Idx elem)
{
    if (i > F.n_log) return;  // a layer the transform does not have: no table row, nothing to write
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const float mine = acc[r];
        const float other = lane_partner(mine, mask_j);
        const int e = elem(r);
        if (!(e & (1 << (i - 1)))) {  // the lane holding the lower element writes
            const int b = e | (1 << (i - 1));
            put_partial(F.at(e, i), (mine - other) * F.scale(e, b, i), F.first);
        }
    }
}
// register layer i pairing register bit J
template <int J, class Idx>
__device__ __forceinline__ void finalize_reg_layer(const FinArgs &F, const float (&acc)[4], int i, Idx elem)
{
    if (i > F.n_log) return;
    int q = 0;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        if (!(r & (1 << J))) {
            const int a = elem(r), b = elem(r | (1 << J));
            put_partial(F.at(a, i), acc[q] * F.scale(a, b, i), F.first);
            ++q;
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
                w[i] = f32x2_to_f16x2_bits(y[2 * i], y[2 * i + 1]);
            } else {
                w[i] = f32x2_to_bf16x2_bits(y[2 * i], y[2 * i + 1]);
            }
        }
        bwd_v4i a = {(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
        __builtin_amdgcn_raw_buffer_store_b128(a, rs, (int)off, 0, 0);
    }
}

// Workgroup barrier that waits for the wave's LDS traffic only.  (__syncthreads() also waits for the wave's
// outstanding global loads and stores, which would end every row's prefetch at the next barrier.)  Everything
// the two wave groups exchange goes through LDS.
__device__ __forceinline__ void wg_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// ---- the fused pass ---------------------------------------------------------------------------------------
// Waves 0..7 (group N, layout N, layers 1..6) and waves 8..15 (group Q, layout Q, layers 7..12) of a workgroup
// pipeline its rows; per iteration `it` and two barriers M and E:
//   N: read H (row it-2: x_6, g_6)          | M | layers 6..1 transposed with sums, dx out; row it: x in, scale
//                                                 E_0, layers 1..6 forward, write XA                           | E
//   Q: read XA (row it-1: w_6)              | M | layers 7..12 forward; dy (row it-1) from the ring; layers
//                                                 12..7 transposed with sums; write H                          | E
// XA and H are read before M and written after it, so one buffer each suffices.  dy reaches group Q through a
// ring of LDS slots filled by direct global->LDS loads (16 bytes per lane, issued by group Q's waves one
// iteration or more ahead); the chunk a lane loads is chosen so that the 4-byte reads of layout Q spread over
// all banks:  position (16-byte units) of chunk q = idx >> 3 in a slot:
//   pos bits 0..2 = q bits 4..6 (idx 7..9), pos bits 3..5 = q bits 0..2 (idx 3..5), pos bits 6..8 = q bits 3, 7, 8.
// x reaches group N through registers (one row ahead).
constexpr int kFusedThreads = 1024;

template <typename T, bool kHalf>
struct FusedLds {
    static constexpr int kSlots = kHalf ? 2 : 3;  // dy ring
    static constexpr uint32_t kHalfRowBytes = G::n * sizeof(T);
    static constexpr uint32_t kSlotBytes = kHalfRowBytes * (kHalf ? 2 : 1);
    // 16-bit rows: x comes through a ring of its own (two slots; a wave reads back only what it loaded itself);
    // 32-bit rows are prefetched in registers
    static constexpr bool kXRing = sizeof(T) == 2;
    static constexpr uint32_t kXSlotBytes = kHalfRowBytes;
    static constexpr size_t kDyRingBytes = (size_t)kSlots * kSlotBytes;
    static constexpr size_t kXRingBytes = kXRing ? 2 * (size_t)kXSlotBytes : 0;
    // n = 8192 with 16-bit rows: group Q is short of registers and parks the coefficients of layer 7 in LDS
    static constexpr bool kPark7 = kHalf && sizeof(T) == 2;
    // n <= 4096 with 16-bit rows: LDS has room for the PARTNER's coefficients of group N's three lane layers, with
    // which the forward recomputation of those layers costs one DPP FMA per element instead of a multiplication
    // and a DPP addition
    static constexpr bool kParkFwd = !kHalf && sizeof(T) == 2;
    // per-thread tables: E_0 (group N); n = 8192: the layer-13 coefficients (group Q); kPark7: layer 7 (group Q);
    // kParkFwd: three layers of partner coefficients (group N)
    static constexpr int kTabFloats = (kHalf ? (kPark7 ? 3 : 2) : kParkFwd ? 4 : 1) * G::n;
    // The rings come first: the LDS address of a direct global->LDS load travels in M0, and the rings' addresses
    // stay below 64 KB this way whatever the field's width.
    static constexpr size_t kRingBytes = kDyRingBytes + kXRingBytes;
    static_assert(kRingBytes <= 65536, "ring addresses must fit 16 bits");
    static constexpr size_t kBytes = kRingBytes + (3 * (size_t)G::kRowFloats + kTabFloats) * sizeof(float);
    static_assert(kBytes <= 160 * 1024, "LDS of a compute unit");
};

template <typename T, bool kDx, bool kHalf, bool kVirt>
__global__ __launch_bounds__(kFusedThreads) void bwd_fused_kernel(BwdFastArgs A)
{
    extern __shared__ float lds[];
    if (plan_is_bad(A)) return;
    using L = FusedLds<T, kHalf>;
    const Part<kHalf, kVirt> pt(A);
    const int ts = pt.ts;
    constexpr int xs = Part<kHalf, kVirt>::xs;
    const int role = threadIdx.x >> 9;  // uniform per wave
    const int tid = threadIdx.x & 511, wave = tid >> 6, lane = tid & 63;
    float *xa = lds + L::kRingBytes / sizeof(float), *hx = xa + G::kRowFloats, *hg = xa + 2 * G::kRowFloats;
    float4 *tab = (float4 *)(xa + 3 * G::kRowFloats);  // per-thread tables: float4 slots [tid] and [512 + tid]
    const int mine = A.rows > (int64_t)pt.slot ? (int)((A.rows - pt.slot + pt.nslots - 1) / pt.nslots) : 0;
    const int iters = mine > 0 ? mine + 2 : 0;
    const float *fg = A.fg_inv;
    FinArgs F;
    F.part = A.partial + (size_t)pt.slot * A.slice_floats;
    F.fw_inv = A.fw_inv;
    F.stride = ts;
    F.tmask = pt.tmask;
    F.pairs = xs / 2;
    F.c0 = pt.c0;
    F.n_log = pt.n_log;
    F.rmask = kVirt ? pt.rmask : 0;
    F.first = A.first_chunk;
    if (role == 0) {
        // ---- group N ----
        const int idx_n = (wave * 64 + lane_chunk(lane)) * 8;
        const int an = lds_addr2(idx_n);
        float cn[6][8];
#pragma unroll
        for (int j = 0; j < 6; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r) cn[j][r] = fg[pt.trow(idx_n, j) + pt.col(idx_n) + r];
        {
            const float *e0 = A.fd_inv + (size_t)pt.head(idx_n) * ts + pt.col(idx_n);
            tab[tid] = *(const float4 *)e0;
            tab[512 + tid] = *(const float4 *)(e0 + 4);
        }
        if (L::kParkFwd) {
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                float pc[8];
#pragma unroll
                for (int r = 0; r < 8; ++r) pc[r] = lane_partner(cn[3 + j][r], j);
                tab[1024 + 1024 * j + tid] = make_float4(pc[0], pc[1], pc[2], pc[3]);
                tab[1024 + 1024 * j + 512 + tid] = make_float4(pc[4], pc[5], pc[6], pc[7]);
            }
        }
        // The empty statements consume the loaded coefficients: the waits for these loads then sit here and not,
        // as waits for everything outstanding, inside the row loop.
#pragma unroll
        for (int j = 0; j < 6; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r) asm volatile("" ::"v"(cn[j][r]));
        NAcc6 acc;
        acc.clear();
        const T *x = (const T *)A.x + A.row0 * A.ld_in + pt.c0;
        T *dx = (T *)A.dx + A.row0 * A.ld_out + pt.c0;  // used only if kDx
        // kVirt: a sub-row missing from the last block reads the block's first row instead (its dy will be zero)
        const uint32_t off_x = pt.off(idx_n, A.sub_ld_in) * (uint32_t)sizeof(T);
        const uint32_t off_x0 = pt.off(idx_n & pt.tmask, A.sub_ld_in) * (uint32_t)sizeof(T);
        const bool gap = pt.in_tail_gap(idx_n);
        const uint32_t off_dx = pt.off(idx_n, A.sub_ld_out) * (uint32_t)sizeof(T);
        const uint32_t block_bytes = (uint32_t)(((G::n >> pt.row_log) - 1) * A.sub_ld_out + pt.rmask + 1) * (uint32_t)sizeof(T);
        const uint32_t tail_bytes = pt.tail > 0 ? (uint32_t)((pt.tail - 1) * A.sub_ld_out + pt.rmask + 1) * (uint32_t)sizeof(T) : 0u;
        auto load_row = [&](int r) {  // 32-bit rows: the thread's 8 elements of kernel row r
            uint32_t off = (gap && r == pt.tail_row) ? off_x0 : off_x;
            asm volatile("" : "+v"(off));
            return load8((const T *)((const char *)(x + r * A.ld_in) + off));
        };
        // 16-bit rows: the x ring.  Lane l of wave w loads the chunk (8 elements) 64 w + l of row j into bytes
        // [1024 w + 16 l, +16) of slot j & 1 and the thread reads its own chunk 64 w + e(l) back: only the wave's
        // own loads are involved, so s_waitcnt vmcnt is the only synchronisation, and the load of row it + 2 can
        // follow the read of row it at once.  Memory operations of a wave complete in issue order: when row `it`
        // is consumed, the younger ones are the load of row it + 1 and the dx stores of two iterations.
        constexpr bool kXRing = L::kXRing;
        constexpr int kStores = kDx ? 1 : 0;
        const uint32_t xring0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds + (uint32_t)L::kDyRingBytes;
        const uint32_t xwave_base = __builtin_amdgcn_readfirstlane(xring0 + (uint32_t)wave * 1024u);
        const uint32_t xrd_addr = xring0 + (uint32_t)(wave * 64 + lane_chunk(lane)) * 16u;
        const int e_xload = (wave * 64 + lane) * 8;
        const uint32_t xvoff = pt.off(e_xload, A.sub_ld_in) * (uint32_t)sizeof(T);
        const uint32_t xvoff0 = pt.off(e_xload & pt.tmask, A.sub_ld_in) * (uint32_t)sizeof(T);
        const bool xgap = pt.in_tail_gap(e_xload);
        auto x_ring_load = [&](int j) {
            const int jj = j < mine ? j : mine - 1;  // past the end: the last row again (unused)
            const int row = pt.slot + jj * pt.nslots;
            const uint32_t vo = (xgap && row == pt.tail_row) ? xvoff0 : xvoff;
            const char *rowp = (const char *)(x + row * A.ld_in);
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2"
                         :
                         : "v"(vo), "s"(xwave_base + (uint32_t)(j & 1) * L::kXSlotBytes), "s"(rowp)
                         : "memory");
        };
        Raw8 raw = {};
        if (mine > 0) {
            if (kXRing) {
                x_ring_load(0);
                x_ring_load(1);
            } else {
                raw = load_row(pt.slot);
            }
        }
        for (int it = 0; it < iters; ++it) {
            float vx[8], vg[8];
            if (it >= 2) {
                lds_read_n2(hx, an, vx);
                lds_read_n2(hg, an, vg);
            }
            wg_barrier();  // M
            if (it >= 2) {
                n_phase6(vx, vg, cn, acc);
                if (kDx) {
                    const int row = pt.slot + (it - 2) * pt.nslots;
                    const float4 da = tab[tid], db = tab[512 + tid];
                    vg[0] *= da.x; vg[1] *= da.y; vg[2] *= da.z; vg[3] *= da.w;
                    vg[4] *= db.x; vg[5] *= db.y; vg[6] *= db.z; vg[7] *= db.w;
                    uint32_t off = off_dx;
                    asm volatile("" : "+v"(off));
                    if (kVirt)  // the short last block stores only the rows it has
                        store8_bounded(dx + row * A.ld_out, row == pt.tail_row ? tail_bytes : block_bytes, off, vg);
                    else
                        store8((T *)((char *)(dx + row * A.ld_out) + off), vg);
                }
            }
            if (it < mine) {
                float w[8];
                if (kXRing) {
                    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                    u32x4 v;
                    const uint32_t ra = xrd_addr + (uint32_t)(it & 1) * L::kXSlotBytes;
                    if (it >= 4)
                        asm volatile("s_waitcnt vmcnt(%2)\n\tds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)"
                                     : "=v"(v) : "v"(ra), "n"(1 + 2 * kStores) : "memory");
                    else  // the pipeline is still filling (fewer stores issued): wait for everything
                        asm volatile("s_waitcnt vmcnt(0)\n\tds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)"
                                     : "=v"(v) : "v"(ra) : "memory");
                    x_ring_load(it + 2);  // refills the slot just read
                    Raw8 r8;
                    r8.lo = make_uint4(v.x, v.y, v.z, v.w);
                    raw = r8;
                }
                const float4 da = tab[tid], db = tab[512 + tid];
                const float e0[8] = {da.x, da.y, da.z, da.w, db.x, db.y, db.z, db.w};
                if constexpr (std::is_same<T, __half>::value) {
                    // w = E_0 * x as a fused multiply-add with a zero addend: the instruction takes the binary16 operand
                    // as it is, which saves the eight conversions
                    const uint32_t xw[4] = {raw.lo.x, raw.lo.y, raw.lo.z, raw.lo.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const __half2 h = *(const __half2 *)&xw[i];
                        w[2 * i] = __builtin_fmaf(e0[2 * i], __low2float(h), 0.0f);
                        w[2 * i + 1] = __builtin_fmaf(e0[2 * i + 1], __high2float(h), 0.0f);
                    }
                } else {
                    unpack8(raw, w, (const T *)nullptr);
#pragma unroll
                    for (int r = 0; r < 8; ++r) w[r] *= e0[r];
                }
                if (!kXRing && it + 1 < mine) raw = load_row(pt.slot + (it + 1) * pt.nslots);
                n_forward<L::kParkFwd>(w, cn, tab, 1024 + tid);
                lds_write_n2(xa, an, w);
            }
            wg_barrier();  // E
        }
        if (kXRing) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        const auto elem = [&](int r) { return idx_n + r; };
        finalize_reg_layer<0>(F, acc.r[0], 1, elem);
        finalize_reg_layer<1>(F, acc.r[1], 2, elem);
        finalize_reg_layer<2>(F, acc.r[2], 3, elem);
        finalize_lane_layer(F, acc.d[0], 4, 0, elem);
        finalize_lane_layer(F, acc.d[1], 5, 1, elem);
        finalize_lane_layer(F, acc.d[2], 6, 2, elem);
    } else {
        // ---- group Q ----
        const int idx_q = base_q(wave, lane);
        const int aq = lds_addr2(idx_q);
        float cq[5][8];
#pragma unroll
        for (int j = 0; j < 5; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r)  // layers above log2 n do not exist: weight zero leaves the element as it is
                cq[j][r] = (!kVirt || 8 + j <= pt.n_log)
                               ? fg[pt.trow(idx_q + p_reg_idx2<K>(r), 7 + j) + pt.col(idx_q + p_reg_idx2<K>(r))]
                               : 0.0f;
        Coef7<L::kPark7> c7;
        {
            float v[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) v[r] = fg[pt.trow(idx_q + p_reg_idx2<K>(r), 6) + pt.col(idx_q + p_reg_idx2<K>(r))];
            c7.init(v, tab, 2048 + tid);
        }
        float acc13[8];  // kHalf only: layer 13 pairs column e with e + 4096
#pragma unroll
        for (int r = 0; r < 8; ++r) acc13[r] = 0.0f;
        if (kHalf) {
            float c13[8];
#pragma unroll
            for (int r = 0; r < 8; ++r) c13[r] = fg[12 * ts + pt.col(idx_q + p_reg_idx2<K>(r))];
            tab[1024 + tid] = make_float4(c13[0], c13[1], c13[2], c13[3]);
            tab[1536 + tid] = make_float4(c13[4], c13[5], c13[6], c13[7]);
        }
#pragma unroll
        for (int j = 0; j < 5; ++j)  // (see group N: pins the waits for the coefficient loads in front of the loop)
#pragma unroll
            for (int r = 0; r < 8; ++r) asm volatile("" ::"v"(cq[j][r]));
        if (!L::kPark7) {
            float c[8];
            c7.get(c);
#pragma unroll
            for (int r = 0; r < 8; ++r) asm volatile("" ::"v"(c[r]));
        }
        QAcc acc;
        acc.clear();
        // -- the dy ring: what this lane loads, and where this thread reads --
        constexpr int kSlots = L::kSlots, kLead = kSlots - 2;
        constexpr int kLoads = ((int)sizeof(T) / 2) * (kHalf ? 2 : 1);  // load instructions per wave and row
        const uint32_t ring0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
        const int q_load = ((lane >> 3) & 7) | ((wave & 1) << 3) | ((lane & 7) << 4) | ((wave >> 1) << 7);  // chunk of 8 elements
        const int e_load = q_load * 8;
        const uint32_t voff = pt.off(e_load, A.sub_ld_in) * (uint32_t)sizeof(T);
        const uint32_t voff0 = pt.off(e_load & pt.tmask, A.sub_ld_in) * (uint32_t)sizeof(T);
        const bool gap_load = pt.in_tail_gap(e_load);
        const uint32_t wave_base = __builtin_amdgcn_readfirstlane(ring0 + (uint32_t)wave * 1024u);
        const T *dy = (const T *)A.dy + A.row0 * A.ld_in + pt.c0;
        const T *dyo = (const T *)A.dy + A.row0 * A.ld_in + (pt.c0 ^ G::n);  // the other half (kHalf)
        auto ring_load = [&](int j) {
            const int jj = j < mine ? j : mine - 1;  // past the end: the last row again (unused)
            const int row = pt.slot + jj * pt.nslots;
            const uint32_t vo = (gap_load && row == pt.tail_row) ? voff0 : voff;
            const uint32_t m0v = wave_base + (uint32_t)(j % kSlots) * L::kSlotBytes;
#pragma unroll
            for (int h = 0; h < (kHalf ? 2 : 1); ++h) {
                const char *rowp = (const char *)((h ? dyo : dy) + row * A.ld_in);
#pragma unroll
                for (int part16 = 0; part16 < (int)sizeof(T) / 2; ++part16) {
                    // 32-bit rows: the two 16-byte halves of a chunk go to two regions of the slot, 8192 bytes apart
                    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2"
                                 :
                                 : "v"(vo + 16u * part16), "s"(m0v + (uint32_t)h * L::kHalfRowBytes + 8192u * part16), "s"(rowp)
                                 : "memory");
                }
            }
        };
        const int c4 = lane_chunk(lane & 15);
        const uint32_t pos = (uint32_t)((c4 & 7) | (wave << 3) | ((c4 >> 3) << 6));
        const uint32_t rd_off = sizeof(T) == 2 ? pos * 16u + (uint32_t)(((lane >> 4) & 1) | (((lane >> 5) & 1) << 1)) * 4u
                                               : pos * 16u + (uint32_t)((lane >> 5) & 1) * 8192u + (uint32_t)((lane >> 4) & 1) * 8u;
        const char *ring = (const char *)lds;
        // elements 2 q and 2 q + 1 of the thread (layout Q) of row j, half h of the slot
        auto ring_read_pair = [&](int j, int h, int q, float &v0, float &v1) {
            const char *p = ring + (j % kSlots) * L::kSlotBytes + h * L::kHalfRowBytes + rd_off + q * 2048;
            if (sizeof(T) == 4) {
                const float2 f = *(const float2 *)p;
                v0 = f.x;
                v1 = f.y;
            } else {
                const uint32_t wd = *(const uint32_t *)p;
                if (std::is_same<T, __half>::value) {
                    const __half2 hh = *(const __half2 *)&wd;
                    v0 = __low2float(hh);
                    v1 = __high2float(hh);
                } else {
                    v0 = __uint_as_float(wd << 16);
                    v1 = __uint_as_float(wd & 0xFFFF0000u);
                }
            }
        };
        // kVirt: which of the thread's elements lie in rows missing from the short last block
        int gap_mask = 0;
        if (kVirt)
#pragma unroll
            for (int r = 0; r < 8; ++r) gap_mask |= pt.in_tail_gap(idx_q + p_reg_idx2<K>(r)) ? (1 << r) : 0;
        if (mine > 0)
            for (int j = 0; j < kLead; ++j) ring_load(j);
        for (int it = 0; it < iters; ++it) {
            ring_load(it + kLead);
            float vx[8], vg[8];
            const bool work = it >= 1 && it <= mine;
            if (work) lds_read_p2<K>(xa, aq, vx);
            wg_barrier();  // M
            if (work) {
                const int row = pt.slot + (it - 1) * pt.nslots;
                q_forward(vx, c7, cq);
                if (!kHalf) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) ring_read_pair(it - 1, 0, q, vg[2 * q], vg[2 * q + 1]);
                } else {
                    // the forward state arrives as E_12 x_12 with E_12 = the cosine of the element's layer-13
                    // pair; the transposed cascade wants x_12 / E_12:  1 / cos^2 = 1 + tan^2, and the layer's
                    // coefficient is -+ tan (both scales still 1)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float2 c13 = *((const float2 *)&tab[(q < 2 ? 1024 : 1536) + tid] + (q & 1));
                        float g[2], go[2];
                        ring_read_pair(it - 1, 0, q, g[0], g[1]);
                        ring_read_pair(it - 1, 1, q, go[0], go[1]);
#pragma unroll
                        for (int b = 0; b < 2; ++b) {
                            const int r = 2 * q + b;
                            const float c = b ? c13.y : c13.x;
                            vx[r] *= __builtin_fmaf(c, c, 1.0f);
                            // transposed layer 13 on g: own half kept, the other half only feeds the layer's sum
                            const float other12 = __builtin_fmaf(-c, g[b], go[b]);
                            acc13[r] = __builtin_fmaf(other12, vx[r], acc13[r]);
                            vg[r] = __builtin_fmaf(c, go[b], g[b]);
                        }
                        asm volatile("" ::: "memory");  // one pair at a time: keeps few values alive
                    }
                }
                if (kVirt && row == pt.tail_row) {
#pragma unroll
                    for (int r = 0; r < 8; ++r)
                        if (gap_mask & (1 << r)) vg[r] = 0.0f;
                }
                q_phase(vx, vg, c7, cq, acc);
                lds_write_p2<K>(hx, aq, vx);
                lds_write_p2<K>(hg, aq, vg);
            }
            // the row group Q consumes in the next iteration has arrived (younger loads may still be in flight)
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLead * kLoads) : "memory");
            wg_barrier();  // E
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        const auto elem = [&](int r) { return idx_q + p_reg_idx2<K>(r); };
        finalize_reg_layer<2>(F, acc.r2, K, elem);
        finalize_reg_layer<1>(F, acc.r1, K - 1, elem);
        finalize_lane_layer(F, acc.d[3], 10, 2, elem);
        finalize_lane_layer(F, acc.d[2], 9, 1, elem);
        finalize_lane_layer(F, acc.d[1], 8, 0, elem);
        finalize_lane_layer(F, acc.d[0], 7, 3, elem);
        if (kHalf) {
            // sum of layer 13 = (scale after the layer)^2 * deferred sum; the lower half's share goes to the
            // layer's place in the slice, the upper half's, negated, behind the slice's regular part
            float *dst = F.part + (size_t)(pt.half ? 13 : 12) * G::n;
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const int e = idx_q + p_reg_idx2<K>(r);
                const float d = A.fw_inv[11 * ts + pt.col(e)];
                const float v = acc13[r] * (d * d);
                put_partial(dst + e, pt.half ? -v : v, A.first_chunk);
            }
        }
    }
}

// out[q] = sum over slices of partial[s][q] (+ the upper-half share of the last layer where a slice has
// one), in double, slice order; skipped for flagged plans
template <typename Out>
__global__ void bwd_reduce_kernel(const float *__restrict__ partial, Out *__restrict__ out, size_t n_angles,
                                  size_t slice_floats, size_t last_layer_at, int n_parts, PlanRef plan)
{
    if (!plan_fast_both(plan)) return;
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
                                PlanRef plan)
{
    if (!plan_fast_both(plan)) return;
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
// Slices = row slots of the kernel, which runs one workgroup per compute unit (n = 8192: two per slot).
static int bwd_fast_slices(int k) { return k == 13 ? 128 : 256; }
// Kernel rows (of 4096 or 8192 elements) per launch: row counters inside the kernel are 32-bit.
static int64_t bwd_fast_chunk_rows(int) { return (int64_t)1 << 22; }
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

// The workspace holds the partial sums only (25 MB; 29 MB for n = 8192; plus the fold buffer for n < 4096).
size_t bwd_fast_workspace_bytes(const Shape &s)
{
    return align256((size_t)bwd_fast_slices(s.k) * bwd_fast_slice_floats(s.k) * sizeof(float)) + bwd_fast_fold_bytes(s.k);
}

// The kernel needs more dynamic LDS than the default limit: raised once per kernel and device.
template <typename T, bool kDx, bool kHalf, bool kVirt>
static hipError_t fused_kernel_ready()
{
    static hipError_t state[64];
    static bool done[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64)
        return hipFuncSetAttribute((const void *)bwd_fused_kernel<T, kDx, kHalf, kVirt>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)FusedLds<T, kHalf>::kBytes);
    if (!done[dev]) {  // (a race between two first calls only repeats the same setting)
        state[dev] = hipFuncSetAttribute((const void *)bwd_fused_kernel<T, kDx, kHalf, kVirt>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)FusedLds<T, kHalf>::kBytes);
        done[dev] = state[dev] == hipSuccess;
    }
    return state[dev];
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
    const size_t lds_bytes = FusedLds<T, kHalf>::kBytes;
    hipError_t e = A.dx ? fused_kernel_ready<T, true, kHalf, kVirt>() : fused_kernel_ready<T, false, kHalf, kVirt>();
    if (e != hipSuccess) return e;
    const int grid = kHalf ? 2 * slices : slices;  // kHalf: a multiple of 16 (see Part)
    for (int64_t r0 = 0; r0 < kernel_rows; r0 += chunk_rows) {
        A.row0 = r0;
        A.rows = kernel_rows - r0 < chunk_rows ? kernel_rows - r0 : chunk_rows;
        A.first_chunk = (r0 == 0);
        // every slice must be written by the first chunk, so the grid does not shrink with the row count
        if (A.dx)
            hipLaunchKernelGGL((bwd_fused_kernel<T, true, kHalf, kVirt>), dim3(grid), dim3(kFusedThreads), lds_bytes, stream, A);
        else
            hipLaunchKernelGGL((bwd_fused_kernel<T, false, kHalf, kVirt>), dim3(grid), dim3(kFusedThreads), lds_bytes, stream, A);
    }
    if (kVirt) {
        const size_t sums = (size_t)s.k * (G::n / 2);  // the layers the transform has
        hipLaunchKernelGGL(bwd_reduce_kernel<double>, dim3((unsigned)((sums + 255) / 256)), dim3(256), 0, stream,
                           (const float *)ws, fold, sums, (size_t)A.slice_floats, sums, slices, A.plan);
        const unsigned angles = (unsigned)(s.heads * s.k * (s.n / 2));
        hipLaunchKernelGGL(bwd_fold_kernel, dim3((angles + 255) / 256), dim3(256), 0, stream, (const double *)fold, dtheta, s.k,
                           s.heads, A.plan);
    } else {
        const size_t angles = (size_t)s.k * (s.n / 2);
        hipLaunchKernelGGL(bwd_reduce_kernel<float>, dim3((unsigned)((angles + 255) / 256)), dim3(256), 0, stream,
                           (const float *)ws, dtheta, angles, (size_t)A.slice_floats, (size_t)(s.k - 1) * (s.n / 2), slices,
                           A.plan);
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
    A.fg_inv = pv.fg_inv;
    A.fd_inv = pv.fd_inv;
    A.fw_inv = pv.fw_inv;
    A.bad_fwd = &pv.hdr->fast_bad_fwd;
    A.bad_inv = &pv.hdr->fast_bad_inv;
    A.plan = pv.ref;
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
