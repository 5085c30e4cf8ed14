// Specialised kernels for n = 4096 (k = 12) and n = 8192 (k = 13): forward, inverse and fused forward +
// quantisation.  Included by one translation unit per width.
//
// One workgroup of 512 threads owns one transform at a time; thread t holds 8 elements.  All
// n*k scale-deferred coefficients (bq_internal.h) of the workgroup's head stay in registers (96 + 8
// per thread) while the workgroup loops over its rows, so a row costs one coalesced 16-byte load per
// thread, 12 FMAs per element, two LDS transposes and one store.
//
//   layout N ("natural"): thread (wave w, lane l) holds idx = 8*chunk + r, chunk = 64 w + e(l),
//                         r = 0..7.  Layers 1-3 pair registers, layers 4-7 pair lanes of a 16-lane
//                         row through DPP (bq_cascade.h).
//   layout P            : thread holds idx = baseP + b0 + 1024 r1 + 2048 r2 (register r' = b0 + 2 r1 +
//                         4 r2): idx bit 0 and idx bits 10, 11 are register bits, idx bits 7, 8, 9 are
//                         the chunk bits of lane bits 0..2 (DPP masks 1, 2, 7), idx bit 2 is lane
//                         bit 3, the remaining idx bits are lane bits 4, 5 and the wave index.
//                         Layers 8, 9, 10 use DPP, layers 11, 12 pair registers.
//   forward : A: load N, layers 1..7, write LDS1 | B: read P, layers 8..12, write LDS2 |
//             C: read N, output scale, quantise or store
//   inverse : A: load N, write LDS1 | B: read P, layers 12..8, write LDS2 | C: read N, layers 7..1,
//             output scale, store
//
// The three phases of consecutive rows are software-pipelined: iteration `it` of a workgroup runs
// C(row it-2), B(row it-1), A(row it) and then ONE barrier; three row buffers rotate through the roles,
// so every read of a buffer is separated from the next write to it by a barrier.  (Some variants use two
// buffers: A then overwrites what C has just read, each thread at the very addresses it read itself.)
//
// LDS accesses are 64-bit (two adjacent floats per lane), which is what reaches the full LDS rate.
// LDS float address of idx is idx + 2 (idx >> 5) + 2 (idx >> 9).  For a group of 16 lanes the N-side
// accesses vary idx bits 3..6 and the P-side accesses idx bits 2, 7, 8, 9; in both cases the four
// bits move the address by 2, 4, 8 and 16 words modulo 32, so the 16 lanes hit 16 different bank
// pairs (the padding terms supply what the plain index lacks).
//
// n = 8192 (kWide): layers 1..12 act inside each half of a row and only layer 13 couples element e with
// e + 4096.  A workgroup of 1024 threads runs the scheme above on both halves side by side (threads 0..511
// on the lower half, 512..1023 on the upper, each with its own row buffers, one barrier for all) and adds
// layer 13 where both halves are in LDS anyway: forward in phase C (a thread reads its own 8 elements and
// the 8 elements of the other half at the same position), inverse at the start of phase B.
//
// If the plan flags the scale-deferred tables as unusable (a cosine too close to zero), the cascade
// of a row runs through LDS with plain (cos, sin) rotations instead; everything else is unchanged.
#pragma once

#include <type_traits>

#include "bq_cascade.h"

namespace bq {

constexpr int kN = 4096, kK = 12, kThreads = 512;
constexpr int kLdsRow = 4368;  // floats: 4095 + 2*127 + 2*7 + 1, rounded up to a multiple of 4
// per half of a row: the input ring (16-bit rows: 3 slots of 8 KB; 32-bit rows: 2 slots of 16 KB) and behind
// it three row buffers (the variants that use two of them fit the same allocation)
constexpr int kFrontFloats = 3 * kN * 2 / 4;  // 6144 floats = 24 KB in front of the row buffers
constexpr size_t kLdsBytes = (kFrontFloats + 3 * kLdsRow) * sizeof(float);
static_assert((2 * kN + 2 * kLdsRow) * sizeof(float) <= kLdsBytes, "32-bit rows: two slots and two buffers must fit");

struct K12Args {
    const void *in;
    void *out;
    const float *fg;   // [heads][k][n] coefficients of the direction
    const float *fd;   // [heads][n] output scales
    const float2 *cs;  // [heads][k][n/2]
    const int *fast_bad;
    PlanRef plan;  // not read by the fixed transform (its coefficients come from the element index)
    int64_t rows, ld_in, ld_out;
    int heads;
    // quantiser
    uint8_t *codes;
    void *scales;
    unsigned long long *hist;  // kFwdFake: 2^bits counters or NULL
    int group, scale_f16;
    // the batch is larger than the memory-side cache (input and output are touched once): the launcher then picks
    // the kNt variants of the plain transforms
    int streaming;
    // transforms of n = 2^n_log < 4096 points (kVirt): a "row" of the kernel is a block of 4096 consecutive
    // elements of the caller's [rows][heads * n] array.  Rows of up to 4096 elements: 2^(12 - row_log) whole rows
    // (row_log = log2 of the row width; ld_in / ld_out are the strides between blocks, sub_ld_* the caller's
    // strides, heads = 1).  Wider rows: block `head` of the heads = width / 4096 blocks of a row (row_log = 12).
    int n, n_log, row_log;
    int64_t sub_ld_in, sub_ld_out;
};

// Element offset, inside a kernel row, of the element with index e (a multiple of 8) of the 4096-point block.
template <bool kVirt, bool kWide = false>
__device__ __forceinline__ uint32_t elem_off(const K12Args &A, int head, int e, int64_t sub_ld)
{
    if (!kVirt) return (uint32_t)(head * (kWide ? 2 * kN : kN) + e);
    return (uint32_t)((e >> A.row_log) * (int)sub_ld + head * kN + (e & ((1 << A.row_log) - 1)));
}
// kVirt: the transform (head of the caller's row) that element e of block `head` belongs to
__device__ __forceinline__ int virt_head(const K12Args &A, int head, int e)
{
    return (head * kN + (e & ((1 << A.row_log) - 1))) >> A.n_log;
}

__device__ __forceinline__ int lds_addr(int idx) { return idx + 2 * (idx >> 5) + 2 * (idx >> 9); }
constexpr int kPStepR1 = 1024 + 2 * 32 + 2 * 2;  // address step of register bit r1 (idx + 1024)
constexpr int kPStepR2 = 2 * kPStepR1;           // register bit r2 (idx + 2048)

// thread's base index in layout P
__device__ __forceinline__ int base_p(int wave, int lane)
{
    const int c3 = lane_chunk(lane & 15) & 7;
    return (c3 << 7) | (((lane >> 3) & 1) << 2) | (((lane >> 4) & 1) << 1) | (((lane >> 5) & 1) << 3) | (wave << 4);
}
__device__ __forceinline__ int p_reg_idx(int r) { return (r & 1) + 1024 * ((r >> 1) & 1) + 2048 * (r >> 2); }

__device__ __forceinline__ void lds_write_n(float *buf, int an, const float (&u)[8])
{
#pragma unroll
    for (int j = 0; j < 4; ++j) *(float2 *)&buf[an + 2 * j] = make_float2(u[2 * j], u[2 * j + 1]);
}
__device__ __forceinline__ void lds_read_n(const float *buf, int an, float (&u)[8])
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float2 v = *(const float2 *)&buf[an + 2 * j];
        u[2 * j] = v.x;
        u[2 * j + 1] = v.y;
    }
}
__device__ __forceinline__ void lds_write_p(float *buf, int ap, const float (&u)[8])
{
#pragma unroll
    for (int j = 0; j < 4; ++j)
        *(float2 *)&buf[ap + (j & 1) * kPStepR1 + (j >> 1) * kPStepR2] = make_float2(u[2 * j], u[2 * j + 1]);
}
__device__ __forceinline__ void lds_read_p(const float *buf, int ap, float (&u)[8])
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float2 v = *(const float2 *)&buf[ap + (j & 1) * kPStepR1 + (j >> 1) * kPStepR2];
        u[2 * j] = v.x;
        u[2 * j + 1] = v.y;
    }
}

// Layer 13 of an 8192-point transform: u[r] += c[r] * (the other half's element at the same position), read
// from the other half's row buffer.
template <bool kLayoutP>
__device__ __forceinline__ void cross_layer(const float *other, int addr, const float (&c)[8], float (&u)[8])
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int a = kLayoutP ? addr + (j & 1) * kPStepR1 + (j >> 1) * kPStepR2 : addr + 2 * j;
        const float2 v = *(const float2 *)&other[a];
        u[2 * j] = __builtin_fmaf(c[2 * j], v.x, u[2 * j]);
        u[2 * j + 1] = __builtin_fmaf(c[2 * j + 1], v.y, u[2 * j + 1]);
    }
}

// slow cascade through LDS with (cos, sin); in: u[] in layout N, out: y[] in layout N (true values)
// n_log < 12: the block holds 4096 >> n_log independent transforms of 2^n_log points (same angles).
// kWide: 1024 threads on one 8192-point transform (idx_n counts inside the whole row).
// row_mask, head0: several transforms with their own angles side by side in the block (see K12Args): element a
// belongs to transform (head0 + (a & row_mask)) >> n_log.
template <bool kInverse, bool kWide = false>
__device__ __forceinline__ void slow_cascade(float (&u)[8], float *buf, const float2 *__restrict__ cs, int idx_n,
                                             int n_log = kWide ? kK + 1 : kK, int row_mask = 0, int head0 = 0)
{
    constexpr int kPoints = kWide ? 2 * kN : kN, kWorkers = kWide ? 2 * kThreads : kThreads;
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 8; ++r) buf[idx_n + r] = u[r];
    __syncthreads();
    const int half_n = 1 << (n_log - 1);
    for (int step = 0; step < n_log; ++step) {
        const int i = kInverse ? (n_log - step) : (step + 1);
        const int h = 1 << (i - 1);
        for (int p = threadIdx.x; p < kPoints / 2; p += kWorkers) {
            const int a = ((p >> (i - 1)) << i) | (p & (h - 1));
            const int hd = (head0 + (a & row_mask)) >> n_log;
            const float2 w = cs[((size_t)hd * n_log + (i - 1)) * half_n + (p & (half_n - 1))];
            const float xa = buf[a], xb = buf[a + h];
            if (!kInverse) {
                buf[a] = __builtin_fmaf(w.x, xa, -(w.y * xb));
                buf[a + h] = __builtin_fmaf(w.y, xa, w.x * xb);
            } else {
                buf[a] = __builtin_fmaf(w.x, xa, w.y * xb);
                buf[a + h] = __builtin_fmaf(w.x, xb, -(w.y * xa));
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) u[r] = buf[idx_n + r];
    __syncthreads();
}

// max |y| over a group of 256 .. 8192 consecutive channels (up to the whole row): 16-lane rows by DPP, the
// wave by two lane shuffles, several waves through `wg_max` (one float per wave) and one workgroup barrier.
// Every thread of the workgroup must call it; successive calls must be separated by a barrier of their own
// (the row loop's is).
__device__ __forceinline__ float big_group_max(const float (&y)[8], int group, int wave_row, float *wg_max)
{
    float m = row16_max(amax8(y));
    m = fmaxf(m, __shfl_xor(m, 16));
    if (group >= 512) m = fmaxf(m, __shfl_xor(m, 32));
    if (group > 512) {
        if ((threadIdx.x & 63) == 0) wg_max[wave_row] = m;
        __syncthreads();
        const int waves = group >> 9, first = wave_row & ~(waves - 1);
        float g = wg_max[first];
        for (int w = 1; w < waves; ++w) g = fmaxf(g, wg_max[first + w]);
        m = g;
    }
    return m;
}

// Epilogue shared by the fast and the slow loop: y[] holds the rotated values in layout N.
// kLanes > 0 fixes the group size (8 * kLanes) and kScale fixes the scale type (0 = float32,
// 1 = binary16) at compile time; kLanes == 0 reads both from the arguments.
// Addresses are a uniform row base plus a 32-bit per-thread offset.
struct NoCount {};
template <int kMode, int kBits>
struct CountOf {
    typedef NoCount type;
};
template <int kBits>
struct CountOf<kFwdFake, kBits> {
    typedef BinCount<kBits> type;
};

// kFwdFake only: kYq = the dequantised row is stored, kHist = the bins are counted.
// chunk: the thread's group of 8 elements, counted inside the whole row.
// kBig: quantiser groups of more than 128 channels (the maximum then comes from big_group_max()).
template <typename T, int kMode, int kBits, int kLanes, int kScale, bool kYq, bool kHist, bool kVirt, bool kWide, bool kBig,
          bool kNt = false>
__device__ __forceinline__ void finish_row(const K12Args &A, const float (&y)[8], int64_t row, int head, int chunk,
                                           typename CountOf<kMode, kBits>::type &bins, unsigned long long *wg_bins,
                                           float *wg_max)
{
    constexpr bool big = kBig;
    if (kMode == kFwdFake) {
        const int lanes = A.group >> 3;  // lanes per group
        float f[8], s;
        bool ordinary;
        if (big)
            rounded8<kBits, true>(y, lanes, A.scale_f16 != 0, f, &s, &ordinary, big_group_max(y, A.group, chunk >> 6, wg_max));
        else
            rounded8<kBits>(y, lanes, A.scale_f16 != 0, f, &s, &ordinary);
        if (kHist) {
            auto &bc = (BinCount<kBits> &)bins;
            count8<kBits>(bc, f, ordinary);
            if (bc.full()) bc.drain(wg_bins);
        }
        if (kYq) {
            float yq[8];
            dequant8(f, s, yq);
            T *out_row = (T *)A.out + row * A.ld_out;
            uint32_t off = elem_off<kVirt, kWide>(A, head, chunk * 8, A.sub_ld_out) * (uint32_t)sizeof(T);
            asm volatile("" : "+v"(off));
            store8((T *)((char *)out_row + off), yq);
        }
    } else if (kMode != kFwdQuant) {
        T *out_row = (T *)A.out + row * A.ld_out;
        uint32_t off = elem_off<kVirt, kWide>(A, head, chunk * 8, A.sub_ld_out) * (uint32_t)sizeof(T);
        asm volatile("" : "+v"(off));
        if (kNt)
            store8_nt((T *)((char *)out_row + off), y);
        else
            store8((T *)((char *)out_row + off), y);
    } else {
        const int lanes = kLanes > 0 ? kLanes : (A.group >> 3);  // lanes per group
        const bool f16 = kLanes > 0 ? (kScale != 0) : (A.scale_f16 != 0);
        float s;
        uint32_t packed;
        if (big)
            packed = quant8<kBits, true>(y, lanes, f16, &s, big_group_max(y, A.group, chunk >> 6, wg_max));
        else
            packed = quant8<kBits>(y, lanes, f16, &s);
        const int64_t unit = row * A.heads + head;
        uint8_t *codes_row = A.codes + unit * ((kWide ? 2 * kN : kN) * kBits / 8);
        uint32_t coff = (uint32_t)(chunk * kBits);
        asm volatile("" : "+v"(coff));
        if (kBits == 2)
            *(uint16_t *)(codes_row + coff) = (uint16_t)packed;
        else
            *(uint32_t *)(codes_row + coff) = packed;
        // every lane of a group stores the group's scale (same value, same address): no divergence
        const int groups = ((kWide ? 2 * kN : kN) / 8) / lanes;
        uint32_t goff = ((uint32_t)chunk / (uint32_t)lanes) * (f16 ? 2u : 4u);
        asm volatile("" : "+v"(goff));
        if (f16)
            *(__half *)((char *)((__half *)A.scales + unit * groups) + goff) = __float2half_rn(s);
        else
            *(float *)((char *)((float *)A.scales + unit * groups) + goff) = s;
    }
}

template <typename T, int kMode, int kBits, int kLanes, int kScale, bool kYq = true, bool kHist = false, bool kVirt = false,
          bool kWide = false, bool kBig = false, bool kNt = false>
__global__ __launch_bounds__(kWide ? 2 * kThreads : kThreads, 4) void k12_kernel(K12Args A)
{
    static_assert(!(kWide && kVirt), "blocks of small transforms are a 4096-point scheme");
    // kNt: rows are loaded and stored with the non-temporal hint.  262144 fp16 rows of n = 4096: forward 0.796 ->
    // 0.778 ms on every box tried.  Not used where it did not hold up: the inverse gained 3.5 % on some boxes and
    // lost as much on others, float32 rows lost 15 - 19 % (0.78 -> 0.93 ms), the fused quantiser stores too little.
    static_assert(!kNt || ((kMode == kFwd || kMode == kHadamard) && sizeof(T) == 2), "16-bit forward transforms only");
    // (the two-phase inverse of 16-bit rows, bq_k12_inv.h, has a variant of its own that does gain)
    static_assert(!kBig || ((kMode == kFwdQuant || kMode == kFwdFake) && kLanes == 0), "large groups: general quantiser variants");
    constexpr int kHalves = kWide ? 2 : 1;
    constexpr int kPoints = kHalves * kN;  // n
    constexpr int kLayers = kWide ? kK + 1 : kK;
    __shared__ unsigned long long wg_bins[16];  // kFwdFake: this workgroup's bin counts
    __shared__ float wg_max[16];                // quantiser groups that span several waves: one maximum per wave
    typename CountOf<kMode, kBits>::type bins;
    if (kMode == kFwdFake && kHist) {
        ((BinCount<kBits> &)bins).clear();
        if (threadIdx.x < 16) wg_bins[threadIdx.x] = 0;
        __syncthreads();
    }
    // kFwdFake: per-thread counts -> workgroup counts -> the caller's counters (every thread gets here)
    auto flush_bins = [&]() {
        if (kMode == kFwdFake && kHist) {
            ((BinCount<kBits> &)bins).drain(wg_bins);
            __syncthreads();
            if (threadIdx.x < (1 << kBits) && wg_bins[threadIdx.x]) atomicAdd(&A.hist[threadIdx.x], wg_bins[threadIdx.x]);
        }
    };
    // LDS: [input ring 3 x 8 KB | output-scale table] first (low addresses), then the row buffers L[0..2]
    extern __shared__ float lds_raw[];
    // (32-bit rows: two ring slots of 16 KB per half in front, two row buffers behind them)
    constexpr bool kRing32 = sizeof(T) == 4;
    float *lds = lds_raw + kHalves * (kRing32 ? 2 * kN : kFrontFloats);
    constexpr bool kInverse = (kMode == kInv);
    // kHadamard: the same cascade with every coefficient +1 (lower element of a pair) or -1 (upper element), i.e.
    // additions and subtractions; nothing is read from a plan.  A layer then maps (a, b) to (a + b, b - a), which
    // is the Sylvester butterfly (a + b, a - b) up to the sign of its second output; over all layers the signs
    // collect to (-1)^popcount(index) per output element, which the single scale 1 / sqrt(n) takes along.
    constexpr bool kHad = (kMode == kHadamard);
    // kWide: `half` selects the half of the row; tid, wave, chunk and idx_n count inside the half
    const int half = kWide ? (int)(threadIdx.x >> 9) : 0;
    const int tid = threadIdx.x & (kThreads - 1), wave = tid >> 6, lane = tid & 63;
    const int chunk = wave * 64 + lane_chunk(lane);
    const int idx_n = chunk * 8;
    const int col0 = half * kN;                 // first column of the half
    const int chunk_row = half * (kN / 8) + chunk;  // the thread's chunk counted inside the whole row
    const int head = blockIdx.x % A.heads;
    const int64_t row_first = blockIdx.x / A.heads;
    const int64_t row_step = gridDim.x / A.heads;
    const uint32_t off_n = elem_off<kVirt, kWide>(A, head, col0 + idx_n, A.sub_ld_in);  // element offset of the thread inside a row
    // tables: rows of n entries, indexed inside the transform the element belongs to
    const int tn = kVirt ? A.n : kPoints;
    const int nk = kVirt ? A.n_log : kLayers;
    const int tmask = tn - 1;
    const T *in = (const T *)A.in;
    if (row_first >= A.rows) return;
    if (!kHad && !plan_matches(A.plan)) return;

    // coefficients: cn[j][r] for layer j+1 (layout N), cp[j][r'] for layer 8+j (layout P), d[r] (layout N)
    const int idx_p = base_p(wave, lane);
    float cn[7][8], cp[5][8];
    float cw[8];  // kWide: layer 13, in layout N (forward, phase C) or layout P (inverse, phase B)
    auto load_coefficients = [&]() {
        if (kHad) {
#pragma unroll
            for (int r = 0; r < 8; ++r) {
#pragma unroll
                for (int j = 0; j < 7; ++j) cn[j][r] = (((idx_n + r) >> j) & 1) ? -1.0f : 1.0f;
#pragma unroll
                for (int j = 0; j < 5; ++j) cp[j][r] = (((idx_p + p_reg_idx(r)) >> (7 + j)) & 1) ? -1.0f : 1.0f;
                cw[r] = half ? -1.0f : 1.0f;
            }
            return;
        }
        // tables are [head][layer][n]; kVirt: the head is the element's own (virt_head)
        const float *fg = A.fg + (kVirt ? 0 : (size_t)head * kLayers * kPoints);
        const float *fg_n = fg + (kVirt ? (size_t)virt_head(A, head, idx_n) * nk * tn : 0);
#pragma unroll
        for (int j = 0; j < 7; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r) cn[j][r] = fg_n[j * tn + ((col0 + idx_n) & tmask) + r];
#pragma unroll
        for (int j = 0; j < 5; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r) {  // layers above log2 n do not exist: weight zero leaves the element as it is
                const int e = col0 + idx_p + p_reg_idx(r);
                const float *fg_p = fg + (kVirt ? (size_t)virt_head(A, head, e) * nk * tn : 0);
                cp[j][r] = (!kVirt || 8 + j <= nk) ? fg_p[(7 + j) * tn + (e & tmask)] : 0.0f;
            }
#pragma unroll
        for (int r = 0; r < 8; ++r)
            cw[r] = !kWide ? 0.0f : kInverse ? fg[kK * tn + col0 + idx_p + p_reg_idx(r)] : fg[kK * tn + col0 + idx_n + r];
    };
    // Transforms and the fused quantiser are also called with a handful of rows (decoding), where the call's
    // latency is a chain of memory round trips: there the coefficient loads are issued in front of the branch
    // on the plan's flag (the empty statements consume their results, which pins them there), so that the two
    // round trips overlap.
    constexpr bool kEarlyLoads = (kMode != kFwdFake) && !kWide;  // (not where registers are short anyway)
    if (kEarlyLoads) {
        load_coefficients();
#pragma unroll
        for (int r = 0; r < 8; ++r) {
#pragma unroll
            for (int j = 0; j < 7; ++j) asm volatile("" ::"v"(cn[j][r]));
#pragma unroll
            for (int j = 0; j < 5; ++j) asm volatile("" ::"v"(cp[j][r]));
            if (kWide) asm volatile("" ::"v"(cw[r]));
        }
    }
    if (!kHad && *A.fast_bad != 0) {  // rare: plain rotations through LDS
        const float2 *cs = A.cs + (kVirt ? 0 : (size_t)head * kLayers * (kPoints / 2));
        for (int64_t row = row_first; row < A.rows; row += row_step) {
            float u[8];
            unpack8(load8(in + row * A.ld_in + off_n), u, (const T *)nullptr);
            slow_cascade<kInverse, kWide>(u, lds, cs, col0 + idx_n, nk, kVirt ? (1 << A.row_log) - 1 : 0, kVirt ? head * kN : 0);
            finish_row<T, kMode, kBits, kLanes, kScale, kYq, kHist, kVirt, kWide, kBig, kNt>(A, u, row, head, chunk_row, bins, wg_bins, wg_max);
        }
        flush_bins();
        return;
    }
    if (!kEarlyLoads) load_coefficients();

    const int an = lds_addr(idx_n);
    const int ap = lds_addr(idx_p);
    // rows of this workgroup: below 2^28 for every batch the library accepts, so the loop counters are 32-bit
    // (64-bit comparisons of uniform values would be done on the vector unit)
    const int n_my = (int)((A.rows - row_first + row_step - 1) / row_step);

    // Phase B of one row: layers 8..12 (or 12..8) on layout P, in place in its LDS buffer.
    // kWide: lb is the buffer of the thread's own half, lo the other half's; the inverse starts with layer 13.
    auto phase_b = [&](float *lb, const float *lo) {
        float u[8];
        lds_read_p(lb, ap, u);
        if (kWide && kInverse) {
            cross_layer<true>(lo, ap, cw, u);
            // both halves must have read the other's values before either overwrites its own
            __syncthreads();
        }
        if (!kInverse) {
            dpp_layer_xor1(u, cp[0]);
            dpp_layer_xor2(u, cp[1]);
            dpp_layer_xor7(u, cp[2]);
            reg_layer<1>(u, cp[3]);
            reg_layer<2>(u, cp[4]);
        } else {
            if (kWide)
                reg_layer<2>(u, cp[4]);
            else
                reg_layer_first<2>(u, cp[4]);
            reg_layer<1>(u, cp[3]);
            dpp_layer_xor7(u, cp[2]);
            dpp_layer_xor2(u, cp[1]);
            dpp_layer_xor1(u, cp[0]);
        }
        lds_write_p(lb, ap, u);
    };
    // Layers of phase A after the first one / layers of phase C before the output scale.
    auto layers_a = [&](float (&u)[8]) {
        if (!kInverse) {
            reg_layer<1>(u, cn[1]);
            reg_layer<2>(u, cn[2]);
            dpp_layer_xor1(u, cn[3]);
            dpp_layer_xor2(u, cn[4]);
            dpp_layer_xor7(u, cn[5]);
            dpp_layer_xor8(u, cn[6]);
        }
    };
    auto layers_c = [&](float (&u)[8]) {
        if (kInverse) {
            dpp_layer_xor8(u, cn[6]);
            dpp_layer_xor7(u, cn[5]);
            dpp_layer_xor2(u, cn[4]);
            dpp_layer_xor1(u, cn[3]);
            reg_layer<2>(u, cn[2]);
            reg_layer<1>(u, cn[1]);
            reg_layer<0>(u, cn[0]);
        }
    };
    // ---- input staged through an LDS ring filled by direct global->LDS loads -------------------
    // Two rows per workgroup have to be in flight from HBM to cover its latency, and there are
    // no registers left to hold them.  global_load_lds_dwordx4 moves 16 bytes per lane straight
    // into LDS (16-bit rows: wave w, lane l -> bytes [1024 w + 16 l, +16) of the ring slot, row order), the
    // thread later reads its own chunk back with ds_read_b128.  A wave only reads what it loaded
    // itself, so s_waitcnt vmcnt is the only synchronisation.  These loads and waits are inline
    // assembly: the compiler would otherwise wait for ALL outstanding loads before any LDS read.
    // Memory operations of a wave complete in issue order, and per iteration a wave issues one
    // ring load (in A) and at least kStores stores (in C); row `it` was requested two iterations
    // earlier, followed by stores, the load of row it+1 and stores again, so at most
    // 2 kStores + 1 younger operations may still be pending when row `it` is consumed.  The
    // first four iterations (pipeline fill, fewer stores issued) wait for everything.
    // 32-bit rows: two such loads per lane and row (kLoads), two stores per lane for a row of output.
    constexpr int kLoads = (int)sizeof(T) / 2;
    constexpr int kStores = (kMode == kFwdQuant) ? 2 : (kMode == kFwdFake && !kYq) ? 0 : kLoads;
    constexpr int kPending = 2 * kStores + kLoads;  // operations younger than the last load of the awaited row
    constexpr uint32_t kSlotBytes = kPoints * sizeof(T);
    // kTwoBuf: two row buffers and two ring slots instead of three.  Phase A of row `it` writes the buffer that
    // phase C of row it-2 has just read (there each thread reads and writes the same addresses, and C comes
    // first), and the load of row it+2 refills the slot that A has just read.  Where the rows are 16-bit the
    // third buffer then holds the output scales, which leave the registers.  Used
    //  - for 32-bit rows (slots twice as large: three of them plus three buffers would not leave room for two
    //    workgroups per compute unit; before, such rows were prefetched in registers, at the price of a dozen
    //    spilled ones: 131072 rows of n = 4096 went from 1.20 / 0.92 / 0.84 ms to 0.81 / 0.80 / 0.53 ms);
    //  - for n = 8192, whose kernels are short of registers (65536 fp16 rows: 0.67 / 0.78 / 0.62 ms ->
    //    0.63 / 0.60 / 0.47 ms forward / inverse / fused quantiser, despite the barrier it adds, see below);
    //  - for two fake-quantising variants of n <= 4096, where it measured faster: the one that stores the row
    //    and counts INT4 codes as well (1.14 -> 1.00 ms for 262144 fp16 rows) and the INT2 one that only counts
    //    (0.82 -> 0.77 ms).  On the other 16-bit variants of n <= 4096 it measured equal or slower.
    constexpr bool kTwoBuf = kRing32 || kWide || (kMode == kFwdFake && kHist && ((kYq && kBits == 4) || (!kYq && kBits == 2)));
    constexpr bool kScaleLds = kTwoBuf && !kRing32;
    float d[8];
    float *dtab = lds + (2 * kHalves + half) * kLdsRow;  // kScaleLds: the third buffer
    {
        if (kHad) {
            const float scale = kWide ? 0.011048543456039806f : 0.015625f;  // 1 / sqrt(8192), 1 / sqrt(4096)
#pragma unroll
            for (int r = 0; r < 8; ++r) d[r] = (__builtin_popcount(col0 + idx_n + r) & 1) ? -scale : scale;
        } else {
            const float *fd = A.fd + (kVirt ? (size_t)virt_head(A, head, idx_n) * tn : (size_t)head * kPoints);
#pragma unroll
            for (int r = 0; r < 8; ++r) d[r] = fd[((col0 + idx_n) & tmask) + r];
        }
        if (kScaleLds) lds_write_n(dtab, an, d);  // read back by the same thread only
    }
    const int wave_row = half * 8 + wave;  // the wave's piece of a row: 512 elements, 1 KB per load
    constexpr int kPer = 16 / (int)sizeof(T);  // elements per lane and load
    const uint32_t ring0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds_raw;
    const uint32_t slice = ring0 + (uint32_t)wave_row * (1024u * kLoads);             // this wave's piece of a slot
    const uint32_t rd_addr = slice + (uint32_t)lane_chunk(lane) * (16u * kLoads);      // this thread's chunk
    // lane's bytes in a row, first and (32-bit rows) second load
    const uint32_t voff = elem_off<kVirt, kWide>(A, head, wave_row * 512 + lane * kPer, A.sub_ld_in) * (uint32_t)sizeof(T);
    const uint32_t voff1 = kLoads == 2 ? elem_off<kVirt, kWide>(A, head, wave_row * 512 + (64 + lane) * kPer, A.sub_ld_in) * (uint32_t)sizeof(T) : 0u;
    const uint32_t slice_s = __builtin_amdgcn_readfirstlane(slice);  // uniform over the wave
    auto ring_load = [&](int j, int slot) {
        const int jj = j < n_my ? j : n_my - 1;  // past the end: re-read the last row (unused)
        const char *rowp = (const char *)(in + (row_first + jj * row_step) * A.ld_in);
        const uint32_t m0v = slice_s + (uint32_t)slot * kSlotBytes;
        if (kNt) {
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2 nt"
                         :
                         : "v"(voff), "s"(m0v), "s"(rowp)
                         : "memory");
            if (kLoads == 2)
                asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2 nt"
                             :
                             : "v"(voff1), "s"(m0v + 1024u), "s"(rowp)
                             : "memory");
        } else {
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2"
                         :
                         : "v"(voff), "s"(m0v), "s"(rowp)
                         : "memory");
            if (kLoads == 2)
                asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2"
                             :
                             : "v"(voff1), "s"(m0v + 1024u), "s"(rowp)
                             : "memory");
        }
    };
    ring_load(0, 0);
    ring_load(1, 1);
    // One pipeline step with the roles of the three buffers fixed at compile time (BA: phase A of row it,
    // BB: phase B of row it-1, BC: phase C of row it-2), so that buffer offsets become immediates of the
    // LDS instructions instead of per-lane address arithmetic.  Three such steps make one turn.
    // n = 8192: whether phase B runs before phase C (see below)
    constexpr bool kBFirst = kWide && (sizeof(T) == 2 ? (kMode == kFwd || kMode == kInv || kHad) : kMode == kFwdFake);
    auto step = [&](auto BA, auto BB, auto BC, int it) {
        constexpr int ba = decltype(BA)::value, bb = decltype(BB)::value, bc = decltype(BC)::value;
        float *la = lds + (ba * kHalves + half) * kLdsRow, *lb = lds + (bb * kHalves + half) * kLdsRow;
        float *lc = lds + (bc * kHalves + half) * kLdsRow;
        const float *lb_other = lds + (bb * kHalves + (half ^ 1)) * kLdsRow;  // kWide only
        const float *lc_other = lds + (bc * kHalves + (half ^ 1)) * kLdsRow;
        auto phase_a = [&]() {  // A(it)
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            u32x4 v, v1;
            constexpr int ro = ba * (int)kSlotBytes;
            if (kLoads == 1) {
                if (it >= 4)
                    asm volatile("s_waitcnt vmcnt(%3)\n\tds_read_b128 %0, %1 offset:%2\n\ts_waitcnt lgkmcnt(0)"
                                 : "=v"(v) : "v"(rd_addr), "n"(ro), "n"(kPending) : "memory");
                else
                    asm volatile("s_waitcnt vmcnt(0)\n\tds_read_b128 %0, %1 offset:%2\n\ts_waitcnt lgkmcnt(0)"
                                 : "=v"(v) : "v"(rd_addr), "n"(ro) : "memory");
            } else {
                if (it >= 4)
                    asm volatile("s_waitcnt vmcnt(%5)\n\tds_read_b128 %0, %2 offset:%3\n\tds_read_b128 %1, %2 offset:%4\n\ts_waitcnt lgkmcnt(0)"
                                 : "=&v"(v), "=&v"(v1) : "v"(rd_addr), "n"(ro), "n"(ro + 16), "n"(kPending) : "memory");
                else
                    asm volatile("s_waitcnt vmcnt(0)\n\tds_read_b128 %0, %2 offset:%3\n\tds_read_b128 %1, %2 offset:%4\n\ts_waitcnt lgkmcnt(0)"
                                 : "=&v"(v), "=&v"(v1) : "v"(rd_addr), "n"(ro), "n"(ro + 16) : "memory");
            }
            // refills the slot of row it-1, consumed in the previous iteration (kTwoBuf: the slot just read)
            ring_load(it + 2, kTwoBuf ? ba : bb);
            Raw8 raw;
            raw.lo = make_uint4(v.x, v.y, v.z, v.w);
            if (kLoads == 2) raw.hi = make_uint4(v1.x, v1.y, v1.z, v1.w);
            float u[8];
            unpack8(raw, u, (const T *)nullptr);
            if (!kInverse) reg_layer_first<0>(u, cn[0]);
            layers_a(u);
            lds_write_n(la, an, u);
        };
        auto phase_c = [&]() {  // C(it-2)
            float u[8];
            lds_read_n(lc, an, u);
            if (kWide && !kInverse) cross_layer<false>(lc_other, an, cw, u);  // layer 13
            layers_c(u);
            if (kScaleLds) {
                float dl[8];
                lds_read_n(dtab, an, dl);
#pragma unroll
                for (int r = 0; r < 8; ++r) u[r] *= dl[r];
            } else {
#pragma unroll
                for (int r = 0; r < 8; ++r) u[r] *= d[r];
            }
            finish_row<T, kMode, kBits, kLanes, kScale, kYq, kHist, kVirt, kWide, kBig, kNt>(A, u, row_first + (it - 2) * row_step, head, chunk_row, bins, wg_bins, wg_max);
        };
        // The phases touch different buffers, so any order is correct as long as C precedes A where the two
        // share a buffer.  n = 4096: C, B, A measured 1-2 % faster than the other orders on all modes.
        // n = 8192 (always two buffers): layer 13 makes phase C of the forward modes read the other half's
        // buffer, which that half's phase A is about to overwrite, hence the extra barrier.  These kernels also
        // spill a few coefficients, and the compiler waits for their reloads with vmcnt(0), which waits for every
        // load and store the wave issued before; which order keeps those waits away from fresh loads depends on
        // where the reloads fall, and was measured per mode (65536 rows: fp16 forward 0.66 -> 0.63 ms and
        // inverse 0.69 -> 0.60 ms with B first, fused quantiser 0.52 -> 0.47 ms with C first).
        if (!kBFirst) {
            if (it >= 2) phase_c();
            if (it >= 1 && it <= n_my) phase_b(lb, lb_other);  // B(it-1)
        } else {
            if (it >= 1 && it <= n_my) phase_b(lb, lb_other);
            if (it >= 2) phase_c();
        }
        if (kWide && !kInverse) __syncthreads();  // the other half's reads in phase C are complete
        if (it < n_my) phase_a();
        __syncthreads();
    };
    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;
    typedef std::integral_constant<int, 2> I2;
    const int end = n_my + 2;
    if (kTwoBuf) {
        for (int it = 0; it < end; it += 2) {  // (A, B, C) buffers: (0, 1, 0) -> (1, 0, 1) -> ...
            step(I0{}, I1{}, I0{}, it);
            if (it + 1 < end) step(I1{}, I0{}, I1{}, it + 1);
        }
    } else {
        for (int it = 0; it < end; it += 3) {  // (A, B, C) buffers: (0, 2, 1) -> (1, 0, 2) -> (2, 1, 0) -> ...
            step(I0{}, I2{}, I1{}, it);
            if (it + 1 < end) step(I1{}, I0{}, I2{}, it + 1);
            if (it + 2 < end) step(I2{}, I1{}, I0{}, it + 2);
        }
    }
    flush_bins();
}

template <typename T, bool kVirt, bool kWide, bool kBig>
static hipError_t launch_k12_t(Mode mode, const K12Args &A, int bits, unsigned grid, hipStream_t stream)
{
    constexpr bool V = kVirt, W = kWide, G = kBig;
    void (*kern)(K12Args) = nullptr;
    if (mode == kFwdFake) {
        if (A.out && A.hist)
            kern = bits == 2 ? k12_kernel<T, kFwdFake, 2, 0, 0, true, true, V, W, G> : k12_kernel<T, kFwdFake, 4, 0, 0, true, true, V, W, G>;
        else if (A.out)
            kern = bits == 2 ? k12_kernel<T, kFwdFake, 2, 0, 0, true, false, V, W, G> : k12_kernel<T, kFwdFake, 4, 0, 0, true, false, V, W, G>;
        else
            kern = bits == 2 ? k12_kernel<T, kFwdFake, 2, 0, 0, false, true, V, W, G> : k12_kernel<T, kFwdFake, 4, 0, 0, false, true, V, W, G>;
    } else if (mode == kFwdQuant && (kBig || kVirt || A.group != 128 || !A.scale_f16)) {
        kern = bits == 2 ? k12_kernel<T, kFwdQuant, 2, 0, 0, true, false, V, W, G> : k12_kernel<T, kFwdQuant, 4, 0, 0, true, false, V, W, G>;
    } else if constexpr (!kBig) {
        if constexpr (!kVirt) {
            if (mode == kHadamard)
                kern = k12_kernel<T, kHadamard, 4, 0, 0, true, false, false, W>;
        }
        if (kern) {
        } else if (mode == kFwd)
            kern = k12_kernel<T, kFwd, 4, 0, 0, true, false, V, W>;
        else if (mode == kInv)
            kern = k12_kernel<T, kInv, 4, 0, 0, true, false, V, W>;
        else  // the common activation format: group 128, binary16 scales
            kern = bits == 2 ? k12_kernel<T, kFwdQuant, 2, 16, 1, true, false, false, W> : k12_kernel<T, kFwdQuant, 4, 16, 1, true, false, false, W>;
    }
    if constexpr (!kBig && sizeof(T) == 2) {  // large batches of 16-bit rows: the non-temporal variants
        if (A.streaming && mode == kFwd) kern = k12_kernel<T, kFwd, 4, 0, 0, true, false, V, W, false, true>;
        if constexpr (!kVirt) {
            if (A.streaming && mode == kHadamard) kern = k12_kernel<T, kHadamard, 4, 0, 0, true, false, false, W, false, true>;
        }
    }
    if (!kern) return hipErrorInvalidValue;
    constexpr size_t lds_bytes = (kWide ? 2 : 1) * kLdsBytes;
    // one record per kernel of this instantiation of the launcher (the modes, bit widths and output choices)
    static LdsLimitOnce once[5][2][3][2];
    const int variant = mode != kFwdFake ? 0 : (A.out && A.hist) ? 0 : A.out ? 1 : 2;
    const int general = (mode == kFwdQuant && (kBig || kVirt || A.group != 128 || !A.scale_f16)) ? 1 : 0;
    hipError_t e = once[mode][bits == 2 ? 0 : 1][mode == kFwdQuant ? general : variant][(A.streaming && sizeof(T) == 2 && (mode == kFwd || mode == kHadamard)) ? 1 : 0].set((const void *)kern, lds_bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kWide ? 2 * kThreads : kThreads), lds_bytes, stream, A);
    return hipGetLastError();
}

template <bool kVirt, bool kWide, bool kBig = false>
static hipError_t launch_k12_dtype(Mode mode, const K12Args &A, int bits, unsigned grid, int dtype, hipStream_t stream)
{
    switch (dtype) {
        case BQ_F32: return launch_k12_t<float, kVirt, kWide, kBig>(mode, A, bits, grid, stream);
        case BQ_F16: return launch_k12_t<__half, kVirt, kWide, kBig>(mode, A, bits, grid, stream);
        default: return launch_k12_t<bf16_t, kVirt, kWide, kBig>(mode, A, bits, grid, stream);
    }
}

// the n = 8192 instantiations live in a translation unit of their own
hipError_t launch_k13_dtype(Mode mode, const K12Args &A, int bits, unsigned grid, int dtype, hipStream_t stream);
// ... and so do those for quantiser groups of more than 128 channels (virt: n < 4096, wide: n = 8192)
hipError_t launch_k12_big_dtype(Mode mode, const K12Args &A, int bits, unsigned grid, int dtype, bool virt, bool wide,
                                hipStream_t stream);

}  // namespace bq
