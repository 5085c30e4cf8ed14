// Inverse transform (layers 12 .. 1, each transposed) of 16-bit rows for n = 256 .. 4096, in two phases instead of
// the three of bq_k12_kernel.h.
//
// The inverse starts with the layers that pair far elements (layout P) and ends with the ones that pair
// neighbours (layout N, which is also the layout of a coalesced store).  The general kernel therefore spends its
// phase A on nothing but a transposition: it converts the row to float32 and writes it to LDS in layout N, only for
// phase B to read it back in layout P.  Here phase B takes its elements straight from the input ring, where the row
// lies as it came from memory (two adjacent 16-bit values per 32-bit read, four reads per thread), which saves
// the conversion, one LDS write and read of the row, one row buffer and one pipeline stage:
//
//   iteration it:  load(row it + 3) | C(row it - 1): read N, layers 7 .. 1, output scale, store |
//                  B(row it): read the ring in layout P, layers 12 .. 8, write LDS | wait for row it + 1 | barrier
//
// A thread of phase B reads what other waves loaded, so every wave waits for its own piece of row it + 1 before the
// barrier that ends iteration it: four ring slots (the row being read, the row waited for, two in flight) and two
// row buffers.
//
// Ring layout.  Wave w loads the 1 KB piece w of a row (elements 512 w .. 512 w + 511) with one direct-to-LDS
// load; lane l deposits its 16 bytes at offset 16 l of the piece, so the order of the 8-element chunks inside the
// piece is free: lane l loads chunk j(l) = ((l & 3) << 4) | (l >> 2), which puts chunk j at position
// pos(j) = (j >> 4) | ((j & 15) << 2), and the pieces are 1088 bytes apart.  A 32-bit read of phase B by the lanes of
// half a wave varies idx bits 1, 2 (the word inside the chunk: address bits 2, 3), idx bits 7, 8 (chunk bits 4, 5:
// position bits 0, 1, address bits 4, 5) and idx bit 9 (the piece: 1088 = 1024 + 64, address bit 6): 32 lanes, 32
// different banks.
#pragma once

#include "bq_k12_kernel.h"

namespace bq {

constexpr int kInvSlots = 4;
constexpr int kInvPiece = 1088;                     // bytes between the pieces of a slot
constexpr int kInvSlotBytes = 8 * kInvPiece;        // 8704
constexpr int kInvRingBytes = kInvSlots * kInvSlotBytes;
constexpr size_t kInvLdsBytes = kInvRingBytes + 2 * kLdsRow * sizeof(float);
static_assert(kInvLdsBytes <= 80 * 1024, "two workgroups per compute unit");

// byte offset inside a ring slot of element idx (even) of the 4096-point block
__device__ __forceinline__ int inv_ring_addr(int idx)
{
    const int j = (idx >> 3) & 63;
    const int pos = (j >> 4) | ((j & 15) << 2);
    return (idx >> 9) * kInvPiece + pos * 16 + (idx & 7) * 2;
}

// Workgroup barrier that waits for the wave's LDS traffic only (the ring loads in flight must stay in flight).
__device__ __forceinline__ void inv_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <typename T>
__device__ __forceinline__ void unpack2(uint32_t w, float &a, float &b);
template <>
__device__ __forceinline__ void unpack2<__half>(uint32_t w, float &a, float &b)
{
    const __half2 h = *(const __half2 *)&w;
    a = __low2float(h);
    b = __high2float(h);
}
template <>
__device__ __forceinline__ void unpack2<bf16_t>(uint32_t w, float &a, float &b)
{
    a = __uint_as_float(w << 16);
    b = __uint_as_float(w & 0xFFFF0000u);
}

// kNt: the batch is larger than the caches; rows are loaded and stored with the non-temporal hint (0.780 -> 0.766 ms
// for 2^30 fp16 elements)
template <typename T, bool kVirt, bool kNt>
__global__ __launch_bounds__(kThreads, 4) void k12_inv_ring_kernel(K12Args A)
{
    static_assert(sizeof(T) == 2, "16-bit rows");
    extern __shared__ __align__(16) float inv_lds[];
    float *bufs = inv_lds + kInvRingBytes / 4;  // two row buffers behind the ring
    unsigned long long *const wg_bins = nullptr;  // (the quantiser's workgroup scratch: not used by a plain transform)
    float *const wg_max = nullptr;
    NoCount bins;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int chunk = wave * 64 + lane_chunk(lane);
    const int idx_n = chunk * 8;
    const int head = blockIdx.x % A.heads;
    const int64_t row_first = blockIdx.x / A.heads;
    const int64_t row_step = gridDim.x / A.heads;
    const int tn = kVirt ? A.n : kN;
    const int nk = kVirt ? A.n_log : kK;
    const int tmask = tn - 1;
    const T *in = (const T *)A.in;
    if (row_first >= A.rows) return;
    if (!plan_matches(A.plan)) return;

    // coefficients: cn[j][r] for layer j+1 (layout N), cp[j][r'] for layer 8+j (layout P), d[r] (layout N)
    const int idx_p = base_p(wave, lane);
    float cn[7][8], cp[5][8], d[8];
    {
        const float *fg = A.fg + (kVirt ? 0 : (size_t)head * kK * kN);
        const float *fg_n = fg + (kVirt ? (size_t)virt_head(A, head, idx_n) * nk * tn : 0);
#pragma unroll
        for (int j = 0; j < 7; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r) cn[j][r] = fg_n[j * tn + (idx_n & tmask) + r];
#pragma unroll
        for (int j = 0; j < 5; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r) {  // layers above log2 n do not exist: weight zero leaves the element as it is
                const int e = idx_p + p_reg_idx(r);
                const float *fg_p = fg + (kVirt ? (size_t)virt_head(A, head, e) * nk * tn : 0);
                cp[j][r] = (!kVirt || 8 + j <= nk) ? fg_p[(7 + j) * tn + (e & tmask)] : 0.0f;
            }
        const float *fd = A.fd + (kVirt ? (size_t)virt_head(A, head, idx_n) * tn : (size_t)head * kN);
#pragma unroll
        for (int r = 0; r < 8; ++r) d[r] = fd[(idx_n & tmask) + r];
        // the empty statements consume the loaded values: their waits then sit here and not inside the row loop
#pragma unroll
        for (int r = 0; r < 8; ++r) {
#pragma unroll
            for (int j = 0; j < 7; ++j) asm volatile("" ::"v"(cn[j][r]));
#pragma unroll
            for (int j = 0; j < 5; ++j) asm volatile("" ::"v"(cp[j][r]));
            asm volatile("" ::"v"(d[r]));
        }
    }
    if (*A.fast_bad != 0) {  // rare: plain rotations through LDS
        const float2 *cs = A.cs + (kVirt ? 0 : (size_t)head * kK * (kN / 2));
        const uint32_t off_n = elem_off<kVirt, false>(A, head, idx_n, A.sub_ld_in);
        for (int64_t row = row_first; row < A.rows; row += row_step) {
            float u[8];
            unpack8(load8(in + row * A.ld_in + off_n), u, (const T *)nullptr);
            slow_cascade<true, false>(u, bufs, cs, idx_n, nk, kVirt ? (1 << A.row_log) - 1 : 0, kVirt ? head * kN : 0);
            finish_row<T, kInv, 4, 0, 0, true, false, kVirt, false, false>(A, u, row, head, chunk, bins, wg_bins, wg_max);
        }
        return;
    }

    const int an = lds_addr(idx_n);
    const int ap = lds_addr(idx_p);
    const int n_my = (int)((A.rows - row_first + row_step - 1) / row_step);

    // ---- input ring ----------------------------------------------------------------------------------------
    const uint32_t ring0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)inv_lds;
    const uint32_t piece_s = __builtin_amdgcn_readfirstlane(ring0 + (uint32_t)wave * (uint32_t)kInvPiece);
    const int jl = ((lane & 3) << 4) | (lane >> 2);  // the chunk this lane loads
    const uint32_t voff = elem_off<kVirt, false>(A, head, wave * 512 + jl * 8, A.sub_ld_in) * (uint32_t)sizeof(T);
    const uint32_t rd_p = ring0 + (uint32_t)inv_ring_addr(idx_p);  // + 2 r1 + 4 r2 pieces for the other register pairs
    auto ring_load = [&](int j, int slot) {
        const int jj = j < n_my ? j : n_my - 1;  // past the end: the last row again (unused)
        const char *rowp = (const char *)(in + (row_first + jj * row_step) * A.ld_in);
        const uint32_t m0v = piece_s + (uint32_t)slot * (uint32_t)kInvSlotBytes;
        if (kNt)
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2 nt" : : "v"(voff), "s"(m0v), "s"(rowp) : "memory");
        else
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2" : : "v"(voff), "s"(m0v), "s"(rowp) : "memory");
    };
    // Memory operations of a wave complete in issue order.  Per iteration a wave issues one ring load (first) and
    // one store (in C).  Row it + 1 was requested at the start of iteration it - 2; younger than that load are the
    // stores of iterations it - 2, it - 1 and it and the loads of rows it + 2 and it + 3: five operations.
    ring_load(0, 0);
    ring_load(1, 1);
    ring_load(2, 2);
    asm volatile("s_waitcnt vmcnt(2)" ::: "memory");  // row 0
    inv_barrier();

    auto step = [&](auto SB, auto BB, int it) {
        constexpr int sb = decltype(SB)::value, bb = decltype(BB)::value;  // ring slot and row buffer of row it
        ring_load(it + 3, (sb + 3) & 3);  // the slot of row it - 1, which every wave has finished reading
        if (it >= 1) {  // C(it - 1)
            float u[8];
            lds_read_n(bufs + (bb ^ 1) * kLdsRow, an, u);
            dpp_layer_xor8(u, cn[6]);
            dpp_layer_xor7(u, cn[5]);
            dpp_layer_xor2(u, cn[4]);
            dpp_layer_xor1(u, cn[3]);
            reg_layer<2>(u, cn[2]);
            reg_layer<1>(u, cn[1]);
            reg_layer<0>(u, cn[0]);
#pragma unroll
            for (int r = 0; r < 8; ++r) u[r] *= d[r];
            finish_row<T, kInv, 4, 0, 0, true, false, kVirt, false, false, kNt>(A, u, row_first + (it - 1) * row_step, head, chunk,
                                                                              bins, wg_bins, wg_max);
        }
        if (it < n_my) {  // B(it)
            uint32_t w0, w1, w2, w3;
            constexpr int so = sb * kInvSlotBytes;
            asm volatile("ds_read_b32 %0, %4 offset:%5\n\tds_read_b32 %1, %4 offset:%6\n\tds_read_b32 %2, %4 offset:%7\n\t"
                         "ds_read_b32 %3, %4 offset:%8\n\ts_waitcnt lgkmcnt(0)"
                         : "=&v"(w0), "=&v"(w1), "=&v"(w2), "=&v"(w3)
                         : "v"(rd_p), "n"(so), "n"(so + 2 * kInvPiece), "n"(so + 4 * kInvPiece), "n"(so + 6 * kInvPiece)
                         : "memory");
            float u[8];  // register r = b0 + 2 r1 + 4 r2
            unpack2<T>(w0, u[0], u[1]);
            unpack2<T>(w1, u[2], u[3]);
            unpack2<T>(w2, u[4], u[5]);
            unpack2<T>(w3, u[6], u[7]);
            reg_layer_first<2>(u, cp[4]);
            reg_layer<1>(u, cp[3]);
            dpp_layer_xor7(u, cp[2]);
            dpp_layer_xor2(u, cp[1]);
            dpp_layer_xor1(u, cp[0]);
            lds_write_p(bufs + bb * kLdsRow, ap, u);
        }
        // this wave's piece of row it + 1 has landed; with the barrier, all of row it + 1 has
        if (it >= 3)
            asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
        else
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        inv_barrier();
    };
    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;
    typedef std::integral_constant<int, 2> I2;
    typedef std::integral_constant<int, 3> I3;
    const int end = n_my + 1;
    for (int it = 0; it < end; it += 4) {
        step(I0{}, I0{}, it);
        if (it + 1 < end) step(I1{}, I1{}, it + 1);
        if (it + 2 < end) step(I2{}, I0{}, it + 2);
        if (it + 3 < end) step(I3{}, I1{}, it + 3);
    }
}

template <bool kVirt>
static hipError_t launch_k12_inv_ring(const K12Args &A, unsigned grid, int dtype, hipStream_t stream)
{
    void (*kern)(K12Args);
    if (A.streaming)
        kern = dtype == BQ_F16 ? k12_inv_ring_kernel<__half, kVirt, true> : k12_inv_ring_kernel<bf16_t, kVirt, true>;
    else
        kern = dtype == BQ_F16 ? k12_inv_ring_kernel<__half, kVirt, false> : k12_inv_ring_kernel<bf16_t, kVirt, false>;
    static LdsLimitOnce once[2][2];
    hipError_t e = once[dtype == BQ_F16 ? 0 : 1][A.streaming ? 1 : 0].set((const void *)kern, kInvLdsBytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), kInvLdsBytes, stream, A);
    return hipGetLastError();
}

}  // namespace bq
