// Specialised kernels for n = 4096 (k = 12): forward, inverse and fused forward + quantisation.
//
// One workgroup of 512 threads owns one transform at a time; thread t holds 8 elements.  All
// n*k scale-deferred coefficients (bq_internal.h) of the workgroup's head stay in registers (96 + 8
// per thread) while the workgroup loops over its rows, so a row costs one coalesced 16-byte load per
// thread, 12 FMAs per element, two LDS transposes and one store.
//
//   layout N ("natural"): thread (wave w, lane l) holds idx = 8*chunk + r, chunk = 64 w + e(l),
//                         r = 0..7.  Layers 1-3 pair registers, layers 4-7 pair lanes of a 16-lane
//                         row through DPP (bq_cascade.h).
//   layout P            : thread holds idx = baseP + 512 r'; idx bits 9,10,11 are the register index,
//                         idx bits 7,8 are lane bits 0,1 (DPP quad_perm), the other seven idx bits are
//                         spread over lane bits 2..5 and the wave index.  Layers 8,9 use DPP,
//                         layers 10-12 pair registers.
//   forward : load N, layers 1..7, LDS N->P, layers 8..12, LDS P->N, scale, quantise/store
//   inverse : load N, LDS N->P, layers 12..8, LDS P->N, layers 7..1, scale, store
//
// LDS float address of idx is idx + (idx >> 5) (one pad word per 32): with 32 banks both the N-side
// accesses (lane stride 8 words) and the P-side accesses (lanes spread over idx bits 0,1,4 and 7,8)
// of a half-wave hit 32 different banks.
//
// If the plan flags the scale-deferred tables as unusable (a cosine too close to zero), the cascade
// of a row runs through LDS with plain (cos, sin) rotations instead; everything else is unchanged.
#include "bq_cascade.h"

namespace bq {

constexpr int kN = 4096, kK = 12, kThreads = 512;
constexpr int kLdsRow = kN + kN / 32;  // padded row

struct K12Args {
    const void *in;
    void *out;
    const float *fg;   // [heads][k][n] coefficients of the direction
    const float *fd;   // [heads][n] output scales
    const float2 *cs;  // [heads][k][n/2]
    const int *fast_bad;
    int64_t rows, ld_in, ld_out;
    int heads;
    // quantiser
    uint8_t *codes;
    void *scales;
    int group, scale_f16;
};

__device__ __forceinline__ int lds_addr(int idx) { return idx + (idx >> 5); }

// thread's base index in layout P (register r' adds 512 r')
__device__ __forceinline__ int base_p(int wave, int lane)
{
    return ((lane & 1) << 7) | (((lane >> 1) & 1) << 8) | (((lane >> 2) & 1) << 0) | (((lane >> 3) & 1) << 1) |
           (((lane >> 4) & 1) << 4) | (((lane >> 5) & 1) << 2) | ((wave & 1) << 3) | (((wave >> 1) & 1) << 5) |
           (((wave >> 2) & 1) << 6);
}

// slow cascade through LDS with (cos, sin); in: u[] in layout N, out: y[] in layout N (true values)
template <bool kInverse>
__device__ __forceinline__ void slow_cascade(float (&u)[8], float *buf, const float2 *__restrict__ cs, int idx_n)
{
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 8; ++r) buf[idx_n + r] = u[r];
    __syncthreads();
    for (int step = 0; step < kK; ++step) {
        const int i = kInverse ? (kK - step) : (step + 1);
        const int h = 1 << (i - 1);
        for (int p = threadIdx.x; p < kN / 2; p += kThreads) {
            const float2 w = cs[(size_t)(i - 1) * (kN / 2) + p];
            const int a = ((p >> (i - 1)) << i) | (p & (h - 1));
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

// Epilogue shared by the fast and the slow loop: y[] holds the rotated values in layout N.
template <typename T, int kMode, int kBits>
__device__ __forceinline__ void finish_row(const K12Args &A, const float (&y)[8], T *out, int64_t row, int head,
                                           int chunk)
{
    if (kMode != kFwdQuant) {
        store8(out + row * A.ld_out, y);
    } else {
        const int lanes = A.group >> 3;  // 1..16 lanes per group
        float s;
        const uint32_t packed = quant8<kBits>(y, lanes, A.scale_f16 != 0, &s);
        const int64_t unit = row * A.heads + head;
        if (kBits == 2)
            *(uint16_t *)(A.codes + unit * (kN / 4) + chunk * 2) = (uint16_t)packed;
        else
            *(uint32_t *)(A.codes + unit * (kN / 2) + chunk * 4) = packed;
        if ((chunk & (lanes - 1)) == 0) {
            const int64_t sidx = unit * (kN / A.group) + (chunk * 8) / A.group;
            if (A.scale_f16)
                ((__half *)A.scales)[sidx] = __float2half_rn(s);
            else
                ((float *)A.scales)[sidx] = s;
        }
    }
}

template <typename T, int kMode, int kBits>
__global__ __launch_bounds__(kThreads, 4) void k12_kernel(K12Args A)
{
    __shared__ float lds1[kLdsRow];
    __shared__ float lds2[kLdsRow];
    constexpr bool kInverse = (kMode == kInv);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int chunk = wave * 64 + lane_chunk(lane);
    const int idx_n = chunk * 8;
    const int head = blockIdx.x % A.heads;
    const int64_t row_first = blockIdx.x / A.heads;
    const int64_t row_step = gridDim.x / A.heads;
    const T *in = (const T *)A.in + (size_t)head * kN + idx_n;
    T *out = (T *)A.out + (size_t)head * kN + idx_n;
    int64_t row = row_first;
    if (row >= A.rows) return;

    if (*A.fast_bad != 0) {  // rare: plain rotations through LDS
        const float2 *cs = A.cs + (size_t)head * kK * (kN / 2);
        for (; row < A.rows; row += row_step) {
            float u[8];
            unpack8(load8(in + row * A.ld_in), u, (const T *)nullptr);
            slow_cascade<kInverse>(u, lds1, cs, idx_n);
            finish_row<T, kMode, kBits>(A, u, out, row, head, chunk);
        }
        return;
    }

    // coefficients: cn[j][r] for layer j+1 (layout N), cp[j][r'] for layer 8+j (layout P), d[r] (layout N)
    const int idx_p = base_p(wave, lane);
    float cn[7][8], cp[5][8], d[8];
    {
        const float *fg = A.fg + (size_t)head * kK * kN;
        const float *fd = A.fd + (size_t)head * kN;
#pragma unroll
        for (int j = 0; j < 7; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r) cn[j][r] = fg[j * kN + idx_n + r];
#pragma unroll
        for (int j = 0; j < 5; ++j)
#pragma unroll
            for (int r = 0; r < 8; ++r) cp[j][r] = fg[(7 + j) * kN + idx_p + 512 * r];
#pragma unroll
        for (int r = 0; r < 8; ++r) d[r] = fd[idx_n + r];
    }
    const int an = lds_addr(idx_n);  // + r
    const int ap = lds_addr(idx_p);  // + 528 r'

    Raw8 raw = load8(in + row * A.ld_in);
    for (; row < A.rows; row += row_step) {
        float u[8];
        unpack8(raw, u, (const T *)nullptr);
        const int64_t next = row + row_step;
        if (next < A.rows) raw = load8(in + next * A.ld_in);  // prefetch the next row of this workgroup

        if (!kInverse) {
            reg_layer<0>(u, cn[0]);
            reg_layer<1>(u, cn[1]);
            reg_layer<2>(u, cn[2]);
            dpp_layer_xor1(u, cn[3]);
            dpp_layer_xor2(u, cn[4]);
            dpp_layer_xor7(u, cn[5]);
            dpp_layer_xor8(u, cn[6]);
        }
        // N -> P
#pragma unroll
        for (int r = 0; r < 8; ++r) lds1[an + r] = u[r];
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 8; ++r) u[r] = lds1[ap + 528 * r];
        if (!kInverse) {
            dpp_layer_xor1(u, cp[0]);
            dpp_layer_xor2(u, cp[1]);
            reg_layer<0>(u, cp[2]);
            reg_layer<1>(u, cp[3]);
            reg_layer<2>(u, cp[4]);
        } else {
            reg_layer<2>(u, cp[4]);
            reg_layer<1>(u, cp[3]);
            reg_layer<0>(u, cp[2]);
            dpp_layer_xor2(u, cp[1]);
            dpp_layer_xor1(u, cp[0]);
        }
        // P -> N
#pragma unroll
        for (int r = 0; r < 8; ++r) lds2[ap + 528 * r] = u[r];
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 8; ++r) u[r] = lds2[an + r];
        if (kInverse) {
            dpp_layer_xor8(u, cn[6]);
            dpp_layer_xor7(u, cn[5]);
            dpp_layer_xor2(u, cn[4]);
            dpp_layer_xor1(u, cn[3]);
            reg_layer<2>(u, cn[2]);
            reg_layer<1>(u, cn[1]);
            reg_layer<0>(u, cn[0]);
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) u[r] *= d[r];
        finish_row<T, kMode, kBits>(A, u, out, row, head, chunk);
    }
}

template <typename T>
static hipError_t launch_k12_t(Mode mode, const K12Args &A, int bits, unsigned grid, hipStream_t stream)
{
    void (*kern)(K12Args) = nullptr;
    if (mode == kFwd)
        kern = k12_kernel<T, kFwd, 4>;
    else if (mode == kInv)
        kern = k12_kernel<T, kInv, 4>;
    else
        kern = bits == 2 ? k12_kernel<T, kFwdQuant, 2> : k12_kernel<T, kFwdQuant, 4>;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), 0, stream, A);
    return hipGetLastError();
}

bool k12_supported(Mode mode, const void *in, const void *out, const Shape &s, const QuantArgs *q)
{
    if (s.n != kN) return false;
    const int isz = s.dtype == BQ_F32 ? 4 : 2;
    const int vec = 16 / isz;  // elements per 16 bytes
    if (((uintptr_t)in & 15) || (s.ld_x % vec)) return false;
    if (mode != kFwdQuant && (((uintptr_t)out & 15) || (s.ld_y % vec))) return false;
    if (s.heads > 512) return false;
    if (mode == kFwdQuant) {
        if (q->group > 128) return false;
        if (((uintptr_t)q->codes & 3)) return false;
    }
    return true;
}

hipError_t launch_k12(Mode mode, const void *in, void *out, const PlanView &pv, const Shape &s,
                      const QuantArgs *q, hipStream_t stream)
{
    K12Args A{};
    A.in = in;
    A.out = out;
    A.fg = mode == kInv ? pv.fg_inv : pv.fg_fwd;
    A.fd = mode == kInv ? pv.fd_inv : pv.fd_fwd;
    A.cs = pv.cs;
    A.fast_bad = mode == kInv ? &pv.hdr->fast_bad_inv : &pv.hdr->fast_bad_fwd;
    A.rows = s.rows;
    A.ld_in = s.ld_x;
    A.ld_out = s.ld_y;
    A.heads = s.heads;
    int bits = 4;
    if (q) {
        A.codes = q->codes;
        A.scales = q->scales;
        A.group = q->group;
        A.scale_f16 = q->scale_f16;
        bits = q->bits;
    }
    // persistent workgroups: two per compute unit, a multiple of the head count
    int64_t per_head = s.rows < (512 / s.heads > 0 ? 512 / s.heads : 1) ? s.rows : (512 / s.heads > 0 ? 512 / s.heads : 1);
    unsigned grid = (unsigned)(per_head * s.heads);
    switch (s.dtype) {
        case BQ_F32: return launch_k12_t<float>(mode, A, bits, grid, stream);
        case BQ_F16: return launch_k12_t<__half>(mode, A, bits, grid, stream);
        default: return launch_k12_t<bf16_t>(mode, A, bits, grid, stream);
    }
}

}  // namespace bq
