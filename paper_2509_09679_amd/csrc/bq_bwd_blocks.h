// Building blocks shared by the backward kernels (gfx950, wave64): the transposed cascade on an activation
// vector and a gradient vector together, with the sums that give dtheta.
//
// Sums are kept in deferred units (see bq_bwd.hip):  acc += v_g[b] v_x[a] - v_g[a] v_x[b]  for a pair that
// sits in two registers of a thread; for a pair that sits in two lanes each lane keeps the product of its own
// element (one v_fmac_f32 with a DPP operand) and the two lanes' sums are subtracted at the end.
#pragma once

#include "bq_cascade.h"

namespace bq {

// acc[r] += vg[r] of lane (lane ^ mask) * vx[r]
#define BQ_DPP_ACC8(MOD)                                                                                     \
    asm volatile("s_nop 1\n\t"                                                                              \
                 "v_fmac_f32_dpp %0, %8, %16 " MOD " row_mask:0xf bank_mask:0xf\n\t"                        \
                 "v_fmac_f32_dpp %1, %9, %17 " MOD " row_mask:0xf bank_mask:0xf\n\t"                        \
                 "v_fmac_f32_dpp %2, %10, %18 " MOD " row_mask:0xf bank_mask:0xf\n\t"                       \
                 "v_fmac_f32_dpp %3, %11, %19 " MOD " row_mask:0xf bank_mask:0xf\n\t"                       \
                 "v_fmac_f32_dpp %4, %12, %20 " MOD " row_mask:0xf bank_mask:0xf\n\t"                       \
                 "v_fmac_f32_dpp %5, %13, %21 " MOD " row_mask:0xf bank_mask:0xf\n\t"                       \
                 "v_fmac_f32_dpp %6, %14, %22 " MOD " row_mask:0xf bank_mask:0xf\n\t"                       \
                 "v_fmac_f32_dpp %7, %15, %23 " MOD " row_mask:0xf bank_mask:0xf"                           \
                 : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(acc[4]), "+v"(acc[5]),        \
                   "+v"(acc[6]), "+v"(acc[7])                                                                \
                 : "v"(vg[0]), "v"(vg[1]), "v"(vg[2]), "v"(vg[3]), "v"(vg[4]), "v"(vg[5]), "v"(vg[6]), "v"(vg[7]), \
                   "v"(vx[0]), "v"(vx[1]), "v"(vx[2]), "v"(vx[3]), "v"(vx[4]), "v"(vx[5]), "v"(vx[6]), "v"(vx[7]))

__device__ __forceinline__ void dpp_acc_xor1(float (&acc)[8], const float (&vg)[8], const float (&vx)[8]) { BQ_DPP_ACC8("quad_perm:[1,0,3,2]"); }
__device__ __forceinline__ void dpp_acc_xor2(float (&acc)[8], const float (&vg)[8], const float (&vx)[8]) { BQ_DPP_ACC8("quad_perm:[2,3,0,1]"); }
__device__ __forceinline__ void dpp_acc_xor7(float (&acc)[8], const float (&vg)[8], const float (&vx)[8]) { BQ_DPP_ACC8("row_half_mirror"); }
__device__ __forceinline__ void dpp_acc_xor8(float (&acc)[8], const float (&vg)[8], const float (&vx)[8]) { BQ_DPP_ACC8("row_ror:8"); }

// register-pair layer J: acc[q] (q = index of the pair among the 4 pairs) += vg[b] vx[a] - vg[a] vx[b]
template <int J>
__device__ __forceinline__ void reg_acc(float (&acc)[4], const float (&vg)[8], const float (&vx)[8])
{
    int q = 0;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        if (!(r & (1 << J))) {
            const int a = r, b = r | (1 << J);
            acc[q] = __builtin_fmaf(vg[b], vx[a], acc[q]);
            acc[q] = __builtin_fmaf(-vg[a], vx[b], acc[q]);
            ++q;
        }
    }
}

template <int CTRL>
__device__ __forceinline__ float dpp_get(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

__device__ __forceinline__ int pair_index(int a, int i) { return ((a >> i) << (i - 1)) | (a & ((1 << (i - 1)) - 1)); }


__device__ __forceinline__ void put_partial(float *p, float v, int first)
{
    if (first)
        *p = v;
    else
        *p += v;
}

struct NAcc {  // deferred sums of phase N: lane layers 4..7, register layers 1..3
    float d[4][8], r[3][4];
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int q = 0; q < 8; ++q) d[j][q] = 0.0f;
#pragma unroll
        for (int j = 0; j < 3; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) r[j][q] = 0.0f;
    }
};

// Coefficients of layers 1..7 held in registers, in the form n_phase() takes them.
struct CoefRegs {
    float c[7][8];
    template <int J>
    __device__ __forceinline__ void get(float (&o)[8]) const
    {
#pragma unroll
        for (int r = 0; r < 8; ++r) o[r] = c[J][r];
    }
};

// layers 7..1 transposed on (vx, vg) held in layout N; on return vg holds g_0 in deferred units
template <class C>
__device__ __forceinline__ void n_phase(float (&vx)[8], float (&vg)[8], const C &cn, NAcc &acc)
{
    float c[8];
    cn.template get<6>(c);
    dpp_acc_xor8(acc.d[3], vg, vx);  // layer 7
    dpp_layer_xor8(vx, c);
    dpp_layer_xor8(vg, c);
    cn.template get<5>(c);
    dpp_acc_xor7(acc.d[2], vg, vx);  // layer 6
    dpp_layer_xor7(vx, c);
    dpp_layer_xor7(vg, c);
    cn.template get<4>(c);
    dpp_acc_xor2(acc.d[1], vg, vx);  // layer 5
    dpp_layer_xor2(vx, c);
    dpp_layer_xor2(vg, c);
    cn.template get<3>(c);
    dpp_acc_xor1(acc.d[0], vg, vx);  // layer 4
    dpp_layer_xor1(vx, c);
    dpp_layer_xor1(vg, c);
    cn.template get<2>(c);
    reg_acc<2>(acc.r[2], vg, vx);  // layer 3
    reg_layer<2>(vx, c);
    reg_layer<2>(vg, c);
    cn.template get<1>(c);
    reg_acc<1>(acc.r[1], vg, vx);  // layer 2
    reg_layer<1>(vx, c);
    reg_layer<1>(vg, c);
    cn.template get<0>(c);
    reg_acc<0>(acc.r[0], vg, vx);  // layer 1 (x is not needed below it)
    reg_layer<0>(vg, c);
}

__device__ __forceinline__ float lane_partner(float v, int j)
{
    return j == 0 ? dpp_get<0xB1>(v) : j == 1 ? dpp_get<0x4E>(v) : j == 2 ? dpp_get<0x141>(v) : dpp_get<0x128>(v);
}

}  // namespace bq
