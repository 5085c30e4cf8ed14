// Register/DPP building blocks of the specialised cascade kernels (gfx950, wave64).
//
// Every thread carries 8 elements of a transform in registers, in the scale-deferred form described
// in bq_internal.h: one layer is  u[e] += coef[e] * u[partner(e)], one FMA per element.
//   * partner in the same thread  -> plain FMAs on register pairs
//   * partner in another lane of the same 16-lane row -> one v_fmac_f32 with a DPP operand; the
//     lane exchange costs no extra instruction.  gfx9 DPP offers the lane XOR masks 1, 2
//     (quad_perm), 7 (row_half_mirror), 8 (row_ror:8) and 15 (row_mirror); the masks {1, 2, 7, 8}
//     are linearly independent over GF(2), so four butterfly layers fit in a 16-lane row if lane l
//     holds the chunk  e(l) = l ^ (l & 4 ? 3 : 0)  (then e(l ^ 7) = e(l) ^ 4).
//
// The DPP instructions are written as inline assembly because the compiler does not fold a DPP move
// into an FMA whose accumulator is the permuted register itself.  A VALU write followed by a DPP
// read of the same VGPR needs two wait states; the compiler does not see inside the assembly, so
// every block starts with s_nop 1, and inside a block the eight instructions touch eight different
// registers.
#pragma once

#include "bq_device.h"

namespace bq {

// chunk held by lane l (only the low four lane bits are permuted)
__device__ __forceinline__ int lane_chunk(int lane) { return lane ^ ((lane & 4) ? 3 : 0); }

#define BQ_DPP_FMAC8(MOD)                                                                              \
    asm volatile("s_nop 1\n\t"                                                                        \
                 "v_fmac_f32_dpp %0, %0, %8 " MOD " row_mask:0xf bank_mask:0xf\n\t"                   \
                 "v_fmac_f32_dpp %1, %1, %9 " MOD " row_mask:0xf bank_mask:0xf\n\t"                   \
                 "v_fmac_f32_dpp %2, %2, %10 " MOD " row_mask:0xf bank_mask:0xf\n\t"                  \
                 "v_fmac_f32_dpp %3, %3, %11 " MOD " row_mask:0xf bank_mask:0xf\n\t"                  \
                 "v_fmac_f32_dpp %4, %4, %12 " MOD " row_mask:0xf bank_mask:0xf\n\t"                  \
                 "v_fmac_f32_dpp %5, %5, %13 " MOD " row_mask:0xf bank_mask:0xf\n\t"                  \
                 "v_fmac_f32_dpp %6, %6, %14 " MOD " row_mask:0xf bank_mask:0xf\n\t"                  \
                 "v_fmac_f32_dpp %7, %7, %15 " MOD " row_mask:0xf bank_mask:0xf"                      \
                 : "+v"(u[0]), "+v"(u[1]), "+v"(u[2]), "+v"(u[3]), "+v"(u[4]), "+v"(u[5]), "+v"(u[6]),  \
                   "+v"(u[7])                                                                          \
                 : "v"(c[0]), "v"(c[1]), "v"(c[2]), "v"(c[3]), "v"(c[4]), "v"(c[5]), "v"(c[6]), "v"(c[7]))

// u[r] += c[r] * u[r] of lane (lane ^ mask), for the four supported masks
__device__ __forceinline__ void dpp_layer_xor1(float (&u)[8], const float (&c)[8]) { BQ_DPP_FMAC8("quad_perm:[1,0,3,2]"); }
__device__ __forceinline__ void dpp_layer_xor2(float (&u)[8], const float (&c)[8]) { BQ_DPP_FMAC8("quad_perm:[2,3,0,1]"); }
__device__ __forceinline__ void dpp_layer_xor7(float (&u)[8], const float (&c)[8]) { BQ_DPP_FMAC8("row_half_mirror"); }
__device__ __forceinline__ void dpp_layer_xor8(float (&u)[8], const float (&c)[8]) { BQ_DPP_FMAC8("row_ror:8"); }

// m = max(m, m of lane ^ mask) over the 16-lane row: after the four steps every lane holds the row max
__device__ __forceinline__ float row16_max(float m)
{
    asm volatile("s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
                 "s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
                 "s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
                 "s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf"
                 : "+v"(m));
    return m;
}

// max over lane groups of 2, 4 or 8 lanes (subsets of the steps above)
__device__ __forceinline__ float lanes_max(float m, int lanes)
{
    if (lanes >= 2)
        asm volatile("s_nop 1\n\tv_max_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf" : "+v"(m));
    if (lanes >= 4)
        asm volatile("s_nop 1\n\tv_max_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf" : "+v"(m));
    if (lanes >= 8)
        asm volatile("s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf" : "+v"(m));
    if (lanes >= 16)
        asm volatile("s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf" : "+v"(m));
    return m;
}

// One layer on register pairs: partner of register r is r ^ (1 << J)
template <int J>
__device__ __forceinline__ void reg_layer(float (&u)[8], const float (&c)[8])
{
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        if (!(r & (1 << J))) {
            const int a = r, b = r | (1 << J);
            const float ua = u[a], ub = u[b];
            u[a] = __builtin_fmaf(c[a], ub, ua);
            u[b] = __builtin_fmaf(c[b], ua, ub);
        }
    }
}

// First layer of a cascade: every element still has scale 1, so the two coefficients of a pair are
// t and -t; only the upper element's coefficient c[b] is read (the negation is an operand modifier).
template <int J>
__device__ __forceinline__ void reg_layer_first(float (&u)[8], const float (&c)[8])
{
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        if (!(r & (1 << J))) {
            const int a = r, b = r | (1 << J);
            const float ua = u[a], ub = u[b];
            u[a] = __builtin_fmaf(-c[b], ub, ua);
            u[b] = __builtin_fmaf(c[b], ua, ub);
        }
    }
}

// ---- row I/O: 8 consecutive elements per thread ------------------------------------------------
struct Raw8 {
    uint4 lo, hi;  // f16/bf16 use lo only
};

template <typename T>
__device__ __forceinline__ Raw8 load8(const T *p)
{
    Raw8 r;
    r.lo = *(const uint4 *)p;
    if (sizeof(T) == 4) r.hi = *((const uint4 *)p + 1);
    return r;
}

__device__ __forceinline__ void unpack8(const Raw8 &r, float (&u)[8], const float *)
{
    u[0] = __uint_as_float(r.lo.x); u[1] = __uint_as_float(r.lo.y); u[2] = __uint_as_float(r.lo.z);
    u[3] = __uint_as_float(r.lo.w); u[4] = __uint_as_float(r.hi.x); u[5] = __uint_as_float(r.hi.y);
    u[6] = __uint_as_float(r.hi.z); u[7] = __uint_as_float(r.hi.w);
}
__device__ __forceinline__ void unpack8(const Raw8 &r, float (&u)[8], const __half *)
{
    const uint32_t w[4] = {r.lo.x, r.lo.y, r.lo.z, r.lo.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const __half2 h = *(const __half2 *)&w[i];
        u[2 * i] = __low2float(h);
        u[2 * i + 1] = __high2float(h);
    }
}
__device__ __forceinline__ void unpack8(const Raw8 &r, float (&u)[8], const bf16_t *)
{
    const uint32_t w[4] = {r.lo.x, r.lo.y, r.lo.z, r.lo.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        u[2 * i] = __uint_as_float(w[i] << 16);
        u[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
}

__device__ __forceinline__ void store8(float *p, const float (&y)[8])
{
    *(float4 *)p = make_float4(y[0], y[1], y[2], y[3]);
    *((float4 *)p + 1) = make_float4(y[4], y[5], y[6], y[7]);
}
__device__ __forceinline__ void store8(__half *p, const float (&y)[8])
{
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = f32x2_to_f16x2_bits(y[2 * i], y[2 * i + 1]);
    *(uint4 *)p = make_uint4(w[0], w[1], w[2], w[3]);
}
__device__ __forceinline__ void store8(bf16_t *p, const float (&y)[8])
{
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        w[i] = f32x2_to_bf16x2_bits(y[2 * i], y[2 * i + 1]);
    *(uint4 *)p = make_uint4(w[0], w[1], w[2], w[3]);
}

// the same stores with the non-temporal hint (output that is not read again before it leaves the caches)
typedef uint32_t nt_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store8_nt(float *p, const float (&y)[8])
{
    const nt_u32x4 a = {__float_as_uint(y[0]), __float_as_uint(y[1]), __float_as_uint(y[2]), __float_as_uint(y[3])};
    const nt_u32x4 b = {__float_as_uint(y[4]), __float_as_uint(y[5]), __float_as_uint(y[6]), __float_as_uint(y[7])};
    __builtin_nontemporal_store(a, (nt_u32x4 *)p);
    __builtin_nontemporal_store(b, (nt_u32x4 *)p + 1);
}
__device__ __forceinline__ void store8_nt(__half *p, const float (&y)[8])
{
    nt_u32x4 w;
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = f32x2_to_f16x2_bits(y[2 * i], y[2 * i + 1]);
    __builtin_nontemporal_store(w, (nt_u32x4 *)p);
}
__device__ __forceinline__ void store8_nt(bf16_t *p, const float (&y)[8])
{
    nt_u32x4 w;
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = f32x2_to_bf16x2_bits(y[2 * i], y[2 * i + 1]);
    __builtin_nontemporal_store(w, (nt_u32x4 *)p);
}

// ---- quantiser epilogue for 8 consecutive channels per thread ----------------------------------
// Reciprocal of a positive normal float whose significand has at most 11 bits (a binary16 value),
// correctly rounded: hardware estimate (1 ulp) plus one Newton step in FMA arithmetic.  Used only
// for binary16-valued scales (2^-24 .. 65504); the parity tests sweep every such value.
__device__ __forceinline__ float rcp_f16_valued(float s)
{
    const float r = __builtin_amdgcn_rcpf(s);
    const float e = __builtin_fmaf(-s, r, 1.0f);
    return __builtin_fmaf(e, r, r);
}

// `lanes` consecutive lanes of a 16-lane row (1, 2, 4, 8 or 16) share one group, i.e. group = 8 * lanes.
// Returns the packed codes of the thread's 8 channels (16 bits for INT2, 32 for INT4) and the stored
// scale.  Same float32 operation sequence as documented in bq.h:
//   amax -> s = amax / qmax -> (binary16 rounding) -> inv = 1 / s -> q = clip(rint(y * inv)).
// The clip is applied to y * inv before rounding (the bounds are integers, so clipping and rounding
// commute) and only for the rare scales that can make |y * inv| exceed qmax (a zero product needs no
// clip either); rint is done by adding 1.5 * 2^23: the adder rounds the sum to an integer, ties to even,
// and the low mantissa bits of the sum hold q in two's complement.  The 8 codes are gathered with one
// shift-add each:  acc = sum (bits(f_j) << j*BITS)  =  sum q_j 2^(j*BITS) + const.  Adding the bias
// 2^(BITS-1) to every field makes all fields non-negative (no borrows between fields); the final
// XOR takes the bias out again, field by field.
// Scale, its reciprocal and the products y * inv (clipped where the clip can act) of the thread's 8 channels.
// max |y| over the thread's 8 channels
__device__ __forceinline__ float amax8(const float (&y)[8])
{
    float m = fmaxf(fmaxf(fabsf(y[0]), fabsf(y[1])), fabsf(y[2]));
    m = fmaxf(fmaxf(m, fabsf(y[3])), fabsf(y[4]));
    m = fmaxf(fmaxf(m, fabsf(y[5])), fabsf(y[6]));
    return fmaxf(m, fabsf(y[7]));
}

// kMaxGiven: group_max is the group's max |y|, formed by the caller (groups that reach beyond a 16-lane row)
//
// The common case is kept short: with binary16 scales, "ordinary" means that the rounded scale is a normal,
// finite binary16 number (one range test on its bit pattern); then no clip can act (|y * inv| <= qmax (1 + 2^-10)),
// the scale is not zero and did not saturate.  Everything else -- a zero or subnormal scale, a scale beyond
// 65504 (which saturates), the clip -- is redone on a cold path from the same inputs.
template <int BITS, bool kMaxGiven = false>
__device__ __forceinline__ void scaled8(const float (&y)[8], int lanes, bool scale_f16, float (&t)[8], float *scale_out,
                                        bool *ordinary_out, float group_max = -1.0f)
{
    const float m = kMaxGiven ? group_max : lanes_max(amax8(y), lanes);
    constexpr float qmax = (float)((1 << (BITS - 1)) - 1);
    constexpr float qmin = -(float)(1 << (BITS - 1));
    float s, inv;
    bool ordinary;
    if (scale_f16) {
        // qmax = 1 for INT2: the division is the identity.  For INT4, m / 7 correctly rounded with
        // three FMA-class operations (multiply by RN(1/7), exact remainder, correction); exact for
        // every normal quotient, and quotients below the binary16 range round to a zero scale anyway.
        float s_exact;
        if (BITS == 2) {
            s_exact = m;
        } else {
            constexpr float kRcp = 1.0f / qmax;
            const float q0 = m * kRcp;
            const float rem = __builtin_fmaf(-qmax, q0, m);
            s_exact = __builtin_fmaf(rem, kRcp, q0);
        }
        // The quotient is pinned as a float32 value: left alone, the compiler merges its last FMA with the
        // conversion below into one instruction that rounds the exact sum once to binary16, which differs from
        // "float32 quotient, then one rounding" where the float32 quotient is a binary16 tie.
        asm volatile("" : "+v"(s_exact));
        const __half hs = __float2half_rn(s_exact);  // beyond the binary16 range: infinity
        const uint16_t hb = __half_as_ushort(hs);
        ordinary = (uint16_t)(hb - 0x0400u) < (uint16_t)0x7800u;  // 2^-14 <= scale <= 65504
        s = __half2float(hs);
        inv = rcp_f16_valued(s);
        if (__builtin_expect(!ordinary, 0)) {  // rare: saturation at 65504, zero scale
            asm volatile("");              // (keeps this a branch: the statements must not join the common path)
            s = __half2float(__float2half_rn(fminf(s_exact, 65504.0f)));
            inv = (s == 0.0f) ? 0.0f : rcp_f16_valued(s);
        }
    } else {
        s = (BITS == 2) ? m : m / qmax;
        inv = 1.0f / s;
        ordinary = s >= 0x1p-100f;
        if (__builtin_expect(!ordinary, 0)) {
            asm volatile("");
            inv = (s == 0.0f) ? 0.0f : inv;
        }
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) t[r] = y[r] * inv;
    if (__builtin_expect(!ordinary, 0)) {  // rare: clip before rounding (the bounds are integers, so the two commute)
#pragma unroll
        for (int r = 0; r < 8; ++r) t[r] = __builtin_amdgcn_fmed3f(t[r], qmin, qmax);
    }
    *scale_out = s;
    *ordinary_out = ordinary;
}

constexpr float kRoundMagic = 12582912.0f;  // 1.5 * 2^23, bits 0x4B400000

// acc = (acc << BITS) + v in one instruction (left to itself the compiler turns the chain into a tree of
// shifts and three-operand adds, half as many instructions again)
template <int BITS>
__device__ __forceinline__ uint32_t shl_add(uint32_t acc, uint32_t v)
{
    uint32_t d;
    asm("v_lshl_add_u32 %0, %1, %2, %3" : "=v"(d) : "v"(acc), "n"(BITS), "v"(v));
    return d;
}

// Rounding and packing: adding 1.5 * 2^23 + 2^(BITS-1) rounds t to an integer (ties to even) and leaves
// q + 2^(BITS-1), a non-negative BITS-bit field, in the low bits of the sum's pattern.  The 8 fields are
// gathered with one shift-add each (no borrows between fields); the upper bits of the patterns do not reach
// the low 16 bits (INT2) or are subtracted as one constant (INT4); the final XOR turns every field
// q + 2^(BITS-1) into q in two's complement.
template <int BITS, bool kMaxGiven = false>
__device__ __forceinline__ uint32_t quant8(const float (&y)[8], int lanes, bool scale_f16, float *scale_out,
                                           float group_max = -1.0f)
{
    float t[8];
    bool ordinary;
    scaled8<BITS, kMaxGiven>(y, lanes, scale_f16, t, scale_out, &ordinary, group_max);
    constexpr float kBiasedMagic = kRoundMagic + (float)(1 << (BITS - 1));
    uint32_t acc = __float_as_uint(t[7] + kBiasedMagic);
#pragma unroll
    for (int r = 6; r >= 0; --r) acc = shl_add<BITS>(acc, __float_as_uint(t[r] + kBiasedMagic));
    uint32_t magic_sum = 0, bias = 0;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        magic_sum += 0x4B400000u << (r * BITS);
        bias |= (1u << (BITS - 1)) << (r * BITS);
    }
    if (BITS == 2) return (acc ^ bias) & 0xFFFFu;
    return (acc - magic_sum) ^ bias;
}

// ---- fake quantisation: Dequant(Quant(y)) and code-bin counting -----------------------------------
// Per-thread counters of the code bins, cheap enough for the row loop; drained into 2^BITS 64-bit counters
// of the workgroup in LDS (`wg`, zeroed by the caller) through drain().  Bin c holds code c - 2^(BITS-1).
template <int BITS>
struct BinCount;

// INT2: with an ordinary scale the codes are -1, 0, 1, so their sum and their sum of squares give the three
// counts; code -2 (possible only where the clip acts) is counted explicitly on that cold path.
//   sum = pos - neg - 2 m2,  squares = pos + neg + 4 m2,  rows * 8 = pos + neg + zero + m2
template <>
struct BinCount<2> {
    int sum, squares, m2, rows;
    __device__ __forceinline__ void clear() { sum = squares = m2 = rows = 0; }
    __device__ __forceinline__ void add(const float (&q)[8], bool ordinary)
    {
        const float a = ((q[0] + q[1]) + (q[2] + q[3])) + ((q[4] + q[5]) + (q[6] + q[7]));
        float b = q[0] * q[0];
#pragma unroll
        for (int r = 1; r < 8; ++r) b = __builtin_fmaf(q[r], q[r], b);
        sum += (int)a;
        squares += (int)b;
        rows += 1;
        if (__builtin_expect(!ordinary, 0)) {
#pragma unroll
            for (int r = 0; r < 8; ++r) m2 += (q[r] == -2.0f) ? 1 : 0;
        }
    }
    __device__ __forceinline__ void drain(unsigned long long *wg)
    {
        const int pos = (sum + squares - 2 * m2) / 2, neg = (squares - sum - 6 * m2) / 2;
        const int zero = 8 * rows - pos - neg - m2;
        if (m2) atomicAdd(&wg[0], (unsigned long long)m2);
        if (neg) atomicAdd(&wg[1], (unsigned long long)neg);
        if (zero) atomicAdd(&wg[2], (unsigned long long)zero);
        if (pos) atomicAdd(&wg[3], (unsigned long long)pos);
        clear();
    }
    __device__ __forceinline__ void skip() {}
    static constexpr int kDrainEvery = 1 << 24;  // rows; int range
    __device__ __forceinline__ bool full() const { return rows >= kDrainEvery; }
};

// INT4: the low four bits of (t + 1.5 * 2^23) are the code in two's complement.  One row's eight codes become
// a 64-bit word of sixteen 4-bit counts (one-hot adds); its even and odd nibbles are added to four words of
// 8-bit counts, which hold 31 rows; then the wave adds them up and one lane of it updates the workgroup's
// counters.
template <>
struct BinCount<4> {
    uint32_t c8[4];  // 8-bit counts: [0] nibbles 0,2,4,6  [1] 1,3,5,7  [2] 8,10,12,14  [3] 9,11,13,15
    int rows;
    __device__ __forceinline__ void clear()
    {
        c8[0] = c8[1] = c8[2] = c8[3] = 0;
        rows = 0;
    }
    __device__ __forceinline__ void add(const uint32_t (&fbits)[8])
    {
        unsigned long long p = 0;
#pragma unroll
        for (int r = 0; r < 8; ++r) p += 1ull << ((fbits[r] & 15u) << 2);
        const uint32_t lo = (uint32_t)p, hi = (uint32_t)(p >> 32);
        c8[0] += lo & 0x0F0F0F0Fu;
        c8[1] += (lo >> 4) & 0x0F0F0F0Fu;
        c8[2] += hi & 0x0F0F0F0Fu;
        c8[3] += (hi >> 4) & 0x0F0F0F0Fu;
        rows += 1;
    }
    __device__ __forceinline__ void skip() { rows += 1; }  // keeps `rows` uniform over the wave
    __device__ __forceinline__ bool full() const { return rows >= 31; }
    // every lane of the wave must call this together
    __device__ __forceinline__ void drain(unsigned long long *wg)
    {
        // 16-bit counts (a wave's total is at most 64 * 248), two per word, added across the 64 lanes; one
        // word of 8-bit counts at a time, so that this rarely executed path keeps few values alive
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t w0 = c8[j] & 0x00FF00FFu;         // fields 0 and 2 of c8[j]
            uint32_t w1 = (c8[j] >> 8) & 0x00FF00FFu;  // fields 1 and 3
#pragma unroll
            for (int m = 1; m < 64; m <<= 1) {
                w0 += (uint32_t)__shfl_xor((int)w0, m, 64);
                w1 += (uint32_t)__shfl_xor((int)w1, m, 64);
            }
            if ((threadIdx.x & 63) == 0) {
#pragma unroll
                for (int f = 0; f < 4; ++f) {
                    // field f of c8[j] counts nibble: (j >> 1) * 8 + 2 f + (j & 1); bin = nibble ^ 8
                    const int nibble = (j >> 1) * 8 + 2 * f + (j & 1);
                    const uint32_t word = (f & 1) ? w1 : w0;
                    const uint32_t v = (f >> 1) ? (word >> 16) : (word & 0xFFFFu);
                    if (v) atomicAdd(&wg[nibble ^ 8], (unsigned long long)v);
                }
            }
        }
        clear();
    }
};

// Fake quantisation of the thread's 8 channels, in two steps so that a caller can count before it forms
// the output (fewer values alive at once): rounded8 gives f = t + 1.5 * 2^23 (the code q is f - 1.5 * 2^23,
// and the low bits of f's pattern hold q in two's complement); Dequant is s * q, one float32 rounding, with
// the same scale and codes as quant8.
template <int BITS, bool kMaxGiven = false>
__device__ __forceinline__ void rounded8(const float (&y)[8], int lanes, bool scale_f16, float (&f)[8], float *s,
                                         bool *ordinary, float group_max = -1.0f)
{
    float t[8];
    scaled8<BITS, kMaxGiven>(y, lanes, scale_f16, t, s, ordinary, group_max);
#pragma unroll
    for (int r = 0; r < 8; ++r) f[r] = t[r] + kRoundMagic;
}

template <int BITS>
__device__ __forceinline__ void count8(BinCount<BITS> &bc, const float (&f)[8], bool ordinary);
template <>
__device__ __forceinline__ void count8<2>(BinCount<2> &bc, const float (&f)[8], bool ordinary)
{
    float q[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) q[r] = f[r] - kRoundMagic;
    bc.add(q, ordinary);
}
template <>
__device__ __forceinline__ void count8<4>(BinCount<4> &bc, const float (&f)[8], bool)
{
    uint32_t fbits[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) fbits[r] = __float_as_uint(f[r]);
    bc.add(fbits);
}

// The product is pinned as a float32 value: left alone, the compiler merges the multiplication with a later
// conversion to binary16 into one v_fma_mixlo_f16, which rounds the exact product once and so differs from
// "float32 product, then one rounding" where the float32 product is a binary16 tie (float32 scales, INT4).
__device__ __forceinline__ void dequant8(const float (&f)[8], float s, float (&yq)[8])
{
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        yq[r] = (f[r] - kRoundMagic) * s;
        asm volatile("" : "+v"(yq[r]));
    }
}

// ---- transforms of n = 8 .. 128 inside 16 lanes (8 consecutive elements per lane, no LDS) -----------
template <int CTRL>
__device__ __forceinline__ float dpp_read(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Plain (cos, sin) cascade for flagged plans: a run-time loop over the layers (kept rolled so that
// this rare path needs few registers); partners come from registers for layers 1-3 and from the
// lanes lane^1, lane^2, lane^7, lane^8 for layers 4-7.
template <int K, bool kInverse>
__device__ __noinline__ void slow_small(float (&u)[8], const float2 *__restrict__ cs_head, int idx)
{
    constexpr int n = 1 << K;
#pragma unroll 1
    for (int step = 0; step < K; ++step) {
        const int i = kInverse ? (K - step) : (step + 1);
        const int h = 1 << (i - 1);
        float p[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            float v;
            switch (i) {
                case 1: v = u[r ^ 1]; break;
                case 2: v = u[r ^ 2]; break;
                case 3: v = u[r ^ 4]; break;
                case 4: v = dpp_read<0xB1>(u[r]); break;   // quad_perm [1,0,3,2]
                case 5: v = dpp_read<0x4E>(u[r]); break;   // quad_perm [2,3,0,1]
                case 6: v = dpp_read<0x141>(u[r]); break;  // row_half_mirror
                default: v = dpp_read<0x128>(u[r]); break; // row_ror:8
            }
            p[r] = v;
        }
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int e = idx + r;
            const int a = e & ~h;
            const int pr = ((a >> i) << (i - 1)) | (a & (h - 1));
            const float2 w = cs_head[(size_t)(i - 1) * (n >> 1) + pr];
            const bool upper = (e & h) != 0;
            // forward: lower  c x - s p, upper  c x + s p ; transposed: the signs swap
            const float sgn = (upper != kInverse) ? w.y : -w.y;
            u[r] = __builtin_fmaf(w.x, u[r], sgn * p[r]);
        }
    }
}

template <int K, bool kInverse>
__device__ __forceinline__ void fast_small(float (&u)[8], const float (&c)[7][8], const float (&d)[8])
{
    if (!kInverse) {
        reg_layer_first<0>(u, c[0]);
        reg_layer<1>(u, c[1]);
        reg_layer<2>(u, c[2]);
        if (K >= 4) dpp_layer_xor1(u, c[3]);
        if (K >= 5) dpp_layer_xor2(u, c[4]);
        if (K >= 6) dpp_layer_xor7(u, c[5]);
        if (K >= 7) dpp_layer_xor8(u, c[6]);
    } else {
        if (K >= 7) dpp_layer_xor8(u, c[6]);
        if (K >= 6) dpp_layer_xor7(u, c[5]);
        if (K >= 5) dpp_layer_xor2(u, c[4]);
        if (K >= 4) dpp_layer_xor1(u, c[3]);
        reg_layer<2>(u, c[2]);
        reg_layer<1>(u, c[1]);
        reg_layer<0>(u, c[0]);
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) u[r] *= d[r];
}

}  // namespace bq
