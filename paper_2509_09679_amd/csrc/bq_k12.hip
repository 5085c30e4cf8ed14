// n = 256 .. 4096 instantiations of the specialised transform kernels, and the choice between them.
#include "bq_k12_kernel.h"
#include "bq_k12_inv.h"

namespace bq {

// n = 4096 or 8192 with any number of heads, or n = 256 .. 2048 where 4096 consecutive elements of the
// [rows][heads * n] array form one block of the kernel: several whole rows (k12_block_rows of them; rows that do
// not fill a block are the caller's to handle) or a 4096-element piece of a wider row.
bool k12_supported(Mode mode, const void *in, const void *out, const Shape &s, const QuantArgs *q)
{
    if (s.n > 2 * kN || s.n < 256) return false;
    const int64_t width = (int64_t)s.n * s.heads;
    if (s.n < kN) {
        const bool rows_per_block = width <= kN && kN % width == 0 && s.rows >= kN / width;
        const bool blocks_per_row = width % kN == 0 && width / kN <= 512;
        if (!rows_per_block && !blocks_per_row) return false;
    }
    const int isz = s.dtype == BQ_F32 ? 4 : 2;
    const int vec = 16 / isz;  // elements per 16 bytes
    if (((uintptr_t)in & 15) || (s.ld_x % vec)) return false;
    if (mode != kFwdQuant && out && (((uintptr_t)out & 15) || (s.ld_y % vec))) return false;
    if (s.n < kN && ((int64_t)k12_block_rows(s) * (s.ld_x > s.ld_y ? s.ld_x : s.ld_y) * isz >= ((int64_t)1 << 31))) return false;
    if (s.n >= kN && s.heads > 512) return false;
    if (mode == kFwdQuant || mode == kFwdFake) {
        if (mode == kFwdQuant && ((uintptr_t)q->codes & 3)) return false;
    }
    return true;
}

bool hadamard_supported(const void *in, const void *out, const Shape &s)
{
    if (s.n != kN && s.n != 2 * kN) return false;
    if (s.heads > 512) return false;
    const int vec = s.dtype == BQ_F32 ? 4 : 8;  // elements per 16 bytes
    if (((uintptr_t)in & 15) || ((uintptr_t)out & 15) || (s.ld_x % vec) || (s.ld_y % vec)) return false;
    return true;
}

hipError_t launch_hadamard(const void *in, void *out, const Shape &s, hipStream_t stream)
{
    K12Args A{};
    A.in = in;
    A.out = out;
    A.rows = s.rows;
    A.ld_in = A.sub_ld_in = s.ld_x;
    A.ld_out = A.sub_ld_out = s.ld_y;
    A.n = s.n;
    A.n_log = s.k;
    // beyond the 256 MB of the memory-side cache neither input nor output is found in a cache again
    A.streaming = (int64_t)s.rows * s.n * s.heads * (s.dtype == BQ_F32 ? 4 : 2) >= ((int64_t)256 << 20) ? 1 : 0;
    A.heads = s.heads;
    const bool wide = s.n > kN;
    int64_t per_head = 256 / A.heads > 0 ? 256 / A.heads : 1;  // as for the forward transform: one workgroup per compute unit
    if (per_head > A.rows) per_head = A.rows;
    const unsigned grid = (unsigned)(per_head * A.heads);
    if (wide) return launch_k13_dtype(kHadamard, A, 4, grid, s.dtype, stream);
    return launch_k12_dtype<false, false>(kHadamard, A, 4, grid, s.dtype, stream);
}

int k12_block_rows(const Shape &s)
{
    const int64_t width = (int64_t)s.n * s.heads;
    return s.n < kN && width < kN ? (int)(kN / width) : 1;
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
    A.plan = pv.ref;
    const bool virt = s.n < kN, wide = s.n > kN;
    const int block_rows = k12_block_rows(s);  // rows of the caller per kernel row
    A.rows = s.rows / block_rows;     // whole blocks only (the caller handles the remainder)
    A.ld_in = s.ld_x * block_rows;
    A.ld_out = s.ld_y * block_rows;
    A.sub_ld_in = s.ld_x;
    A.sub_ld_out = s.ld_y;
    A.n = s.n;
    A.n_log = s.k;
    // beyond the 256 MB of the memory-side cache neither input nor output is found in a cache again
    A.streaming = (int64_t)s.rows * s.n * s.heads * (s.dtype == BQ_F32 ? 4 : 2) >= ((int64_t)256 << 20) ? 1 : 0;
    const int64_t width = (int64_t)s.n * s.heads;
    A.heads = virt ? (width > kN ? (int)(width / kN) : 1) : s.heads;  // virt: 4096-element blocks per row
    A.row_log = virt ? (width >= kN ? kK : ilog2_exact((int)width)) : 0;
    int bits = 4;
    if (q) {
        A.codes = q->codes;
        A.scales = q->scales;
        A.hist = q->hist;
        A.group = q->group;
        A.scale_f16 = q->scale_f16;
        bits = q->bits;
    }
    // Persistent workgroups, a multiple of the head count.  Two fit on a compute unit at a time.  Swept on
    // large batches (same box, 512 .. 2304, after a long warm-up): the fused kernels (VALU-bound) do not care
    // (768 .. 2048 within 1 %), the plain transforms (HBM-bound) are fastest with an odd multiple of 256
    // (768, 1280, 1792, 2304 alike) and 6 .. 18 % slower with anything else tried (512, 640, 896, 1000, 1024,
    // 1152, 1536, 2048).  The forward transform is faster still with ONE workgroup per compute unit (256: 0.84 ->
    // 0.79 ms for 2^30 16-bit elements at every n from 256 to 4096, float32 rows 0.793 -> 0.776 ms, small
    // batches too).  The three-phase inverse was not on 16-bit rows (0.88 against 0.855 ms), which now take the two-phase
    // kernel; on float32 rows, which it still serves, it is.
    // n = 8192: one workgroup of 1024 threads per compute unit at a time.
    // The two-phase inverse of 16-bit rows (bq_k12_inv.h) also runs best with one workgroup per compute unit (256: 0.78 ms,
    // 512: 0.86, 768: 0.85, 1024: 0.99, 1280: 0.85, 2048: 0.95 ms for 2^30 fp16 elements).
    const bool inv_ring = mode == kInv && !wide && s.dtype != BQ_F32;
    // (and so does the three-phase inverse on float32 rows: 0.798 -> 0.779 ms for 2^29 elements)
    const int target = (mode == kFwdQuant || mode == kFwdFake) && !wide ? 1280 : 256;
    int64_t per_head = target / A.heads > 0 ? target / A.heads : 1;
    if (per_head > A.rows) per_head = A.rows;
    unsigned grid = (unsigned)(per_head * A.heads);
    if ((mode == kFwdQuant || mode == kFwdFake) && q->group > 128)
        return launch_k12_big_dtype(mode, A, bits, grid, s.dtype, virt, wide, stream);
    if (wide) return launch_k13_dtype(mode, A, bits, grid, s.dtype, stream);
    if (inv_ring)  // 16-bit rows: the two-phase inverse
        return virt ? launch_k12_inv_ring<true>(A, grid, s.dtype, stream) : launch_k12_inv_ring<false>(A, grid, s.dtype, stream);
    if (virt) return launch_k12_dtype<true, false>(mode, A, bits, grid, s.dtype, stream);
    return launch_k12_dtype<false, false>(mode, A, bits, grid, s.dtype, stream);
}

}  // namespace bq
