/*
 * bq.h — C ABI of the MI355X (gfx950) butterfly-transform + low-bit quantisation library.
 *
 * The library implements the data-parallel hot path of ButterflyQuant (arXiv 2509.09679):
 * applying the learnable orthogonal butterfly transform B(theta) to batches of activation rows,
 * its transpose, the fused transform + symmetric INT4/INT2 quantisation, and the backward pass
 * (dx and dtheta summed over rows) used for calibration.
 *
 * The transform (paper, section "Structure and Parameterization"): for n = 2^k,
 *     B(theta) = B_k ... B_2 B_1,
 * where layer i consists of n/2 Givens rotations G(t) = [[cos t, -sin t], [sin t, cos t]] acting on
 * the index pairs (a, a + 2^(i-1)).  Layer 1 (stride 1) is applied to the input first, as in the
 * data-flow diagram of the appendix "The Butterfly Pattern Visualization"; the j-th angle of layer i
 * belongs to the j-th pair in increasing order of a, which reproduces the 8x8 layer matrices printed
 * in the appendix "Concrete Example: Butterfly Matrix Structure for n=8".
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller, unless stated otherwise.  The
 *     library never allocates, frees or synchronises; every call only enqueues kernels on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream) and returns.
 *   - The descriptor structs (bq_rows, bq_quant) are HOST pointers, read during the call.
 *   - theta / dtheta: float32, layout [heads][k][n/2] (layer-major, pair index j as above).
 *   - A row consists of `heads` independent blocks of n contiguous elements; block h is transformed
 *     with theta[h] (a block-diagonal transform; heads = 1 is the plain case).
 *   - Errors are reported by return code only; on any code other than BQ_OK nothing was launched.
 *     bq_last_error() returns a thread-local text for the last failing call of the calling thread.
 *   - rows == 0 is valid: BQ_OK, nothing is launched.
 */
#ifndef BQ_H
#define BQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BQ_OK = 0,
    BQ_ERR_NULL = 1,        /* a required pointer is NULL                                   */
    BQ_ERR_SHAPE = 2,       /* n not a power of two in [2, 16384], heads < 1, rows < 0, ld too small,
                               group does not divide n, ...                                 */
    BQ_ERR_DTYPE = 3,       /* unknown element / scale type                                 */
    BQ_ERR_ALIGN = 4,       /* pointer or leading dimension not aligned as documented       */
    BQ_ERR_WORKSPACE = 5,   /* plan or workspace buffer smaller than the size query returns */
    BQ_ERR_UNSUPPORTED = 6, /* valid in principle but not implemented (e.g. bits = 3)       */
    BQ_ERR_HIP = 7          /* a HIP runtime call failed (text in bq_last_error)            */
} bq_status;

typedef enum { BQ_F32 = 0, BQ_F16 = 1, BQ_BF16 = 2 } bq_dtype;

/* One batch of rows.  Element pointers must be aligned to their element size (else BQ_ERR_ALIGN).
 * The specialised kernels additionally need 16-byte aligned pointers and ld_* that are multiples of
 * 16 bytes worth of elements (4 for f32, 8 for f16/bf16); rows that do not meet this are processed by
 * the slower general kernels, with the same results. */
typedef struct {
    int64_t rows;  /* T >= 0                                                                  */
    int32_t n;     /* transform size, power of two, 2 <= n <= 16384                           */
    int32_t heads; /* H >= 1 transforms side by side; logical row width = H * n <= 2^24,
                      and rows * H * n <= 2^40 (else BQ_ERR_SHAPE)                            */
    int64_t ld_x;  /* row stride, in elements, of the input operand(s)  (>= H * n)            */
    int64_t ld_y;  /* row stride, in elements, of the output operand    (>= H * n);
                      rows * max(ld_x, ld_y) <= 2^44 (else BQ_ERR_SHAPE)                      */
    int32_t dtype; /* bq_dtype of the row operands (inputs and outputs share it)              */
    int32_t reserved;
} bq_rows;

/* Quantiser parameters (paper, equation for Quant/Dequant in section "Loss Function"). */
typedef struct {
    int32_t bits;        /* 4 or 2                                                            */
    int32_t group;       /* channels per scale: power of two, 8 <= group <= n, divides n;
                            group == n gives one scale per row and head                       */
    int32_t scale_dtype; /* BQ_F32 or BQ_F16                                                  */
    int32_t reserved;
} bq_quant;

/* ---- plan: everything derived from theta alone --------------------------------------------- */

/* Size in bytes of the device buffer bq_plan_build fills for (n, heads); 0 if the shape is invalid. */
size_t bq_plan_bytes(int32_t n, int32_t heads);

/* Derive from theta what the hot calls need (the paper's "pre-computed cos/sin twiddle factors stored
 * in a lookup table", section "Inference Efficiency" and appendix "Inference FLOP Analysis"; kept in
 * float32) into `plan`, a caller-owned device buffer of at least bq_plan_bytes(n, heads) bytes,
 * aligned to 256 bytes.  Asynchronous on `stream`; call it again whenever theta changes.  The plan's
 * layout is private to the library.  cos/sin are evaluated in double from the float32 angle and
 * rounded once.
 * The plan records the (n, heads) it was built for.  The calls below cannot read it on the host without
 * a synchronisation, so their kernels compare it with the call's shape on the device, before the first
 * table access: given a buffer that bq_plan_build has not filled for exactly this (n, heads) (never
 * built, or built for another shape) they return at once, nothing is read beyond the plan's header,
 * the call still returns BQ_OK and its outputs keep their previous contents (bq_butterfly_fwd_fakequant:
 * hist is set to zero; bq_kron_*: the output is unspecified where the mix with q1 runs as a pass of
 * its own).  The buffer must in every case be readable for its first 256 bytes. */
bq_status bq_plan_build(const float *theta, int32_t n, int32_t heads, void *plan, size_t plan_bytes,
                        void *stream);

/* ---- hot path ------------------------------------------------------------------------------ */

/* y = B(theta) x for every row (paper: x' = Bx, equations of "Structure and Parameterization").
 * x: [rows][ld_x], y: [rows][ld_y], both of rows->dtype; arithmetic in float32, one rounding to the
 * output type.  y == x (with ld_y == ld_x) is allowed. */
bq_status bq_butterfly_fwd(const void *x, void *y, const void *plan, const bq_rows *rows, void *stream);

/* x = B(theta)^T y: the layers in reverse order, each transposed ("orthogonality by construction";
 * computational invariance y = (W B^T)(B x)).  Input y: [rows][ld_x]; output x: [rows][ld_y]. */
bq_status bq_butterfly_inv(const void *y, void *x, const void *plan, const bq_rows *rows, void *stream);

/* Fused Quant(B(theta) x) (activation side of the reconstruction loss; Quant as in the paper:
 * q = clip(round(v / s), -2^(b-1), 2^(b-1)-1), s = max|v| / (2^(b-1)-1) per group of `group`
 * consecutive channels of a rotated row).  The rotated values stay in float32 registers; they are
 * not rounded to rows->dtype first.  The quantiser is the following sequence of correctly rounded
 * float32 operations: amax = max|v|; s = amax / qmax; if scale_dtype is BQ_F16, s = half(s) with
 * round-to-nearest-even, saturating at 65504; inv = (s == 0) ? 0 : 1 / s; q = clip(rint(v * inv)).
 *   codes : [rows][H*n*bits/8] bytes, dense.  Two's-complement fields, lowest channel in the lowest
 *           bits (INT4: byte j/2 = (q_j & 15) | (q_{j+1} & 15) << 4; INT2: four channels per byte).
 *   scales: [rows][H*n/group] of scale_dtype, dense; the stored value is s. */
bq_status bq_butterfly_fwd_quant(const void *x, const void *plan, uint8_t *codes, void *scales,
                                 const bq_quant *quant, const bq_rows *rows, void *stream);

/* Fake-quantised forward: yq = Dequant(Quant(B(theta) x)) = s * q, the activation factor of the
 * reconstruction loss, and the occupancy of the 2^bits code bins, from which the uniformity regulariser
 * D_KL(P_bins || U) follows (paper, sections "Loss Function" and "Uniformity Regularization").  Quant is
 * exactly the quantiser of bq_butterfly_fwd_quant (same operation sequence, same scales and codes);
 * Dequant is one float32 multiplication of the stored scale with the code.
 *   yq  : [rows][ld_y] of rows->dtype, the float32 product rounded once to that type; may be NULL
 *   hist: 2^bits uint64 counters on the device, OVERWRITTEN: hist[c] = number of channels, over all rows
 *         and heads of this call, whose code is c - 2^(bits-1); may be NULL
 * At least one of yq and hist must be given. */
bq_status bq_butterfly_fwd_fakequant(const void *x, const void *plan, void *yq, uint64_t *hist,
                                     const bq_quant *quant, const bq_rows *rows, void *stream);

/* Bytes of device scratch bq_butterfly_bwd needs for this batch shape (0 if the shape is invalid). */
size_t bq_butterfly_bwd_workspace_bytes(const bq_rows *rows);

/* Backward pass (paper, "Gradient Flow Through Butterfly Layers": dG/dt = [[-sin,-cos],[cos,-sin]]).
 * Given upstream dy = dL/d(Bx):  dx = B^T dy  ([rows][ld_y], rows->dtype) and
 * dtheta[h][i][j] = sum over rows of  g_i[b] * x_i[a] - g_i[a] * x_i[b]   (float32, OVERWRITTEN),
 * where x_i / g_i are the activations / gradients at the output of layer i and (a, b) is the pair of
 * angle (i, j).  x and dy: [rows][ld_x].  Partial
 * sums are kept per workgroup and combined in a fixed order in a second pass: the result does not
 * depend on scheduling.  workspace: device scratch of at least the queried size, 256-byte aligned;
 * its contents on entry are ignored.  dx may be NULL to skip it; dtheta may be NULL to skip it.
 * rows == 0: dtheta (if given) is set to zero, nothing else is read or written, x, dy, plan and workspace may
 * be NULL. */
bq_status bq_butterfly_bwd(const void *x, const void *dy, const void *plan, void *dx, float *dtheta,
                           void *workspace, size_t workspace_bytes, const bq_rows *rows, void *stream);

/* The same pass for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The scratch is a fixed array in the
 * library's device image (bq_butterfly_bwd_static_max_bytes() bytes, 32 MiB, held on every GPU the library
 * runs on until the process ends); the call allocates and frees nothing.  Same arguments, results and error
 * codes as bq_butterfly_bwd without the workspace pair; a batch whose bq_butterfly_bwd_workspace_bytes exceeds
 * the array is refused with BQ_ERR_WORKSPACE and nothing is launched.  All calls on one GPU share the one
 * array (its previous contents are ignored), so calls that overlap in time on the same GPU, on different
 * streams, race: serialise them.  The array's address is looked up once per GPU, on the first call there. */
bq_status bq_butterfly_bwd_static(const void *x, const void *dy, const void *plan, void *dx, float *dtheta,
                                  const bq_rows *rows, void *stream);
size_t bq_butterfly_bwd_static_max_bytes(void);

/* ---- fixed Hadamard rotation (the baseline the learned transform is compared with) ------------ */

/* y = H_n x / sqrt(n) for every block of n elements of every row, H_n the Sylvester-ordered Walsh-Hadamard
 * matrix (paper, "Hadamard Transform": H_2n = [[H_n, H_n], [H_n, -H_n]]; the fixed rotation of QuIP / QuaRot that
 * the learned butterfly replaces, and the "FHT" column of the appendix "Inference FLOP Analysis").  Additions and
 * subtractions in float32, one multiplication by 1 / sqrt(n) at the end, one rounding to rows->dtype; no plan, no
 * angles.  H_n / sqrt(n) is symmetric and orthogonal: the same call is its own inverse.  Implemented for
 * n = 4096 and n = 8192 (heads <= 512, 16-byte aligned pointers, leading dimensions multiples of 16 bytes);
 * other shapes return BQ_ERR_UNSUPPORTED.  y == x (with ld_y == ld_x) is allowed. */
bq_status bq_hadamard_fwd(const void *x, void *y, const bq_rows *rows, void *stream);

/* ---- widths that are not powers of two ------------------------------------------------------ */

/* Orthogonal factor for a width d = d1 * d2 with d1 not a power of two (paper, "Concrete Example for
 * d = 5120"): Q1 = (I - A)(I + A)^-1 with A skew-symmetric.  params: the d1 (d1 - 1) / 2 entries of A's
 * strict upper triangle, row by row (A[i][j] = p, A[j][i] = -p for i < j), float32 on the device.
 * q1: [d1][d1] float32, row-major, on the device.  2 <= d1 <= 64.  Evaluated in double (Gauss-Jordan
 * with partial pivoting; I + A is never singular) and rounded once. */
bq_status bq_cayley_build(const float *params, int32_t d1, float *q1, void *stream);

/* y = (Q1 (x) B(theta)) x  (paper, "Kronecker Product Formulation": Q_composite = Q1 (x) Q2 with a
 * butterfly for the power-of-two factor).  A row has d1 * d2 elements, element (i, j) at i * d2 + j:
 * with X the d1 x d2 matrix of a row, the result is Q1 X B^T.  rows->n = d2, rows->heads must be 1,
 * rows->ld_x = rows->ld_y = d1 * d2 (dense rows).  plan: a plan for (n = d2, heads = 1).  y == x is allowed.
 * Arithmetic: d2 = 128 with d1 <= 40: one pass, the butterflies in float32 and the product with Q1 on the
 * matrix cores with float32 accumulation, one rounding to rows->dtype; the product's operands are float32 for
 * float32 and bfloat16 rows, and two-way bfloat16 splits of both factors (three products, relative error of
 * a term below 3 * 2^-16) for binary16 rows.  Other shapes: two passes, the butterfly factor first, its result
 * passing through y in rows->dtype (a second rounding), then the product with Q1 in float32. */
bq_status bq_kron_fwd(const void *x, void *y, const float *q1, int32_t d1, const void *plan,
                      const bq_rows *rows, void *stream);

/* x = (Q1 (x) B(theta))^T y, the inverse of bq_kron_fwd; same conventions. */
bq_status bq_kron_inv(const void *y, void *x, const float *q1, int32_t d1, const void *plan,
                      const bq_rows *rows, void *stream);

/* ---- measurement helpers (not part of the method) ------------------------------------------- */

/* dst[0, bytes) = src[0, bytes): a plain streaming copy (16 bytes per lane), the reference for what the memory
 * system delivers.  Device pointers aligned to 16 bytes, bytes a multiple of 16; asynchronous on `stream`. */
bq_status bq_probe_copy(const void *src, void *dst, size_t bytes, void *stream);

/* The read side alone: every lane of a fixed grid loads its share of src[0, bytes) (16 bytes per lane and access)
 * and stores one 16-byte checksum into `sink`, a device buffer of bq_probe_read_sink_bytes() bytes.  Same alignment
 * rules; asynchronous on `stream`. */
bq_status bq_probe_read(const void *src, size_t bytes, void *sink, void *stream);
size_t bq_probe_read_sink_bytes(void);

/* A float32 FMA issue-rate loop: every lane of a fixed grid runs 16 independent chains of `iters` FMAs, in the
 * instructions this library is built from (no packed float32).  out: device buffer of
 * bq_probe_fma_out_floats() floats (receives one checksum per lane).  Returns the number of lane-FMAs the
 * launch performs (2 flops each), or -1 on a bad argument or launch failure.  Asynchronous on `stream`. */
int64_t bq_probe_fma(float *out, int32_t iters, void *stream);
size_t bq_probe_fma_out_floats(void);

/* ---- helpers ------------------------------------------------------------------------------- */

const char *bq_status_string(bq_status s);
const char *bq_last_error(void); /* thread-local; "" if the last call succeeded */
int bq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BQ_H */
