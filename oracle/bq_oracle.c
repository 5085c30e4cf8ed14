/*
 * CPU oracle for the butterfly-transform + quantisation path of ButterflyQuant (arXiv 2509.09679).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the method computes,
 * written from the paper.  It shares no code, tables or helpers with the HIP library and must
 * never be called from the product path; only tests, the smoke check and the benchmark's
 * cpu_baseline leg may use it.
 *
 * Arithmetic: the transform and its gradient are evaluated in IEEE double.  The quantiser is a
 * fixed sequence of IEEE single-precision operations (so integer codes are reproducible bit for
 * bit); build with -ffp-contract=off and without any fast-math option.
 *
 * Notation (paper, "Structure and Parameterization"):  n = 2^k.  Layer i = 1..k consists of n/2
 * Givens rotations G(theta) = [[cos, -sin], [sin, cos]] acting on index pairs (a, a + 2^(i-1)).
 * The j-th rotation of layer i (j = 0..n/2-1, the paper's theta_{i,j+1}) acts on the j-th such
 * pair in increasing order of a, which reproduces the three 8x8 layer matrices printed in the
 * appendix "Concrete Example: Butterfly Matrix Structure for n=8".
 * Layer 1 (stride 1) is applied to the input first and layer k last, as in the appendix's
 * data-flow diagram (Input -> Layer 1 -> Layer 2 -> Layer 3 -> Output).
 *
 * theta is float32, layout [heads][k][n/2]; each value is converted exactly to double before
 * cos/sin.  A row holds `heads` independent blocks of n contiguous elements; block h uses
 * theta[h] (block-diagonal transform).
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py (dense-matrix definition
 * on tiny n, printed 8x8 layers, Hadamard special case, Kronecker closed form, orthogonality,
 * finite differences, hand-computed quantiser vectors; Dequant, the bin histogram and the uniformity
 * KL by hand-worked values, closed forms and library routines in tests/test_oracle_fakequant.py).  The bit layout of packed codes and the
 * treatment of an all-zero group are this project's choices, not the paper's: "parity unpinned"
 * for bq_oracle_pack_codes and for the zero-group rule.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* index of the lower element of pair j in layer i (1-based), stride h = 2^(i-1) */
static inline long pair_lo(long j, int i)
{
    long h = 1L << (i - 1);
    return ((j >> (i - 1)) << i) | (j & (h - 1));
}

static void cos_sin_tables(const float *theta, int n, int k, int heads, double **c_out, double **s_out)
{
    size_t m = (size_t)heads * (size_t)k * (size_t)(n / 2);
    double *c = (double *)malloc(m * sizeof(double));
    double *s = (double *)malloc(m * sizeof(double));
    for (size_t q = 0; q < m; ++q) {
        double t = (double)theta[q];
        c[q] = cos(t);
        s[q] = sin(t);
    }
    *c_out = c;
    *s_out = s;
}

static int ilog2_exact(int n)
{
    int k = 0;
    while ((1 << k) < n) ++k;
    return ((1 << k) == n && n >= 2) ? k : -1;
}

/* One layer applied in place to one block v[0..n): v <- B_i v.
 * (Eq. "G(theta)" and the layer structure "B_i = P_i diag(G...) P_i^T".) */
static void layer_apply(double *v, const double *c, const double *s, int n, int i)
{
    long h = 1L << (i - 1);
    for (long j = 0; j < n / 2; ++j) {
        long a = pair_lo(j, i), b = a + h;
        double xa = v[a], xb = v[b];
        v[a] = c[j] * xa - s[j] * xb;
        v[b] = s[j] * xa + c[j] * xb;
    }
}

/* Transposed layer in place: v <- B_i^T v  (G(theta)^T = G(-theta) = [[cos, sin], [-sin, cos]]). */
static void layer_apply_T(double *v, const double *c, const double *s, int n, int i)
{
    long h = 1L << (i - 1);
    for (long j = 0; j < n / 2; ++j) {
        long a = pair_lo(j, i), b = a + h;
        double ya = v[a], yb = v[b];
        v[a] = c[j] * ya + s[j] * yb;
        v[b] = -s[j] * ya + c[j] * yb;
    }
}

/* y = B(theta) x for `rows` rows of heads*n doubles.  B = B_k ... B_2 B_1.  Returns 0, or -1 on a
 * bad shape. */
int bq_oracle_fwd(const double *x, double *y, const float *theta, long rows, int n, int heads)
{
    int k = ilog2_exact(n);
    if (k < 0 || heads < 1 || rows < 0) return -1;
    double *c, *s;
    cos_sin_tables(theta, n, k, heads, &c, &s);
    long w = (long)n * heads;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        for (int hd = 0; hd < heads; ++hd) {
            double *v = y + r * w + (long)hd * n;
            memcpy(v, x + r * w + (long)hd * n, (size_t)n * sizeof(double));
            for (int i = 1; i <= k; ++i) {
                size_t off = ((size_t)hd * k + (size_t)(i - 1)) * (size_t)(n / 2);
                layer_apply(v, c + off, s + off, n, i);
            }
        }
    }
    free(c);
    free(s);
    return 0;
}

/* x = B(theta)^T y: layers in reverse order, each transposed (orthogonality by construction). */
int bq_oracle_inv(const double *y, double *x, const float *theta, long rows, int n, int heads)
{
    int k = ilog2_exact(n);
    if (k < 0 || heads < 1 || rows < 0) return -1;
    double *c, *s;
    cos_sin_tables(theta, n, k, heads, &c, &s);
    long w = (long)n * heads;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        for (int hd = 0; hd < heads; ++hd) {
            double *v = x + r * w + (long)hd * n;
            memcpy(v, y + r * w + (long)hd * n, (size_t)n * sizeof(double));
            for (int i = k; i >= 1; --i) {
                size_t off = ((size_t)hd * k + (size_t)(i - 1)) * (size_t)(n / 2);
                layer_apply_T(v, c + off, s + off, n, i);
            }
        }
    }
    free(c);
    free(s);
    return 0;
}

/* Gradients of L = sum_rows <dy, B(theta) x> w.r.t. x and theta (section "Gradient Flow Through
 * Butterfly Layers").  With x_0 = x, x_i = B_i x_{i-1}, g_k = dy, g_{i-1} = B_i^T g_i:
 *     dL/dtheta_{i,j} = g_i[a,b] . (dG/dtheta)(theta_{i,j}) . x_{i-1}[a,b],
 *     dG/dtheta = [[-sin, -cos], [cos, -sin]],
 * summed over rows;  dx = g_0.  All layer inputs x_{i-1} of a row are kept (no recomputation).
 * dtheta (double, layout of theta) is overwritten.  absacc, if not NULL, receives for every angle
 * the sum over rows of the absolute values of the four products entering its gradient; tests use it
 * as the scale of the rounding-error bound. */
int bq_oracle_bwd(const double *x, const double *dy, const float *theta, double *dx, double *dtheta,
                  double *absacc, long rows, int n, int heads)
{
    int k = ilog2_exact(n);
    if (k < 0 || heads < 1 || rows < 0) return -1;
    double *c, *s;
    cos_sin_tables(theta, n, k, heads, &c, &s);
    long w = (long)n * heads;
    size_t m = (size_t)heads * (size_t)k * (size_t)(n / 2);
    memset(dtheta, 0, m * sizeof(double));
    if (absacc) memset(absacc, 0, m * sizeof(double));
    /* Rows are split into contiguous chunks, one per thread; every thread sums its rows in order into
     * its own accumulator, and the accumulators are added in thread order afterwards: the result is
     * reproducible for a given thread count. */
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#endif
    if (nthreads > rows) nthreads = rows > 0 ? (int)rows : 1;
    double *acc_all = (double *)calloc((size_t)nthreads * m * (absacc ? 2 : 1), sizeof(double));
#pragma omp parallel num_threads(nthreads)
    {
        int tid = 0;
#ifdef _OPENMP
        tid = omp_get_thread_num();
#endif
        double *acc = acc_all + (size_t)tid * m * (absacc ? 2 : 1);
        double *aab = absacc ? acc + m : NULL;
        double *xs = (double *)malloc((size_t)(k + 1) * (size_t)n * sizeof(double));
        double *g = (double *)malloc((size_t)n * sizeof(double));
        long r0 = rows * tid / nthreads, r1 = rows * (tid + 1) / nthreads;
        for (long r = r0; r < r1; ++r) {
            for (int hd = 0; hd < heads; ++hd) {
                memcpy(xs, x + r * w + (long)hd * n, (size_t)n * sizeof(double));
                for (int i = 1; i <= k; ++i) {
                    size_t off = ((size_t)hd * k + (size_t)(i - 1)) * (size_t)(n / 2);
                    double *cur = xs + (size_t)i * n;
                    memcpy(cur, xs + (size_t)(i - 1) * n, (size_t)n * sizeof(double));
                    layer_apply(cur, c + off, s + off, n, i);
                }
                memcpy(g, dy + r * w + (long)hd * n, (size_t)n * sizeof(double));
                for (int i = k; i >= 1; --i) {
                    size_t off = ((size_t)hd * k + (size_t)(i - 1)) * (size_t)(n / 2);
                    const double *xin = xs + (size_t)(i - 1) * n;
                    long h = 1L << (i - 1);
                    for (long j = 0; j < n / 2; ++j) {
                        long a = pair_lo(j, i), b = a + h;
                        double cc = c[off + j], ss = s[off + j];
                        double da = -ss * xin[a] - cc * xin[b]; /* row 1 of dG/dtheta times x_{i-1} */
                        double db = cc * xin[a] - ss * xin[b];  /* row 2 */
                        acc[off + j] += g[a] * da + g[b] * db;
                        if (aab)
                            aab[off + j] += fabs(g[a] * ss * xin[a]) + fabs(g[a] * cc * xin[b]) +
                                            fabs(g[b] * cc * xin[a]) + fabs(g[b] * ss * xin[b]);
                    }
                    layer_apply_T(g, c + off, s + off, n, i);
                }
                memcpy(dx + r * w + (long)hd * n, g, (size_t)n * sizeof(double));
            }
        }
        free(xs);
        free(g);
    }
    for (int t = 0; t < nthreads; ++t) {
        const double *acc = acc_all + (size_t)t * m * (absacc ? 2 : 1);
        for (size_t q = 0; q < m; ++q) dtheta[q] += acc[q];
        if (absacc)
            for (size_t q = 0; q < m; ++q) absacc[q] += acc[m + q];
    }
    free(acc_all);
    free(c);
    free(s);
    return 0;
}

/* ------------------------------------------------------------------------------------------- */
/* float <-> IEEE binary16, round to nearest even, written out on the bits                      */

static uint16_t f32_to_f16_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t sign = (u >> 16) & 0x8000u;
    uint32_t ex = (u >> 23) & 0xFFu;
    uint32_t man = u & 0x7FFFFFu;
    if (ex == 0xFFu) return (uint16_t)(sign | 0x7C00u | (man ? 0x200u : 0u));
    int e = (int)ex - 127 + 15;
    if (e >= 31) return (uint16_t)(sign | 0x7C00u); /* overflow -> inf */
    if (e <= 0) {
        if (e < -10) return (uint16_t)sign; /* below half of the smallest subnormal -> 0 */
        man |= 0x800000u;
        int shift = 14 - e; /* 14..24 */
        uint32_t q = man >> shift;
        uint32_t rem = man & ((1u << shift) - 1u);
        uint32_t half = 1u << (shift - 1);
        if (rem > half || (rem == half && (q & 1u))) ++q;
        return (uint16_t)(sign | q);
    }
    uint32_t q = ((uint32_t)e << 10) | (man >> 13);
    uint32_t rem = man & 0x1FFFu;
    if (rem > 0x1000u || (rem == 0x1000u && (q & 1u))) ++q; /* may carry into the exponent: correct */
    return (uint16_t)(sign | q);
}

static float f16_bits_to_f32(uint16_t hbits)
{
    uint32_t sign = ((uint32_t)hbits & 0x8000u) << 16;
    int e = (hbits >> 10) & 0x1F;
    uint32_t man = hbits & 0x3FFu;
    float v;
    if (e == 0)
        v = ldexpf((float)man, -24);
    else if (e == 31)
        v = man ? NAN : INFINITY;
    else
        v = ldexpf((float)(man | 0x400u), e - 25);
    uint32_t u;
    memcpy(&u, &v, 4);
    u |= sign;
    memcpy(&v, &u, 4);
    return v;
}

uint16_t bq_oracle_f32_to_f16_bits(float f) { return f32_to_f16_bits(f); }
float bq_oracle_f16_bits_to_f32(uint16_t h) { return f16_bits_to_f32(h); }

/* Symmetric uniform quantiser (equation "Quant(x) = clip(round(x/s), -2^(b-1), 2^(b-1)-1)" with
 * s = max|x| / (2^(b-1)-1) per group).  A group is `group` consecutive channels of one row.
 * Every step is one correctly rounded float operation, in this order:
 *     amax = max_j |y_j|
 *     s    = amax / qmax                      (qmax = 2^(b-1)-1)
 *     if scales are stored as binary16: s = float(half_rne(s)), an overflow saturating to 65504
 *     inv  = (s == 0) ? 0 : 1 / s
 *     q_j  = clip(rint(y_j * inv), -2^(b-1), 2^(b-1)-1)     (rint = ties to even)
 * The stored scale is s.  codes: one int8 per element; scales: one float per group.
 * Returns 0, -1 on a bad argument. */
int bq_oracle_quant(const float *y, long rows, long width, int group, int bits, int scale_f16,
                    int8_t *codes, float *scales)
{
    if (bits < 2 || bits > 8 || group < 1 || width % group != 0 || rows < 0) return -1;
    const float qmax = (float)((1 << (bits - 1)) - 1);
    const float qmin = -(float)(1 << (bits - 1));
    long ng = width / group;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        for (long gi = 0; gi < ng; ++gi) {
            const float *v = y + r * width + gi * group;
            float amax = 0.0f;
            for (int j = 0; j < group; ++j) {
                float a = fabsf(v[j]);
                if (a > amax) amax = a;
            }
            float s = amax / qmax;
            if (scale_f16) {
                if (s > 65504.0f) s = 65504.0f;
                s = f16_bits_to_f32(f32_to_f16_bits(s));
            }
            float inv = (s == 0.0f) ? 0.0f : 1.0f / s;
            for (int j = 0; j < group; ++j) {
                float t = v[j] * inv;
                float q = rintf(t);
                if (q > qmax) q = qmax;
                if (q < qmin) q = qmin;
                codes[r * width + gi * group + j] = (int8_t)q;
            }
            scales[r * ng + gi] = s;
        }
    }
    return 0;
}

/* Dequant(q) = s * q (paper, "Loss Function"): one float multiplication per element, the group's stored
 * scale times the code.  yq: [rows][width] float.  Returns 0, -1 on a bad argument. */
int bq_oracle_dequant(const int8_t *codes, const float *scales, long rows, long width, int group, float *yq)
{
    if (group < 1 || width % group != 0 || rows < 0) return -1;
    long ng = width / group;
    for (long r = 0; r < rows; ++r)
        for (long j = 0; j < width; ++j)
            yq[r * width + j] = scales[r * ng + j / group] * (float)codes[r * width + j];
    return 0;
}

/* Occupancy of the 2^b quantisation bins (the empirical distribution P_bins of the uniformity
 * regulariser, before normalisation): hist[c] = number of codes equal to c - 2^(b-1). */
int bq_oracle_bin_histogram(const int8_t *codes, long count, int bits, uint64_t *hist)
{
    if (bits < 2 || bits > 8 || count < 0) return -1;
    int nb = 1 << bits, off = 1 << (bits - 1);
    for (int c = 0; c < nb; ++c) hist[c] = 0;
    for (long i = 0; i < count; ++i) {
        int c = (int)codes[i] + off;
        if (c < 0 || c >= nb) return -1;
        hist[c] += 1;
    }
    return 0;
}

/* L_uniform = D_KL(P_bins || U) = sum_c P_c log(P_c * 2^b), P_c = hist[c] / total, 0 log 0 = 0
 * (paper, "Uniformity Regularization"); natural logarithm. */
double bq_oracle_uniformity_kl(const uint64_t *hist, int bits)
{
    int nb = 1 << bits;
    double total = 0.0, kl = 0.0;
    for (int c = 0; c < nb; ++c) total += (double)hist[c];
    if (total == 0.0) return 0.0;
    for (int c = 0; c < nb; ++c) {
        double pc = (double)hist[c] / total;
        if (pc > 0.0) kl += pc * log(pc * (double)nb);
    }
    return kl;
}

/* Pack signed codes into bytes: two's-complement fields of `bits` bits, element j of a row in
 * bits [(j % per)*bits, ...) of byte j / per, per = 8 / bits (lowest-index element in the lowest
 * bits).  This layout is this project's choice; the paper does not define one. */
int bq_oracle_pack_codes(const int8_t *codes, long rows, long width, int bits, uint8_t *packed)
{
    if (!(bits == 2 || bits == 4 || bits == 8) || width % (8 / bits) != 0) return -1;
    int per = 8 / bits;
    unsigned mask = (1u << bits) - 1u;
    long wb = width / per;
    for (long r = 0; r < rows; ++r)
        for (long q = 0; q < wb; ++q) {
            unsigned byte = 0;
            for (int e = 0; e < per; ++e)
                byte |= ((unsigned)codes[r * width + q * per + e] & mask) << (e * bits);
            packed[r * wb + q] = (uint8_t)byte;
        }
    return 0;
}

int bq_oracle_num_threads(void)
{
    int nt = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        nt = omp_get_num_threads();
    }
#endif
    return nt;
}
