/*
 * CPU oracle for the 8-bit floating point training primitive of
 * "Mixed Precision Training With 8-bit Floating Point" (arXiv 1905.12334).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously
 * correct statement of what the GPU library must compute.  It is written in
 * double precision with <math.h> only, shares no code, header, table or helper
 * with the HIP library, and may be used only by the tests, the smoke check and
 * the cpu_baseline leg of the benchmark.
 *
 * Every function names the passage of the paper it follows.  Where the paper is
 * silent or garbled the reading taken is stated next to the code.
 *
 * Build:  gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC mp8_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

#define ORC_RNE 0
#define ORC_SR 1
#define ORC_FLAG_SATURATE 1

typedef struct {
    uint32_t amax_bits; /* max over elements of the FP32 bit pattern of |y|      */
    uint32_t nonfinite; /* outputs that are an Inf or NaN code                   */
    uint32_t zeroed;    /* inputs with y != 0 whose output code is +0 or -0      */
    uint32_t rsvd;
} orc_stats;

/* ------------------------------------------------------------------------- */
/* Number formats (Section 3, Table 1)                                        */
/* ------------------------------------------------------------------------- */

/*
 * Value of a sign / 5-bit exponent / `mbits`-bit mantissa code.
 * Section 3 fixes the 8-bit format as (s,e,m) = (1,5,2); Table 1 prints
 * max normal 57344, min normal 6.10e-5 and min subnormal 1.52e-5 for it, and the
 * IEEE half row (1,5,10) next to it.  Those three numbers force bias 15, gradual
 * underflow and a reserved top exponent (Inf / NaN): without the reserved
 * exponent the maximum would be 114688.  Both formats are therefore decoded by
 * the same IEEE rule, with mbits = 2 or 10.
 */
static double small_float_decode(uint32_t code, int mbits)
{
    uint32_t mmask = (1u << mbits) - 1u;
    uint32_t m = code & mmask;
    uint32_t e = (code >> mbits) & 31u;
    uint32_t s = (code >> (mbits + 5)) & 1u;
    double v;
    if (e == 31u)
        v = (m == 0u) ? INFINITY : NAN;
    else if (e == 0u)
        v = ldexp((double)m, -14 - mbits); /* subnormal: m * 2^(1-15-mbits) */
    else
        v = ldexp((double)((1u << mbits) + m), (int)e - 15 - mbits);
    return s ? -v : v;
}

double orc_e5m2_decode(uint8_t code) { return small_float_decode(code, 2); }
double orc_fp16_decode(uint16_t code) { return small_float_decode(code, 10); }

/*
 * Round a finite magnitude ax >= 0 onto the (5-bit exponent, mbits mantissa) grid
 * and return the magnitude code.  May return the Inf code (31 << mbits).
 *
 * Grid: with e = floor(log2 ax), the spacing around ax is 2^(max(e,-14) - mbits)
 * (fixed spacing 2^(-14-mbits) in the subnormal range).  lo = spacing * floor(ax /
 * spacing) is the neighbour toward zero and lo + spacing the one away from zero;
 * above the largest normal the "away" neighbour is the would-be 2^16, which the
 * format spells Inf.
 *
 * mode ORC_RNE (Section 3.2, round to nearest even): nearest neighbour, a tie goes
 * to the neighbour whose code is even.  One rounding, straight from the source
 * value.
 *
 * mode ORC_SR (Section 3.2, the two-case definition of round(x,k)): the printed
 * formula puts the random draw r inside the probability.  Reading taken: epsilon
 * is the grid spacing at x, r is uniform on [0,1), and the value goes to the
 * neighbour away from zero exactly when (|x| - lo)/epsilon + r >= 1, which happens
 * with probability (|x| - lo)/epsilon, so the expectation is x.  r is supplied as
 * a 16-bit integer r16 (r = r16 / 65536) and the fraction is truncated to 16 bits:
 * F = floor((|x| - lo)/epsilon * 65536); up  <=>  F + r16 >= 65536.
 * Rounding acts on the magnitude; the sign is kept by the caller.
 *
 * Because codes of one sign are ordered like their values, "lo's code + 1" is the
 * code of the neighbour away from zero, across binade and subnormal/normal
 * boundaries and into Inf.
 */
static uint32_t grid_round_mag(double ax, int mbits, int mode, uint32_t r16)
{
    const uint32_t inf_code = 31u << mbits;
    int e;
    double q, n, frac;
    uint32_t code;
    int up;

    if (ax == 0.0)
        return 0u;
    (void)frexp(ax, &e); /* ax = f * 2^e, f in [0.5,1)  =>  floor(log2 ax) = e-1 */
    e -= 1;
    if (e > 15)
        return inf_code; /* ax >= 65536: beyond the virtual top neighbour */
    {
        int eq = (e < -14 ? -14 : e) - mbits; /* log2 of the spacing */
        q = ldexp(ax, -eq);                   /* exact: power-of-two scaling */
    }
    n = floor(q);
    frac = q - n; /* exact */
    if (e < -14)
        code = (uint32_t)n; /* subnormal: code is the integer count of quanta */
    else
        code = ((uint32_t)(e + 15) << mbits) + ((uint32_t)n - (1u << mbits));
    if (mode == ORC_RNE) {
        up = (frac > 0.5) || (frac == 0.5 && (((uint32_t)n) & 1u));
    } else {
        uint32_t F = (uint32_t)floor(frac * 65536.0);
        up = (F + (r16 & 0xFFFFu)) >= 65536u;
    }
    return code + (uint32_t)up;
}

/*
 * Double -> E5M2 code.  NaN -> 0x7F, one canonical code whatever the sign or payload
 * of the source NaN (a convention of this build: processors differ in the NaN they
 * produce); +-Inf stays Inf (also when saturating); finite values that round to or
 * beyond the Inf code give Inf, or the largest normal 57344 (0x7B) when `saturate`
 * is set.  The paper does not say what
 * overflow does; IEEE (non-saturating) is the default here because its dynamic
 * loss scaling (Section 3.1) works by detecting overflow.
 */
uint8_t orc_e5m2_encode(double y, int mode, uint32_t r16, int saturate)
{
    uint32_t s = signbit(y) ? 0x80u : 0u;
    uint32_t mag;
    if (isnan(y))
        return (uint8_t)0x7Fu;
    if (isinf(y))
        return (uint8_t)(s | 0x7Cu);
    mag = grid_round_mag(fabs(y), 2, mode, r16);
    if (mag >= 0x7Cu)
        mag = saturate ? 0x7Bu : 0x7Cu;
    return (uint8_t)(s | mag);
}

/* Double -> IEEE half code, same rule on the 10-bit-mantissa grid (no saturation). */
uint16_t orc_fp16_encode(double y, int mode, uint32_t r16)
{
    uint32_t s = signbit(y) ? 0x8000u : 0u;
    uint32_t mag;
    if (isnan(y))
        return (uint16_t)0x7E00u; /* canonical quiet NaN */
    if (isinf(y))
        return (uint16_t)(s | 0x7C00u);
    mag = grid_round_mag(fabs(y), 10, mode, r16);
    if (mag >= 0x7C00u)
        mag = 0x7C00u;
    return (uint16_t)(s | mag);
}

/* ------------------------------------------------------------------------- */
/* Random numbers for stochastic rounding                                     */
/* ------------------------------------------------------------------------- */

/*
 * Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).  Section 3.2 leaves
 * the generator behind its random value r open; a counter-based one is used so
 * that a result depends on (seed, offset, element index) alone.
 */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    int round;
    for (round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * The 16 random bits of the element with row-major linear index i of a tensor:
 * key = (seed low, seed high); counter = (low32(i/8), high32(i/8), low32(offset),
 * high32(offset)); the call gives four words, i.e. eight halfwords, and element i
 * takes halfword i mod 8 (low half of a word first).  `offset` tells calls apart.
 * This layout is a convention of this build, not of the paper.
 */
uint32_t orc_sr_bits(uint64_t seed, uint64_t offset, uint64_t i)
{
    uint32_t ctr[4], key[2], w[4];
    uint64_t blk = i >> 3;
    uint32_t h = (uint32_t)(i & 7u);
    ctr[0] = (uint32_t)blk;
    ctr[1] = (uint32_t)(blk >> 32);
    ctr[2] = (uint32_t)offset;
    ctr[3] = (uint32_t)(offset >> 32);
    key[0] = (uint32_t)seed;
    key[1] = (uint32_t)(seed >> 32);
    orc_philox4x32_10(ctr, key, w);
    return (w[h >> 1] >> (16u * (h & 1u))) & 0xFFFFu;
}

/* ------------------------------------------------------------------------- */
/* Q node: FP32 -> E5M2 (Section 3, Figure 1a)                                */
/* ------------------------------------------------------------------------- */

static uint32_t f32_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return u;
}

/*
 * dst[i] = Q(fl32(src[i] * scale)) for a row-major [rows, cols] tensor; dst_t, if
 * given, receives the same codes transposed ([cols, rows]).  The multiply is one
 * IEEE single-precision multiply (this is where the loss scale of Section 3.1 is
 * applied to errors); rounding happens once, on that product.  src is FP32, or
 * IEEE half codes when src_is_f16 is set.  stats, if given, is accumulated into.
 */
void orc_quantize_e5m2(const void *src, int src_is_f16, uint8_t *dst, uint8_t *dst_t,
                       int64_t rows, int64_t cols, float scale, int mode, int flags,
                       uint64_t seed, uint64_t offset, orc_stats *stats)
{
    int64_t n = rows * cols, i;
    uint32_t amax = stats ? stats->amax_bits : 0u;
    uint32_t nonfinite = 0u, zeroed = 0u;
#pragma omp parallel for reduction(max : amax) reduction(+ : nonfinite, zeroed)
    for (i = 0; i < n; ++i) {
        float x = src_is_f16 ? (float)orc_fp16_decode(((const uint16_t *)src)[i])
                             : ((const float *)src)[i];
        volatile float y = x * scale;
        uint32_t r16 = (mode == ORC_SR) ? orc_sr_bits(seed, offset, (uint64_t)i) : 0u;
        uint8_t c = orc_e5m2_encode((double)y, mode, r16, flags & ORC_FLAG_SATURATE);
        /* |y| as a bit pattern; every NaN counts as the canonical 0x7FC00000 */
        uint32_t ab = isnan(y) ? 0x7FC00000u : (f32_bits(y) & 0x7FFFFFFFu);
        dst[i] = c;
        if (dst_t)
            dst_t[(i % cols) * rows + (i / cols)] = c;
        if (ab > amax)
            amax = ab;
        if ((c & 0x7Cu) == 0x7Cu)
            nonfinite++;
        if ((c & 0x7Fu) == 0u && ab != 0u)
            zeroed++;
    }
    if (stats) {
        stats->amax_bits = amax;
        stats->nonfinite += nonfinite;
        stats->zeroed += zeroed;
    }
}

/* FP32 -> IEEE half over an array, element i using the random bits of index i. */
void orc_fp16_encode_array(const float *src, int64_t n, int mode, uint64_t seed,
                           uint64_t offset, uint16_t *dst)
{
    int64_t i;
#pragma omp parallel for
    for (i = 0; i < n; ++i) {
        uint32_t r16 = (mode == ORC_SR) ? orc_sr_bits(seed, offset, (uint64_t)i) : 0u;
        dst[i] = orc_fp16_encode((double)src[i], mode, r16);
    }
}

/* ------------------------------------------------------------------------- */
/* GEMM reference (Section 3: two FP8 tensors in, wide accumulator)           */
/* ------------------------------------------------------------------------- */

/*
 * ref[r,c] = sum_j a[r,j] * b[c,j] over the contraction index j in increasing
 * order, every operand decoded exactly and the sum kept in double;
 * absref[r,c] = sum_j |a[r,j]| * |b[c,j]|.  Both operands are given with the
 * contraction index contiguous (a: [rows, kc] leading dim lda; b: [cols, kc]
 * leading dim ldb).  If row_idx is non-NULL only those nrows rows of the output
 * are computed and ref/absref are [nrows, cols].
 */
void orc_gemm_ref(const uint8_t *a, int64_t lda, const uint8_t *b, int64_t ldb,
                  int64_t rows, int64_t cols, int64_t kc, const int64_t *row_idx,
                  int64_t nrows, double *ref, double *absref)
{
    double table[256];
    int64_t t, count = row_idx ? nrows : rows;
    int c;
    for (c = 0; c < 256; ++c)
        table[c] = orc_e5m2_decode((uint8_t)c);
#pragma omp parallel for schedule(dynamic, 1)
    for (t = 0; t < count; ++t) {
        int64_t r = row_idx ? row_idx[t] : t;
        const uint8_t *ar = a + r * lda;
        int64_t cc, j;
        for (cc = 0; cc < cols; ++cc) {
            const uint8_t *bc = b + cc * ldb;
            double s = 0.0, sa = 0.0;
            for (j = 0; j < kc; ++j) {
                double p = table[ar[j]] * table[bc[j]];
                s += p;
                sa += fabs(p);
            }
            ref[t * cols + cc] = s;
            if (absref)
                absref[t * cols + cc] = sa;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* 3x3 convolution reference (Section 3 puts every convolution and GEMM        */
/* kernel in the 8-bit format; Section 4: the ResNet layers)                   */
/* ------------------------------------------------------------------------- */

/*
 * The paper applies the 8-bit primitive to convolutions as it does to GEMMs but
 * does not restate the operation; the reading taken is the one of the residual
 * networks it trains: stride 1, zero padding 1, cross-correlation (no kernel
 * flip), activations stored [B, H, W, C] (channel fastest), weights
 * [3, 3, Cin, Cout].  All three functions decode the codes exactly, sum in double
 * in the index order written below, and also return the sum of absolute products.
 *
 *   forward        y[b,h,w,co]    = sum_{r,s,ci} x[b,h+r-1,w+s-1,ci] * wt[r,s,ci,co]
 *   backward data  dx[b,h,w,ci]   = sum_{r,s,co} e[b,h-r+1,w-s+1,co] * wt[r,s,ci,co]
 *   weight grad    dw[r,s,ci,co]  = sum_{b,h,w}  x[b,h+r-1,w+s-1,ci] * e[b,h,w,co]
 * with every out-of-range pixel read as zero.  Backward data and weight gradient
 * are the derivatives of sum(y * e) with respect to x and wt.
 */
static void conv_tables(double *table)
{
    int c;
    for (c = 0; c < 256; ++c)
        table[c] = orc_e5m2_decode((uint8_t)c);
}

void orc_conv3x3_fwd_ref(const uint8_t *x, const uint8_t *wt, int64_t B, int64_t H, int64_t W,
                         int64_t Ci, int64_t Co, double *ref, double *absref)
{
    double table[256];
    int64_t pix;
    conv_tables(table);
#pragma omp parallel for schedule(dynamic, 16)
    for (pix = 0; pix < B * H * W; ++pix) {
        int64_t b = pix / (H * W), h = (pix / W) % H, w = pix % W, co;
        for (co = 0; co < Co; ++co) {
            double s = 0.0, sa = 0.0;
            int r, t;
            for (r = 0; r < 3; ++r)
                for (t = 0; t < 3; ++t) {
                    int64_t hh = h + r - 1, ww = w + t - 1, ci;
                    if (hh < 0 || hh >= H || ww < 0 || ww >= W)
                        continue;
                    for (ci = 0; ci < Ci; ++ci) {
                        double p = table[x[((b * H + hh) * W + ww) * Ci + ci]] *
                                   table[wt[((r * 3 + t) * Ci + ci) * Co + co]];
                        s += p;
                        sa += fabs(p);
                    }
                }
            ref[pix * Co + co] = s;
            if (absref)
                absref[pix * Co + co] = sa;
        }
    }
}

void orc_conv3x3_bwd_data_ref(const uint8_t *e, const uint8_t *wt, int64_t B, int64_t H,
                              int64_t W, int64_t Ci, int64_t Co, double *ref, double *absref)
{
    double table[256];
    int64_t pix;
    conv_tables(table);
#pragma omp parallel for schedule(dynamic, 16)
    for (pix = 0; pix < B * H * W; ++pix) {
        int64_t b = pix / (H * W), h = (pix / W) % H, w = pix % W, ci;
        for (ci = 0; ci < Ci; ++ci) {
            double s = 0.0, sa = 0.0;
            int r, t;
            for (r = 0; r < 3; ++r)
                for (t = 0; t < 3; ++t) {
                    int64_t hh = h - r + 1, ww = w - t + 1, co;
                    if (hh < 0 || hh >= H || ww < 0 || ww >= W)
                        continue;
                    for (co = 0; co < Co; ++co) {
                        double p = table[e[((b * H + hh) * W + ww) * Co + co]] *
                                   table[wt[((r * 3 + t) * Ci + ci) * Co + co]];
                        s += p;
                        sa += fabs(p);
                    }
                }
            ref[pix * Ci + ci] = s;
            if (absref)
                absref[pix * Ci + ci] = sa;
        }
    }
}

void orc_conv3x3_wgrad_ref(const uint8_t *x, const uint8_t *e, int64_t B, int64_t H, int64_t W,
                           int64_t Ci, int64_t Co, double *ref, double *absref)
{
    double table[256];
    int64_t row;
    conv_tables(table);
#pragma omp parallel for schedule(dynamic, 4)
    for (row = 0; row < 9 * Ci; ++row) {
        int64_t tap = row / Ci, ci = row % Ci, r = tap / 3, t = tap % 3, co;
        for (co = 0; co < Co; ++co) {
            double s = 0.0, sa = 0.0;
            int64_t b, h, w;
            for (b = 0; b < B; ++b)
                for (h = 0; h < H; ++h)
                    for (w = 0; w < W; ++w) {
                        int64_t hh = h + r - 1, ww = w + t - 1;
                        double p;
                        if (hh < 0 || hh >= H || ww < 0 || ww >= W)
                            continue;
                        p = table[x[((b * H + hh) * W + ww) * Ci + ci]] *
                            table[e[((b * H + h) * W + w) * Co + co]];
                        s += p;
                        sa += fabs(p);
                    }
            ref[row * Co + co] = s;
            if (absref)
                absref[row * Co + co] = sa;
        }
    }
}

/*
 * Exact dot products for small cases.  Every finite E5M2 value is an integer
 * multiple of 2^-16 below 2^32 in those units, so each product is an integer
 * below 2^64 in units of 2^-32 and a 128-bit integer holds any sum of them.
 * out_hi/out_lo receive the two's-complement 128-bit sum (value = sum * 2^-32).
 * Returns the number of output elements that met a non-finite operand code
 * (their sums are left as zero).
 */
int64_t orc_gemm_exact(const uint8_t *a, int64_t lda, const uint8_t *b, int64_t ldb,
                       int64_t rows, int64_t cols, int64_t kc, int64_t *out_hi,
                       uint64_t *out_lo)
{
    int64_t r, c, j, bad = 0;
    for (r = 0; r < rows; ++r) {
        for (c = 0; c < cols; ++c) {
            __int128 s = 0;
            int nonfinite = 0;
            for (j = 0; j < kc; ++j) {
                double va = orc_e5m2_decode(a[r * lda + j]);
                double vb = orc_e5m2_decode(b[c * ldb + j]);
                if (!isfinite(va) || !isfinite(vb)) {
                    nonfinite = 1;
                    break;
                }
                {
                    int64_t ia = (int64_t)ldexp(va, 16); /* exact integers */
                    int64_t ib = (int64_t)ldexp(vb, 16);
                    s += (__int128)ia * (__int128)ib;
                }
            }
            if (nonfinite) {
                s = 0;
                bad++;
            }
            out_hi[r * cols + c] = (int64_t)(s >> 64);
            out_lo[r * cols + c] = (uint64_t)s;
        }
    }
    return bad;
}

/* out[i] = Q(alpha * ref[i]) straight from the double reference, RNE. */
void orc_round_ref_e5m2(const double *ref, int64_t n, double alpha, int flags, uint8_t *out)
{
    int64_t i;
    for (i = 0; i < n; ++i)
        out[i] = orc_e5m2_encode(alpha * ref[i], ORC_RNE, 0u, flags & ORC_FLAG_SATURATE);
}

/* ------------------------------------------------------------------------- */
/* Master-weight update (Section 3, Figure 1b)                                */
/* ------------------------------------------------------------------------- */

/*
 * Per element, in the order the paper gives for the weight-update path:
 *   g   = fl32(value(g8) * inv_loss_scale)      un-scale in full precision
 *   w   = value(w16) as FP32                    half -> single is exact
 *   w'  = fmaf(-lr, g, w)                       the update is a 32-bit operation
 *   w16 = half(w')  rounded by `mode`           stored back as 16 bits
 * The paper does not name the rounding of the final store nor the operation
 * order; one fused multiply-add and a selectable RNE / stochastic store are the
 * readings taken.  Division by the loss scale is a multiply by the caller's
 * reciprocal.  If *skip is non-zero nothing is changed (overflow step skipped).
 * w8_out, if given, receives Q_RNE of the new half weight (the next step's W8).
 * stats->nonfinite counts Inf/NaN gradient codes.
 */
void orc_sgd_update_fp16(uint16_t *w16, const uint8_t *g8, int64_t n, float lr,
                         float inv_loss_scale, int mode, uint64_t seed, uint64_t offset,
                         const uint32_t *skip, uint8_t *w8_out, orc_stats *stats)
{
    int64_t i;
    uint32_t nonfinite = 0u;
#pragma omp parallel for reduction(+ : nonfinite)
    for (i = 0; i < n; ++i)
        if ((g8[i] & 0x7Cu) == 0x7Cu)
            nonfinite++;
    if (stats)
        stats->nonfinite += nonfinite;
    if (skip && *skip != 0u)
        return;
#pragma omp parallel for
    for (i = 0; i < n; ++i) {
        volatile float g = (float)orc_e5m2_decode(g8[i]) * inv_loss_scale;
        float w = (float)orc_fp16_decode(w16[i]);
        float wn = fmaf(-lr, g, w);
        uint32_t r16 = (mode == ORC_SR) ? orc_sr_bits(seed, offset, (uint64_t)i) : 0u;
        uint16_t h = orc_fp16_encode((double)wn, mode, r16);
        w16[i] = h;
        if (w8_out)
            w8_out[i] = orc_e5m2_encode(orc_fp16_decode(h), ORC_RNE, 0u, 0);
    }
}

/*
 * The same path with the momentum optimizer that Figure 1b draws between the
 * un-scaled gradient and the master weights, and the L2 regularisation term of
 * Eq. 1 (loss + lambda * sum w^2, whose gradient 2 * lambda * w enters as
 * weight_decay * w):
 *   g   = fl32(value(g8) * inv_loss_scale)
 *   w   = value(w16) as FP32
 *   g   = fmaf(weight_decay, w, g)              regularisation gradient
 *   v'  = fmaf(momentum, v, g)                  velocity, kept in FP32
 *   w'  = fmaf(-lr, v', w)
 *   w16 = half(w') rounded by `mode`
 * The paper does not give the precision of the velocity; FP32 is the reading
 * taken (Section 3 carries out the whole update path in 32 bits).  With
 * momentum = 0 and weight_decay = 0 this is orc_sgd_update_fp16 exactly.
 */
void orc_sgd_momentum_fp16(uint16_t *w16, float *vel, const uint8_t *g8, int64_t n, float lr,
                           float inv_loss_scale, float momentum, float weight_decay, int mode,
                           uint64_t seed, uint64_t offset, const uint32_t *skip,
                           uint8_t *w8_out, orc_stats *stats)
{
    int64_t i;
    uint32_t nonfinite = 0u;
#pragma omp parallel for reduction(+ : nonfinite)
    for (i = 0; i < n; ++i)
        if ((g8[i] & 0x7Cu) == 0x7Cu)
            nonfinite++;
    if (stats)
        stats->nonfinite += nonfinite;
    if (skip && *skip != 0u)
        return;
#pragma omp parallel for
    for (i = 0; i < n; ++i) {
        volatile float g0 = (float)orc_e5m2_decode(g8[i]) * inv_loss_scale;
        float w = (float)orc_fp16_decode(w16[i]);
        float g = fmaf(weight_decay, w, g0);
        float v = fmaf(momentum, vel[i], g);
        float wn = fmaf(-lr, v, w);
        uint32_t r16 = (mode == ORC_SR) ? orc_sr_bits(seed, offset, (uint64_t)i) : 0u;
        uint16_t h = orc_fp16_encode((double)wn, mode, r16);
        vel[i] = v;
        w16[i] = h;
        if (w8_out)
            w8_out[i] = orc_e5m2_encode(orc_fp16_decode(h), ORC_RNE, 0u, 0);
    }
}

/*
 * The same path with the ADAM optimizer, which Section 4 names for the
 * translation networks (GNMT, Transformer).  The paper gives no formula; this
 * is the published algorithm (Kingma & Ba, Algorithm 1) with the L2
 * regularisation gradient of Eq. 1 added to the un-scaled gradient as in
 * orc_sgd_momentum_fp16.  Every operation is a separately rounded FP32
 * operation (Section 3 carries out the weight update in 32 bits), the two
 * moments are kept in FP32 (the paper is
 * silent on the precision of optimizer state; same reading as the velocity):
 *   g    = fl32(value(g8) * inv_loss_scale);  w = value(w16)
 *   g    = fmaf(weight_decay, w, g)
 *   m'   = fmaf(beta1, m, fl32((1 - beta1) * g))
 *   v'   = fmaf(beta2, v, fl32((1 - beta2) * fl32(g * g)))
 *   mhat = m' / c1,  vhat = v' / c2     c_i = fl32(1 - beta_i^step), step >= 1
 *   w'   = fmaf(-lr, mhat / (sqrt(vhat) + eps), w)
 *   w16  = half(w') rounded by `mode`
 * (1 - beta_i) is the FP32 difference; beta_i^step is taken in double.
 */
void orc_adam_fp16(uint16_t *w16, float *m, float *v, const uint8_t *g8, int64_t n, float lr,
                   float inv_loss_scale, float beta1, float beta2, float eps, float weight_decay,
                   int64_t step, int mode, uint64_t seed, uint64_t offset, const uint32_t *skip,
                   uint8_t *w8_out, orc_stats *stats)
{
    int64_t i;
    uint32_t nonfinite = 0u;
    const float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
    const float c1 = (float)(1.0 - pow((double)beta1, (double)step));
    const float c2 = (float)(1.0 - pow((double)beta2, (double)step));
#pragma omp parallel for reduction(+ : nonfinite)
    for (i = 0; i < n; ++i)
        if ((g8[i] & 0x7Cu) == 0x7Cu)
            nonfinite++;
    if (stats)
        stats->nonfinite += nonfinite;
    if (skip && *skip != 0u)
        return;
#pragma omp parallel for
    for (i = 0; i < n; ++i) {
        volatile float g0 = (float)orc_e5m2_decode(g8[i]) * inv_loss_scale;
        float w = (float)orc_fp16_decode(w16[i]);
        float g = fmaf(weight_decay, w, g0);
        volatile float t1 = omb1 * g;
        volatile float gg = g * g;
        volatile float t2 = omb2 * gg;
        float mn = fmaf(beta1, m[i], t1);
        float vn = fmaf(beta2, v[i], t2);
        volatile float mhat = mn / c1;
        volatile float vhat = vn / c2;
        volatile float root = sqrtf(vhat);
        volatile float den = root + eps;
        volatile float upd = mhat / den;
        float wn = fmaf(-lr, upd, w);
        uint32_t r16 = (mode == ORC_SR) ? orc_sr_bits(seed, offset, (uint64_t)i) : 0u;
        uint16_t h = orc_fp16_encode((double)wn, mode, r16);
        m[i] = mn;
        v[i] = vn;
        w16[i] = h;
        if (w8_out)
            w8_out[i] = orc_e5m2_encode(orc_fp16_decode(h), ORC_RNE, 0u, 0);
    }
}

/* ------------------------------------------------------------------------- */
/* Loss scaler (Section 3.1)                                                  */
/* ------------------------------------------------------------------------- */

typedef struct {
    double scale;            /* current loss scale                               */
    double floor;            /* the caller-raised minimum threshold              */
    int64_t growth_interval; /* clean steps before the scale doubles             */
    int64_t good_steps;      /* clean steps since the last change                */
} orc_scaler;

/*
 * Back-off dynamic loss scaling with a minimum threshold.  The paper gives the
 * idea (halve on overflow, grow again after a while, and never go below a floor
 * that the user raises as training proceeds) but no constants; taken here:
 * overflow -> scale = max(scale/2, floor), step skipped, counter reset;
 * growth_interval clean steps in a row -> scale = min(2 * scale, 2^32): growth
 * stops at 2^32 (an overflow-free run would otherwise double without end; up to
 * there the scale and its reciprocal are exact single-precision numbers, and
 * with the smallest 8-bit subnormal at 2^-16 a larger scale could only rescue
 * errors below 2^-48).  Returns 1 if the step must be skipped.
 */
#define ORC_SCALER_MAX 4294967296.0
int orc_scaler_update(orc_scaler *s, uint32_t nonfinite)
{
    if (nonfinite != 0u) {
        s->scale = s->scale / 2.0;
        if (s->scale < s->floor)
            s->scale = s->floor;
        s->good_steps = 0;
        return 1;
    }
    s->good_steps += 1;
    if (s->good_steps >= s->growth_interval) {
        if (s->scale < ORC_SCALER_MAX) {   /* a floor above the limit is left alone */
            s->scale *= 2.0;
            if (s->scale > ORC_SCALER_MAX)
                s->scale = ORC_SCALER_MAX;
        }
        s->good_steps = 0;
    }
    return 0;
}

void orc_scaler_set_floor(orc_scaler *s, double floor_value)
{
    s->floor = floor_value;
    if (s->scale < floor_value)
        s->scale = floor_value;
}
