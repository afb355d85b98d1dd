/*
 * CPU oracle for the 2:4 semi-structured-sparse convolution.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the GPU library is
 * checked against.  Only the tests, the smoke check and the benchmark's CPU-baseline leg may
 * call it; the product path never does.  It shares no code, header, table or helper with the
 * HIP sources.
 *
 * What it follows (paper: "Inducing Semi-Structured Sparsity by Masking for Efficient Model
 * Inference in Convolutional Networks"):
 *   - Sec. 3.1, Eq. (2): the mask M is row-major, tiled left to right by blocks of 4 contiguous
 *     entries, each block holding exactly two ones (N:M sparsity with N=2, M=4; six patterns).
 *   - Fig. 1: the structured representation keeps only the surviving values plus a 2-bit
 *     position index for each of them.
 *   - Sec. 3.3, Eq. (4): direct 2-D convolution with zero padding (a cross-correlation: the
 *     input index is the sum of the output index and the kernel offset).
 *   - Sec. 3.3, Eq. (6): the masked convolution is the convolution with M (.) W in place of W.
 *
 * Arithmetic: inputs are the exact values of their fp16 / bf16 bit patterns; every product and
 * the running sum are fp64; the bias is fp32 widened to fp64; the result is NOT rounded.
 *
 * Tail of a layer (the paper's layer model sigma(Wx + b), Lemma 3.1, inside a residual block):
 * z = conv + bias + residual (the residual is a 16-bit NHWC tensor of the output's shape, taken
 * at its exact value), then act(z): identity, ReLU max(z, 0), or GELU z * Phi(z) with the exact
 * standard normal CDF Phi(z) = (1 + erf(z / sqrt 2)) / 2.
 *
 * Weight matrices are [cout][K] with K = cin*kh*kw and one of two flattenings of (c, r, t):
 *   korder 0 ("CRS", the paper's: channel slowest, kernel column fastest)  k = (c*kh + r)*kw + t
 *   korder 1 ("RSC", channels-last flattening)                             k = (r*kw + t)*cin + c
 * Activations are NHWC, outputs are NHWC.
 *
 * Parity pins (tests, CPU only): unfold+matmul (Eq. 5) in numpy, a float64 library conv,
 * one-hot-kernel shifts, all-ones closed forms, linearity, 1x1 == matmul, brute-force over the
 * six patterns, round trip, byte count 9/16; the tail by W = 0 closed forms, the identity
 * gelu(z) - gelu(-z) = z, tabulated values of Phi, and a library normal CDF.  No function here
 * is "parity unpinned".  The weight update's rounding is pinned against numpy's float16 and torch's bfloat16
 * conversions (all 65536 patterns x a spread of addends: ties, carries, subnormals, overflow).
 * The 8-bit integer functions are pinned against an int64 unfold + matmul in numpy, a float64 library convolution
 * (exact on these integers), the 16-bit functions above on the same small integers, and closed forms.
 * The FP8 functions are pinned by a library's E4M3 conversion on all 256 bytes, closed-form values, and the binary16
 * functions above on the same values (every E4M3 value is exact in binary16).
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <stdlib.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* dtype: 0 = IEEE binary16, 1 = bfloat16.  Exact widening of a 16-bit pattern to double. */
double ss_oracle_bits_to_double(uint16_t bits, int dtype)
{
    if (dtype == 1) {
        uint32_t u = ((uint32_t)bits) << 16;
        float f;
        memcpy(&f, &u, sizeof f);
        return (double)f;
    }
    int sign = (bits >> 15) & 1;
    int expo = (bits >> 10) & 0x1f;
    int frac = bits & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);            /* subnormal: frac * 2^-10 * 2^-14 */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(frac + 1024), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
    }
    return sign ? -v : v;
}

/* Round-to-nearest-even of a float to a 16-bit pattern (dtype 0: binary16, 1: bfloat16), done on the bits so that
 * it does not depend on the compiler's half-precision support.  A NaN maps to a quiet NaN of the same sign. */
static uint16_t float_to_bits16(float f, int dtype)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    uint32_t sign = u >> 31, mag = u & 0x7fffffffu;
    if (dtype == 1) {
        if (mag > 0x7f800000u) return (uint16_t)((sign << 15) | 0x7fc0u);
        uint32_t r = mag + 0x7fffu + ((mag >> 16) & 1u);           /* ties to even on the kept bit */
        return (uint16_t)((sign << 15) | (r >> 16));
    }
    if (mag > 0x7f800000u) return (uint16_t)((sign << 15) | 0x7e00u);
    if (mag >= 0x47800000u) return (uint16_t)((sign << 15) | 0x7c00u);   /* >= 65536, or infinity */
    if (mag < 0x33000000u) return (uint16_t)(sign << 15);                  /* < 2^-25: rounds to zero */
    int e = (int)(mag >> 23) - 127;                     /* unbiased exponent, -25 .. 15 */
    uint32_t m = (mag & 0x7fffffu) | 0x800000u;         /* 24-bit significand with the hidden one */
    /* binary16 keeps 10 fraction bits for e >= -14; below that the value is a multiple of 2^-24 */
    int drop = (e >= -14) ? 13 : (13 + (-14 - e));      /* low bits of m to round away (13 .. 24) */
    uint32_t kept = m >> drop;
    uint32_t rem = m & ((1u << drop) - 1u), half = 1u << (drop - 1);
    if (rem > half || (rem == half && (kept & 1u))) kept++;
    uint32_t bits;
    if (e >= -14)
        bits = ((uint32_t)(e + 15) << 10) + (kept - 0x400u);   /* a carry out of the significand bumps the exponent */
    else
        bits = kept;                                            /* subnormal (or the smallest normal after a carry) */
    if (bits >= 0x7c00u) bits = 0x7c00u;                        /* rounded up to infinity */
    return (uint16_t)((sign << 15) | bits);
}

/* Weight update in the storage type (Sec. 3.2, combined effect of masking and updating: the model moves to
 * V = W + U and keeps its mask): V[i] = round16( float(W[i]) + float(U[i]) ), the sum taken in binary32 (itself
 * rounded to nearest even) as a framework adding two 16-bit tensors does.  In place over W. */
void ss_oracle_update(uint16_t *W, const uint16_t *U, int64_t n, int dtype)
{
    for (int64_t i = 0; i < n; i++) {
        float a = (float)ss_oracle_bits_to_double(W[i], dtype);    /* exact: every 16-bit value is a float */
        float b = (float)ss_oracle_bits_to_double(U[i], dtype);
        volatile float sum = a + b;                                 /* one binary32 rounding, no wider intermediate */
        W[i] = float_to_bits16(sum, dtype);
    }
}

int ss_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sec. 3.1 / Eq. (2): every block of 4 consecutive entries of a row of M holds exactly two
 * ones and every entry is 0 or 1.  Returns 0 if valid, else 1 and the first offending
 * (row, group) in row-major order. */
int ss_oracle_mask_check(const uint8_t *M, int64_t cout, int64_t K, int64_t *bad_row, int64_t *bad_group)
{
    if (K % 4 != 0) {
        if (bad_row) *bad_row = -1;
        if (bad_group) *bad_group = -1;
        return 2;
    }
    for (int64_t o = 0; o < cout; o++) {
        for (int64_t g = 0; g < K / 4; g++) {
            int ones = 0, ok = 1;
            for (int e = 0; e < 4; e++) {
                uint8_t m = M[o * K + 4 * g + e];
                if (m > 1) ok = 0;
                ones += (m == 1);
            }
            if (!ok || ones != 2) {
                if (bad_row) *bad_row = o;
                if (bad_group) *bad_group = g;
                return 1;
            }
        }
    }
    return 0;
}

/* Fig. 1: canonical structured representation.
 *   vals[o][2g], vals[o][2g+1] = the bit patterns of the two kept weights of group g, in
 *                                ascending position order (copied, never converted);
 *   meta[o][g]                 = i0 | (i1 << 2), one byte per group (values 0..15), where
 *                                i0 < i1 are the kept positions inside the group.
 * Returns 0, or the mask-check status if the mask is invalid (outputs then undefined). */
int ss_oracle_compress(const uint16_t *W, const uint8_t *M, int64_t cout, int64_t K,
                       uint16_t *vals, uint8_t *meta)
{
    int st = ss_oracle_mask_check(M, cout, K, NULL, NULL);
    if (st) return st;
    int64_t G = K / 4;
    for (int64_t o = 0; o < cout; o++) {
        for (int64_t g = 0; g < G; g++) {
            int pos[2], n = 0;
            for (int e = 0; e < 4; e++)
                if (M[o * K + 4 * g + e]) pos[n++] = e;
            vals[o * (K / 2) + 2 * g + 0] = W[o * K + 4 * g + pos[0]];
            vals[o * (K / 2) + 2 * g + 1] = W[o * K + 4 * g + pos[1]];
            meta[o * G + g] = (uint8_t)(pos[0] | (pos[1] << 2));
        }
    }
    return 0;
}

/* Inverse of the above: rebuilds M (.) W, writing +0 at the two dropped positions. */
void ss_oracle_decompress(const uint16_t *vals, const uint8_t *meta, int64_t cout, int64_t K,
                          uint16_t *Wm)
{
    int64_t G = K / 4;
    for (int64_t o = 0; o < cout; o++) {
        for (int64_t g = 0; g < G; g++) {
            for (int e = 0; e < 4; e++) Wm[o * K + 4 * g + e] = 0;
            int i0 = meta[o * G + g] & 3, i1 = (meta[o * G + g] >> 2) & 3;
            Wm[o * K + 4 * g + i0] = vals[o * (K / 2) + 2 * g + 0];
            Wm[o * K + 4 * g + i1] = vals[o * (K / 2) + 2 * g + 1];
        }
    }
}

static int64_t kflat(int korder, int64_t c, int64_t r, int64_t t, int64_t cin, int64_t kh, int64_t kw)
{
    return korder == 0 ? (c * kh + r) * kw + t : (r * kw + t) * cin + c;
}

/* act: 0 identity, 1 ReLU (a NaN stays a NaN), 2 GELU with the exact normal CDF. */
static double layer_tail(double z, int act)
{
    if (act == 1) return (z > 0.0 || z != z) ? z : 0.0;
    if (act == 2) return z * 0.5 * (1.0 + erf(z / sqrt(2.0)));
    return z;
}

/* Eq. (4) with H <- M (.) W (Eq. 6), for cout kernels, a batch of N inputs, strides and
 * symmetric zero padding; bias and activation follow the layer model sigma(Wx + b) of
 * Lemma 3.1 with sigma in {identity (act=0), ReLU (act=1)}.
 *   x    [N][H][Wd][cin]     16-bit patterns (dtype)
 *   W    [cout][K]           16-bit patterns, flattening per korder
 *   M    [cout][K]           0/1 bytes; NULL means all ones (plain dense convolution)
 *   bias [cout] fp32 or NULL
 *   residual [N][Ho][Wo][cout] 16-bit patterns of `dtype`, or NULL: added before the activation
 *   y    [N][Ho][Wo][cout]   fp64, not rounded
 * Returns 0, or 3 if the output would be empty. */
int ss_oracle_conv2d(const uint16_t *x, int64_t N, int64_t H, int64_t Wd, int64_t cin,
                     const uint16_t *W, const uint8_t *M, int64_t cout, int64_t kh, int64_t kw,
                     int korder, int dtype, const float *bias, const uint16_t *residual,
                     int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w, int act,
                     double *y)
{
    int64_t Ho = (H + 2 * pad_h - kh) / stride_h + 1;
    int64_t Wo = (Wd + 2 * pad_w - kw) / stride_w + 1;
    if (H + 2 * pad_h < kh || Wd + 2 * pad_w < kw || Ho <= 0 || Wo <= 0) return 3;
    int64_t K = cin * kh * kw;

    /* exact widening of the operands, and the entry-wise product M (.) W */
    double *xd = (double *)malloc(sizeof(double) * (size_t)(N * H * Wd * cin));
    double *wd = (double *)malloc(sizeof(double) * (size_t)(cout * K));
    if (!xd || !wd) { free(xd); free(wd); return 4; }
    for (int64_t i = 0; i < N * H * Wd * cin; i++) xd[i] = ss_oracle_bits_to_double(x[i], dtype);
    for (int64_t i = 0; i < cout * K; i++)
        wd[i] = (M == NULL || M[i]) ? ss_oracle_bits_to_double(W[i], dtype) : 0.0;

#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; n++) {
        for (int64_t ho = 0; ho < Ho; ho++) {
            for (int64_t wo = 0; wo < Wo; wo++) {
                for (int64_t o = 0; o < cout; o++) {
                    double acc = 0.0;
                    for (int64_t c = 0; c < cin; c++) {
                        for (int64_t r = 0; r < kh; r++) {
                            int64_t ih = ho * stride_h - pad_h + r;
                            if (ih < 0 || ih >= H) continue;          /* zero padding */
                            for (int64_t t = 0; t < kw; t++) {
                                int64_t iw = wo * stride_w - pad_w + t;
                                if (iw < 0 || iw >= Wd) continue;     /* zero padding */
                                acc += wd[o * K + kflat(korder, c, r, t, cin, kh, kw)] *
                                       xd[((n * H + ih) * Wd + iw) * cin + c];
                            }
                        }
                    }
                    if (bias) acc += (double)bias[o];
                    int64_t yi = ((n * Ho + ho) * Wo + wo) * cout + o;
                    if (residual) acc += ss_oracle_bits_to_double(residual[yi], dtype);
                    y[yi] = layer_tail(acc, act);
                }
            }
        }
    }
    free(xd);
    free(wd);
    return 0;
}

/* Same definition, evaluated only at `npts` sampled outputs (flat NHWC indices into y);
 * out[i] receives y[flat_idx[i]].  Used for parity at sizes where the full tensor would
 * take the CPU too long. */
int ss_oracle_conv2d_points(const uint16_t *x, int64_t N, int64_t H, int64_t Wd, int64_t cin,
                            const uint16_t *W, const uint8_t *M, int64_t cout, int64_t kh, int64_t kw,
                            int korder, int dtype, const float *bias, const uint16_t *residual,
                            int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w, int act,
                            const int64_t *flat_idx, int64_t npts, double *out)
{
    int64_t Ho = (H + 2 * pad_h - kh) / stride_h + 1;
    int64_t Wo = (Wd + 2 * pad_w - kw) / stride_w + 1;
    if (H + 2 * pad_h < kh || Wd + 2 * pad_w < kw || Ho <= 0 || Wo <= 0) return 3;
    int64_t K = cin * kh * kw;
    (void)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < npts; i++) {
        int64_t f = flat_idx[i];
        const int64_t yi = f;
        int64_t o = f % cout; f /= cout;
        int64_t wo = f % Wo; f /= Wo;
        int64_t ho = f % Ho; f /= Ho;
        int64_t n = f;
        double acc = 0.0;
        for (int64_t c = 0; c < cin; c++)
            for (int64_t r = 0; r < kh; r++) {
                int64_t ih = ho * stride_h - pad_h + r;
                if (ih < 0 || ih >= H) continue;
                for (int64_t t = 0; t < kw; t++) {
                    int64_t iw = wo * stride_w - pad_w + t;
                    if (iw < 0 || iw >= Wd) continue;
                    int64_t k = kflat(korder, c, r, t, cin, kh, kw);
                    if (M != NULL && !M[o * K + k]) continue;
                    acc += ss_oracle_bits_to_double(W[o * K + k], dtype) *
                           ss_oracle_bits_to_double(x[((n * H + ih) * Wd + iw) * cin + c], dtype);
                }
            }
        if (bias) acc += (double)bias[o];
        if (residual) acc += ss_oracle_bits_to_double(residual[yi], dtype);
        out[i] = layer_tail(acc, act);
    }
    return 0;
}

/* ---------------------------------------------------------------------------------------------
 * 8-bit integer precision point.  The same definitions (Fig. 1 for the representation, Eq. (4) with
 * H <- M (.) W, Eq. 6, for the convolution) on signed 8-bit operands: weights and activations are the
 * integers their bytes encode, every product and the running sum are exact (int64), and the layer output is
 *     y = act( scale[o] * acc + bias[o] )
 * in fp64, with a per-output-channel fp32 scale (the product of the weight and activation quantisation steps
 * of a symmetric quantiser; NULL means 1).  The paper itself stops at 16-bit floats; this is the integer
 * analogue of its Eq. (6), not something it defines.
 * --------------------------------------------------------------------------------------------- */

/* Fig. 1 on bytes: vals[o][2g], vals[o][2g+1] = the two kept bytes of group g in ascending position order,
 * meta[o][g] = i0 | (i1 << 2). */
int ss_oracle_compress8(const uint8_t *W, const uint8_t *M, int64_t cout, int64_t K, uint8_t *vals, uint8_t *meta)
{
    int st = ss_oracle_mask_check(M, cout, K, NULL, NULL);
    if (st) return st;
    int64_t G = K / 4;
    for (int64_t o = 0; o < cout; o++) {
        for (int64_t g = 0; g < G; g++) {
            int pos[2], n = 0;
            for (int e = 0; e < 4; e++)
                if (M[o * K + 4 * g + e]) pos[n++] = e;
            vals[o * (K / 2) + 2 * g + 0] = W[o * K + 4 * g + pos[0]];
            vals[o * (K / 2) + 2 * g + 1] = W[o * K + 4 * g + pos[1]];
            meta[o * G + g] = (uint8_t)(pos[0] | (pos[1] << 2));
        }
    }
    return 0;
}

void ss_oracle_decompress8(const uint8_t *vals, const uint8_t *meta, int64_t cout, int64_t K, uint8_t *Wm)
{
    int64_t G = K / 4;
    for (int64_t o = 0; o < cout; o++) {
        for (int64_t g = 0; g < G; g++) {
            for (int e = 0; e < 4; e++) Wm[o * K + 4 * g + e] = 0;
            int i0 = meta[o * G + g] & 3, i1 = (meta[o * G + g] >> 2) & 3;
            Wm[o * K + 4 * g + i0] = vals[o * (K / 2) + 2 * g + 0];
            Wm[o * K + 4 * g + i1] = vals[o * (K / 2) + 2 * g + 1];
        }
    }
}

/* One output of the integer convolution: the exact sum of Eq. (4) / Eq. (6) at (n, ho, wo, o). */
static int64_t q8_sum(const int8_t *x, int64_t H, int64_t Wd, int64_t cin, const int8_t *W, const uint8_t *M,
                      int64_t kh, int64_t kw, int korder, int64_t stride_h, int64_t stride_w, int64_t pad_h,
                      int64_t pad_w, int64_t n, int64_t ho, int64_t wo, int64_t o)
{
    int64_t K = cin * kh * kw, acc = 0;
    for (int64_t c = 0; c < cin; c++)
        for (int64_t r = 0; r < kh; r++) {
            int64_t ih = ho * stride_h - pad_h + r;
            if (ih < 0 || ih >= H) continue;                  /* zero padding */
            for (int64_t t = 0; t < kw; t++) {
                int64_t iw = wo * stride_w - pad_w + t;
                if (iw < 0 || iw >= Wd) continue;             /* zero padding */
                int64_t k = kflat(korder, c, r, t, cin, kh, kw);
                if (M != NULL && !M[o * K + k]) continue;     /* M (.) W */
                acc += (int64_t)W[o * K + k] * (int64_t)x[((n * H + ih) * Wd + iw) * cin + c];
            }
        }
    return acc;
}

/*   x [N][H][Wd][cin] int8, W [cout][K] int8, M [cout][K] 0/1 bytes or NULL, scale [cout] fp32 or NULL (= 1),
 *   bias [cout] fp32 or NULL, y [N][Ho][Wo][cout] fp64, not rounded. */
int ss_oracle_conv2d_q8(const int8_t *x, int64_t N, int64_t H, int64_t Wd, int64_t cin, const int8_t *W,
                        const uint8_t *M, int64_t cout, int64_t kh, int64_t kw, int korder, const float *scale,
                        const float *bias, int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                        int act, double *y)
{
    int64_t Ho = (H + 2 * pad_h - kh) / stride_h + 1;
    int64_t Wo = (Wd + 2 * pad_w - kw) / stride_w + 1;
    if (H + 2 * pad_h < kh || Wd + 2 * pad_w < kw || Ho <= 0 || Wo <= 0) return 3;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; n++)
        for (int64_t ho = 0; ho < Ho; ho++)
            for (int64_t wo = 0; wo < Wo; wo++)
                for (int64_t o = 0; o < cout; o++) {
                    int64_t acc = q8_sum(x, H, Wd, cin, W, M, kh, kw, korder, stride_h, stride_w, pad_h, pad_w,
                                         n, ho, wo, o);
                    double z = (double)acc * (scale ? (double)scale[o] : 1.0);
                    if (bias) z += (double)bias[o];
                    y[((n * Ho + ho) * Wo + wo) * cout + o] = layer_tail(z, act);
                }
    return 0;
}

/* The same at sampled outputs (flat NHWC indices), for sizes the full tensor would take too long. */
int ss_oracle_conv2d_q8_points(const int8_t *x, int64_t N, int64_t H, int64_t Wd, int64_t cin, const int8_t *W,
                               const uint8_t *M, int64_t cout, int64_t kh, int64_t kw, int korder,
                               const float *scale, const float *bias, int64_t stride_h, int64_t stride_w,
                               int64_t pad_h, int64_t pad_w, int act, const int64_t *flat_idx, int64_t npts,
                               double *out)
{
    int64_t Ho = (H + 2 * pad_h - kh) / stride_h + 1;
    int64_t Wo = (Wd + 2 * pad_w - kw) / stride_w + 1;
    if (H + 2 * pad_h < kh || Wd + 2 * pad_w < kw || Ho <= 0 || Wo <= 0) return 3;
    (void)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < npts; i++) {
        int64_t f = flat_idx[i];
        int64_t o = f % cout; f /= cout;
        int64_t wo = f % Wo; f /= Wo;
        int64_t ho = f % Ho; f /= Ho;
        int64_t acc = q8_sum(x, H, Wd, cin, W, M, kh, kw, korder, stride_h, stride_w, pad_h, pad_w, f, ho, wo, o);
        double z = (double)acc * (scale ? (double)scale[o] : 1.0);
        if (bias) z += (double)bias[o];
        out[i] = layer_tail(z, act);
    }
    return 0;
}

/* ---------------------------------------------------------------------------------------------
 * 8-bit float precision point: operands are OCP FP8 E4M3 bytes (1 sign, 4 exponent bits with bias 7, 3 fraction
 * bits; no infinities; S.1111.111 is NaN; exponent field 0 holds the subnormals m/8 * 2^-6).  Same definition as
 * above with every byte widened exactly to fp64, fp64 products and sums, and the tail act(scale[o]*sum + bias[o]).
 * --------------------------------------------------------------------------------------------- */
double ss_oracle_e4m3_to_double(uint8_t b)
{
    int sign = b >> 7, expo = (b >> 3) & 0xf, frac = b & 7;
    double v;
    if (expo == 15 && frac == 7) return NAN;
    if (expo == 0) v = ldexp((double)frac, -9);               /* frac/8 * 2^-6 */
    else v = ldexp((double)(8 + frac), expo - 10);            /* (1 + frac/8) * 2^(expo-7) */
    return sign ? -v : v;
}

static double f8_sum(const uint8_t *x, int64_t H, int64_t Wd, int64_t cin, const uint8_t *W, const uint8_t *M,
                     int64_t kh, int64_t kw, int korder, int64_t stride_h, int64_t stride_w, int64_t pad_h,
                     int64_t pad_w, int64_t n, int64_t ho, int64_t wo, int64_t o)
{
    int64_t K = cin * kh * kw;
    double acc = 0.0;
    for (int64_t c = 0; c < cin; c++)
        for (int64_t r = 0; r < kh; r++) {
            int64_t ih = ho * stride_h - pad_h + r;
            if (ih < 0 || ih >= H) continue;                  /* zero padding */
            for (int64_t t = 0; t < kw; t++) {
                int64_t iw = wo * stride_w - pad_w + t;
                if (iw < 0 || iw >= Wd) continue;             /* zero padding */
                int64_t k = kflat(korder, c, r, t, cin, kh, kw);
                if (M != NULL && !M[o * K + k]) continue;     /* M (.) W */
                acc += ss_oracle_e4m3_to_double(W[o * K + k]) *
                       ss_oracle_e4m3_to_double(x[((n * H + ih) * Wd + iw) * cin + c]);
            }
        }
    return acc;
}

int ss_oracle_conv2d_f8(const uint8_t *x, int64_t N, int64_t H, int64_t Wd, int64_t cin, const uint8_t *W,
                        const uint8_t *M, int64_t cout, int64_t kh, int64_t kw, int korder, const float *scale,
                        const float *bias, int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                        int act, double *y)
{
    int64_t Ho = (H + 2 * pad_h - kh) / stride_h + 1;
    int64_t Wo = (Wd + 2 * pad_w - kw) / stride_w + 1;
    if (H + 2 * pad_h < kh || Wd + 2 * pad_w < kw || Ho <= 0 || Wo <= 0) return 3;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; n++)
        for (int64_t ho = 0; ho < Ho; ho++)
            for (int64_t wo = 0; wo < Wo; wo++)
                for (int64_t o = 0; o < cout; o++) {
                    double z = f8_sum(x, H, Wd, cin, W, M, kh, kw, korder, stride_h, stride_w, pad_h, pad_w,
                                      n, ho, wo, o) * (scale ? (double)scale[o] : 1.0);
                    if (bias) z += (double)bias[o];
                    y[((n * Ho + ho) * Wo + wo) * cout + o] = layer_tail(z, act);
                }
    return 0;
}

int ss_oracle_conv2d_f8_points(const uint8_t *x, int64_t N, int64_t H, int64_t Wd, int64_t cin, const uint8_t *W,
                               const uint8_t *M, int64_t cout, int64_t kh, int64_t kw, int korder,
                               const float *scale, const float *bias, int64_t stride_h, int64_t stride_w,
                               int64_t pad_h, int64_t pad_w, int act, const int64_t *flat_idx, int64_t npts,
                               double *out)
{
    int64_t Ho = (H + 2 * pad_h - kh) / stride_h + 1;
    int64_t Wo = (Wd + 2 * pad_w - kw) / stride_w + 1;
    if (H + 2 * pad_h < kh || Wd + 2 * pad_w < kw || Ho <= 0 || Wo <= 0) return 3;
    (void)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < npts; i++) {
        int64_t f = flat_idx[i];
        int64_t o = f % cout; f /= cout;
        int64_t wo = f % Wo; f /= Wo;
        int64_t ho = f % Ho; f /= Ho;
        double z = f8_sum(x, H, Wd, cin, W, M, kh, kw, korder, stride_h, stride_w, pad_h, pad_w, f, ho, wo, o) *
                   (scale ? (double)scale[o] : 1.0);
        if (bias) z += (double)bias[o];
        out[i] = layer_tail(z, act);
    }
    return 0;
}

/* Max pooling, NHWC, k x k window, given stride and symmetric zero-extent padding: the maximum over the window
 * positions that lie inside the image (the pooling layer between the stem and the first residual block of the
 * ResNet models the paper evaluates, Sec. 4).  Values are compared as their exact fp64 widenings; the output is the
 * 16-bit pattern of the winner (first one in row-major window order among equals); a NaN, once met, stays. */
int ss_oracle_maxpool2d(const uint16_t *x, int64_t N, int64_t H, int64_t Wd, int64_t C, int dtype,
                        int64_t k, int64_t stride, int64_t pad, uint16_t *y)
{
    int64_t Ho = (H + 2 * pad - k) / stride + 1, Wo = (Wd + 2 * pad - k) / stride + 1;
    if (H + 2 * pad < k || Wd + 2 * pad < k || Ho <= 0 || Wo <= 0) return 3;
    for (int64_t n = 0; n < N; n++)
        for (int64_t ho = 0; ho < Ho; ho++)
            for (int64_t wo = 0; wo < Wo; wo++)
                for (int64_t c = 0; c < C; c++) {
                    int have = 0;
                    uint16_t best = 0;
                    double bestv = 0.0;
                    for (int64_t r = 0; r < k; r++)
                        for (int64_t t = 0; t < k; t++) {
                            int64_t ih = ho * stride - pad + r, iw = wo * stride - pad + t;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= Wd) continue;
                            uint16_t b = x[((n * H + ih) * Wd + iw) * C + c];
                            double v = ss_oracle_bits_to_double(b, dtype);
                            if (!have) { have = 1; best = b; bestv = v; continue; }
                            if (bestv != bestv) continue;                       /* NaN stays */
                            if (v != v || v > bestv) { best = b; bestv = v; }
                        }
                    y[((n * Ho + ho) * Wo + wo) * C + c] = have ? best : 0;
                }
    return 0;
}

/* Depthwise convolution (one filter per channel; the grouped convolutions that stay dense in the paper, Sec. 4),
 * stride 1, zero padding, NHWC.  Eq. (4) restricted to its diagonal: the output channel c only sees input channel c.
 *   x [N][H][Wd][C], w [kh][kw][C] (channel fastest), bias [C] fp32 or NULL, y [N][Ho][Wo][C] fp64, not rounded. */
int ss_oracle_dwconv2d(const uint16_t *x, int64_t N, int64_t H, int64_t Wd, int64_t C, int dtype,
                       const uint16_t *w, const float *bias, int64_t kh, int64_t kw, int64_t pad_h, int64_t pad_w,
                       int act, double *y)
{
    int64_t Ho = H + 2 * pad_h - kh + 1, Wo = Wd + 2 * pad_w - kw + 1;
    if (Ho <= 0 || Wo <= 0) return 3;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; n++)
        for (int64_t ho = 0; ho < Ho; ho++)
            for (int64_t wo = 0; wo < Wo; wo++)
                for (int64_t c = 0; c < C; c++) {
                    double acc = 0.0;
                    for (int64_t r = 0; r < kh; r++) {
                        int64_t ih = ho - pad_h + r;
                        if (ih < 0 || ih >= H) continue;
                        for (int64_t t = 0; t < kw; t++) {
                            int64_t iw = wo - pad_w + t;
                            if (iw < 0 || iw >= Wd) continue;
                            acc += ss_oracle_bits_to_double(w[(r * kw + t) * C + c], dtype) *
                                   ss_oracle_bits_to_double(x[((n * H + ih) * Wd + iw) * C + c], dtype);
                        }
                    }
                    if (bias) acc += (double)bias[c];
                    y[((n * Ho + ho) * Wo + wo) * C + c] = layer_tail(acc, act);
                }
    return 0;
}
