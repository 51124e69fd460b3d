/*
 * TORQ CPU oracle -- TEST INFRASTRUCTURE ONLY (see torq_oracle.h).
 *
 * Every function names the passage of the paper it follows.  Nothing here is
 * blocked, fused or vectorised by hand: a reader should be able to check each
 * loop against the paper by eye.
 */
#include "torq_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define PI 3.14159265358979323846
#define BLK 32 /* K in the paper's notation: elements per microscaling block */

/* ------------------------------------------------------------------ bf16 -- */

/* bf16 is the upper half of an IEEE binary32 pattern, so widening is a shift. */
float torq_o_bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* Round-to-nearest-even on the 16 discarded bits.  NaN keeps a quiet payload. */
uint16_t torq_o_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu) != 0)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t kept_lsb = (u >> 16) & 1u;
    uint32_t dropped = u & 0xFFFFu;
    uint32_t up = (dropped > 0x8000u) || (dropped == 0x8000u && kept_lsb);
    return (uint16_t)((u >> 16) + up);
}

/* -------------------------------------------------------------- rotation -- */

/* Algorithm 3, step 2: Y = R_inter X.  X is the B x 32 view of one token; the
 * G x G matrix acts on each run of G consecutive blocks (block-diagonal over
 * the row, Appendix A.7 "decomposed into block-diagonal"); G = B is the
 * algorithm exactly as printed. */
void torq_o_rotate_inter(const double *x, int64_t M, int d, int G,
                         const float *R_inter, double *y)
{
    const int B = d / BLK;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const double *X = x + m * (int64_t)d;
        double *Y = y + m * (int64_t)d;
        for (int g0 = 0; g0 < B; g0 += G)
            for (int b = 0; b < G; ++b)
                for (int k = 0; k < BLK; ++k) {
                    double acc = 0.0;
                    for (int bp = 0; bp < G; ++bp)
                        acc += (double)R_inter[b * G + bp] * X[(g0 + bp) * BLK + k];
                    Y[(g0 + b) * BLK + k] = acc;
                }
    }
}

/* Algorithm 3, step 3: Z = Y R_intra, i.e. every block (a row of Y) is
 * multiplied on the right by the 32 x 32 matrix. */
void torq_o_rotate_intra(const double *y, int64_t M, int d,
                         const float *R_intra, double *z)
{
    const int B = d / BLK;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const double *Y = y + m * (int64_t)d;
        double *Z = z + m * (int64_t)d;
        for (int b = 0; b < B; ++b)
            for (int k = 0; k < BLK; ++k) {
                double acc = 0.0;
                for (int kp = 0; kp < BLK; ++kp)
                    acc += Y[b * BLK + kp] * (double)R_intra[kp * BLK + k];
                Z[b * BLK + k] = acc;
            }
    }
}

/* Algorithm 3, steps 1-3 on bf16 input rows. */
void torq_o_rotate(const uint16_t *x_bf16, int64_t M, int d, int G,
                   const float *R_inter, const float *R_intra,
                   float *z_f32, double *z_f64)
{
    const int64_t n = M * (int64_t)d;
    double *x = (double *)malloc(sizeof(double) * (size_t)(n ? n : 1));
    double *y = (double *)malloc(sizeof(double) * (size_t)(n ? n : 1));
    double *z = (double *)malloc(sizeof(double) * (size_t)(n ? n : 1));
    for (int64_t i = 0; i < n; ++i)          /* step 1: reshape is indexing */
        x[i] = (double)torq_o_bf16_to_f32(x_bf16[i]);
    torq_o_rotate_inter(x, M, d, G, R_inter, y);   /* step 2 */
    torq_o_rotate_intra(y, M, d, R_intra, z);      /* step 3 */
    for (int64_t i = 0; i < n; ++i) {
        if (z_f32) z_f32[i] = (float)z[i];
        if (z_f64) z_f64[i] = z[i];
    }
    free(x); free(y); free(z);
}

/* Algorithm 3, step 5 option A (explicit inverse), scales already applied:
 * X = R_inter^T (Z R_intra^T).  Used by tests for the round-trip identity of
 * Section 5.2 ("under full precision ... an identity mapping"). */
void torq_o_rotate_inverse(const double *z, int64_t M, int d, int G,
                           const float *R_inter, const float *R_intra,
                           double *x)
{
    const int B = d / BLK;
    for (int64_t m = 0; m < M; ++m) {
        const double *Z = z + m * (int64_t)d;
        double *X = x + m * (int64_t)d;
        double *Y = (double *)malloc(sizeof(double) * (size_t)d);
        for (int b = 0; b < B; ++b)
            for (int kp = 0; kp < BLK; ++kp) {
                double acc = 0.0;
                for (int k = 0; k < BLK; ++k)
                    acc += Z[b * BLK + k] * (double)R_intra[kp * BLK + k];
                Y[b * BLK + kp] = acc;
            }
        for (int g0 = 0; g0 < B; g0 += G)
            for (int bp = 0; bp < G; ++bp)
                for (int k = 0; k < BLK; ++k) {
                    double acc = 0.0;
                    for (int b = 0; b < G; ++b)
                        acc += (double)R_inter[b * G + bp] * Y[(g0 + b) * BLK + k];
                    X[(g0 + bp) * BLK + k] = acc;
                }
        free(Y);
    }
}

/* ----------------------------------------------------------------- MXFP4 -- */

/* Shared scale, Eq. 1.  The printed s_b = 2^floor(log2 max|z_b|) would leave
 * the codewords 3, 4 and 6 unused; the MX format rule subtracts the exponent
 * of the largest e2m1 magnitude (6 = 1.5 * 2^2), so the scale exponent is
 * floor(log2 amax) - 2 and the normalised maximum lands in [4, 8).  For a
 * normal fp32 amax, floor(log2 amax) is the exponent field minus 127, hence
 * byte = field - 2.  Zero, subnormal and tiny amax clamp to byte 0. */
uint8_t torq_o_e8m0_from_amax(float amax)
{
    uint32_t u;
    memcpy(&u, &amax, 4);
    int field = (int)((u >> 23) & 0xFFu);
    int byte = field - 2;
    if (byte < 0) byte = 0;
    if (byte > 254) byte = 254;
    return (uint8_t)byte;
}

static const float E2M1_MAG[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};

float torq_o_e2m1_value(uint8_t code)
{
    float v = E2M1_MAG[code & 7u];
    return (code & 8u) ? -v : v;
}

/* Nearest-neighbour projection onto the e2m1 codebook of Eq. 1.  Midpoints
 * between neighbouring magnitudes are 0.25 0.75 1.25 1.75 2.5 3.5 5; a value
 * exactly on a midpoint goes to the neighbour with the even index (0, 1, 2, 4:
 * indices 0, 2, 4, 6), the IEEE default.  The sign bit is copied, so a small
 * negative value becomes -0 (code 8). */
uint8_t torq_o_e2m1_from_f32(float a)
{
    uint32_t u;
    memcpy(&u, &a, 4);
    uint8_t sign = (uint8_t)((u >> 31) << 3);
    float m = fabsf(a);
    uint8_t idx;
    if      (m <= 0.25f) idx = 0;   /* tie 0.25 -> 0   (index 0, even) */
    else if (m <  0.75f) idx = 1;   /* tie 0.75 -> 1   (index 2)       */
    else if (m <= 1.25f) idx = 2;   /* tie 1.25 -> 1   (index 2)       */
    else if (m <  1.75f) idx = 3;   /* tie 1.75 -> 2   (index 4)       */
    else if (m <= 2.5f)  idx = 4;   /* tie 2.5  -> 2   (index 4)       */
    else if (m <  3.5f)  idx = 5;   /* tie 3.5  -> 4   (index 6)       */
    else if (m <= 5.0f)  idx = 6;   /* tie 5    -> 4   (index 6)       */
    else                 idx = 7;   /* (5, inf): 6, saturating above 6 */
    return (uint8_t)(sign | idx);
}

/* Algorithm 3, step 4, for every block of every row: amax, shared scale,
 * normalise a = z / s (a power-of-two scaling, exact), project, pack.
 * Two codes per byte, element 2j in the low nibble of byte j. */
void torq_o_quantize(const float *z, int64_t M, int d,
                     uint8_t *codes, uint8_t *scales)
{
    const int B = d / BLK;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *zr = z + m * (int64_t)d;
        uint8_t *cr = codes + m * (int64_t)(d / 2);
        uint8_t *sr = scales + m * (int64_t)B;
        for (int b = 0; b < B; ++b) {
            float amax = 0.0f;
            for (int k = 0; k < BLK; ++k) {
                float v = fabsf(zr[b * BLK + k]);
                if (v > amax) amax = v;
            }
            uint8_t byte = torq_o_e8m0_from_amax(amax);
            sr[b] = byte;
            uint8_t c[BLK];
            for (int k = 0; k < BLK; ++k) {
                /* a = z / 2^(byte-127).  A power-of-two scaling with |a| < 8:
                 * exact, except that an element ~2^100 times smaller than its
                 * block's amax may land in the subnormal range and round
                 * there -- far below the first threshold, so it is code 0
                 * (or -0) either way. */
                float a = ldexpf(zr[b * BLK + k], 127 - (int)byte);
                c[k] = torq_o_e2m1_from_f32(a);
            }
            for (int j = 0; j < BLK / 2; ++j)
                cr[b * (BLK / 2) + j] = (uint8_t)(c[2 * j] | (c[2 * j + 1] << 4));
        }
    }
}

/* "De-quantize" line of Algorithm 3 step 4: zhat = s_b * ahat. */
void torq_o_dequantize(const uint8_t *codes, const uint8_t *scales,
                       int64_t M, int d, float *zhat)
{
    const int B = d / BLK;
    for (int64_t m = 0; m < M; ++m)
        for (int b = 0; b < B; ++b) {
            int e = (int)scales[m * (int64_t)B + b] - 127;
            for (int k = 0; k < BLK; ++k) {
                int64_t j = m * (int64_t)d + b * BLK + k;
                uint8_t byte = codes[j / 2];
                uint8_t code = (j & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 15u);
                zhat[j] = ldexpf(torq_o_e2m1_value(code), e);
            }
        }
}

/* ------------------------------------------------- other 4-bit formats -- */
/* Section 6 ("Generalizability to Other Formats", Table 5) applies the same rotations in front
 * of two other block formats.  The paper defines neither; the readings taken are stated here.
 *
 * MXINT4: the microscaling layout of MXFP4 (32 elements, one E8M0 scale chosen by the same rule)
 * with integer elements: a = z / s rounded to the nearest integer, ties to even, clamped to
 * [-7, 7] (symmetric), stored as a two's-complement nibble.
 *
 * NVFP4: blocks of 16 elements, each with an FP8 E4M3 scale, on top of one fp32 scale s_g for the
 * whole tensor (an input here), elements e2m1.  Block scale: the E4M3 value nearest to
 * amax / (6 s_g) (ties to the even code, saturating at 448); effective scale S = value * s_g;
 * a = z / S; e2m1 code as for MXFP4.  All of it in fp32, in exactly this order of operations. */

/* OCP FP8 E4M3: 1 sign, 4 exponent (bias 7), 3 mantissa bits; no infinities, S.1111.111 is NaN,
 * so the largest magnitude is S.1111.110 = 448; exponent field 0 = subnormals m/8 * 2^-6. */
float torq_o_e4m3_value(uint8_t code)
{
    int e = (code >> 3) & 15, m = code & 7;
    float v = e ? ldexpf(1.0f + (float)m / 8.0f, e - 7) : ldexpf((float)m / 8.0f, -6);
    return (code & 0x80u) ? -v : v;
}

/* nearest non-negative E4M3 value to t >= 0: a search over all 127 of them; of two equally near
 * neighbours the one with the even code; anything above 448 gives 448 */
uint8_t torq_o_e4m3_from_f32(float t)
{
    uint8_t best = 0;
    double best_err = fabs((double)t - 0.0);
    for (int c = 1; c <= 0x7E; ++c) {
        double err = fabs((double)t - (double)torq_o_e4m3_value((uint8_t)c));
        if (err < best_err || (err == best_err && (c & 1) == 0)) {
            best_err = err;
            best = (uint8_t)c;
        }
    }
    return best;
}

void torq_o_quantize_mxint4(const float *z, int64_t M, int d, uint8_t *codes, uint8_t *scales)
{
    const int B = d / BLK;
    for (int64_t m = 0; m < M; ++m)
        for (int b = 0; b < B; ++b) {
            const float *zb = z + m * (int64_t)d + b * BLK;
            float amax = 0.0f;
            for (int k = 0; k < BLK; ++k)
                if (fabsf(zb[k]) > amax) amax = fabsf(zb[k]);
            uint8_t byte = torq_o_e8m0_from_amax(amax);
            scales[m * (int64_t)B + b] = byte;
            uint8_t c[BLK];
            for (int k = 0; k < BLK; ++k) {
                float r = rintf(ldexpf(zb[k], 127 - (int)byte));   /* to nearest, ties to even */
                if (r > 7.0f) r = 7.0f;
                if (r < -7.0f) r = -7.0f;
                c[k] = (uint8_t)((int)r & 15);
            }
            for (int j = 0; j < BLK / 2; ++j)
                codes[m * (int64_t)(d / 2) + b * (BLK / 2) + j] = (uint8_t)(c[2 * j] | (c[2 * j + 1] << 4));
        }
}

void torq_o_dequantize_mxint4(const uint8_t *codes, const uint8_t *scales, int64_t M, int d, float *zhat)
{
    for (int64_t j = 0; j < M * (int64_t)d; ++j) {
        uint8_t byte = codes[j / 2];
        int nib = (j & 1) ? (byte >> 4) : (byte & 15);
        int v = nib >= 8 ? nib - 16 : nib;
        zhat[j] = ldexpf((float)v, (int)scales[j / BLK] - 127);
    }
}

void torq_o_quantize_nvfp4(const float *z, int64_t M, int d, float global_scale, uint8_t *codes,
                           uint8_t *scales_e4m3)
{
    const int B16 = d / 16;
    const float D = 6.0f * global_scale;
    for (int64_t m = 0; m < M; ++m)
        for (int b = 0; b < B16; ++b) {
            const float *zb = z + m * (int64_t)d + b * 16;
            float amax = 0.0f;
            for (int k = 0; k < 16; ++k)
                if (fabsf(zb[k]) > amax) amax = fabsf(zb[k]);
            const uint8_t q = torq_o_e4m3_from_f32(amax / D);
            scales_e4m3[m * (int64_t)B16 + b] = q;
            const float S = torq_o_e4m3_value(q) * global_scale;
            uint8_t c[16];
            for (int k = 0; k < 16; ++k) {
                /* a block whose scale rounds to zero keeps only the signs */
                c[k] = (S > 0.0f) ? torq_o_e2m1_from_f32(zb[k] / S) : torq_o_e2m1_from_f32(copysignf(0.0f, zb[k]));
            }
            for (int j = 0; j < 8; ++j)
                codes[m * (int64_t)(d / 2) + b * 8 + j] = (uint8_t)(c[2 * j] | (c[2 * j + 1] << 4));
        }
}

void torq_o_dequantize_nvfp4(const uint8_t *codes, const uint8_t *scales_e4m3, int64_t M, int d,
                             float global_scale, float *zhat)
{
    for (int64_t j = 0; j < M * (int64_t)d; ++j) {
        uint8_t byte = codes[j / 2];
        uint8_t code = (j & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 15u);
        zhat[j] = torq_o_e2m1_value(code) * (torq_o_e4m3_value(scales_e4m3[j / 16]) * global_scale);
    }
}

void torq_o_rotate_quantize(const uint16_t *x_bf16, int64_t M, int d, int G,
                            const float *R_inter, const float *R_intra,
                            uint8_t *codes, uint8_t *scales)
{
    const int64_t n = M * (int64_t)d;
    float *z = (float *)malloc(sizeof(float) * (size_t)(n ? n : 1));
    torq_o_rotate(x_bf16, M, d, G, R_inter, R_intra, z, NULL);
    torq_o_quantize(z, M, d, codes, scales);
    free(z);
}

/* ------------------------------------------------------------------ GEMM -- */

/* one output of the linear layer that consumes the quantised activations
 * (Algorithm 3 "Return"): the dot product of a dequantised activation row and
 * a dequantised fused-weight row, summed in double in index order. */
static double dot_dequant(const uint8_t *aq, const uint8_t *as,
                          const uint8_t *wq, const uint8_t *ws, int d)
{
    double acc = 0.0;
    for (int j = 0; j < d; ++j) {
        uint8_t ab = aq[j / 2], wb = wq[j / 2];
        uint8_t ac = (j & 1) ? (uint8_t)(ab >> 4) : (uint8_t)(ab & 15u);
        uint8_t wc = (j & 1) ? (uint8_t)(wb >> 4) : (uint8_t)(wb & 15u);
        double av = ldexp((double)torq_o_e2m1_value(ac), (int)as[j / BLK] - 127);
        double wv = ldexp((double)torq_o_e2m1_value(wc), (int)ws[j / BLK] - 127);
        acc += av * wv;
    }
    return acc;
}

void torq_o_gemm(const uint8_t *A_q, const uint8_t *A_s,
                 const uint8_t *W_q, const uint8_t *W_s,
                 int64_t M, int64_t N, int d,
                 uint16_t *out_bf16, double *out_f64)
{
    const int B = d / BLK;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double v = dot_dequant(A_q + m * (int64_t)(d / 2), A_s + m * (int64_t)B,
                                   W_q + n * (int64_t)(d / 2), W_s + n * (int64_t)B, d);
            if (out_bf16) out_bf16[m * N + n] = torq_o_f32_to_bf16((float)v);
            if (out_f64) out_f64[m * N + n] = v;
        }
}

void torq_o_gemm_sampled(const uint8_t *A_q, const uint8_t *A_s,
                         const uint8_t *W_q, const uint8_t *W_s,
                         int d, int64_t count,
                         const int64_t *ms, const int64_t *ns,
                         uint16_t *out_bf16, double *out_f64)
{
    const int B = d / BLK;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        int64_t m = ms[i], n = ns[i];
        double v = dot_dequant(A_q + m * (int64_t)(d / 2), A_s + m * (int64_t)B,
                               W_q + n * (int64_t)(d / 2), W_s + n * (int64_t)B, d);
        if (out_bf16) out_bf16[i] = torq_o_f32_to_bf16((float)v);
        if (out_f64) out_f64[i] = v;
    }
}

/* ------------------------------------------------- variance equalisation -- */

/* Section 5.1: the covariance of the block view that Algorithm 1 equalises.  With one shared
 * R_inter for all in-block positions, the quantity that R_inter acts on is the Gram matrix of
 * the blocks, Sigma[b][b'] = E <x_b, x_b'>; diag(R Sigma R^T) are then the block energies
 * sigma_b^2 = E ||z_b||^2 of Theorem 4.1 after the rotation.  The expectation is the plain mean
 * over all runs of G blocks in the sample. */
void torq_o_block_gram(const uint16_t *x_bf16, int64_t M, int d, int G, double *Sigma)
{
    const int B = d / BLK;
    const int64_t groups = M * (int64_t)(B / G);
    for (int i = 0; i < G * G; ++i) Sigma[i] = 0.0;
    for (int64_t m = 0; m < M; ++m)
        for (int g0 = 0; g0 < B; g0 += G) {
            const uint16_t *X = x_bf16 + m * (int64_t)d + (int64_t)g0 * BLK;
            for (int b = 0; b < G; ++b)
                for (int bp = 0; bp < G; ++bp) {
                    double acc = 0.0;
                    for (int k = 0; k < BLK; ++k)
                        acc += (double)torq_o_bf16_to_f32(X[b * BLK + k]) *
                               (double)torq_o_bf16_to_f32(X[bp * BLK + k]);
                    Sigma[b * G + bp] += acc;
                }
        }
    if (groups > 0)
        for (int i = 0; i < G * G; ++i) Sigma[i] /= (double)groups;
}

/* The same statistic kept apart by the position k inside a block: the covariance matrices
 * Sigma_k of Theorem 4.1 (one per position, B x B each; the calibration cost analysis counts
 * "covariance matrices for all K positions"):
 *
 *   Sigma_pos[k][b][b'] = mean over the runs of G blocks of  X[b][k] X[b'][k]
 *
 * so that the sum over k is torq_o_block_gram's Sigma. */
void torq_o_block_gram_positions(const uint16_t *x_bf16, int64_t M, int d, int G, double *Sigma_pos)
{
    const int B = d / BLK;
    const int64_t groups = M * (int64_t)(B / G);
    for (int64_t i = 0; i < (int64_t)BLK * G * G; ++i) Sigma_pos[i] = 0.0;
    for (int64_t m = 0; m < M; ++m)
        for (int g0 = 0; g0 < B; g0 += G) {
            const uint16_t *Xg = x_bf16 + m * (int64_t)d + (int64_t)g0 * BLK;
            for (int k = 0; k < BLK; ++k)
                for (int b = 0; b < G; ++b)
                    for (int bp = 0; bp < G; ++bp)
                        Sigma_pos[((int64_t)k * G + b) * G + bp] +=
                            (double)torq_o_bf16_to_f32(Xg[b * BLK + k]) *
                            (double)torq_o_bf16_to_f32(Xg[bp * BLK + k]);
        }
    if (groups > 0)
        for (int64_t i = 0; i < (int64_t)BLK * G * G; ++i) Sigma_pos[i] /= (double)groups;
}

/* Algorithm 1 (Section 5.1): plane rotations until diag(R Sigma R^T) = c 1,
 * c = tr(Sigma) / B.  Each step takes the block i furthest above c and the
 * block j furthest below it (opposite deviation signs, as the algorithm asks)
 * and turns the (i, j) plane by the angle that puts sigma_ii exactly on c:
 *
 *   sigma_ii' = cos^2 a + 2 sin cos g + sin^2 b      (a, b, g = s_ii, s_jj, s_ij)
 *   set to c and divide by cos^2:  (b-c) t^2 + 2 g t + (a-c) = 0,  t = tan(theta)
 *
 * The discriminant g^2 - (a-c)(b-c) is positive because (a-c)(b-c) < 0.  The
 * root of smaller magnitude is taken in its cancellation-free form.  Trace is
 * conserved (Appendix A.1, step 1), so sigma_jj' = a + b - c, and after at most
 * B-1 steps every diagonal entry equals c.  The angle printed in Algorithm 1 is
 * the Jacobi diagonalising angle, which moves the two entries apart; it cannot
 * meet the algorithm's own output condition, so the equalising angle is used. */
int torq_o_equalize(double *Sigma, int B, double eps, double *R)
{
    double tr = 0.0;
    for (int i = 0; i < B; ++i) tr += Sigma[i * B + i];
    const double c = tr / B;
    for (int i = 0; i < B; ++i)
        for (int j = 0; j < B; ++j) R[i * B + j] = (i == j) ? 1.0 : 0.0;

    int steps = 0;
    for (;;) {
        int i = -1, j = -1;
        double hi = 0.0, lo = 0.0, worst = 0.0;
        for (int q = 0; q < B; ++q) {
            double dev = Sigma[q * B + q] - c;
            if (fabs(dev) > worst) worst = fabs(dev);
            if (dev > hi) { hi = dev; i = q; }
            if (dev < lo) { lo = dev; j = q; }
        }
        if (worst <= eps) break;
        if (i < 0 || j < 0) return -1;
        if (steps >= 4 * B) return -1;

        const double a = Sigma[i * B + i], b = Sigma[j * B + j], g = Sigma[i * B + j];
        const double D = sqrt(g * g - (a - c) * (b - c));
        const double t = -(a - c) / (g + (g >= 0.0 ? D : -D));
        const double cs = 1.0 / sqrt(1.0 + t * t);
        const double sn = t * cs;

        /* Sigma <- G Sigma G^T and R <- G R, where G mixes rows i and j:
         * row_i' = cs row_i + sn row_j ; row_j' = -sn row_i + cs row_j. */
        for (int q = 0; q < B; ++q) {             /* rows of Sigma and of R */
            double si = Sigma[i * B + q], sj = Sigma[j * B + q];
            Sigma[i * B + q] = cs * si + sn * sj;
            Sigma[j * B + q] = -sn * si + cs * sj;
            double ri = R[i * B + q], rj = R[j * B + q];
            R[i * B + q] = cs * ri + sn * rj;
            R[j * B + q] = -sn * ri + cs * rj;
        }
        for (int q = 0; q < B; ++q) {             /* columns of Sigma */
            double si = Sigma[q * B + i], sj = Sigma[q * B + j];
            Sigma[q * B + i] = cs * si + sn * sj;
            Sigma[q * B + j] = -sn * si + cs * sj;
        }
        ++steps;
    }
    return steps;
}

/* The same goal -- an orthogonal R with diag(R Sigma R^T) = c 1 (Theorem 4.1, Section 5.1) --
 * reached with plane rotations arranged as a butterfly, so that the result can be applied online
 * in log2(B) rounds of B/2 independent plane rotations instead of as a dense matrix (Algorithm 1
 * picks its pairs greedily, one after the other; the Schur-Horn argument does not care which
 * orthogonal matrix reaches the constant diagonal).  B is a power of two.  Round t = 0, 1, ...
 * pairs row p with row q = p + h, h = B / 2^(t+1), for every p whose bit h is clear, and turns
 * the pair by the angle that makes its two diagonal entries EQUAL:
 *
 *   row_p' = cos row_p + sin row_q,  row_q' = -sin row_p + cos row_q
 *   s_pp' - s_qq' = (a - b) cos 2theta + 2 g sin 2theta = 0   (a, b, g = s_pp, s_qq, s_pq)
 *   theta = atan((b - a) / (2 g)) / 2 in (-pi/4, pi/4);  g = 0: pi/4 if a != b, else 0.
 *
 * After round t the diagonal is constant on every residue class of the row index modulo h (the
 * mean of the 2^(t+1) entries it replaces), so after the last round it is the overall mean c.
 * tangents[t * B/2 + i] = tan(theta) of the i-th pair (in increasing p) of round t. */
void torq_o_equalize_butterfly(double *Sigma, int B, double *R, double *tangents)
{
    for (int i = 0; i < B; ++i)
        for (int j = 0; j < B; ++j) R[i * B + j] = (i == j) ? 1.0 : 0.0;
    int round = 0;
    for (int h = B / 2; h >= 1; h /= 2, ++round) {
        int pair = 0;
        for (int p = 0; p < B; ++p) {
            if (p & h) continue;
            const int q = p + h;
            const double a = Sigma[p * B + p], b = Sigma[q * B + q], g = Sigma[p * B + q];
            double theta;
            if (g != 0.0) theta = 0.5 * atan((b - a) / (2.0 * g));
            else theta = (a != b) ? PI / 4.0 : 0.0;
            const double cs = cos(theta), sn = sin(theta);
            tangents[round * (B / 2) + pair++] = tan(theta);
            for (int k = 0; k < B; ++k) {             /* rows of Sigma and of R */
                double sp = Sigma[p * B + k], sq = Sigma[q * B + k];
                Sigma[p * B + k] = cs * sp + sn * sq;
                Sigma[q * B + k] = -sn * sp + cs * sq;
                double rp = R[p * B + k], rq = R[q * B + k];
                R[p * B + k] = cs * rp + sn * rq;
                R[q * B + k] = -sn * rp + cs * rq;
            }
            for (int k = 0; k < B; ++k) {             /* columns of Sigma */
                double sp = Sigma[k * B + p], sq = Sigma[k * B + q];
                Sigma[k * B + p] = cs * sp + sn * sq;
                Sigma[k * B + q] = -sn * sp + cs * sq;
            }
        }
    }
}

/* ------------------------------------------- intra-block calibration -- */

void torq_o_code_histogram(const uint8_t *codes, int64_t M, int d, uint64_t *counts)
{
    for (int i = 0; i < BLK * 8; ++i) counts[i] = 0;
    for (int64_t m = 0; m < M; ++m)
        for (int j = 0; j < d; ++j) {
            uint8_t byte = codes[m * (int64_t)(d / 2) + j / 2];
            uint8_t code = (j & 1) ? (uint8_t)(byte >> 4) : (uint8_t)(byte & 15u);
            counts[(j % BLK) * 8 + (code & 7u)] += 1;
        }
}

double torq_o_code_loss(const uint64_t n[8])
{
    double total = 0.0, loss = 0.0;
    for (int j = 0; j < 8; ++j) total += (double)n[j];
    if (total == 0.0) return 0.0;
    for (int j = 0; j < 8; ++j) {
        double dev = (double)n[j] / total - 1.0 / 8.0;
        loss += dev * dev;
    }
    return loss;
}

void torq_o_pair_scores(const uint64_t *counts, double lambda, double *h, double *H)
{
    double dev[BLK][8];
    for (int k = 0; k < BLK; ++k) {
        double total = 0.0;
        for (int j = 0; j < 8; ++j) total += (double)counts[k * 8 + j];
        h[k] = 0.0;
        for (int j = 0; j < 8; ++j) {
            dev[k][j] = (total > 0.0 ? (double)counts[k * 8 + j] / total : 0.0) - 1.0 / 8.0;
            h[k] += dev[k][j] * dev[k][j];
        }
    }
    for (int k = 0; k < BLK; ++k)
        for (int l = 0; l < BLK; ++l) {
            double c = 0.0;
            for (int j = 0; j < 8; ++j) c -= dev[k][j] * dev[l][j];
            H[k * BLK + l] = h[k] + h[l] + lambda * c;
        }
}

/* Magnitude codeword of a normalised value: the index j of the interval I_j between the decision
 * boundaries d_j (the midpoints of neighbouring e2m1 magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6) that
 * holds |a|; a value on a boundary goes to the neighbour with the even mantissa, as round-to-
 * nearest-even does. */
int torq_o_mag_code(double a)
{
    const double m = fabs(a);
    if (m <= 0.25) return 0;
    if (m < 0.75) return 1;
    if (m <= 1.25) return 2;
    if (m < 1.75) return 3;
    if (m <= 2.5) return 4;
    if (m < 3.5) return 5;
    if (m <= 5.0) return 6;
    return 7;
}

/* occupancy of the 8 codewords when the pair (u, v) is turned by theta, on top of `rest` */
static void counts_at(const double *u, const double *v, int64_t n, const uint64_t rest[8], double theta,
                      uint64_t cnt[8])
{
    const double c = cos(theta), s = sin(theta);
    for (int j = 0; j < 8; ++j) cnt[j] = rest[j];
    for (int64_t b = 0; b < n; ++b) {
        cnt[torq_o_mag_code(u[b] * c + v[b] * s)] += 1;
        cnt[torq_o_mag_code(-u[b] * s + v[b] * c)] += 1;
    }
}

/* sum_j n_j^2: because sum_j n_j does not depend on theta, the loss sum_j (n_j / N - 1/8)^2 =
 * (sum_j n_j^2) / N^2 - 1/8 orders the angles exactly as this integer does, so angles are compared
 * on it and equal losses are recognised exactly */
static unsigned __int128 sum_squares(const uint64_t cnt[8])
{
    unsigned __int128 t = 0;
    for (int j = 0; j < 8; ++j) t += (unsigned __int128)cnt[j] * cnt[j];
    return t;
}

static int cmp_double(const void *a, const void *b)
{
    double x = *(const double *)a, y = *(const double *)b;
    return (x > y) - (x < y);
}

int64_t torq_o_best_angle(const double *u, const double *v, int64_t n, const uint64_t rest[8],
                          double *theta, double *loss)
{
    static const double bound[7] = {0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0};
    const double two_pi = 2.0 * PI;
    uint64_t cnt[8];
    /* at most 7 boundaries x 2 axes x 4 angles per sample */
    double *tau = (double *)malloc(sizeof(double) * (size_t)(n * 56 + 1));
    int64_t count = 0;
    for (int64_t b = 0; b < n; ++b) {
        const double r = sqrt(u[b] * u[b] + v[b] * v[b]);
        const double phi = atan2(v[b], u[b]);
        for (int j = 0; j < 7; ++j) {
            if (r < bound[j]) continue;
            const double alpha = acos(bound[j] / r);
            for (int axis = 0; axis < 2; ++axis) {
                /* |cos(phi_axis - theta)| = d / r: theta = phi_axis -+ alpha, and the same + pi */
                const double base = phi - (axis ? PI / 2.0 : 0.0);
                const double cand[4] = {base - alpha, base + alpha, base - alpha + PI, base + alpha + PI};
                for (int t = 0; t < 4; ++t) {
                    double a = fmod(cand[t], two_pi);
                    if (a < 0.0) a += two_pi;
                    if (a >= two_pi) a -= two_pi;
                    tau[count++] = a;
                }
            }
        }
    }
    if (count == 0) {
        counts_at(u, v, n, rest, 0.0, cnt);
        *theta = 0.0;
        *loss = torq_o_code_loss(cnt);
        free(tau);
        return 0;
    }
    qsort(tau, (size_t)count, sizeof(double), cmp_double);
    int64_t uniq = 1;
    for (int64_t i = 1; i < count; ++i)
        if (tau[i] != tau[uniq - 1]) tau[uniq++] = tau[i];
    double best_theta = 0.0;
    unsigned __int128 best_key = 0;
    int have = 0;
    /* i = -1 is the interval that wraps around 2 pi, from the last critical angle to the first */
    for (int64_t i = -1; i + 1 < uniq; ++i) {
        double mid;
        if (i < 0) {
            mid = 0.5 * (tau[uniq - 1] + tau[0] + two_pi);
            if (mid >= two_pi) mid -= two_pi;
        } else {
            mid = 0.5 * (tau[i] + tau[i + 1]);
        }
        counts_at(u, v, n, rest, mid, cnt);
        const unsigned __int128 key = sum_squares(cnt);
        if (!have || key < best_key || (key == best_key && mid < best_theta)) {
            best_key = key;
            best_theta = mid;
            have = 1;
        }
    }
    counts_at(u, v, n, rest, best_theta, cnt);
    *theta = best_theta;
    *loss = torq_o_code_loss(cnt);
    free(tau);
    return uniq;
}

/* Algorithm 2.  X: n blocks of 32 values (after the inter-block rotation).  Each pass evaluates the
 * current rotation (S-step: s_b from the block maximum of Z = X R by the quantiser's own rule;
 * histograms and the loss of Z / s), stops when the loss fell by no more than eps since the last
 * pass, and otherwise takes the R-step: the k_top most imbalanced columns form the pool, the P
 * best-scoring disjoint pairs of the pool are taken in order of their score, and each pair is turned
 * by its exact best angle (the histograms follow every turn).  A last evaluation follows the last
 * R-step.  losses[i] is the loss seen by evaluation i (at most max_iter + 1 of them, *n_eval says
 * how many); R is the rotation of the evaluation with the smallest loss, the earliest among equals. */
void torq_o_intra_rotation(const double *X, int64_t n, int max_iter, int k_top, int P, double lambda,
                           double eps, double *R_out, double *losses, int *n_eval)
{
    double R[BLK][BLK], best_R[BLK][BLK];
    double *Z = (double *)malloc(sizeof(double) * (size_t)n * BLK);
    double *u = (double *)malloc(sizeof(double) * (size_t)n);
    double *v = (double *)malloc(sizeof(double) * (size_t)n);
    double h[BLK], H[BLK * BLK], best_loss = 0.0;
    uint64_t counts[BLK * 8], total[8];
    for (int i = 0; i < BLK; ++i)
        for (int j = 0; j < BLK; ++j) R[i][j] = (i == j) ? 1.0 : 0.0;
    *n_eval = 0;
    for (int iter = 0;; ++iter) {
        /* S-step and evaluation: Z = S^-1 X R */
        for (int64_t b = 0; b < n; ++b) {
            double amax = 0.0;
            for (int k = 0; k < BLK; ++k) {
                double acc = 0.0;
                for (int i = 0; i < BLK; ++i) acc += X[b * BLK + i] * R[i][k];
                Z[b * BLK + k] = acc;
                if (fabs(acc) > amax) amax = fabs(acc);
            }
            const double s = ldexp(1.0, (int)torq_o_e8m0_from_amax((float)amax) - 127);
            for (int k = 0; k < BLK; ++k) Z[b * BLK + k] /= s;
        }
        for (int i = 0; i < BLK * 8; ++i) counts[i] = 0;
        for (int64_t b = 0; b < n; ++b)
            for (int k = 0; k < BLK; ++k) counts[k * 8 + torq_o_mag_code(Z[b * BLK + k])] += 1;
        for (int j = 0; j < 8; ++j) {
            total[j] = 0;
            for (int k = 0; k < BLK; ++k) total[j] += counts[k * 8 + j];
        }
        const double loss = torq_o_code_loss(total);
        losses[*n_eval] = loss;
        if (*n_eval == 0 || loss < best_loss) {
            best_loss = loss;
            memcpy(best_R, R, sizeof(R));
        }
        *n_eval += 1;
        if (iter >= max_iter) break;
        if (iter > 0 && !(losses[iter - 1] - loss > eps)) break;

        /* R-step: pool, pairs */
        torq_o_pair_scores(counts, lambda, h, H);
        int in_pool[BLK], used[BLK];
        for (int k = 0; k < BLK; ++k) in_pool[k] = used[k] = 0;
        for (int t = 0; t < k_top && t < BLK; ++t) {
            int arg = -1;
            for (int k = 0; k < BLK; ++k)
                if (!in_pool[k] && (arg < 0 || h[k] > h[arg])) arg = k;
            in_pool[arg] = 1;
        }
        for (int l = 0; l < P; ++l) {
            int bp = -1, bq = -1;
            for (int p = 0; p < BLK; ++p)
                for (int q = p + 1; q < BLK; ++q) {
                    if (!in_pool[p] || !in_pool[q] || used[p] || used[q]) continue;
                    if (bp < 0 || H[p * BLK + q] > H[bp * BLK + bq]) {
                        bp = p;
                        bq = q;
                    }
                }
            if (bp < 0) break;
            used[bp] = used[bq] = 1;
            /* the pair's columns, the occupancy of all the others, the exact angle */
            uint64_t rest[8];
            for (int j = 0; j < 8; ++j) rest[j] = total[j] - counts[bp * 8 + j] - counts[bq * 8 + j];
            for (int64_t b = 0; b < n; ++b) {
                u[b] = Z[b * BLK + bp];
                v[b] = Z[b * BLK + bq];
            }
            double theta, l_pair;
            torq_o_best_angle(u, v, n, rest, &theta, &l_pair);
            /* R <- R G_(p,q)(theta), Z <- Z G_(p,q)(theta): column p becomes p cos + q sin,
             * column q becomes -p sin + q cos */
            const double c = cos(theta), sn = sin(theta);
            for (int i = 0; i < BLK; ++i) {
                const double rp = R[i][bp], rq = R[i][bq];
                R[i][bp] = rp * c + rq * sn;
                R[i][bq] = -rp * sn + rq * c;
            }
            for (int j = 0; j < 8; ++j) counts[bp * 8 + j] = counts[bq * 8 + j] = 0;
            for (int64_t b = 0; b < n; ++b) {
                const double zp = u[b] * c + v[b] * sn, zq = -u[b] * sn + v[b] * c;
                Z[b * BLK + bp] = zp;
                Z[b * BLK + bq] = zq;
                counts[bp * 8 + torq_o_mag_code(zp)] += 1;
                counts[bq * 8 + torq_o_mag_code(zq)] += 1;
            }
            for (int j = 0; j < 8; ++j) total[j] = rest[j] + counts[bp * 8 + j] + counts[bq * 8 + j];
        }
    }
    memcpy(R_out, best_R, sizeof(best_R));
    free(Z);
    free(u);
    free(v);
}

int torq_o_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
