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

int torq_o_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
