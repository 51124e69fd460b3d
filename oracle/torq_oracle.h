/*
 * TORQ CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, step-by-step C implementation of the online inference path of
 * TORQ (Appendix A.3, Algorithm 3) and of the MXFP4 quantiser (Section 4,
 * Eq. 1), written from the paper.  It exists so that the GPU library can be
 * checked against something independent of it.  It shares no code, header,
 * table or constant with the HIP path, and nothing in the product may call it:
 * only the tests, the smoke check and the benchmark's CPU-baseline leg do.
 *
 * Arithmetic is C double except where the format fixes a precision (bf16 and
 * fp32 bit patterns, the e2m1 / E8M0 encodings).  Loops follow the paper's
 * index order; the only concession to speed is an OpenMP "parallel for" over
 * independent token rows, which does not reorder any sum.
 *
 * Notation (Section 4, "Notations"): a token row x of d features is viewed as
 * X[b][k] = x[32*b + k], B = d/32 microscaling blocks of 32 elements.  R_inter
 * is G x G and acts on each run of G consecutive blocks (G divides B; G = B is
 * Algorithm 3 as printed).  R_intra is 32 x 32.
 *
 * Parity status of the pieces:
 *   - bf16 conversion, E8M0 scale, e2m1 rounding, nibble packing, rotation,
 *     reference GEMM, variance equaliser (greedy and butterfly), block Gram matrix (whole and per
 *     position), MXINT4 / NVFP4 quantisers, code histogram,
 *     occupancy loss, pair scores, exact angle solver and the Algorithm 2 loop:
 *     pinned by tests/test_oracle_*.py.  Algorithm 2 leaves its loop control
 *     open (what the loss change is measured between, which rotation is
 *     returned, the rounding rule of the scale): the definition of
 *     torq_o_intra_rotation states the reading taken.
 *   - rotations that the paper would obtain by calibrating on real model
 *     activations: parity unpinned (no such data exists here); seeded random
 *     orthogonal matrices and the equaliser below stand in for them.
 */
#ifndef TORQ_ORACLE_H
#define TORQ_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* bf16 <-> fp32.  Widening is exact; narrowing is round-to-nearest-even. */
float    torq_o_bf16_to_f32(uint16_t h);
uint16_t torq_o_f32_to_bf16(float f);

/* Algorithm 3 step 2 alone: Y = R_inter X on every run of G blocks, double. */
void torq_o_rotate_inter(const double *x, int64_t M, int d, int G,
                         const float *R_inter, double *y);
/* Algorithm 3 step 3 alone: Z = Y R_intra on every block, double. */
void torq_o_rotate_intra(const double *y, int64_t M, int d,
                         const float *R_intra, double *z);

/* Algorithm 3 steps 1-3 on bf16 rows.  z_f32 (may be NULL) receives the result
 * rounded once to fp32; z_f64 (may be NULL) the unrounded doubles. */
void torq_o_rotate(const uint16_t *x_bf16, int64_t M, int d, int G,
                   const float *R_inter, const float *R_intra,
                   float *z_f32, double *z_f64);

/* Algorithm 3 step 5 option A without the scales (they are already inside the
 * dequantised values): x = R_inter^T Z R_intra^T, double.  Test use only. */
void torq_o_rotate_inverse(const double *z, int64_t M, int d, int G,
                           const float *R_inter, const float *R_intra,
                           double *x);

/* Shared scale of one block (Eq. 1 read with the OCP MX rule): E8M0 byte such
 * that 2^(byte-127) = 2^(floor(log2 amax) - 2), clamped to [0, 254]. */
uint8_t torq_o_e8m0_from_amax(float amax);

/* Nearest e2m1 code (Eq. 1's projection Q) of an already-normalised value:
 * bit 3 = sign, bits 2..0 index {0, .5, 1, 1.5, 2, 3, 4, 6}; ties go to the
 * code whose index is even; magnitudes above 6 saturate. */
uint8_t torq_o_e2m1_from_f32(float a);
/* value of a 4-bit code */
float   torq_o_e2m1_value(uint8_t code);

/* Algorithm 3 step 4 on fp32 rows: scales[M][d/32], codes[M][d/2] with the
 * even element in the low nibble. */
void torq_o_quantize(const float *z, int64_t M, int d,
                     uint8_t *codes, uint8_t *scales);
/* "De-quantize" line of step 4: zhat = value(code) * 2^(byte-127), fp32 exact */
void torq_o_dequantize(const uint8_t *codes, const uint8_t *scales,
                       int64_t M, int d, float *zhat);

/* Other 4-bit block formats behind the same rotations (Section 6, Table 5); the paper defines
 * neither, the definitions state the readings.  MXINT4: 32-element blocks, E8M0 scale as above,
 * integer elements in [-7, 7] as two's-complement nibbles.  NVFP4: 16-element blocks, an FP8 E4M3
 * scale byte per block ([M][d/16]) on top of the tensor-wide fp32 scale global_scale > 0, e2m1
 * elements.  Packing as above. */
float   torq_o_e4m3_value(uint8_t code);
uint8_t torq_o_e4m3_from_f32(float t);   /* t >= 0: nearest, ties to the even code, saturating at 448 */
void torq_o_quantize_mxint4(const float *z, int64_t M, int d, uint8_t *codes, uint8_t *scales);
void torq_o_dequantize_mxint4(const uint8_t *codes, const uint8_t *scales, int64_t M, int d, float *zhat);
void torq_o_quantize_nvfp4(const float *z, int64_t M, int d, float global_scale, uint8_t *codes,
                           uint8_t *scales_e4m3);
void torq_o_dequantize_nvfp4(const uint8_t *codes, const uint8_t *scales_e4m3, int64_t M, int d,
                             float global_scale, float *zhat);

/* steps 1-4 in one call (rotate in double, round to fp32, quantise) */
void torq_o_rotate_quantize(const uint16_t *x_bf16, int64_t M, int d, int G,
                            const float *R_inter, const float *R_intra,
                            uint8_t *codes, uint8_t *scales);

/* Algorithm 3 "Return": y = W' vec(Zhat) for every token.
 * out[m][n] = sum_j zhatA[m][j] * zhatW[n][j], accumulated in double in
 * index order, rounded once to bf16.  out_f64 (may be NULL) is unrounded. */
void torq_o_gemm(const uint8_t *A_q, const uint8_t *A_s,
                 const uint8_t *W_q, const uint8_t *W_s,
                 int64_t M, int64_t N, int d,
                 uint16_t *out_bf16, double *out_f64);
/* the same sum for `count` chosen (m, n) pairs */
void torq_o_gemm_sampled(const uint8_t *A_q, const uint8_t *A_s,
                         const uint8_t *W_q, const uint8_t *W_s,
                         int d, int64_t count,
                         const int64_t *ms, const int64_t *ns,
                         uint16_t *out_bf16, double *out_f64);

/* The statistic Algorithm 1 starts from (Section 5.1; Section 4.2, sigma_b^2 = E||z_b||^2): the
 * block Gram matrix Sigma[b][b'] = mean over token-groups of <x_b, x_b'>, a token-group being one
 * run of G consecutive 32-element blocks of one row (every row of [M, d] holds d/32/G of them).
 * Sigma is G x G, row-major, double.  Its diagonal holds the mean block energies. */
void torq_o_block_gram(const uint16_t *x_bf16, int64_t M, int d, int G, double *Sigma);
/* Section 4.2, Theorem 4.1: the per-position covariance matrices Sigma_k, [32][G][G]; their sum is Sigma. */
void torq_o_block_gram_positions(const uint16_t *x_bf16, int64_t M, int d, int G, double *Sigma_pos);

/* Algorithm 1 with the equalising angle (the printed Jacobi angle separates
 * the two diagonal entries instead of moving one onto the target).  Sigma is
 * B x B symmetric, overwritten by R Sigma R^T; R receives the rotation.
 * Returns the number of plane rotations used (at most B-1), or -1 if a pair
 * with opposite deviation signs could not be found. */
int torq_o_equalize(double *Sigma, int B, double eps, double *R);

/* The same output condition reached by a butterfly of plane rotations (B a power of two): round t
 * turns the B/2 pairs (p, p + B / 2^(t+1)) by the angles that make each pair's two diagonal entries
 * equal.  Sigma is overwritten with R Sigma R^T; R: B*B; tangents: log2(B) * B/2, the tangent of
 * every pair's angle, rounds in order, pairs in increasing p. */
void torq_o_equalize_butterfly(double *Sigma, int B, double *R, double *tangents);

/* ---- intra-block calibration (Section 5.2, Algorithm 2, Appendix A.4 / A.5) ---- */

/* Column-wise codebook histogram (Appendix A.5, N_j^(k)): counts[k * 8 + j] = number of blocks,
 * over all rows, whose element k carries the magnitude codeword j (the code's low three bits). */
void torq_o_code_histogram(const uint8_t *codes, int64_t M, int d, uint64_t *counts);

/* Codebook occupancy equilibrium loss (Section 5.2): sum_j (p_j - 1/8)^2 with p_j = n[j] / sum n. */
double torq_o_code_loss(const uint64_t n[8]);

/* Appendix A.5: imbalance h_k of every column, and the pair score
 * H[k][l] = h_k + h_l + lambda * c_kl, c_kl = - sum_j (p_j^(k) - 1/8)(p_j^(l) - 1/8). */
void torq_o_pair_scores(const uint64_t *counts /* [32][8] */, double lambda, double *h /* [32] */,
                        double *H /* [32][32] */);

/* Index j of the magnitude interval I_j (Section 5.2, decision boundaries d_j) that holds |a|. */
int torq_o_mag_code(double a);

/* Appendix A.4: the Givens angle that minimises the occupancy loss for one column pair.
 * u, v: the n normalised values z / s of the two columns (S is fixed in the R-step); rest[j]:
 * occupancy counts of all other columns.  Under the angle theta the columns become
 * u cos + v sin and -u sin + v cos.  Every critical angle (a sample's projected magnitude on
 * either axis equal to a decision boundary) is enumerated, the occupancy is counted afresh at the
 * midpoint of every interval between neighbouring critical angles (including the one that wraps
 * around 2 pi), and the smallest loss wins, the smallest angle among equals.  Returns the number of
 * intervals examined; with no critical angle at all the loss is constant and theta = 0. */
int64_t torq_o_best_angle(const double *u, const double *v, int64_t n, const uint64_t rest[8],
                          double *theta, double *loss);

/* Algorithm 2 on n sample blocks X[n][32]; see the definition for the reading of the loop. */
void torq_o_intra_rotation(const double *X, int64_t n, int max_iter, int k_top, int P, double lambda,
                           double eps, double *R /* [32][32] */, double *losses /* [max_iter + 1] */,
                           int *n_eval);

/* number of OpenMP threads the row loops will use */
int torq_o_threads(void);

#ifdef __cplusplus
}
#endif
#endif
