// Host-side declarations shared by the translation units of libtorq.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/torq.h"

struct torq_rotation {
  int d;
  int G;
  int KS;            // ceil(G / 32): k-steps of the inter-block contraction
  int device;        // device the tables live on
  // R_inter as bf16 hi and lo parts, [G][KS*32] row-major, zero-padded columns
  uint16_t *inter_hi, *inter_lo;
  // the same values in the order in which the lanes of v_mfma_f32_32x32x16_bf16 take them as B operand,
  // [tile NW = ceil(G/32)][k-step 2 NW][lane 64][8], zero past G, so that a wave's load of one operand is
  // 1 KiB of consecutive bytes (from the row-major table it touches 32 cache lines)
  uint16_t *inter32f_hi, *inter32f_lo;
  // R_intra^T rows permuted for the accumulator layout, bf16 hi and lo, [32][32]
  uint16_t *intra_hi, *intra_lo;
  // the same matrix as the A operand of v_mfma_f32_32x32x16_bf16 (two k-steps), bf16 hi and lo
  uint16_t *intra32_hi, *intra32_lo;
  // optional: R_inter as a butterfly of plane rotations (rotate_butterfly.hip), the per-lane
  // coefficient table [butterfly_coef_count(G)][32]; nullptr for a dense R_inter
  float *butterfly;
  // DECODE_CTR_WORDS counters (zero between launches) on which torq_linear_single_launch synchronises
  // its rotating and its multiplying workgroups (mxfp4_gemm_skinny.hip)
  unsigned *decode_ctr;
};
constexpr int DECODE_CTR_WORDS = 32 * 131;
constexpr int DECODE_ERR = 32 * 130;      // the sticky "a workgroup gave up" word among them

namespace torq {

// fp32 rows -> a 4-bit block format (FMT_* of torq_device.h = TORQ_FMT_* of torq.h).  nblk = number
// of 32-element blocks (M * d / 32); global_scale is NVFP4's tensor-wide scale, else ignored.
hipError_t launch_quantize_f32(const float *z, int64_t nblk, int format, float global_scale, uint8_t *codes,
                               uint8_t *scales, hipStream_t stream);

// Two-level rotation (+ quantisation).  Exactly one of (codes, scales) / z_out is used:
// z_out != nullptr writes the rotated fp32 values instead of quantising to `format`.
hipError_t launch_rotate(const torq_rotation *r, const void *x_bf16, int64_t M, int format, float global_scale,
                         uint8_t *codes, uint8_t *scales, float *z_out, hipStream_t stream);

// The same for a handle whose R_inter is a butterfly (r->butterfly != nullptr; G in 32, 64, 128, 256).
int butterfly_coef_count(int G);
hipError_t launch_rotate_butterfly(const torq_rotation *r, const void *x_bf16, int64_t M, int format,
                                   float global_scale, uint8_t *codes, uint8_t *scales, float *z_out,
                                   hipStream_t stream);

// workspace: optional device scratch of mxfp4_gemm_workspace_bytes(M, N, d) bytes; with it, shapes
// with few output tiles and a long reduction are cut along k (fp32 pieces added in a fixed order).
size_t mxfp4_gemm_workspace_bytes(int64_t M, int64_t N, int d);
// what launch_mxfp4_gemm would do with a workspace of that size (operands assumed 16-byte aligned)
void mxfp4_gemm_plan(int64_t M, int64_t N, int d, size_t workspace_bytes, int *skinny, int *tile_m, int *tile_n,
                     int *splits);
// the tiled kernel on a given plan: tile 0 ... 3 = 256x256, 256x128, 128x128, 128x64; k_pieces > 1 needs the
// workspace (k_pieces * M * N floats) and d / 512 divisible by it; deep: the deeper load pipeline (tiles 2, 3)
hipError_t launch_mxfp4_gemm_forced(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                                    void *out_bf16, int64_t M, int64_t N, int d, int tile, int k_pieces, int deep,
                                    void *workspace, size_t workspace_bytes, hipStream_t stream);
// N, or the leading output columns that a first launch of whole rounds of 256 x 256 tiles takes (the plan
// above is then that launch's; the remaining columns are a product of their own with its own plan)
int64_t mxfp4_gemm_main_columns(int64_t M, int64_t N, int d, size_t workspace_bytes);
hipError_t launch_mxfp4_gemm(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q,
                             const uint8_t *W_s, void *out_bf16, int64_t M, int64_t N, int d,
                             void *workspace, size_t workspace_bytes, hipStream_t stream);

// The same product for 1 <= M <= 64 (weight-streaming layout); called by launch_mxfp4_gemm when
// mxfp4_gemm_skinny_fits (the scale rows it stages fit the LDS).
bool mxfp4_gemm_skinny_fits(int64_t M, int d);
hipError_t launch_mxfp4_gemm_skinny(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q,
                                    const uint8_t *W_s, void *out_bf16, int64_t M, int64_t N, int d,
                                    hipStream_t stream);
// torq_linear for at most 64 rows in one launch: rotate + quantise (the 16-block body, G = 128) in the
// first workgroups of the weight-streaming GEMM.  Preconditions: r->G == 128, dense R_inter,
// 1 <= M <= 64, mxfp4_gemm_skinny_fits(M, r->d); A_q / A_s are the workspace's code and scale areas.
// spin_limit: polls before a waiting workgroup gives up; raise_ready = 0 withholds the hand-off
// (test of the give-up path: every workgroup still exits).
hipError_t launch_torq_linear_decode(const torq_rotation *r, const void *x_bf16, uint8_t *A_q, uint8_t *A_s,
                                     const uint8_t *W_q, const uint8_t *W_s, void *out, int64_t M, int64_t N,
                                     int spin_limit, int raise_ready, hipStream_t stream);
// torq_linear for a few token-groups with rotate + quantise inside every workgroup of the GEMM's launch
// (no hand-off between workgroups, the packed activations stay in LDS; workgroup 0 leaves a copy in
// A_q / A_s).  torq_linear_local_fits: dense R_inter, G = 112 or 128, at most four token-groups.
bool torq_linear_local_fits(const torq_rotation *r, int64_t M);
// ... and is measured faster than the two launches (what torq_linear itself then does)
bool torq_linear_local_pays(const torq_rotation *r, int64_t M, int64_t N);
hipError_t launch_torq_linear_local(const torq_rotation *r, const void *x_bf16, uint8_t *A_q, uint8_t *A_s,
                                    const uint8_t *W_q, const uint8_t *W_s, void *out, int64_t M, int64_t N,
                                    hipStream_t stream);
// all of the handle's counters back to zero, the sticky error word included
hipError_t launch_decode_ctr_reset(const torq_rotation *r, hipStream_t stream);

// Block Gram matrix of the runs of G blocks (block_gram.hip): TG token-groups of G * 32 bf16 each.
size_t block_gram_workspace_bytes(int G);
hipError_t launch_block_gram(const void *x_bf16, int64_t TG, int G, int position, double *Sigma, void *workspace,
                             hipStream_t stream);

// Codeword histogram per in-block position (code_histogram.hip): nblk blocks of 16 code bytes.
size_t code_histogram_workspace_bytes();
hipError_t launch_code_histogram(const uint8_t *codes, int64_t nblk, uint64_t *counts, void *workspace,
                                 hipStream_t stream);

// Host side of the intra-block calibration (intra_calib.hip).
void intra_pair_scores(const uint64_t *counts, double lambda, double *h, double *H);
int64_t intra_best_angle(const double *u, const double *v, int64_t n, const uint64_t rest[8], double *theta,
                         double *loss);
void intra_rotation(const float *X, int64_t n, int max_iter, int k_top, int P, double lambda, double eps,
                    double *R_out, double *losses, int *n_eval);

// 1024 x 256 lanes issue iters x 16 MFMAs each on operands taken from `words` (see diag.hip).
hipError_t launch_mfma_burn(int kind, const uint32_t *words, uint32_t n_words, int iters, float *sink,
                            hipStream_t stream);

// The two headline kernels with parts of their work left out (SKIP bits documented at the kernels):
// what each part costs in time on this machine.  Outputs are meaningless by design.
hipError_t launch_mxfp4_gemm_ablated(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                                     void *out_bf16, int64_t M, int64_t N, int d, int skip, hipStream_t stream);
// the persistent form of the tiled GEMM (tile 0: 256 x 256, 1: 256 x 128) on `workgroups` workgroups
hipError_t launch_mxfp4_gemm_persistent(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                                        void *out_bf16, int64_t M, int64_t N, int d, int tile, int workgroups,
                                        hipStream_t stream);
hipError_t launch_rotate_ablated(const torq_rotation *r, const void *x, int64_t M, uint8_t *codes, uint8_t *scales,
                                 int skip, hipStream_t stream);
// plain copy of `bytes` (a multiple of 16) device bytes, the traffic counters' yardstick (diag.hip)
hipError_t launch_diag_copy(const void *src, void *dst, size_t bytes, hipStream_t stream);

}  // namespace torq
