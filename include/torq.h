/*
 * libtorq -- MI355X (gfx950) kernels for the online path of TORQ:
 * two-level orthogonal rotation of bf16 activations, MXFP4 quantisation of the
 * result, and the W4A4 MXFP4 GEMM that consumes it.
 *
 * Plain C ABI.  Unless a parameter is named *_host, every pointer is a DEVICE
 * pointer owned by the caller (allocated by whatever the caller likes, e.g.
 * torch); the library never frees or keeps it.  `stream` is a hipStream_t
 * passed as void* (NULL = the default stream).  Every compute call only
 * enqueues work on that stream and returns; it allocates nothing.  Calls on
 * different streams may overlap; a rotation handle is immutable after creation
 * and may be shared by any number of concurrent calls.
 *
 * Notation (paper, Section 4 "Notations"): a token row x has d features and is
 * viewed as X[b][k] = x[32 b + k]: B = d/32 microscaling blocks of 32 elements.
 *
 * Return value: TORQ_OK (0) or a negative error code; on error nothing has been
 * launched and no output has been touched.  M = 0 (or N = 0) is TORQ_OK and a
 * no-op.  Inputs are assumed finite; a block that holds Inf/NaN gets scale
 * byte 0xFF or 0xFD.. and unspecified codes.
 */
#ifndef TORQ_H
#define TORQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    TORQ_OK          =  0,
    TORQ_EINVAL      = -1,  /* null pointer, negative size, d % 32 != 0, G does not divide d/32,
                               G not a multiple of 16 or above TORQ_MAX_G, N or d beyond the limits below */
    TORQ_EALIGN      = -2,  /* a device pointer is not 16-byte aligned */
    TORQ_EWORKSPACE  = -3,  /* workspace smaller than torq_linear_workspace_bytes() */
    TORQ_EHIP        = -4,  /* the HIP runtime reported an error (allocation, copy or launch) */
    TORQ_ENODEVICE   = -5,  /* no gfx950 device is current */
    TORQ_ECONVERGE   = -6,  /* torq_equalize_inter: no pair of blocks with deviations of opposite sign is
                               left although the tolerance is not met (Sigma not symmetric, or eps below
                               what double precision can reach) */
    TORQ_ETOOBIG     = -7,  /* torq_linear_static: the packed activations do not fit TORQ_STATIC_SCRATCH_BYTES */
    TORQ_ENOMEM      = -8   /* a host routine (handle creation, the equalisers, the intra-block calibration)
                               could not allocate host memory */
};

#define TORQ_BLOCK 32       /* elements per microscaling block (the paper's K) */
#define TORQ_MAX_G 256      /* largest supported inter-block rotation */

/* Text for a status code (static storage, never NULL). */
const char *torq_status_string(int status);

/* ------------------------------------------------------------------------ */
/* Rotation handle: the offline parameters R_inter and R_intra of Algorithm 3
 * (Appendix A.3, "Offline parameters"), uploaded once and laid out for the
 * matrix cores.
 *
 *   d             feature dimension, multiple of 32
 *   G             size of R_inter.  R_inter acts on each run of G consecutive
 *                 blocks of a row (block-diagonal over the row, Appendix A.7
 *                 "decomposed into block-diagonal"); G = d/32 is Algorithm 3
 *                 as printed.  G must be a multiple of 16, at most TORQ_MAX_G,
 *                 and divide d/32.
 *   R_inter_host  HOST pointer, G*G floats, row-major: Y = R_inter X
 *                 (Algorithm 3, step 2: Y[b][k] = sum_b' R_inter[b][b'] X[b'][k])
 *   R_intra_host  HOST pointer, 32*32 floats, row-major: Z = Y R_intra
 *                 (Algorithm 3, step 3: Z[b][k] = sum_k' Y[b][k'] R_intra[k'][k])
 *
 * The handle owns a few hundred KiB of device memory on the device that is
 * current at creation; it must be used on that device.  Creation synchronises
 * with the device (not a hot call).  Orthogonality is not checked. */
typedef struct torq_rotation torq_rotation_t;

int  torq_rotation_create(torq_rotation_t **out, int d, int G,
                          const float *R_inter_host, const float *R_intra_host);
void torq_rotation_destroy(torq_rotation_t *r);   /* NULL is allowed */
int  torq_rotation_d(const torq_rotation_t *r);
int  torq_rotation_G(const torq_rotation_t *r);

/* ------------------------------------------------------------------------ */
/* Algorithm 3 steps 1-4 (Appendix A.3): reshape, inter-block rotation,
 * intra-block rotation, MXFP4 quantisation (Section 4, Eq. 1).
 *
 *   x_bf16  [M][d] bf16, row-major
 *   codes   [M][d/2] bytes: e2m1 codes (bit 3 sign, bits 2..0 index into
 *           {0, .5, 1, 1.5, 2, 3, 4, 6}), element 2j in the low nibble of byte j
 *   scales  [M][d/32] bytes: E8M0 shared exponent of each block, value
 *           2^(byte-127) = 2^(floor(log2 amax) - 2), clamped to [0, 254]
 *
 * The rotation is computed on the matrix cores in split bf16 with fp32
 * accumulation; the rotated values differ from exact arithmetic by far less
 * than 1e-3 of the row RMS, so a code or scale can differ from an exact
 * computation only where a rotated value sits on a rounding boundary. */
int torq_rotate_quantize(const torq_rotation_t *r, const void *x_bf16, int64_t M,
                         uint8_t *codes, uint8_t *scales, void *stream);

/* Algorithm 3 steps 1-3 only: the rotated values Z as fp32 [M][d].  Test hook
 * for the accuracy of the rotation; same arithmetic as torq_rotate_quantize. */
int torq_rotate(const torq_rotation_t *r, const void *x_bf16, int64_t M,
                float *z_f32, void *stream);

/* Algorithm 3 step 4 only (Section 4, Eq. 1) on fp32 input z [M][d]: per block
 * amax -> E8M0 scale -> round to nearest e2m1 (ties to the even code, values
 * above 6 saturate, sign bit copied) -> packed codes.  Same quantiser code as
 * inside torq_rotate_quantize; bit-exact by specification. */
int torq_quantize_f32(const float *z_f32, int64_t M, int d,
                      uint8_t *codes, uint8_t *scales, void *stream);

/* The linear layer that consumes the quantised activations with the inverse
 * rotation folded into its weights (Section 5; Algorithm 3 "Return"):
 *
 *   out[m][n] = sum_kb 2^(A_s[m][kb] + W_s[n][kb] - 254)
 *                 * sum_{k<32} val(A[m][32 kb + k]) * val(W[n][32 kb + k])
 *
 * on the block-scaled fp4 matrix cores, fp32 accumulation, one rounding to
 * bf16 (nearest even).  A_q [M][d/2], A_s [M][d/32], W_q [N][d/2],
 * W_s [N][d/32] in the layout torq_rotate_quantize writes; out [M][N] bf16
 * row-major.  d must be a multiple of 128.  One or two kernel launches on
 * `stream` (mxfp4_gemm_main_columns below says which); every output is the sum
 * over k in the same order either way.  Weights are prepared offline by
 * running torq_rotate_quantize over the rows of W (the map x -> z is
 * orthogonal, so rotating W's rows is the weight fusion W' of Section 5). */
int mxfp4_gemm(const uint8_t *A_q, const uint8_t *A_s,
               const uint8_t *W_q, const uint8_t *W_s,
               void *out_bf16, int64_t M, int64_t N, int d, void *stream);

/* The same two calls for the other 4-bit block formats that Section 6 ("Generalizability to Other
 * Formats", Table 5) puts behind the rotations.  The paper names the formats without defining them;
 * the readings taken (all arithmetic in fp32, in this order):
 *   TORQ_FMT_MXFP4   as torq_rotate_quantize / torq_quantize_f32.
 *   TORQ_FMT_MXINT4  32-element blocks and the E8M0 scale of MXFP4; elements round(z / scale) to the
 *                    nearest integer, ties to even, clamped to [-7, 7], two's-complement nibbles.
 *   TORQ_FMT_NVFP4   16-element blocks, each with an OCP FP8 E4M3 scale byte, scales [M][d/16], on
 *                    top of the tensor-wide fp32 `global_scale` (finite, > 0; ignored by the other
 *                    formats): byte = E4M3 nearest to amax / (6 * global_scale) (ties to the even
 *                    code, saturating at 448 = 0x7E), S = value(byte) * global_scale, element = e2m1
 *                    code of z / S as in MXFP4 (a block whose byte is 0 keeps only the signs).
 * Nibble packing, alignment and error codes as above; an unknown format is TORQ_EINVAL.  Only the
 * quantisers exist for these formats: the GEMM of this library consumes MXFP4. */
#define TORQ_FMT_MXFP4  0
#define TORQ_FMT_MXINT4 1
#define TORQ_FMT_NVFP4  2
int torq_rotate_quantize_fmt(const torq_rotation_t *r, const void *x_bf16, int64_t M, int format,
                             float global_scale, uint8_t *codes, uint8_t *scales, void *stream);
int torq_quantize_f32_fmt(const float *z_f32, int64_t M, int d, int format, float global_scale,
                          uint8_t *codes, uint8_t *scales, void *stream);

/* mxfp4_gemm with scratch memory.  Same operands, same result up to the order of the fp32 sums.
 * When the output has too few tiles to occupy the GPU and the reduction is long (a few hundred
 * activation rows, e.g. a decode batch or a prefill chunk against a down projection), the k range
 * is cut into pieces that run as separate workgroups; their fp32 tiles go through `workspace` and a
 * second kernel adds them in a fixed order (deterministic) and rounds once to bf16.
 *   workspace  device, 16-byte aligned, at least mxfp4_gemm_workspace_bytes(M, N, d) bytes (0 for
 *              shapes that are not cut); NULL or too small: exactly mxfp4_gemm. */
size_t mxfp4_gemm_workspace_bytes(int64_t M, int64_t N, int d);
/* Which kernel the product of that shape runs on, given a workspace of that many bytes (0: as
 * mxfp4_gemm) and 16-byte aligned scale arrays: *weight_streaming = 1 for the kernel that streams
 * 16-row weight strips (at most 64 activation rows), else 0 and *tile_m x *tile_n is the output
 * tile; *k_pieces > 1 if the k range is cut.  Host only, launches nothing; for logs and tests. */
int mxfp4_gemm_plan(int64_t M, int64_t N, int d, size_t workspace_bytes, int *weight_streaming, int *tile_m,
                    int *tile_n, int *k_pieces);
/* A tile count just above a whole number of rounds (one 256 x 256 tile per compute unit) would leave
 * the last round mostly empty.  Such a product runs as two: a first launch computes the leading
 * output columns that make up whole rounds, and the remaining columns are a product of their own
 * (weight rows from that column on, same activations, same output rows).  Returns the number of those
 * leading columns (a multiple of 256), or N when the product is one: mxfp4_gemm_plan above then
 * describes the first launch, and mxfp4_gemm_plan(M, N - that, d, workspace_bytes) the remainder.
 * 0 for arguments that mxfp4_gemm_plan rejects.  Host only, launches nothing; for logs and tests. */
int64_t mxfp4_gemm_main_columns(int64_t M, int64_t N, int d, size_t workspace_bytes);
int mxfp4_gemm_ws(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                  void *out_bf16, int64_t M, int64_t N, int d, void *workspace, size_t workspace_bytes,
                  void *stream);

/* Algorithm 3 end to end ("output of the linear layer"): torq_rotate_quantize
 * into `workspace`, then mxfp4_gemm, on one stream.  workspace is device
 * memory of at least torq_linear_workspace_bytes(M, d) bytes, 256-byte aligned
 * sizes; its contents afterwards are the packed activations (codes, then
 * scales at offset M*d/2 rounded up to 256).  For a row or two of a decode step
 * (at most four token-groups, G = 112 or 128, packed weights up to 16 - 20 MB) both
 * steps run in ONE launch whose workgroups each rotate the rows themselves (form
 * (1) of torq_linear_single_launch): same codes, same outputs, bit for bit. */
size_t torq_linear_workspace_bytes(int64_t M, int d);
/* The same plus the scratch that lets the GEMM inside cut its k range (see mxfp4_gemm_ws);
 * torq_linear uses whatever it is given beyond torq_linear_workspace_bytes(M, d) for that. */
size_t torq_linear_workspace_bytes_n(int64_t M, int64_t N, int d);
int torq_linear(const torq_rotation_t *r, const void *x_bf16,
                const uint8_t *W_q, const uint8_t *W_s, void *out_bf16,
                int64_t M, int64_t N, void *workspace, size_t workspace_bytes,
                void *stream);

/* torq_linear for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operands, same
 * kernels and the same result, bit for bit, as torq_linear with a workspace of exactly
 * torq_linear_workspace_bytes(M, d) bytes (so the GEMM inside never cuts its k range); the packed
 * activations pass through an array of TORQ_STATIC_SCRATCH_BYTES bytes that is part of the library's
 * device image (every GPU the library runs on holds its own copy until the process ends).  The call
 * allocates nothing and frees nothing.
 *   torq_linear_workspace_bytes(M, d) must not exceed TORQ_STATIC_SCRATCH_BYTES (e.g. 64 rows of
 *   d = 28672, 1900 rows of d = 4096), else TORQ_ETOOBIG and nothing is launched.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams, different threads) race on it -- order them on one stream.  The array keeps the packed
 * activations of the last call; nothing in it has to start at zero, every call overwrites the part
 * it reads.  The first call on a device looks the array's address up (no allocation; not a call to
 * make for the first time under stream capture). */
#define TORQ_STATIC_SCRATCH_BYTES ((size_t)4 << 20)
int torq_linear_static(const torq_rotation_t *r, const void *x_bf16, const uint8_t *W_q, const uint8_t *W_s,
                       void *out_bf16, int64_t M, int64_t N, void *stream);

/* torq_linear for decode sizes in ONE kernel launch (Algorithm 3, steps 1-4 and "Return").  Same
 * arguments and workspace as torq_linear.  Two forms, chosen by the size:
 *
 * (1) Up to four token-groups in all (M * d / (32 G) <= 4: e.g. four rows of d = 4096, one of d = 14336
 *     or 16384), G = 112 or 128, a dense R_inter: EVERY workgroup of the weight-streaming GEMM rotates and
 *     quantises all rows itself into its LDS, behind its own weight reads; nothing is handed over between
 *     workgroups, the packed activations never leave the chip (workgroup 0 stores a copy to the workspace
 *     for the caller to inspect, which the launch does not read), and the handle's counters are neither
 *     read nor written.  The codes are torq_rotate_quantize's, bit for bit, and the product is mxfp4_gemm
 *     of them.  torq_linear itself takes this launch where it is measured faster than its two launches
 *     with weights that come from HBM (up to 20 MB of packed weights for one or two token-groups, 16 MB for
 *     three or four: [1, 4096] -> 4096 6.2 against 7.7 us, -> 8192 8.3 against 9.0, -> 14336 11.4 against 11.6).
 *
 * (2) Otherwise, up to 64 rows, G = 128, a dense R_inter: the first workgroups rotate and quantise one
 *     token-group each while the others, one per strip of weight rows, already have their weight scales
 *     and codes on the way and wait for the activations at a counter in device memory.
 *     The packed activations are left in the workspace as by torq_linear: torq_rotate_quantize's codes
 * and scale bytes, bit for bit, and the product is mxfp4_gemm of them.  Every workgroup exits: the wait is bounded.  A workgroup whose wait runs
 * out writes NaN to its outputs and raises an error word among the handle's counters that no launch
 * clears: from then on every launch of form (2) on that handle writes NaN to all of `out`
 * (the counters of the failed launch cannot be trusted any more) until
 * torq_linear_single_launch_reset has run; the calls themselves keep returning TORQ_OK, as they only
 * enqueue.  Calls on one
 * handle must not overlap in time (they share the handle's counters; stream order is enough).  On
 * this part the hand-off between workgroups costs what the second launch costs: measured against
 * torq_linear 13.1 against 13.5 us at [16, 4096] -> 14336,
 * 36.5 against 34.3 us at [16, 8192] -> 28672 and 85 against 37 us at [64, 8192] -> 28672 (where
 * torq_linear takes a tiled GEMM kernel), which is why torq_linear does not use form (2).
 *
 * Limits of both: d a multiple of 128 whose scale rows fit the LDS (every d up to 28672 does);
 * 0 <= M <= 64.  Anything else is TORQ_EINVAL. */
int torq_linear_single_launch(const torq_rotation_t *r, const void *x_bf16, const uint8_t *W_q, const uint8_t *W_s,
                              void *out_bf16, int64_t M, int64_t N, void *workspace, size_t workspace_bytes,
                              void *stream);
/* torq_linear_single_launch_reset: every counter of the handle back to zero, the error word included
 *   (one small kernel on `stream`; allowed under stream capture).
 * torq_linear_single_launch_gave_up: *gave_up = 1 if a launch on this handle has given up since the last
 *   reset, else 0.  Copies one word from the device with a blocking copy: not a hot call.
 * torq_linear_single_launch_probe: form (2) of torq_linear_single_launch (at any size it covers) with its
 *   two internal constants exposed, for tests of the give-up path that let every workgroup exit normally: spin_limit = how often a
 *   waiting workgroup polls before it gives up (1 .. 2^18; torq_linear_single_launch uses 2^18),
 *   withhold_ready != 0 = the rotating workgroups do their work but never hand over, so every
 *   multiplying workgroup gives up after spin_limit polls. */
int torq_linear_single_launch_reset(const torq_rotation_t *r, void *stream);
int torq_linear_single_launch_gave_up(const torq_rotation_t *r, int *gave_up);
int torq_linear_single_launch_probe(const torq_rotation_t *r, const void *x_bf16, const uint8_t *W_q,
                                    const uint8_t *W_s, void *out_bf16, int64_t M, int64_t N, void *workspace,
                                    size_t workspace_bytes, int spin_limit, int withhold_ready, void *stream);

/* ------------------------------------------------------------------------ */
/* Calibration of the inter-block rotation (Section 5.1, Algorithm 1).  Not part of the online
 * path: run once on calibration activations to obtain R_inter for torq_rotation_create.
 *
 * torq_block_gram: the statistic Algorithm 1 equalises,
 *   Sigma[b][b'] = mean over token-groups of sum_k X[b][k] X[b'][k],
 * a token-group being one run of G consecutive blocks of one row of x (Section 4.2: the diagonal
 * holds the block energies sigma_b^2 = E||x_b||^2 of Theorem 4.1).
 *   x_bf16     device, [M][d] bf16 row-major, 16-byte aligned; d % 32 == 0, (d/32) % G == 0,
 *              G a multiple of 16, at most TORQ_MAX_G
 *   Sigma      device, G*G doubles, row-major, overwritten (symmetric)
 *   workspace  device, at least torq_block_gram_workspace_bytes(G) bytes, 16-byte aligned, scratch
 * M = 0 is TORQ_EINVAL (a mean over nothing).  Sums are fp32 inside a workgroup and double across
 * workgroups, in a fixed order: the result is deterministic.
 *
 * torq_block_gram_positions: the same statistic kept apart by the position k inside a block, the
 * covariance matrices Sigma_k of Theorem 4.1 (Section 4.2; the calibration cost analysis of the
 * appendix counts "covariance matrices for all K positions"),
 *   Sigma_pos[k][b][b'] = mean over token-groups of X[b][k] X[b'][k],   k < 32,
 * whose sum over k is Sigma.  Arguments as torq_block_gram, with
 *   Sigma_pos  device, 32*G*G doubles, [k][b][b'], overwritten
 * One pass over x per position (32 launches of the same kernel on the stream).  Each matrix can be
 * handed to torq_equalize_inter; the online path of Algorithm 3 applies ONE R_inter to all
 * positions, so a per-position rotation is not something torq_rotation_create takes.
 *
 * torq_equalize_inter: Algorithm 1 on the HOST, in double.  Plane rotations of the pair (block
 * furthest above the mean energy c = tr(Sigma)/G, block furthest below it) until every diagonal
 * entry of R Sigma R^T is within eps of c; at most G-1 of them.  The rotation angle is the one that
 * puts the first block exactly on c (the angle printed in Algorithm 1 diagonalises the pair, which
 * moves the two energies apart and cannot meet the algorithm's own output condition).
 *   Sigma_host    HOST, G*G doubles, symmetric, not modified
 *   eps           absolute tolerance on the diagonal, >= 0 (e.g. 1e-12 * c)
 *   R_inter_host  HOST, G*G floats out, row-major, for torq_rotation_create (Y = R_inter X)
 *   steps         HOST, optional: number of plane rotations used
 * Returns TORQ_OK, TORQ_EINVAL (also for a Sigma with a NaN or an infinity), TORQ_ECONVERGE or
 * TORQ_ENOMEM. */
/* The inter-block rotation as a BUTTERFLY of plane rotations (what Section 5.1 calls an efficient
 * implementation of R_inter; Algorithm 1 itself picks its pairs greedily, one after the other, which
 * leaves a dense G x G matrix to multiply online).  Round t = 0 .. log2(G) - 1 turns the G/2
 * independent pairs of block rows (p, p + G / 2^(t+1)) by the angle that makes each pair's two
 * diagonal entries of Sigma equal; after the last round diag(R Sigma R^T) = tr(Sigma)/G * 1, the
 * same output condition (the equality case of Theorem 4.1).  Online this costs one fused
 * multiply-add per element and round in fp32 (log2(G) + 1 in all) instead of a dense G x G
 * contraction.
 *
 * torq_equalize_inter_butterfly (HOST, double):
 *   Sigma_host     G*G doubles, symmetric, finite, not modified; G in {32, 64, 128, 256}
 *   R_inter_host   optional, G*G floats out: the dense matrix of the returned tangents, for
 *                  checking, for weights prepared elsewhere, or for torq_rotation_create
 *   tangents_host  log2(G) * G/2 floats out: tan(theta) of every pair, rounds in order, pairs in
 *                  increasing p; |tan| <= 1
 * torq_rotation_create_butterfly: a handle whose inter-block rotation is that butterfly.  The rotation
 * is orthogonal whatever the tangents are, but the kernel carries every row divided by the product of
 * the cosines it has met, in fp32: |tan| must not exceed TORQ_BUTTERFLY_MAX_TAN (then that product
 * stays above 2^-65 and every coefficient below 2^73); beyond it, or for a NaN, TORQ_EINVAL.  Every
 * entry point that takes a handle works on it; destroy it with torq_rotation_destroy.  Other errors
 * as torq_rotation_create. */
#define TORQ_BUTTERFLY_MAX_TAN 256.0f
int torq_equalize_inter_butterfly(const double *Sigma_host, int G, float *R_inter_host, float *tangents_host);
int torq_rotation_create_butterfly(torq_rotation_t **out, int d, int G, const float *tangents_host,
                                   const float *R_intra_host);
size_t torq_block_gram_workspace_bytes(int G);
int torq_block_gram(const void *x_bf16, int64_t M, int d, int G, double *Sigma,
                    void *workspace, size_t workspace_bytes, void *stream);
int torq_block_gram_positions(const void *x_bf16, int64_t M, int d, int G, double *Sigma_pos,
                              void *workspace, size_t workspace_bytes, void *stream);
int torq_equalize_inter(const double *Sigma_host, int G, double eps, float *R_inter_host, int *steps);

/* ------------------------------------------------------------------------ */
/* Calibration of the intra-block rotation (Section 5.2, Algorithm 2; Appendix A.4, A.5).  Not part
 * of the online path: run once to obtain R_intra for torq_rotation_create.
 *
 * torq_code_histogram: the column-wise codebook histogram N_j^(k) of Appendix A.5 over packed codes
 * as the quantiser wrote them (the S-step of Section 5.2 is the quantiser's own scale, so the codes
 * of torq_rotate_quantize under the current R_intra are the occupancy that the loss of Section 5.2
 * measures):  counts[k * 8 + j] = number of 32-element blocks whose element k has the magnitude
 * codeword j = code & 7 (the sign bit is ignored).
 *   codes      device, [M][d/2] bytes as torq_rotate_quantize writes them, 16-byte aligned
 *   counts     device, 256 uint64, 8-byte aligned, overwritten
 *   workspace  device, at least torq_code_histogram_workspace_bytes() bytes, 16-byte aligned, scratch
 * M = 0 gives all-zero counts.  Integer work: the result is exact and deterministic.
 *
 * The remaining entry points run on the HOST, in double, on HOST arrays.
 *
 * torq_intra_pair_scores (Appendix A.5): h[k] = sum_j (p_j^(k) - 1/8)^2 and
 * H[k][l] = h[k] + h[l] + lambda * c_kl with c_kl = -sum_j (p_j^(k) - 1/8)(p_j^(l) - 1/8), from
 * counts[32][8] (a column without counts has p = 0).  h: 32 doubles, H: 32*32 doubles.
 *
 * torq_intra_best_angle (Appendix A.4): for the n normalised values (u, v) of one column pair and
 * the occupancy `rest` (8 counts) of all other columns, the angle theta in [0, 2 pi) that minimises
 * the loss when the pair becomes (u cos + v sin, -u sin + v cos): the midpoint of the best interval
 * between neighbouring critical angles, the smallest such midpoint among equally good intervals;
 * theta = 0 if there is no critical angle.  Equal losses are recognised exactly (the comparison is
 * made on the integer sum of squared counts).  `critical` (optional) receives the number of distinct
 * critical angles.  n <= TORQ_INTRA_MAX_SAMPLE; up to 56 events of 16 bytes per sample are held.
 *
 * torq_calibrate_intra (Algorithm 2) on a sample of n blocks X[n][32] (fp32, after the inter-block
 * rotation, e.g. rows of torq_rotate's output under R_intra = I).  Readings of the loop that
 * Algorithm 2 leaves open: an evaluation is the S-step (scale of each block from the maximum of
 * Z = X R by the quantiser's rule 2^(floor(log2 amax) - 2)) followed by the loss of Z / s; the loop
 * stops after max_iter R-steps or when the loss fell by no more than eps since the previous
 * evaluation; one R-step takes the k_top columns of largest h as the pool and turns the P
 * best-scoring disjoint pairs of the pool in order of their score, each by its exact angle with the
 * occupancy as the earlier turns left it (lower index first among equal scores); the result is the
 * rotation of the evaluation with the smallest loss.
 *   R_intra_host  32*32 floats out, row-major, Z = X R_intra (the layout torq_rotation_create takes)
 *   losses_host   max_iter + 1 doubles out: the loss of every evaluation
 *   n_eval        out: how many evaluations were made
 *   1 <= k_top <= 32, 1 <= P <= 16, 0 <= max_iter <= 1000, lambda >= 0, eps >= 0
 * All return TORQ_OK or TORQ_EINVAL (torq_code_histogram also TORQ_EALIGN, TORQ_EWORKSPACE, TORQ_EHIP). */
#define TORQ_INTRA_MAX_SAMPLE (1 << 22)
size_t torq_code_histogram_workspace_bytes(void);
int torq_code_histogram(const uint8_t *codes, int64_t M, int d, uint64_t *counts, void *workspace,
                        size_t workspace_bytes, void *stream);
int torq_intra_pair_scores(const uint64_t *counts_host, double lambda, double *h_host, double *H_host);
int torq_intra_best_angle(const double *u_host, const double *v_host, int64_t n, const uint64_t *rest_host,
                          double *theta, double *loss, int64_t *critical);
int torq_calibrate_intra(const float *X_host, int64_t n, int max_iter, int k_top, int P, double lambda,
                         double eps, float *R_intra_host, double *losses_host, int *n_eval);

/* ------------------------------------------------------------------------ */
/* Diagnostics (not a step of Algorithm 3): the rate the matrix cores sustain on
 * this machine with nothing else running, on operands the caller supplies --
 * the ceiling to read the MFMA-bound kernels against, since the part lowers its
 * clock under matrix work on non-trivial operands.
 *
 *   kind      TORQ_DIAG_FP4  the block-scaled e2m1 MFMA of mxfp4_gemm (unit scales), or
 *             TORQ_DIAG_BF16 the bf16 MFMA of the rotation
 *   operands  device, 4-byte aligned, n_bytes >= 128: every lane fills its operand
 *             registers from it (packed codes for FP4, bf16 values for BF16;
 *             wraps around)
 *   iters     rounds of 16 MFMAs per wave, > 0
 *   sink      device, TORQ_DIAG_SINK_FLOATS floats, overwritten
 *
 * Enqueues one kernel that executes TORQ_DIAG_FLOP_PER_ITER_FP4 (or _BF16) * iters
 * floating-point operations; the caller times it.  Errors: TORQ_EINVAL, TORQ_EALIGN,
 * TORQ_EHIP. */
#define TORQ_DIAG_FP4  0
#define TORQ_DIAG_BF16 1
#define TORQ_DIAG_SINK_FLOATS (1024 * 256)
#define TORQ_DIAG_FLOP_PER_ITER_FP4  (1024.0 * 4 * 16 * 2 * 32 * 32 * 64)
#define TORQ_DIAG_FLOP_PER_ITER_BF16 (1024.0 * 4 * 16 * 2 * 32 * 32 * 16)
int torq_diag_mfma_burn(int kind, const void *operands, size_t n_bytes, int iters, float *sink,
                        void *stream);
/* The two headline kernels with parts of their work left out, to measure on the machine at hand what
 * each part costs (the kernels run at the board's power limit, so a part's cost is the time by which
 * the launch shortens without it, not its instruction count).  Operands, shapes and launch shape are
 * those of mxfp4_gemm's 256 x 256-tile kernel (d a multiple of 512, all five pointers 16-byte aligned)
 * and of torq_rotate_quantize at G = 128 (dense R_inter).  skip = 0 is the product kernel (the GEMM's in
 * its plain form, one workgroup per tile, which mxfp4_gemm runs below four tiles per compute unit); with any
 * other value the OUTPUT IS MEANINGLESS (every access stays within the same buffers).
 *   torq_diag_gemm_ablation    skip: 1 no buffer loads in the k loop (it multiplies what the prologue
 *                              staged); 3 also no LDS stores; 7 also no fragment reads (MFMAs and the
 *                              barrier only); 15 also no barrier; 4 no fragment reads only
 *   torq_diag_rotate_ablation  skip bits: 1 no low-part pass over R_inter; 2 no hi/lo split of Y on the
 *                              vector ALU; 4 no amax / conversion in step 4; 8 one R_intra pass instead
 *                              of three; supported: 0, 1, 2, 4, 6, 8, 9, 15
 * Any other skip, shape or handle: TORQ_EINVAL. */
int torq_diag_gemm_ablation(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                            void *out_bf16, int64_t M, int64_t N, int d, int skip, void *stream);
int torq_diag_rotate_ablation(const torq_rotation_t *r, const void *x_bf16, int64_t M, uint8_t *codes,
                              uint8_t *scales, int skip, void *stream);
/* mxfp4_gemm's tiled kernel in its persistent form -- a workgroup takes several output tiles in turn and its
 * k loop runs through the tile boundaries (the last two iterations of a tile request the first two of the
 * workgroup's next one) -- on `workgroups` workgroups, whatever the shape.  mxfp4_gemm takes this form only
 * from a round and a half of tiles on; this entry point exists so that tests can walk it over several tiles per
 * workgroup on shapes small enough to check every output.  The result is mxfp4_gemm's, bit for bit.
 *   tile        0: 256 x 256 output tile, 1: 256 x 128
 *   d           a multiple of 1024; all five pointers 16-byte aligned; 1 <= workgroups <= 65536
 * Anything else: TORQ_EINVAL / TORQ_EALIGN. */
int torq_diag_gemm_persistent(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                              void *out_bf16, int64_t M, int64_t N, int d, int tile, int workgroups, void *stream);
/* mxfp4_gemm's tiled kernel on a plan of the caller's choice, whatever the planner would take for the
 * shape: for measuring the planner's alternatives against each other and for checking every form of the
 * kernel on shapes small enough to compare every output.  Never the weight-streaming kernel, the
 * persistent form or two launches.  The result is mxfp4_gemm's bit for bit when k_pieces = 1, and
 * mxfp4_gemm_ws's for the same tile and k_pieces otherwise.
 *   tile        0: 256 x 256 output tile, 1: 256 x 128, 2: 128 x 128, 3: 128 x 64
 *   k_pieces    1, or into how many pieces the k range is cut: d / 512 must be a multiple of it, N a multiple of
 *               8, and workspace (device, 16-byte aligned) hold k_pieces * M * N floats
 *   deep        != 0: the deeper load pipeline (tiles 2 and 3 only)
 *   tile 3, k_pieces > 1 and deep need d a multiple of 512 and 16-byte aligned scale arrays
 * Anything else: TORQ_EINVAL / TORQ_EALIGN. */
int torq_diag_gemm_plan(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                        void *out_bf16, int64_t M, int64_t N, int d, int tile, int k_pieces, int deep,
                        void *workspace, size_t workspace_bytes, void *stream);
/* A plain device-to-device copy of n_bytes (a multiple of 16; src and dst 16-byte aligned, not
 * overlapping) by a kernel of this library, `torq::diag_copy_kernel`: it reads n_bytes and writes
 * n_bytes, nothing else, which makes it the yardstick for memory-traffic counters (run it in the same
 * counter collection as the kernel under study and scale by what the counter reads for it).
 * Errors: TORQ_EINVAL, TORQ_EALIGN, TORQ_EHIP. */
int torq_diag_copy(const void *src, void *dst, size_t n_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TORQ_H */
