// mxfp4_gemm: the W4A4 linear layer that consumes the quantised, rotated
// activations (Section 5, weight fusion; Algorithm 3, "Return").
//
//   out[m][n] = sum_kb 2^(A_s[m][kb] + W_s[n][kb] - 254) * sum_{k<32} val(A[m][32kb+k]) val(W[n][32kb+k])
//
// on v_mfma_scale_f32_32x32x64_f8f6f4 with both operands in e2m1: one lane holds
// the 32 codes (16 bytes) of one microscaling block of one row, and one E8M0
// byte per lane scales exactly that block -- the MX format maps onto the
// instruction without any repacking of the row-major code arrays.
//
// The product is formed transposed (first operand = weight rows n, second =
// activation rows m), so that an accumulator lane holds runs of four
// consecutive n for one m and the bf16 epilogue stores 8 bytes per lane.
//
// Workgroup = 4 waves (2 x 2), one per SIMD; each wave owns a (32 WM) x (32 WN)
// piece of the (64 WM) x (64 WN) output tile and keeps it in accumulator
// registers (tiles: 256 x 256, 256 x 128, 128 x 128, chosen per problem size).  The k loop advances 256 elements per iteration (128 bytes of
// codes per row = one full cache line, 8 scale bytes per row):
//   * codes: buffer loads (tile-relative 32-bit offsets, hardware bounds check
//     returns zero for rows past M or N) -> registers -> LDS, double-buffered in
//     LDS; the loads of iteration kt+2 are issued right after the LDS stores of
//     iteration kt+1;
//   * scales: staged through LDS in pieces of 16 bytes per row (two iterations)
//     so that their global loads are not 8-byte gathers;
//   * operand fragments are read from LDS one k-step (64 elements) ahead of the
//     MFMAs that use them.
// LDS rows are 128 bytes; the 16-byte chunk index is XOR-swizzled with
// (row >> 1) & 7, which makes both the row-wise stores and the column-wise
// 16-byte fragment reads bank-conflict free.
#include "torq_device.h"
#include "torq_internal.h"

namespace torq {

constexpr int GEMM_GROUP_M = 8;       // tile rows per scheduling group

typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

// SPLIT: blockIdx.y = which of gridDim.y equal pieces of the k range this workgroup multiplies
// (each a whole, even number of iterations); the tile's fp32 sums go to partial[blockIdx.y][M][N]
// and mxfp4_gemm_splitk_reduce_kernel adds the pieces.  Needs FULLK.
// SKIP (diagnostic builds only, torq_diag_gemm_ablation): parts of the k loop left out to measure what
// each costs -- 1: the buffer loads, 2: the LDS stores (only with 1: their data would be dead), 4: the
// fragment and scale reads, 8: the barrier.
// What is left out is never replaced by anything else: the loop then multiplies the operands that the
// prologue staged, again and again, and the output is meaningless.  SKIP = 0 is the product.
// PERSIST (needs FULLK, no SPLIT, no DEEP, a k range of a multiple of four iterations): the workgroup takes
// the tiles blockIdx.x, blockIdx.x + gridDim.x, ... and the k loop runs THROUGH the tile boundary.  The loop
// requests operands two iterations ahead anyway (its last two iterations used to load data nobody reads);
// here those requests go to the first two iterations of the workgroup's NEXT tile, so that after the
// epilogue the next tile starts in the state the loop expects -- stage 0 and its scale bytes in LDS, the
// second iteration in the staging registers, the first fragments read -- with no prologue and no wait for
// memory.  The epilogue then may only use the LDS of stage 1 (a quarter of the tile at a time), and the
// accumulators are cleared where it has read them.
template <int WM, int WN, bool FULLK, bool SPLIT, bool DEEP = false, int SKIP = 0, bool PERSIST = false>
__global__ void __launch_bounds__(256)
mxfp4_gemm_kernel(const uint8_t *__restrict__ A_q, const uint8_t *__restrict__ A_s,
                  const uint8_t *__restrict__ W_q, const uint8_t *__restrict__ W_s,
                  uint16_t *__restrict__ out, float *__restrict__ partial, int64_t M, int64_t N, int d,
                  int tiles_m, int tiles_n, int64_t ldc) {
  static_assert(FULLK || !SPLIT, "split-k needs whole iterations");
  constexpr int BM = 64 * WM, BN = 64 * WN;
  constexpr int A_CH = BM / 32, W_CH = BN / 32;          // 16-byte code chunks per thread per iteration
  constexpr int ROWS = (BM + BN + 255) / 256 * 256;      // scale rows staged: padded so that every thread
  constexpr int S_CH = ROWS / 256;                       // stages S_CH 16-byte chunks per 2 iterations
  // LDS map: [A stage 0 | A stage 1 | W stage 0 | W stage 1 | scales buffer 0 | scales buffer 1]
  constexpr int A_STAGE = BM * 128, W_STAGE = BN * 128;
  constexpr int W_BASE = 2 * A_STAGE;
  constexpr int S_BASE = W_BASE + 2 * W_STAGE;
  constexpr int SSTAGE = ROWS * 16;
  extern __shared__ __attribute__((aligned(16))) char lds[];

  static_assert(!PERSIST || (FULLK && !SPLIT && !DEEP && SKIP == 0), "the persistent form is the plain full-k kernel");
  // ---- which output tile: contiguous runs of tiles per XCD, groups of GEMM_GROUP_M tile rows.  seq: the
  // position in launch order (the block index; PERSIST: + a multiple of the grid, itself a multiple of 8)
  const int total = tiles_m * tiles_n;
  int64_t m0, n0;
  int rows_a, rows_w;
  auto tile_at = [&](int seq, int64_t &tm0, int64_t &tn0, int &ra, int &rw) {
    int lid = seq;
    if (total % 8 == 0) lid = (seq % 8) * (total / 8) + seq / 8;
    const int width = GEMM_GROUP_M * tiles_n;
    const int group = lid / width;
    const int first_m = group * GEMM_GROUP_M;
    const int gsz = (tiles_m - first_m < GEMM_GROUP_M) ? tiles_m - first_m : GEMM_GROUP_M;
    const int tm = first_m + (lid % width) % gsz;
    const int tn = (lid % width) / gsz;
    tm0 = (int64_t)tm * BM;
    tn0 = (int64_t)tn * BN;
    ra = (M - tm0 < BM) ? (int)(M - tm0) : BM;
    rw = (N - tn0 < BN) ? (int)(N - tn0) : BN;
  };
  tile_at(blockIdx.x, m0, n0, rows_a, rows_w);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wy = wave >> 1, wx = wave & 1;
  const int lrow = lane & 31, g = lane >> 5;
  const int row_bytes = d / 2, srow_bytes = d / 32;
  const int KT = (d + 255) / 256;
  // Iterations past the end (the pipeline always loads two ahead) wrap around to a valid k.
  const int kt_count = SPLIT ? KT / (int)gridDim.y : ((KT + 1) & ~1);   // even; odd KT only without FULLK
  const int kt0 = SPLIT ? (int)blockIdx.y * kt_count : 0;
#define PHYS_KT(KT_) (PERSIST ? ((KT_) + l_kt_off) : FULLK ? (((KT_) + kt0) % KT) : (KT_))

  // ---- global side: buffer resources over the rows of the tile that is being LOADED (PERSIST: the next
  // tile's during the last two iterations of a tile); reads past them return 0
  __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(A_q + m0 * row_bytes, (uint32_t)rows_a * row_bytes);
  __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(W_q + n0 * row_bytes, (uint32_t)rows_w * row_bytes);
  __amdgpu_buffer_rsrc_t as_rsrc = make_rsrc(A_s + m0 * srow_bytes, (uint32_t)rows_a * srow_bytes);
  __amdgpu_buffer_rsrc_t ws_rsrc = make_rsrc(W_s + n0 * srow_bytes, (uint32_t)rows_w * srow_bytes);
  int l_kt_off = 0;                                // PERSIST: - kt_count while the next tile is loaded
  // code chunk id = tid + 256 i: row = tid/8 + 32 i, chunk = tid%8
  const int c_chunk = tid & 7, c_row = tid >> 3;
  const int c_voff = c_row * row_bytes + c_chunk * 16;   // + 32 i rows + 128 kt via the scalar offset
  const int c_lds = c_row * 128 + ((c_chunk ^ ((c_row >> 1) & 7)) * 16);   // + 32 i * 128 (same swizzle)

  // DEEP: two sets of staging registers, filled alternately, so that the codes of an iteration
  // are requested three iterations before they are multiplied instead of two (for the shapes
  // whose pace is set by the latency of the weight stream; costs A_CH + W_CH more registers)
  constexpr int NSET = DEEP ? 2 : 1;
  constexpr int AHEAD = DEEP ? 3 : 2;
  u32x4 a_regs[NSET][A_CH], w_regs[NSET][W_CH], s_regs[S_CH];

  // The codes of iteration k pass through register set k % NSET and LDS stage k % 2.
#define G_LOAD_Q(SET_, KT_, Q_)                 /* quarter Q_ (0..3) of an iteration's chunks */ \
  {                                                                                               \
    const int kt_ = PHYS_KT(KT_);                                                                 \
    constexpr int set_ = DEEP ? (SET_) : 0;                                                       \
    const bool ok_ = FULLK || (kt_ * 128 + c_chunk * 16 < row_bytes);                             \
    _Pragma("unroll") for (int i = (Q_) * A_CH / 4; i < ((Q_) + 1) * A_CH / 4; ++i) {             \
      a_regs[set_][i] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, c_voff, i * 32 * row_bytes + kt_ * 128, 0); \
      if (!FULLK && !ok_) a_regs[set_][i] = u32x4{0, 0, 0, 0};                                    \
    }                                                                                             \
    _Pragma("unroll") for (int i = (Q_) * W_CH / 4; i < ((Q_) + 1) * W_CH / 4; ++i) {             \
      w_regs[set_][i] = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, c_voff, i * 32 * row_bytes + kt_ * 128, 0); \
      if (!FULLK && !ok_) w_regs[set_][i] = u32x4{0, 0, 0, 0};                                    \
    }                                                                                             \
  }
#define G_LOAD(SET_, KT_) { G_LOAD_Q(SET_, KT_, 0) G_LOAD_Q(SET_, KT_, 1) G_LOAD_Q(SET_, KT_, 2) G_LOAD_Q(SET_, KT_, 3) }
#define L_STORE(P_, Q_)                         /* quarter Q_ (0..3) of stage P_'s chunks */     \
  {                                                                                               \
    constexpr int set_ = DEEP ? (P_) : 0;                                                         \
    _Pragma("unroll") for (int i = (Q_) * A_CH / 4; i < ((Q_) + 1) * A_CH / 4; ++i)               \
        *reinterpret_cast<u32x4 *>(lds + c_lds + (P_) * A_STAGE + i * 32 * 128) = a_regs[set_][i]; \
    _Pragma("unroll") for (int i = (Q_) * W_CH / 4; i < ((Q_) + 1) * W_CH / 4; ++i)               \
        *reinterpret_cast<u32x4 *>(lds + c_lds + W_BASE + (P_) * W_STAGE + i * 32 * 128) = w_regs[set_][i]; \
  }
  // scales of iterations 2 SC_ and 2 SC_ + 1: 16 bytes per row; staged row id = tid + 256 i
  // (A rows first, then W rows)
#define S_LOAD(SC_)                                                                               \
  {                                                                                               \
    const int sc_ = (SC_);                                                                        \
    _Pragma("unroll") for (int i = 0; i < S_CH; ++i) {                                            \
      const int r_ = tid + 256 * i;                                                               \
      /* 64 divides BM, so a wave stages either A rows or W rows: a scalar choice; padding rows  \
         are past the end of the W buffer and read zeros */                                        \
      const bool is_a_ = __builtin_amdgcn_readfirstlane(r_) < BM;                                 \
      const int vo_ = (is_a_ ? r_ : r_ - BM) * srow_bytes;                                        \
      const __amdgpu_buffer_rsrc_t rs_ = is_a_ ? as_rsrc : ws_rsrc;                               \
      if (FULLK) {                                                                                \
        s_regs[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_, vo_, sc_ * 16, 0);                 \
      } else {                                                                                    \
        _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                           \
          const uint32_t v_ = __builtin_amdgcn_raw_buffer_load_b32(rs_, vo_, sc_ * 16 + e * 4, 0); \
          s_regs[i][e] = (sc_ * 16 + e * 4 < srow_bytes) ? v_ : 0x7F7F7F7Fu;                      \
        }                                                                                         \
      }                                                                                           \
    }                                                                                             \
  }
#define S_STORE(B_)                                                                               \
  {                                                                                               \
    _Pragma("unroll") for (int i = 0; i < S_CH; ++i)                                              \
        *reinterpret_cast<u32x4 *>(lds + S_BASE + (B_) * SSTAGE + (tid + 256 * i) * 16) = s_regs[i]; \
  }

  f32x16 acc[WN][WM];
#pragma unroll
  for (int j = 0; j < WN; ++j)
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

  // ---- fragment addressing.  The 64 k of one MFMA are two microscaling blocks: lanes 0..31
  // (g = 0) supply one, lanes 32..63 (g = 1) the other.  Which two blocks of the iteration a
  // k-step multiplies is free as long as both operands agree; k-step ks takes blocks ks (g = 0)
  // and 4 + ks (g = 1), so that a lane's four scale bytes of the iteration are one aligned
  // dword (bytes 4 g .. 4 g + 3 of the row's 8) and the byte select of the MFMA is just ks.
  // Lane (lrow, g) reads chunk 4 g + ks of rows lrow + 32 i of its wave's strip; (row >> 1) & 7
  // is the same for all those rows, so one swizzled offset per ks serves every fragment and the
  // row strips become immediate offsets.
  const int f_sw = (lrow >> 1) & 7;
  int fa_off[4], fw_off[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int ch = ((4 * g + ks) ^ f_sw) * 16;
    fa_off[ks] = (wy * WM * 32 + lrow) * 128 + ch;
    fw_off[ks] = W_BASE + (wx * WN * 32 + lrow) * 128 + ch;
  }
  const int sa_off = S_BASE + (wy * WM * 32 + lrow) * 16 + 4 * g;
  const int sw_off = S_BASE + (BM + wx * WN * 32 + lrow) * 16 + 4 * g;

  i32x4 fa[2][WM], fw[2][WN];
  uint32_t sa[2][WM], sw[2][WN];                   // [iteration parity][frag]: the lane's 4 scale bytes

#define F_LOAD(SET_, P_, KS_)                                                                     \
  {                                                                                               \
    _Pragma("unroll") for (int i = 0; i < WM; ++i)                                                \
        fa[SET_][i] = *reinterpret_cast<const i32x4 *>(lds + fa_off[KS_] + (P_) * A_STAGE + i * 32 * 128); \
    _Pragma("unroll") for (int j = 0; j < WN; ++j)                                                \
        fw[SET_][j] = *reinterpret_cast<const i32x4 *>(lds + fw_off[KS_] + (P_) * W_STAGE + j * 32 * 128); \
  }
  // this lane's 4 scale bytes of each row for iteration KT_, into register set PAR_
#define SC_LOAD(PAR_, KT_)                                                                        \
  {                                                                                               \
    const int o_ = (((KT_) >> 1) & 1) * SSTAGE + ((KT_) & 1) * 8;                                 \
    _Pragma("unroll") for (int i = 0; i < WM; ++i)                                                \
        sa[PAR_][i] = *reinterpret_cast<const uint32_t *>(lds + sa_off + o_ + i * 32 * 16);       \
    _Pragma("unroll") for (int j = 0; j < WN; ++j)                                                \
        sw[PAR_][j] = *reinterpret_cast<const uint32_t *>(lds + sw_off + o_ + j * 32 * 16);       \
  }
#define MFMA_ONE(SET_, PAR_, KS_, J_, I_)                                                         \
  acc[J_][I_] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(                                  \
      i32x8{fw[SET_][J_][0], fw[SET_][J_][1], fw[SET_][J_][2], fw[SET_][J_][3], 0, 0, 0, 0},      \
      i32x8{fa[SET_][I_][0], fa[SET_][I_][1], fa[SET_][I_][2], fa[SET_][I_][3], 0, 0, 0, 0},      \
      acc[J_][I_], 4, 4, KS_, sw[PAR_][J_], KS_, sa[PAR_][I_]);
#define MFMA_HALF(SET_, PAR_, KS_, J0_, J1_)                                                      \
  _Pragma("unroll") for (int j = (J0_); j < (J1_); ++j)                                           \
      _Pragma("unroll") for (int i = 0; i < WM; ++i) { MFMA_ONE(SET_, PAR_, KS_, j, i) }

  // ---- prologue
  G_LOAD(0, 0);
  S_LOAD(PHYS_KT(0) >> 1);
  L_STORE(0, 0);
  L_STORE(0, 1);
  L_STORE(0, 2);
  L_STORE(0, 3);
  S_STORE(0);
  G_LOAD(1, 1);
  if (DEEP) G_LOAD(0, 2);
  __syncthreads();
  SC_LOAD(0, 0);
  F_LOAD(0, 0, 0);
  if constexpr ((SKIP & 4) != 0) { F_LOAD(1, 0, 1); SC_LOAD(1, 0); }   // every register set holds staged operands

  // One k iteration is two scheduling regions, split by the workgroup barrier.  Each region ends
  // with a sched_group_barrier pipeline that tells the machine scheduler how to interleave MFMAs
  // with LDS and buffer traffic (left alone it hoists every load of the iteration to the top and
  // runs out of registers).  P = kt & 1 is a literal so that the LDS stage and the scale staging
  // phase are compile-time.  Every iteration runs the same code: the last two also load and stage
  // data that nobody will read (wrapped around to a valid k), which is cheaper than separate tail
  // code.  The LDS stores of the next stage are spread over k-steps 1, 2 and 3 so that they do
  // not arrive at the LDS in one burst in front of the barrier.
#define SGB(MASK_, N_) __builtin_amdgcn_sched_group_barrier(MASK_, N_, 0);
#define SG_MFMA 0x008
#define SG_VMEM_RD 0x020
#define SG_DS_RD 0x100
#define SG_DS_WR 0x200
#define ITER(P, KT_)                                                                              \
  {                                                                                               \
    const int kt_i = (KT_);                                                                       \
    if constexpr (!(SKIP & 4)) F_LOAD(1, P, 1);                                                                              \
    MFMA_HALF(0, P, 0, 0, WN);                                                                    \
    if constexpr (!(SKIP & 4)) F_LOAD(0, P, 2);                                                                              \
    if constexpr (!(SKIP & 2)) L_STORE((P) ^ 1, 0);                                                                          \
    if constexpr (!(SKIP & 1)) G_LOAD_Q((P) ^ 1, kt_i + AHEAD, 0);                                                           \
    MFMA_HALF(1, P, 1, 0, WN);                                                                    \
    if constexpr (!(SKIP & 4)) F_LOAD(1, P, 3);                                                                              \
    if constexpr (!(SKIP & 2)) L_STORE((P) ^ 1, 1);                                                                          \
    if constexpr (!(SKIP & 1)) G_LOAD_Q((P) ^ 1, kt_i + AHEAD, 1);                                                           \
    MFMA_HALF(0, P, 2, 0, WN);                                                                    \
    if constexpr (!(SKIP & 2)) L_STORE((P) ^ 1, 2);                                                                          \
    if constexpr (!(SKIP & 2)) L_STORE((P) ^ 1, 3);                                                                          \
    if constexpr (!(SKIP & 2)) if ((P) == 1) S_STORE(((kt_i + 1) >> 1) & 1);                                                 \
    MFMA_HALF(1, P, 3, 0, WN / 2);                                                                \
    /* k-step 0: its MFMAs hide the fragment reads of k-step 1 */                                 \
    _Pragma("unroll") for (int n_ = 0; n_ < WM + WN; ++n_) { SGB(SG_MFMA, 1) SGB(SG_DS_RD, 1) }   \
    SGB(SG_MFMA, WM * WN - (WM + WN) > 0 ? WM * WN - (WM + WN) : 0)                               \
    /* k-steps 1 and 2: per two MFMAs one fragment read of the next k-step; a quarter of the     \
       next stage's LDS stores along the way, each followed by the buffer loads that refill the  \
       staging registers it freed (for the iteration after next) */                               \
    _Pragma("unroll") for (int n_ = 0; n_ < 2; ++n_) {                                            \
      _Pragma("unroll") for (int q_ = 0; q_ < WM + WN; ++q_) {                                    \
        SGB(SG_MFMA, WM * WN / (WM + WN)) SGB(SG_DS_RD, 1)                                        \
        if (q_ % 2 == 1) { SGB(SG_DS_WR, 1) SGB(SG_VMEM_RD, 1) }                                  \
      }                                                                                           \
    }                                                                                             \
    /* first half of k-step 3: the rest of the LDS stores */                                      \
    _Pragma("unroll") for (int n_ = 0; n_ < WM * WN / 2; ++n_) { SGB(SG_MFMA, 1) SGB(SG_DS_WR, 2) } \
    if constexpr (!(SKIP & 8)) __syncthreads();                                                                              \
    if constexpr (!(SKIP & 4)) SC_LOAD((P) ^ 1, kt_i + 1);                                                                   \
    if constexpr (!(SKIP & 4)) F_LOAD(0, (P) ^ 1, 0);                                                                        \
    if constexpr (!(SKIP & 1)) G_LOAD_Q((P) ^ 1, kt_i + AHEAD, 2);                                                           \
    if constexpr (!(SKIP & 1)) G_LOAD_Q((P) ^ 1, kt_i + AHEAD, 3);                                                           \
    if constexpr (!(SKIP & 1)) if ((P) == 0) S_LOAD(PHYS_KT(kt_i + 2) >> 1);                                                 \
    MFMA_HALF(1, P, 3, WN / 2, WN);                                                               \
    /* second half of k-step 3: fragment and scale reads of the next iteration first, then      \
       the remaining buffer loads */                                                              \
    _Pragma("unroll") for (int n_ = 0; n_ < WM * WN / 2; ++n_) { SGB(SG_MFMA, 1) SGB(SG_DS_RD, 2) SGB(SG_VMEM_RD, 2) } \
    __builtin_amdgcn_sched_barrier(0);                                                            \
  }
  if constexpr (!PERSIST) {
    // an odd KT (only without FULLK) gets one all-zero iteration
    for (int kt = 0; kt < kt_count; kt += 2) {
      ITER(0, kt);
      ITER(1, kt + 1);
    }
  }
  if constexpr (PERSIST) {
    // ---- the workgroup's tiles, one after the other, the k loop running through the boundaries
    constexpr int ROW_E = 64 * WN;               // bytes of one output row of a wave's piece
    constexpr int PITCH_E = ROW_E + 16;
    constexpr int CH_ROW = ROW_E / 16;           // 16-byte chunks per row
    static_assert(2 * 32 * PITCH_E <= A_STAGE && 2 * 32 * PITCH_E <= W_STAGE, "two waves' quarter pieces per stage-1 buffer");
    // stage 1 of the codes is dead once the last barrier of a tile's k loop has been passed (the loop's
    // tail reads stage 0, which already holds the next tile): waves 0, 1 transpose through A's, 2, 3 through W's
    const bool vec_ok = (N & 7) == 0;
    for (int seq = blockIdx.x; seq < total; seq += gridDim.x) {
      // the tile whose first two iterations this tile's last two request: the next one, or this one
      // again (requests nobody reads, as in the plain kernel)
      int64_t nm0 = m0, nn0 = n0;
      int nra = rows_a, nrw = rows_w;
      if (seq + (int)gridDim.x < total) tile_at(seq + gridDim.x, nm0, nn0, nra, nrw);
      for (int kt = 0; kt < kt_count; kt += 2) {
        if (kt == kt_count - 2) {                  // from here on the requests are the next tile's
          a_rsrc = make_rsrc(A_q + nm0 * row_bytes, (uint32_t)nra * row_bytes);
          w_rsrc = make_rsrc(W_q + nn0 * row_bytes, (uint32_t)nrw * row_bytes);
          as_rsrc = make_rsrc(A_s + nm0 * srow_bytes, (uint32_t)nra * srow_bytes);
          ws_rsrc = make_rsrc(W_s + nn0 * srow_bytes, (uint32_t)nrw * srow_bytes);
          l_kt_off = -kt_count;
        }
        ITER(0, kt);
        ITER(1, kt + 1);
      }
      l_kt_off = 0;

      // ---- epilogue of the tile at (m0, n0), a quarter (32 rows per wave) at a time; see the plain
      // kernel's for the layout.  The accumulators are cleared as they are read.
      // (Its addresses are derived here from copies of the lane's coordinates that the compiler cannot see
      // through: computed ahead of the tile loop they would stay live through the k loop, which has no
      // register to spare.)
      int lrow_e = lrow, g_e = g, lane_e = lane, wave_e = __builtin_amdgcn_readfirstlane(wave);
      asm volatile("" : "+v"(lrow_e), "+v"(g_e), "+v"(lane_e), "+s"(wave_e));
      const int wy_e = wave_e >> 1, wx_e = wave_e & 1;
      char *const ep = lds + (wave_e < 2 ? A_STAGE : W_BASE + W_STAGE) + (wave_e & 1) * 32 * PITCH_E;
#pragma unroll
      for (int i = 0; i < WM; ++i) {
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
          for (int rr = 0; rr < 4; ++rr) {
            bf16x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              v[e] = (__bf16)acc[j][i][4 * rr + e];
              acc[j][i][4 * rr + e] = 0.f;
            }
            *reinterpret_cast<bf16x4 *>(ep + lrow_e * PITCH_E + (32 * j + 8 * rr + 4 * g_e) * 2) = v;
          }
#pragma unroll
        for (int t = 0; t < 32 * CH_ROW / 64; ++t) {
          const int idx = t * 64 + lane_e;
          const int row = idx / CH_ROW, ch = idx % CH_ROW;
          const u32x4 v = *reinterpret_cast<const u32x4 *>(ep + row * PITCH_E + ch * 16);
          const int64_t m = m0 + (wy_e * WM + i) * 32 + row;
          const int64_t n = n0 + wx_e * WN * 32 + ch * 8;
          if (m < M) {
            uint16_t *dst = out + m * N + n;
            if (vec_ok && n + 8 <= N) {
              *reinterpret_cast<u32x4 *>(dst) = v;
            } else {
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (n + e < N) dst[e] = (uint16_t)(v[e >> 1] >> (16 * (e & 1)));
            }
          }
        }
      }
      // every wave is done with stage 1 before the next tile's first iteration stores into it
      __syncthreads();
      m0 = nm0;
      n0 = nn0;
      rows_a = nra;
      rows_w = nrw;
    }
  }
#undef ITER
#undef SGB

  // ---- epilogue.  acc[j][i][r] = out[m = .. + lane%32][n = .. + 8*(r/4) + 4*(lane/32) + r%4]:
  // a lane holds 8-byte pieces of one output row.  Storing those directly makes every 128-byte
  // line of the output arrive in 16 separate partial writes, so the wave first transposes its
  // piece through LDS (free after the last barrier of the k loop; each wave uses a private
  // region) and then stores 16 bytes per lane with 8 adjacent lanes covering one full line.
  if constexpr (PERSIST) {
    // (stored tile by tile above)
  } else if (SPLIT) {
    // fp32 sums of this k piece: 16 bytes per lane and register quad, straight from the accumulators
    float *const dstp = partial + (size_t)blockIdx.y * (size_t)M * (size_t)N;
#pragma unroll
    for (int i = 0; i < WM; ++i) {
      const int64_t m = m0 + (wy * WM + i) * 32 + lrow;
#pragma unroll
      for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const int64_t n = n0 + (wx * WN + j) * 32 + 8 * rr + 4 * g;
          if (m < M && n + 4 <= N)
            *reinterpret_cast<f32x4 *>(dstp + m * N + n) =
                f32x4{acc[j][i][4 * rr], acc[j][i][4 * rr + 1], acc[j][i][4 * rr + 2], acc[j][i][4 * rr + 3]};
        }
    }
  } else {
    constexpr int ROW_E = 64 * WN;               // bytes of one output row of this wave's piece
    constexpr int PITCH_E = ROW_E + 16;
    constexpr int CH_ROW = ROW_E / 16;           // 16-byte chunks per row
    char *const ep = lds + wave * (32 * WM) * PITCH_E;
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (__bf16)acc[j][i][4 * rr + e];
          *reinterpret_cast<bf16x4 *>(ep + (i * 32 + lrow) * PITCH_E + (32 * j + 8 * rr + 4 * g) * 2) = v;
        }
    const bool vec_ok = (ldc & 7) == 0;           // (out itself is 16-byte aligned: checked by the host)
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int t = 0; t < 32 * CH_ROW / 64; ++t) {
        const int idx = t * 64 + lane;
        const int row = idx / CH_ROW, ch = idx % CH_ROW;
        const u32x4 v = *reinterpret_cast<const u32x4 *>(ep + (i * 32 + row) * PITCH_E + ch * 16);
        const int64_t m = m0 + (wy * WM + i) * 32 + row;
        const int64_t n = n0 + wx * WN * 32 + ch * 8;
        if (m < M) {
          uint16_t *dst = out + m * ldc + n;
          if (vec_ok && n + 8 <= N) {
            *reinterpret_cast<u32x4 *>(dst) = v;
          } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
              if (n + e < N) dst[e] = (uint16_t)(v[e >> 1] >> (16 * (e & 1)));
          }
        }
      }
  }
#undef G_LOAD
#undef G_LOAD_Q
#undef PHYS_KT
#undef L_STORE
#undef S_LOAD
#undef S_STORE
#undef F_LOAD
#undef SC_LOAD
#undef MFMA_ONE
#undef MFMA_HALF
}

// out[m][n] = bf16(sum over the k pieces, in order, of partial[s][m][n]); 8 outputs per thread; the rows
// of out are ldc elements apart (N and ldc multiples of 8)
__global__ void __launch_bounds__(256)
mxfp4_gemm_splitk_reduce_kernel(const float *__restrict__ partial, int splits, int64_t MN, int64_t N, int64_t ldc,
                                uint16_t *__restrict__ out) {
  const int64_t e0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (e0 >= MN) return;                          // MN is a multiple of 8
  f32x4 lo = *reinterpret_cast<const f32x4 *>(partial + e0), hi = *reinterpret_cast<const f32x4 *>(partial + e0 + 4);
  // four pieces requested at a time, added in order (the sums are those of one piece after the other)
  int s = 1;
  for (; s + 4 <= splits; s += 4) {
    f32x4 l[4], h[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      l[u] = *reinterpret_cast<const f32x4 *>(partial + (size_t)(s + u) * MN + e0);
      h[u] = *reinterpret_cast<const f32x4 *>(partial + (size_t)(s + u) * MN + e0 + 4);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      lo += l[u];
      hi += h[u];
    }
  }
  if (s + 2 <= splits) {
    const f32x4 l0 = *reinterpret_cast<const f32x4 *>(partial + (size_t)s * MN + e0);
    const f32x4 h0 = *reinterpret_cast<const f32x4 *>(partial + (size_t)s * MN + e0 + 4);
    const f32x4 l1 = *reinterpret_cast<const f32x4 *>(partial + (size_t)(s + 1) * MN + e0);
    const f32x4 h1 = *reinterpret_cast<const f32x4 *>(partial + (size_t)(s + 1) * MN + e0 + 4);
    lo += l0;
    hi += h0;
    lo += l1;
    hi += h1;
    s += 2;
  }
  if (s < splits) {
    lo += *reinterpret_cast<const f32x4 *>(partial + (size_t)s * MN + e0);
    hi += *reinterpret_cast<const f32x4 *>(partial + (size_t)s * MN + e0 + 4);
  }
  bf16x4 a, b;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    a[e] = (__bf16)lo[e];
    b[e] = (__bf16)hi[e];
  }
  typedef __attribute__((__vector_size__(2 * sizeof(uint64_t)))) uint64_t u64x2;
  const int64_t o0 = ldc == N ? e0 : (e0 / N) * ldc + e0 % N;
  *reinterpret_cast<u64x2 *>(out + o0) = u64x2{__builtin_bit_cast(uint64_t, a), __builtin_bit_cast(uint64_t, b)};
}

// compute units of the current device (256 on this part), asked once
static int compute_units() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cus = n;
    else
      cus = 256;
  }
  return cus;
}

// Whether the persistent form (PERSIST above) takes the launch: more than a round and a half of tiles, so
// that most workgroups have a second tile to run into, and a k range of a multiple of four iterations.
// Measured on the same machine against the plain form: [8192, 28672, 8192] (14 tiles per CU) 925 -> 909 us,
// [4096, 25600, 5120] (6 per CU) 288.4 -> 283.5, [8192, 8192, 28672] (4 per CU) 868 -> 865; and with the
// weights from HBM (launches cycling over weight copies of 600 MB): [4096, 14336, 4096] (3.5 per CU)
// 154.9 -> 148.7, [8192, 5120, 4096] (2.5) 114.7 -> 110.7, [4096, 8192, 4096] (2) 82.5 -> 81.0,
// [2048, 14336, 4096] (1.75) 78.9 -> 77.1; equal within 1 % at d = 8192 from 1.75 to 2.7 per CU.
static bool persistent_pays(int64_t tiles, int d) { return 2 * tiles > 3 * (int64_t)compute_units() && d % 1024 == 0; }

template <int WM, int WN, bool FULLK, bool SPLIT, bool DEEP = false, int SKIP = 0, bool PERSIST = false>
static hipError_t launch_tile(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q,
                              const uint8_t *W_s, void *out, float *partial, int splits, int64_t M, int64_t N,
                              int d, hipStream_t stream, int persist_grid = 0, int64_t ldc = 0, int64_t walk_n = 0) {
  // ldc: elements between the rows of out (0: N; the persistent form only knows N);
  // walk_n: only the tiles of the first walk_n tile columns are computed (0: all)
  constexpr int BM = 64 * WM, BN = 64 * WN;
  if (ldc == 0) ldc = N;
  if (PERSIST && ldc != N) return hipErrorInvalidValue;
  const int64_t tiles_m = (M + BM - 1) / BM, tiles_n = walk_n > 0 ? walk_n : (N + BN - 1) / BN;
  if (tiles_n > (N + BN - 1) / BN) return hipErrorInvalidValue;
  if (tiles_m * tiles_n > 0x7FFFFFFF) return hipErrorInvalidValue;
  const size_t lds_bytes = 2 * (size_t)(BM + BN) * 128 + 2 * (size_t)((BM + BN + 255) / 256 * 256) * 16;
  auto kern = mxfp4_gemm_kernel<WM, WN, FULLK, SPLIT, DEEP, SKIP, PERSIST>;
  // PERSIST: one workgroup per CU, or persist_grid of them (a multiple of 8 where the tile count is one,
  // so that a workgroup's tiles stay on its XCD's run)
  int64_t grid = tiles_m * tiles_n;
  if (PERSIST) {
    const int64_t want = persist_grid > 0 ? persist_grid : compute_units();
    grid = grid < want ? grid : want;
    if ((tiles_m * tiles_n) % 8 == 0 && grid >= 8) grid -= grid % 8;
  }
  if (lds_bytes > 64 * 1024) {
    // raise the dynamic LDS limit once per process and kernel variant (the call is slow)
    static bool raised = false;
    if (!raised) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
      if (e != hipSuccess) return e;
      raised = true;
    }
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)grid, SPLIT ? splits : 1), dim3(256), lds_bytes, stream, A_q,
                     A_s, W_q, W_s, reinterpret_cast<uint16_t *>(out), partial, M, N, d, (int)tiles_m, (int)tiles_n, ldc);
  hipError_t e = hipGetLastError();
  if (!SPLIT || e != hipSuccess) return e;
  const int64_t MN = M * N;
  hipLaunchKernelGGL(mxfp4_gemm_splitk_reduce_kernel, dim3((unsigned)((MN / 8 + 255) / 256)), dim3(256), 0, stream,
                     partial, splits, MN, N, ldc, reinterpret_cast<uint16_t *>(out));
  return hipGetLastError();
}

// Which output tile: 0 = 256 x 256, 1 = 256 x 128, 2 = 128 x 128.  Every CU holds one workgroup
// of the two larger tiles (or two of the smallest), so a launch takes ceil(tiles / 256) rounds;
// a round of the three tile shapes costs 1 : 0.60 : 0.33 (measured at full rounds; the larger the
// tile, the fewer operand bytes per flop).  Take the cheapest, the larger tile on a tie.
static int choose_tile(int64_t M, int64_t N) {
  auto rounds = [&](int bm, int bn) { return (double)((((M + bm - 1) / bm) * ((N + bn - 1) / bn) + 255) / 256); };
  const double c0 = rounds(256, 256), c1 = 0.60 * rounds(256, 128), c2 = 0.33 * rounds(128, 128);
  if (c0 <= c1 && c0 <= c2) return 0;
  return c1 <= c2 ? 1 : 2;
}

// the tile shapes: 0 = 256 x 256, 1 = 256 x 128, 2 = 128 x 128, 3 = 128 x 64
static const int TILE_M[4] = {256, 256, 128, 128}, TILE_N[4] = {256, 128, 128, 64};

// How a product is run: the weight-streaming kernel (mxfp4_gemm_skinny.hip), or the tiled kernel
// with tile shape `cfg` and its k range cut into `splits` pieces (1 = not cut).
struct GemmPlan {
  bool skinny;
  int cfg;
  int splits;
  bool deep;      // the tiled kernel's deeper load pipeline (128-row-wide tiles, weight-bound shapes)
  double us;      // the model's estimate of the launch time
};

// Several rounds of tiles: microseconds of a launch of `tiles` tiles of shape cfg over KT iterations.
// A launch costs 6 us; a round (256 tiles, 512 of the smallest shape) a + b KT with (a, b) fitted to
// [4096, 4096 / 24576, 5120] and [4096, 4096, 25600] (256 x 256: 49, 262, 203 us), [2048, 4096, 4096 / 14336]
// (256 x 128: 25.5, 68.5) and [4096, 5120, 5120 / 25600] (128 x 128: 71.5, 322).
static double rounds_us(int cfg, double tiles, double KT) {
  static const double A[3] = {4.8, 2.3, 0.9}, B[3] = {1.9, 1.075, 1.044};
  const double slots = cfg == 2 ? 512.0 : 256.0;
  const double rounds = (double)(int64_t)((tiles + slots - 1) / slots);
  return 6.0 + rounds * (A[cfg] + B[cfg] * KT);
}
// ... and never less than the weights' stream from HBM at 4.7 TB/s (few activation rows against many weight rows)
static double rounds_us(int cfg, double tiles, double KT, int64_t N, int d) {
  const double t = rounds_us(cfg, tiles, KT), stream = 6.0 + (double)N * (double)d * 0.53125 / 1e6 * 0.214;
  return t > stream ? t : stream;
}

// Up to one round of 256 x 256 tiles the choice is wide: four tile shapes, the k range whole or cut into
// pieces that run side by side (a piece is a whole even number of iterations; the pieces' fp32 tiles go
// through the caller's workspace and a second kernel adds them), the deeper load pipeline for the two small
// tiles, and with at most 64 activation rows the weight-streaming kernel.  The planner prices every
// candidate with a model fitted to measurements and takes the cheapest.  The measurements: 238 shapes
// (M = 1 ... 2048, N = 1024 ... 28672, d = 4096 ... 28672, powers of two and not), every candidate of each
// forced through torq_diag_gemm_plan, HIP-graph replays over weight copies of 600 MB in all (weights come
// from HBM, as they do in a model; activations from the caches).  Microseconds:
//   tiled:  a + b * iterations of one workgroup,  b = (b_lo + (b_hi - b_lo) * clamp((w - 128) / 128, 0, 1)) *
//           (1 + (rounds - 1) * m)  with rounds = ceil(workgroups / 256) and w = workgroups / rounds: up to
//           half the CUs busy an iteration costs b_lo (latency), a full round b_hi (the power limit), a CU
//           that holds several workgroups m times more for each further one; never less than the weights'
//           stream from HBM; a cut adds the second launch, the pieces' traffic and 0.25 us per piece.
//   weight-streaming:  the larger of a latency term (iterations x 16-row activation tiles) and the stream.
// Over the measured shapes the choice is within 0.5 % of the best candidate on average (5 - 13 % before, when
// the 128 x 64 tile did not exist and cuts were priced by rule of thumb); the worst case is 7 %.
struct TileCost { double a, b_lo, b_hi; };
static const TileCost TILE_COST[4][2] = {      // [tile][deep]
    {{7.47, 1.40, 2.11}, {7.47, 1.40, 2.11}}, {{5.24, 0.96, 1.10}, {5.24, 0.96, 1.10}},
    {{4.65, 0.84, 0.76}, {3.75, 0.68, 0.83}}, {{4.36, 0.67, 0.65}, {3.12, 0.59, 0.63}}};
static const double TILE_SHARE[4] = {1.0, 1.11, 0.82, 0.70};

static double tiled_us(int tile, int s, bool deep, int64_t M, int64_t N, int d) {
  const double tiles = (double)(((M + TILE_M[tile] - 1) / TILE_M[tile]) * ((N + TILE_N[tile] - 1) / TILE_N[tile]));
  const double wgs = tiles * s, iters = (double)((d + 255) / 256) / s;
  const TileCost &c = TILE_COST[tile][deep ? 1 : 0];
  const double rounds = (double)(int64_t)((wgs + 255.0) / 256.0), w = wgs / rounds;
  double ramp = (w - 128.0) / 128.0;
  ramp = ramp < 0.0 ? 0.0 : ramp > 1.0 ? 1.0 : ramp;
  const double b = (c.b_lo + (c.b_hi - c.b_lo) * ramp) * (1.0 + (rounds - 1.0) * TILE_SHARE[tile]);
  double t = c.a + b * iters;
  const double stream = c.a + (double)N * (double)d * 0.53125 / 1e6 * 0.211;     // 4.7 TB/s
  if (t < stream) t = stream;
  if (s > 1) t += 0.72 + 1.75 * (double)s * (double)M * (double)N / 1e6 + 0.25 * s;
  return t;
}

static double skinny_us(int64_t M, int64_t N, int d) {
  const double mt = (double)((M + 15) / 16), iters = (double)((d + 255) / 256);
  const double w_mb = (double)N * (double)d * 0.53125 / 1e6;
  // beyond d = 16384 a workgroup no longer keeps its activation rows across strips: every further 16-row
  // activation tile costs up to 2.3 times more (d = 28672)
  const double f = d > 16384 ? 1.0 + 1.74 * (double)(d - 16384) / 16384.0 : 1.0;
  const double latency = 2.66 + iters * (0.0565 + 0.0801 * mt * f);
  const double stream = 2.75 + w_mb * (0.2104 + 0.0726 * (mt - 1.0) * f);
  return latency > stream ? latency : stream;
}

static GemmPlan choose_plan(int64_t M, int64_t N, int d, bool allow_split) {
  const bool can_skinny = mxfp4_gemm_skinny_fits(M, d);
  const double KT = (d + 255) / 256;
  auto tiles_of = [&](int tile) { return ((M + TILE_M[tile] - 1) / TILE_M[tile]) * ((N + TILE_N[tile] - 1) / TILE_N[tile]); };
  GemmPlan plan{false, 0, 1, false, 0.0};
  if (tiles_of(0) > 256) {
    // more than a round of the largest tile: by rounds (choose_tile), never cut
    plan.cfg = choose_tile(M, N);
    plan.us = rounds_us(plan.cfg, (double)tiles_of(plan.cfg), KT, N, d);
  } else {
    const bool may_split = allow_split && d % 512 == 0 && N % 8 == 0;
    const int pairs = d / 512;
    double best = -1.0;
    for (int tile = 0; tile < 4; ++tile) {
      if (tile == 3 && d % 512 != 0) continue;                       // (the 128 x 64 tile only has the whole-pieces form)
      for (int s = 1; s <= 16 && s <= (may_split && tile != 0 ? pairs : 1); ++s) {   // the largest tile is never cut
        if (s > 1 && (pairs % s != 0 || tiles_of(tile) * s > 1024)) continue;
        if (s == 1 && tile != 0 && tiles_of(tile) > 1024) continue;
        // the two small tiles, not cut, always on the deeper load pipeline: 10 - 19 % faster up to 256 tiles
        // with weights from HBM, within 3 % beyond; cut, up to 256 workgroups (2 - 7 % faster there, 1 - 2 %
        // slower beyond; priced like the plain pipeline)
        const bool deep = tile >= 2 && d % 512 == 0 && (s == 1 || tiles_of(tile) * s <= 256);
        const double t = tiled_us(tile, s, deep && s == 1, M, N, d);
        if (best < 0.0 || t < best) {
          best = t;
          plan = GemmPlan{false, tile, s, deep, t};
        }
      }
    }
  }
  if (can_skinny) {
    // near a tie the streaming kernel wins: one launch, no tile padding
    const double t = skinny_us(M, N, d);
    if (0.95 * t <= plan.us) plan = GemmPlan{true, 0, 1, false, t};
  }
  return plan;
}

// Whole rounds first.  A tile count just above a whole number of rounds leaves the last round mostly empty
// (Qwen3-32B's [4096, 5120, d]: 320 tiles of 256 x 256 are a round and a quarter; smaller tiles fill the
// rounds better and use the operands worse).  Then the leading columns that make up whole rounds of
// 256 x 256 tiles go first, as one launch that walks only those tile columns, and the remaining columns
// are a product of their own (any plan, its k range cut where that pays) on the same output rows, which
// are N elements apart.  Returns those leading columns, or N: one launch.  Taken when the last round would
// be at most half full and the model promises a gain: measured [4096, 5120, 25600] 322 -> 279 us,
// [4096, 5120, 5120] 71.5 -> 66.3, [4096, 25600, 5120] 291 -> 279; every output is the sum it was before
// (same k order in every tile shape; where the remainder's k range is cut, up to the order of its fp32 sums,
// as for any product that mxfp4_gemm_ws cuts).
static GemmPlan plan_with(int64_t M, int64_t N, int d, bool allow_split, size_t workspace_bytes);
static int64_t choose_main_columns(int64_t M, int64_t N, int d, bool allow_split, size_t workspace_bytes, const GemmPlan &whole) {
  if (whole.skinny || whole.splits > 1 || whole.cfg > 2 || d % 512 != 0 || N % 8 != 0 || M <= 64) return N;
  const int64_t tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256, tiles = tiles_m * tiles_n;
  const int64_t full = tiles / 256;
  if (full < 1 || tiles % 256 == 0 || tiles % 256 > 128 || tiles_m > 256) return N;
  const int64_t cols = full * 256 / tiles_m;                        // whole tile columns of the first launch
  if (cols < 1 || cols >= tiles_n) return N;
  const double KT = (d + 255) / 256;
  // the one launch: by rounds where it takes more than one (choose_plan's own figure is for less)
  const int tm = TILE_M[whole.cfg], tn = TILE_N[whole.cfg];
  const double tiles_whole = (double)(((M + tm - 1) / tm) * ((N + tn - 1) / tn));
  const double one = tiles_whole > (whole.cfg == 2 ? 512.0 : 256.0) ? rounds_us(whole.cfg, tiles_whole, KT) : whole.us;
  const GemmPlan tail = plan_with(M, N - 256 * cols, d, allow_split, workspace_bytes);
  const double two = rounds_us(0, (double)(tiles_m * cols), KT) + tail.us;
  return two < 0.985 * one ? 256 * cols : N;
}
#ifndef GEMM_PLAN
#define GEMM_PLAN(M_, N_, d_, allow_) choose_plan(M_, N_, d_, allow_)
#endif

// the plan of a product given the workspace it may use (a cut k range needs its pieces' fp32 tiles there)
static GemmPlan plan_with(int64_t M, int64_t N, int d, bool allow_split, size_t workspace_bytes) {
  GemmPlan plan = GEMM_PLAN(M, N, d, allow_split);
  if (plan.splits > 1 && workspace_bytes < (size_t)plan.splits * (size_t)M * (size_t)N * sizeof(float))
    plan = GEMM_PLAN(M, N, d, false);
  return plan;
}

int64_t mxfp4_gemm_main_columns(int64_t M, int64_t N, int d, size_t workspace_bytes) {
  const bool allow = d % 512 == 0;
  return choose_main_columns(M, N, d, allow, workspace_bytes, plan_with(M, N, d, allow, workspace_bytes));
}

void mxfp4_gemm_plan(int64_t M, int64_t N, int d, size_t workspace_bytes, int *skinny, int *tile_m, int *tile_n,
                     int *splits) {
  GemmPlan plan = plan_with(M, N, d, d % 512 == 0, workspace_bytes);
  if (mxfp4_gemm_main_columns(M, N, d, workspace_bytes) < N) plan = GemmPlan{false, 0, 1, false, 0.0};   // the first launch
  *skinny = plan.skinny;
  *tile_m = plan.skinny ? 0 : TILE_M[plan.cfg];
  *tile_n = plan.skinny ? 16 : TILE_N[plan.cfg];
  *splits = plan.splits;
}

size_t mxfp4_gemm_workspace_bytes(int64_t M, int64_t N, int d) {
  const GemmPlan plan = GEMM_PLAN(M, N, d, true);
  const int64_t main_n = choose_main_columns(M, N, d, true, ~(size_t)0, plan);
  if (main_n < N) {
    const GemmPlan tail = GEMM_PLAN(M, N - main_n, d, true);
    return tail.splits > 1 ? (size_t)tail.splits * (size_t)M * (size_t)(N - main_n) * sizeof(float) : 0;
  }
  return plan.splits > 1 ? (size_t)plan.splits * (size_t)M * (size_t)N * sizeof(float) : 0;
}

// one product by a given plan of the tiled kernel: out's rows are ldc elements apart.  fullk: d is a whole
// number of 512-element pieces and the scale arrays are 16-byte aligned (needed by every form but the plain
// one of the three larger tiles); persist: the persistent form where it pays (the two larger tiles, ldc = N)
static hipError_t launch_by_plan(const GemmPlan &plan, const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q,
                                 const uint8_t *W_s, void *out_bf16, int64_t M, int64_t N, int d, int64_t ldc,
                                 bool fullk, bool persist, float *partial, hipStream_t stream) {
  const int splits = plan.splits;
  if ((splits > 1 || plan.deep || plan.cfg == 3) && !fullk) return hipErrorInvalidValue;
  if (splits > 1 && !partial) return hipErrorInvalidValue;
  if (plan.deep && splits > 1)
    return plan.cfg == 2   ? launch_tile<2, 2, true, true, true>(A_q, A_s, W_q, W_s, out_bf16, partial, splits, M, N, d, stream, 0, ldc)
           : plan.cfg == 3 ? launch_tile<2, 1, true, true, true>(A_q, A_s, W_q, W_s, out_bf16, partial, splits, M, N, d, stream, 0, ldc)
                           : hipErrorInvalidValue;
  if (plan.deep)
    return plan.cfg == 2   ? launch_tile<2, 2, true, false, true>(A_q, A_s, W_q, W_s, out_bf16, nullptr, 1, M, N, d, stream, 0, ldc)
           : plan.cfg == 3 ? launch_tile<2, 1, true, false, true>(A_q, A_s, W_q, W_s, out_bf16, nullptr, 1, M, N, d, stream, 0, ldc)
                           : hipErrorInvalidValue;
#define TORQ_GEMM_LAUNCH(WM_, WN_)                                                                             \
  if (persist && splits == 1 && fullk && ldc == N &&                                                           \
      persistent_pays(((M + 64 * WM_ - 1) / (64 * WM_)) * ((N + 64 * WN_ - 1) / (64 * WN_)), d))               \
    return launch_tile<WM_, WN_, true, false, false, 0, true>(A_q, A_s, W_q, W_s, out_bf16, nullptr, 1, M, N, d, stream); \
  return splits > 1 ? launch_tile<WM_, WN_, true, true>(A_q, A_s, W_q, W_s, out_bf16, partial, splits, M, N, d, stream, 0, ldc) \
         : fullk    ? launch_tile<WM_, WN_, true, false>(A_q, A_s, W_q, W_s, out_bf16, nullptr, 1, M, N, d, stream, 0, ldc)     \
                    : launch_tile<WM_, WN_, false, false>(A_q, A_s, W_q, W_s, out_bf16, nullptr, 1, M, N, d, stream, 0, ldc);
  if (plan.cfg == 0) { TORQ_GEMM_LAUNCH(4, 4) }
  if (plan.cfg == 1) { TORQ_GEMM_LAUNCH(4, 2) }
#undef TORQ_GEMM_LAUNCH
  // (two workgroups of the 128 x 128 tile share a CU: the persistent form, one per CU, measured slower)
  if (plan.cfg == 2)
    return splits > 1 ? launch_tile<2, 2, true, true>(A_q, A_s, W_q, W_s, out_bf16, partial, splits, M, N, d, stream, 0, ldc)
           : fullk    ? launch_tile<2, 2, true, false>(A_q, A_s, W_q, W_s, out_bf16, nullptr, 1, M, N, d, stream, 0, ldc)
                      : launch_tile<2, 2, false, false>(A_q, A_s, W_q, W_s, out_bf16, nullptr, 1, M, N, d, stream, 0, ldc);
  if (plan.cfg == 3)
    return splits > 1 ? launch_tile<2, 1, true, true>(A_q, A_s, W_q, W_s, out_bf16, partial, splits, M, N, d, stream, 0, ldc)
                      : launch_tile<2, 1, true, false>(A_q, A_s, W_q, W_s, out_bf16, nullptr, 1, M, N, d, stream, 0, ldc);
  return hipErrorInvalidValue;
}

// one product by the planner's plan
static hipError_t launch_planned(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                                 void *out_bf16, int64_t M, int64_t N, int d, int64_t ldc, bool fullk, bool ws_ok,
                                 void *workspace, size_t workspace_bytes, hipStream_t stream) {
  GemmPlan plan = plan_with(M, N, d, ws_ok, ws_ok ? workspace_bytes : 0);
  if (plan.skinny) {
    if (ldc != N) return hipErrorInvalidValue;            // (never planned for a remainder: see launch_mxfp4_gemm)
    return launch_mxfp4_gemm_skinny(A_q, A_s, W_q, W_s, out_bf16, M, N, d, stream);
  }
  if (!fullk) {                                           // the plain form of the three larger tiles takes any d
    plan.deep = false;
    if (plan.cfg == 3) plan.cfg = 2;
  }
  return launch_by_plan(plan, A_q, A_s, W_q, W_s, out_bf16, M, N, d, ldc, fullk, true, static_cast<float *>(workspace), stream);
}

// torq_diag_gemm_plan: the tiled kernel on a plan of the caller's choice, whatever the planner would take
hipError_t launch_mxfp4_gemm_forced(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                                    void *out_bf16, int64_t M, int64_t N, int d, int tile, int k_pieces, int deep,
                                    void *workspace, size_t workspace_bytes, hipStream_t stream) {
  if ((int64_t)d * 128 >= 0x7FFFFFFF || tile < 0 || tile > 3 || k_pieces < 1) return hipErrorInvalidValue;
  const bool fullk = (d % 512 == 0) && ((reinterpret_cast<uintptr_t>(A_s) & 15u) == 0) &&
                     ((reinterpret_cast<uintptr_t>(W_s) & 15u) == 0);
  if (k_pieces > 1) {
    if (d % 512 != 0 || (d / 512) % k_pieces != 0 || N % 8 != 0 || !workspace) return hipErrorInvalidValue;
    if ((reinterpret_cast<uintptr_t>(workspace) & 15u) != 0) return hipErrorInvalidValue;
    if (workspace_bytes < (size_t)k_pieces * (size_t)M * (size_t)N * sizeof(float)) return hipErrorInvalidValue;
  }
  if (deep && tile < 2) return hipErrorInvalidValue;
  const GemmPlan plan{false, tile, k_pieces, deep != 0, 0.0};
  return launch_by_plan(plan, A_q, A_s, W_q, W_s, out_bf16, M, N, d, N, fullk, false, static_cast<float *>(workspace), stream);
}

hipError_t launch_mxfp4_gemm(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q,
                             const uint8_t *W_s, void *out_bf16, int64_t M, int64_t N, int d,
                             void *workspace, size_t workspace_bytes, hipStream_t stream) {
  // a tile's rows must be addressable with 32-bit offsets: 256 rows of d/2 bytes
  if ((int64_t)d * 128 >= 0x7FFFFFFF) return hipErrorInvalidValue;
  // The fast k loop needs whole 512-element pieces per row and 16-byte aligned scale rows.
  const bool fullk = (d % 512 == 0) && ((reinterpret_cast<uintptr_t>(A_s) & 15u) == 0) &&
                     ((reinterpret_cast<uintptr_t>(W_s) & 15u) == 0);
  // cut along k only with a workspace that holds the pieces (16-byte aligned fp32 rows)
  const bool ws_ok = fullk && workspace && (reinterpret_cast<uintptr_t>(workspace) & 15u) == 0;
  // whole rounds of 256 x 256 tiles first, the remaining columns as a product of their own?
  const size_t ws_bytes = ws_ok ? workspace_bytes : 0;
  const int64_t main_n = fullk ? choose_main_columns(M, N, d, ws_ok, ws_bytes, plan_with(M, N, d, ws_ok, ws_bytes)) : N;
  if (main_n < N) {
    const int64_t walk = main_n / 256, tiles = ((M + 255) / 256) * walk;
    // (the persistent form where it pays: it walks the tile columns it is given like the plain one)
    hipError_t e = persistent_pays(tiles, d)
                       ? launch_tile<4, 4, true, false, false, 0, true>(A_q, A_s, W_q, W_s, out_bf16, nullptr, 1, M, N, d, stream, 0, 0, walk)
                       : launch_tile<4, 4, true, false>(A_q, A_s, W_q, W_s, out_bf16, nullptr, 1, M, N, d, stream, 0, 0, walk);
    if (e != hipSuccess) return e;
    // the remainder: rows main_n ... of W, columns main_n ... of out (a multiple of 256: every alignment
    // of the whole product holds for it); too few rows for the weight-streaming kernel never get here
    // (a remainder exists only with more than 256 tiles)
    return launch_planned(A_q, A_s, W_q + (size_t)main_n * (size_t)(d / 2), W_s + (size_t)main_n * (size_t)(d / 32),
                          static_cast<uint16_t *>(out_bf16) + main_n, M, N - main_n, d, N, fullk, ws_ok, workspace,
                          workspace_bytes, stream);
  }
  return launch_planned(A_q, A_s, W_q, W_s, out_bf16, M, N, d, N, fullk, ws_ok, workspace, workspace_bytes, stream);
}

// torq_diag_gemm_ablation: the 256 x 256-tile kernel with parts of its k loop left out (see SKIP above).
hipError_t launch_mxfp4_gemm_ablated(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                                     void *out_bf16, int64_t M, int64_t N, int d, int skip, hipStream_t stream) {
  if ((int64_t)d * 128 >= 0x7FFFFFFF || d % 512 != 0) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(A_s) & 15u) || (reinterpret_cast<uintptr_t>(W_s) & 15u)) return hipErrorInvalidValue;
  switch (skip) {
#define TORQ_ABLATE(S_) \
  case S_: return launch_tile<4, 4, true, false, false, S_>(A_q, A_s, W_q, W_s, out_bf16, nullptr, 1, M, N, d, stream);
    TORQ_ABLATE(0) TORQ_ABLATE(1) TORQ_ABLATE(3) TORQ_ABLATE(4) TORQ_ABLATE(7) TORQ_ABLATE(15)
#undef TORQ_ABLATE
    default: return hipErrorInvalidValue;
  }
}

// torq_diag_gemm_persistent: the persistent form of the tiled kernel on `workgroups` workgroups, whatever
// the shape (mxfp4_gemm only takes it from a round and a half of tiles on), so that its walk over several tiles per
// workgroup can be checked output by output on small shapes.
hipError_t launch_mxfp4_gemm_persistent(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                                        void *out_bf16, int64_t M, int64_t N, int d, int tile, int workgroups,
                                        hipStream_t stream) {
  if ((int64_t)d * 128 >= 0x7FFFFFFF || d % 1024 != 0 || workgroups < 1) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(A_s) & 15u) || (reinterpret_cast<uintptr_t>(W_s) & 15u)) return hipErrorInvalidValue;
  if (tile == 0)
    return launch_tile<4, 4, true, false, false, 0, true>(A_q, A_s, W_q, W_s, out_bf16, nullptr, 1, M, N, d, stream, workgroups);
  if (tile == 1)
    return launch_tile<4, 2, true, false, false, 0, true>(A_q, A_s, W_q, W_s, out_bf16, nullptr, 1, M, N, d, stream, workgroups);
  return hipErrorInvalidValue;
}

}  // namespace torq
