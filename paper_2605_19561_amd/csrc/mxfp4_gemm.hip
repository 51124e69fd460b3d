// mxfp4_gemm: the W4A4 linear layer that consumes the quantised, rotated
// activations (Section 5, weight fusion; Algorithm 3, "Return").
//
//   out[m][n] = sum_kb 2^(A_s[m][kb] + W_s[n][kb] - 254) * sum_{k<32} val(A[m][32kb+k]) val(W[n][32kb+k])
//
// on v_mfma_scale_f32_32x32x64_f8f6f4 with both operands in e2m1: one lane holds
// the 32 codes (16 bytes) of one microscaling block of one row, and one E8M0
// byte per lane scales exactly that block -- the MX format maps onto the
// instruction without any repacking of the row-major code and scale arrays.
//
// The product is formed transposed (first operand = weight rows n, second =
// activation rows m), so that an accumulator lane holds runs of four
// consecutive n for one m and the bf16 epilogue stores 8 bytes per lane.
//
// Workgroup = 4 waves (2 x 2); each wave owns a (32*WM) x (32*WN) piece of the
// output tile.  The k loop advances 128 elements (64 bytes of codes, 4 scale
// bytes per row) per iteration: global -> registers -> LDS, double-buffered,
// one barrier per iteration.  LDS rows are padded from 64 to 80 bytes so that
// the 16-byte operand reads of 8 consecutive rows fall into distinct banks.
#include "torq_device.h"
#include "torq_internal.h"

namespace torq {

constexpr int GEMM_BK_BYTES = 64;     // 128 e2m1 codes per row per iteration
constexpr int GEMM_PITCH = 80;        // padded LDS row pitch in bytes
constexpr int GEMM_GROUP_M = 8;       // tile rows per scheduling group

template <int WM, int WN>
__global__ void __launch_bounds__(256)
mxfp4_gemm_kernel(const uint8_t *__restrict__ A_q, const uint8_t *__restrict__ A_s,
                  const uint8_t *__restrict__ W_q, const uint8_t *__restrict__ W_s,
                  uint16_t *__restrict__ out, int64_t M, int64_t N, int d,
                  int tiles_m, int tiles_n) {
  constexpr int BM = 64 * WM, BN = 64 * WN;
  constexpr int A_CHUNKS = BM * 4 / 256, W_CHUNKS = BN * 4 / 256;   // 16-byte chunks per thread
  constexpr int A_TILE = BM * GEMM_PITCH, W_TILE = BN * GEMM_PITCH;
  constexpr int STAGE = A_TILE + W_TILE;
  extern __shared__ __attribute__((aligned(16))) char lds[];

  // ---- which output tile: spread contiguous runs of tiles over the 8 XCDs, and
  // walk groups of GEMM_GROUP_M tile rows so that co-resident tiles share operands in L2
  const int total = tiles_m * tiles_n;
  int lid = blockIdx.x;
  if (total % 8 == 0) lid = (blockIdx.x % 8) * (total / 8) + blockIdx.x / 8;
  const int width = GEMM_GROUP_M * tiles_n;
  const int group = lid / width;
  const int first_m = group * GEMM_GROUP_M;
  const int gsz = (tiles_m - first_m < GEMM_GROUP_M) ? tiles_m - first_m : GEMM_GROUP_M;
  const int tm = first_m + (lid % width) % gsz;
  const int tn = (lid % width) / gsz;
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wy = wave >> 1, wx = wave & 1;
  const int lrow = lane & 31, g = lane >> 5;
  const int row_bytes = d / 2, srow = d / 32;

  // ---- global -> LDS staging: thread handles chunk c = tid + i*256; row = c/4, piece = c%4
  const uint8_t *a_src[A_CHUNKS];
  const uint8_t *w_src[W_CHUNKS];
  int a_dst[A_CHUNKS], w_dst[W_CHUNKS];
#pragma unroll
  for (int i = 0; i < A_CHUNKS; ++i) {
    const int c = tid + i * 256, r = c >> 2, p = c & 3;
    int64_t gr = m0 + r;
    if (gr >= M) gr = M - 1;                       // clamp: rows past the edge are never stored
    a_src[i] = A_q + gr * row_bytes + p * 16;
    a_dst[i] = r * GEMM_PITCH + p * 16;
  }
#pragma unroll
  for (int i = 0; i < W_CHUNKS; ++i) {
    const int c = tid + i * 256, r = c >> 2, p = c & 3;
    int64_t gr = n0 + r;
    if (gr >= N) gr = N - 1;
    w_src[i] = W_q + gr * row_bytes + p * 16;
    w_dst[i] = A_TILE + r * GEMM_PITCH + p * 16;
  }
  // ---- scale rows of this lane's operand fragments (read straight from global)
  const uint8_t *as_src[WM];
  const uint8_t *ws_src[WN];
#pragma unroll
  for (int i = 0; i < WM; ++i) {
    int64_t gr = m0 + (wy * WM + i) * 32 + lrow;
    if (gr >= M) gr = M - 1;
    as_src[i] = A_s + gr * srow;
  }
#pragma unroll
  for (int i = 0; i < WN; ++i) {
    int64_t gr = n0 + (wx * WN + i) * 32 + lrow;
    if (gr >= N) gr = N - 1;
    ws_src[i] = W_s + gr * srow;
  }

  f32x16 acc[WN][WM];
#pragma unroll
  for (int j = 0; j < WN; ++j)
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

  uint4 a_regs[A_CHUNKS], w_regs[W_CHUNKS];
  uint32_t as_regs[WM], ws_regs[WN], as_next[WM], ws_next[WN];
  auto g_load = [&](int kt) {
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) a_regs[i] = *reinterpret_cast<const uint4 *>(a_src[i] + kt * GEMM_BK_BYTES);
#pragma unroll
    for (int i = 0; i < W_CHUNKS; ++i) w_regs[i] = *reinterpret_cast<const uint4 *>(w_src[i] + kt * GEMM_BK_BYTES);
#pragma unroll
    for (int i = 0; i < WM; ++i) as_next[i] = *reinterpret_cast<const uint32_t *>(as_src[i] + kt * 4);
#pragma unroll
    for (int i = 0; i < WN; ++i) ws_next[i] = *reinterpret_cast<const uint32_t *>(ws_src[i] + kt * 4);
  };
  auto l_store = [&](int buf) {
    char *base = lds + buf * STAGE;
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) *reinterpret_cast<uint4 *>(base + a_dst[i]) = a_regs[i];
#pragma unroll
    for (int i = 0; i < W_CHUNKS; ++i) *reinterpret_cast<uint4 *>(base + w_dst[i]) = w_regs[i];
  };

  const int KT = d / 128;
  g_load(0);
  l_store(0);
#pragma unroll
  for (int i = 0; i < WM; ++i) as_regs[i] = as_next[i] >> (8 * g);
#pragma unroll
  for (int i = 0; i < WN; ++i) ws_regs[i] = ws_next[i] >> (8 * g);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    const bool have_next = kt + 1 < KT;
    if (have_next) g_load(kt + 1);

    const char *sa = lds + buf * STAGE + (wy * WM * 32 + lrow) * GEMM_PITCH + g * 16;
    const char *sw = lds + buf * STAGE + A_TILE + (wx * WN * 32 + lrow) * GEMM_PITCH + g * 16;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      i32x8 af[WM], wf[WN];
#pragma unroll
      for (int i = 0; i < WM; ++i) {
        const i32x4 v = *reinterpret_cast<const i32x4 *>(sa + i * 32 * GEMM_PITCH + ks * 32);
        af[i] = i32x8{v[0], v[1], v[2], v[3], 0, 0, 0, 0};
      }
#pragma unroll
      for (int j = 0; j < WN; ++j) {
        const i32x4 v = *reinterpret_cast<const i32x4 *>(sw + j * 32 * GEMM_PITCH + ks * 32);
        wf[j] = i32x8{v[0], v[1], v[2], v[3], 0, 0, 0, 0};
      }
#pragma unroll
      for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int i = 0; i < WM; ++i) {
          // lane (row, g) of a fragment carries block 2*ks + g of this iteration; its scale
          // byte sits in byte 2*ks of the lane-shifted scale dword
          if (ks == 0)
            acc[j][i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wf[j], af[i], acc[j][i], 4, 4, 0,
                                                                        ws_regs[j], 0, as_regs[i]);
          else
            acc[j][i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wf[j], af[i], acc[j][i], 4, 4, 2,
                                                                        ws_regs[j], 2, as_regs[i]);
        }
    }

    if (have_next) {
      l_store(buf ^ 1);
#pragma unroll
      for (int i = 0; i < WM; ++i) as_regs[i] = as_next[i] >> (8 * g);
#pragma unroll
      for (int i = 0; i < WN; ++i) ws_regs[i] = ws_next[i] >> (8 * g);
    }
    __syncthreads();
  }

  // ---- epilogue: acc[j][i][r] = out[m = .. + lane%32][n = .. + 8*(r/4) + 4*(lane/32) + r%4]
#pragma unroll
  for (int i = 0; i < WM; ++i) {
    const int64_t m = m0 + (wy * WM + i) * 32 + lrow;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < WN; ++j) {
      const int64_t nb = n0 + (wx * WN + j) * 32 + 4 * g;
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const int64_t n = nb + 8 * rr;
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (__bf16)acc[j][i][4 * rr + e];
        uint16_t *dst = out + m * N + n;
        if (n + 3 < N && ((N & 3) == 0)) {
          *reinterpret_cast<bf16x4 *>(dst) = v;
        } else {
          const uint64_t bits = __builtin_bit_cast(uint64_t, v);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (n + e < N) dst[e] = (uint16_t)(bits >> (16 * e));
        }
      }
    }
  }
}

template <int WM, int WN>
static hipError_t launch_tile(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q,
                              const uint8_t *W_s, void *out, int64_t M, int64_t N, int d,
                              hipStream_t stream) {
  constexpr int BM = 64 * WM, BN = 64 * WN;
  const int64_t tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  if (tiles_m * tiles_n > 0x7FFFFFFF) return hipErrorInvalidValue;
  const size_t lds_bytes = 2 * (size_t)(BM + BN) * GEMM_PITCH;
  auto kern = mxfp4_gemm_kernel<WM, WN>;
  if (lds_bytes > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(256), lds_bytes, stream, A_q, A_s, W_q,
                     W_s, reinterpret_cast<uint16_t *>(out), M, N, d, (int)tiles_m, (int)tiles_n);
  return hipGetLastError();
}

hipError_t launch_mxfp4_gemm(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q,
                             const uint8_t *W_s, void *out_bf16, int64_t M, int64_t N, int d,
                             hipStream_t stream) {
  // large tile when it still gives every CU work; small tile otherwise
  const int64_t big_tiles = ((M + 255) / 256) * ((N + 255) / 256);
  if (big_tiles >= 256) return launch_tile<4, 4>(A_q, A_s, W_q, W_s, out_bf16, M, N, d, stream);
  return launch_tile<2, 2>(A_q, A_s, W_q, W_s, out_bf16, M, N, d, stream);
}

}  // namespace torq
