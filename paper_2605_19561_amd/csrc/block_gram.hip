// torq_block_gram: the statistic that the inter-block calibration starts from (Section 5.1,
// Algorithm 1 input; Section 4.2, sigma_b^2 = E ||z_b||^2):
//
//   Sigma[b][b'] = mean over token-groups of  sum_k X[b][k] X[b'][k]
//
// where a token-group is one run of G consecutive 32-element blocks of one row, i.e. G rows of
// 64 contiguous bytes.  The contraction index is the position inside a block (K = 32), which is
// exactly one v_mfma_f32_16x16x32_bf16: lane (m = l % 16, q = l / 16) of an operand holds the 8
// consecutive elements 8 q .. 8 q + 7 of block row m -- 16 contiguous bytes of the row-major input,
// so an operand is 16 rows x one 16-byte chunk and nothing is transposed.  bf16 products are exact
// in fp32; the sums are fp32 per workgroup and fp64 across workgroups.
//
// Workgroup = ceil(G / 32) waves; wave w owns the block rows 32 w .. 32 w + 31 (two 16-row tiles)
// against all G columns (NT = G / 16 tiles): 2 NT accumulator tiles of 4 registers.  Every wave
// needs the whole token-group as its column operand, so the workgroup stages it once through LDS
// (global -> registers -> LDS, two stages, one barrier per trip of two token-groups) instead of
// letting each wave fetch it from the L1 (that version was bound by the L1's request rate, 5 requests
// per byte).  Workgroups are persistent; each writes its partial Sigma to the workspace, and two
// small kernels add the partials in a fixed order in double and divide by the number of
// token-groups.  HBM bound: 2 bytes per element, read once.
#include "torq_device.h"
#include "torq_internal.h"

namespace torq {

constexpr int GRAM_MAX_WG = 512;      // partial results (2 resident workgroups per CU)
constexpr int GRAM_GROUPS_PER_TRIP = 2;

template <int NT>
__global__ void __launch_bounds__(64 * ((NT + 1) / 2))
block_gram_kernel(const uint4 *__restrict__ x, int64_t TG, int position, float *__restrict__ partial) {
  constexpr int G = 16 * NT;
  constexpr int NTHR = 64 * ((NT + 1) / 2);
  constexpr int CHUNKS = 4 * G;                          // 16-byte chunks of one token-group
  constexpr int CH = (CHUNKS + NTHR - 1) / NTHR;         // chunks per thread per token-group (2)
  constexpr int U = GRAM_GROUPS_PER_TRIP;
  constexpr int TG_BYTES = G * 64, STAGE_BYTES = U * TG_BYTES;
  extern __shared__ __attribute__((aligned(16))) char lds[];   // two stages of U token-groups

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m = lane & 15, q = lane >> 4;
  const int rt0 = 2 * wave, rt1 = 2 * wave + 1;          // this wave's row tiles; rt1 may not exist
  const bool has1 = rt1 < NT;

  f32x4 acc0[NT], acc1[NT];
#pragma unroll
  for (int ct = 0; ct < NT; ++ct) acc0[ct] = acc1[ct] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Chunk c of a token-group = (block row c / 4, elements 8 (c % 4) .. + 7).  In LDS the chunk
  // index inside a 64-byte row is XORed with (row >> 2) & 3, so that the 16 lanes that read one
  // operand (16 consecutive rows, same chunk) hit 16 different bank groups.  For a tile's rows
  // 16 t + m that term is (m >> 2) & 3: one lane offset serves every tile.
  const int frag_off = m * 64 + ((q ^ ((m >> 2) & 3)) * 16);
  int st_off[CH];
#pragma unroll
  for (int i = 0; i < CH; ++i) {
    const int c = tid + i * NTHR, r = c >> 2;
    st_off[i] = r * 64 + (((c & 3) ^ ((r >> 2) & 3)) * 16);
  }

  // Which bits of this thread's chunks count: all of them for Sigma (position < 0); for Sigma_k only
  // element `position` of every block, i.e. one half of word (position / 2) % 4 of chunk position / 8.
  uint32_t keep[CH][4];
#pragma unroll
  for (int i = 0; i < CH; ++i)
#pragma unroll
    for (int w = 0; w < 4; ++w)
      keep[i][w] = position < 0 ? 0xFFFFFFFFu
                 : ((((tid + i * NTHR) & 3) == ((position >> 3) & 3) && w == ((position >> 1) & 3))
                        ? ((position & 1) ? 0xFFFF0000u : 0x0000FFFFu) : 0u);

  // a trip = U token-groups; trips are dealt to the workgroups round robin
  const int64_t ntrip = (TG + U - 1) / U;
  uint4 regs[U][CH];
  auto load_trip = [&](int64_t trip) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t tg = trip * U + u;
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        const int c = tid + i * NTHR;
        regs[u][i] = (tg < TG && c < CHUNKS) ? x[tg * CHUNKS + c] : make_uint4(0, 0, 0, 0);
        regs[u][i].x &= keep[i][0];
        regs[u][i].y &= keep[i][1];
        regs[u][i].z &= keep[i][2];
        regs[u][i].w &= keep[i][3];
      }
    }
  };
  auto store_trip = [&](int stage) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int i = 0; i < CH; ++i)
        if (tid + i * NTHR < CHUNKS)
          *reinterpret_cast<uint4 *>(lds + stage * STAGE_BYTES + u * TG_BYTES + st_off[i]) = regs[u][i];
  };

  int64_t trip = blockIdx.x;
  if (trip < ntrip) {
    load_trip(trip);
    store_trip(0);
  }
  __syncthreads();
  int stage = 0;
  for (; trip < ntrip; trip += gridDim.x, stage ^= 1) {
    const int64_t next = trip + gridDim.x;
    const bool have_next = next < ntrip;
    if (have_next) load_trip(next);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const char *g = lds + stage * STAGE_BYTES + u * TG_BYTES + frag_off;
      const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(g + rt0 * 1024);
      const bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(g + (has1 ? rt1 : rt0) * 1024);
#pragma unroll
      for (int ct = 0; ct < NT; ++ct) {
        const bf16x8 col = *reinterpret_cast<const bf16x8 *>(g + ct * 1024);
        acc0[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, col, acc0[ct], 0, 0, 0);
        acc1[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, col, acc1[ct], 0, 0, 0);
      }
    }
    if (have_next) store_trip(stage ^ 1);
    __syncthreads();
  }

  // accumulator lane (n = l % 16, q), register r: row 4 q + r of the row tile, column n of the column tile
  float *out = partial + (size_t)blockIdx.x * (G * G);
#pragma unroll
  for (int ct = 0; ct < NT; ++ct)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      out[(16 * rt0 + 4 * q + r) * G + 16 * ct + m] = acc0[ct][r];
      if (has1) out[(16 * rt1 + 4 * q + r) * G + 16 * ct + m] = acc1[ct][r];
    }
}

// Two-stage sum of the partial results, in double and in a fixed order.  Stage 1: slice s of
// GRAM_SLICES adds its share of the workgroups' partials; stage 2 adds the slices and divides by
// the number of token-groups.
constexpr int GRAM_SLICES = 16;

__global__ void __launch_bounds__(256)
block_gram_reduce1_kernel(const float *__restrict__ partial, int n_partial, int GG, double *__restrict__ slices) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= GG) return;
  const int per = (n_partial + GRAM_SLICES - 1) / GRAM_SLICES;
  const int p0 = blockIdx.y * per, p1 = (p0 + per < n_partial) ? p0 + per : n_partial;
  double s = 0.0;
  int p = p0;
  for (; p + 8 <= p1; p += 8) {                  // eight loads in flight, added in order
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = partial[(size_t)(p + u) * GG + i];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += (double)v[u];
  }
  for (; p < p1; ++p) s += (double)partial[(size_t)p * GG + i];
  slices[(size_t)blockIdx.y * GG + i] = s;
}

__global__ void __launch_bounds__(256)
block_gram_reduce2_kernel(const double *__restrict__ slices, int GG, double inv_groups, double *__restrict__ Sigma) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= GG) return;
  double s = 0.0;
#pragma unroll
  for (int p = 0; p < GRAM_SLICES; ++p) s += slices[(size_t)p * GG + i];
  Sigma[i] = s * inv_groups;
}

// [GRAM_MAX_WG][G * G] floats, then [GRAM_SLICES][G * G] doubles
size_t block_gram_workspace_bytes(int G) {
  return (size_t)GRAM_MAX_WG * G * G * sizeof(float) + (size_t)GRAM_SLICES * G * G * sizeof(double);
}

template <int NT>
static hipError_t launch_nt(const void *x, int64_t TG, int position, double *Sigma, void *workspace, hipStream_t stream) {
  constexpr int G = 16 * NT;
  float *partial = static_cast<float *>(workspace);
  double *slices = reinterpret_cast<double *>(static_cast<char *>(workspace) + (size_t)GRAM_MAX_WG * G * G * sizeof(float));
  const int64_t ntrip = (TG + GRAM_GROUPS_PER_TRIP - 1) / GRAM_GROUPS_PER_TRIP;
  const int n_wg = (int)(ntrip < GRAM_MAX_WG ? ntrip : GRAM_MAX_WG);
  const size_t lds_bytes = 2 * (size_t)GRAM_GROUPS_PER_TRIP * G * 64;
  hipLaunchKernelGGL((block_gram_kernel<NT>), dim3(n_wg), dim3(64 * ((NT + 1) / 2)), lds_bytes, stream,
                     reinterpret_cast<const uint4 *>(x), TG, position, partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(block_gram_reduce1_kernel, dim3((G * G + 255) / 256, GRAM_SLICES), dim3(256), 0, stream, partial,
                     n_wg, G * G, slices);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(block_gram_reduce2_kernel, dim3((G * G + 255) / 256), dim3(256), 0, stream, slices, G * G,
                     1.0 / (double)TG, Sigma);
  return hipGetLastError();
}

// G a multiple of 16 in [16, 256], TG > 0 token-groups, workspace of block_gram_workspace_bytes(G)
// position: -1 for Sigma, 0 .. 31 for the per-position matrix Sigma_k (every other element of a block
// counts as zero)
hipError_t launch_block_gram(const void *x_bf16, int64_t TG, int G, int position, double *Sigma, void *workspace,
                             hipStream_t stream) {
  switch (G / 16) {
#define TORQ_GRAM_CASE(NT_) \
  case NT_: return launch_nt<NT_>(x_bf16, TG, position, Sigma, workspace, stream);
    TORQ_GRAM_CASE(1) TORQ_GRAM_CASE(2) TORQ_GRAM_CASE(3) TORQ_GRAM_CASE(4)
    TORQ_GRAM_CASE(5) TORQ_GRAM_CASE(6) TORQ_GRAM_CASE(7) TORQ_GRAM_CASE(8)
    TORQ_GRAM_CASE(9) TORQ_GRAM_CASE(10) TORQ_GRAM_CASE(11) TORQ_GRAM_CASE(12)
    TORQ_GRAM_CASE(13) TORQ_GRAM_CASE(14) TORQ_GRAM_CASE(15) TORQ_GRAM_CASE(16)
#undef TORQ_GRAM_CASE
  }
  return hipErrorInvalidValue;
}

}  // namespace torq
