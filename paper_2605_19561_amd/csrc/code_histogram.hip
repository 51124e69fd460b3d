// torq_code_histogram: the column-wise codebook histogram of the intra-block calibration
// (Appendix A.5, N_j^(k); Section 5.2, the occupancy that the equilibrium loss is made of):
//
//   counts[k][j] = number of 32-element blocks whose element k carries the magnitude codeword j
//
// over the packed e2m1 codes that the quantiser wrote (the sign bit of a code is ignored).
//
// One lane = one block = one 16-byte load; dword w of it holds the elements 8 w .. 8 w + 7, one per
// nibble, element 8 w in the lowest.  Nothing is decoded element by element.  With b0 b1 b2 the
// three magnitude bits of a nibble, the lane counts, per nibble position, the seven monomials
//   b0, b1, b2, b0 b1, b0 b2, b1 b2, b0 b1 b2
// eight positions at a time with whole-dword AND / shift / ADD into nibble-packed counters (nine
// logic operations and seven additions per dword).  The eight codeword counts follow from the
// monomial sums and the number of blocks by inclusion-exclusion, once, in the final kernel.
// Nibble counters hold 15, so after 15 blocks they are widened into byte-packed counters, which
// hold 255 = 17 such chunks; then the workgroup adds its lanes' byte counters through LDS into
// 32-bit per-thread totals.  Loads are buffer loads in groups of five with two groups in flight
// beyond the one being counted; a block past the end of the input reads as zeros (the buffer's range
// check), and a zero nibble adds to no monomial.  Every workgroup writes its 224 totals; the final kernel adds them (integers: any order
// gives the same result).
// HBM bound: half a byte per element, read once.
#include "torq_device.h"
#include "torq_internal.h"

namespace torq {

constexpr int HIST_THREADS = 256;
constexpr int HIST_MAX_WG = 512;          // two resident workgroups per CU: one round
constexpr int HIST_GROUP = 5;             // blocks per lane per group of loads
constexpr int HIST_CHUNK = 3 * HIST_GROUP; // blocks per lane before a nibble counter could overflow
constexpr int HIST_WIDEN_PER_PASS = 17;   // chunks before a byte counter could overflow
constexpr int HIST_MONO = 7;
constexpr int HIST_WORDS = 2 * HIST_MONO * 4;  // byte-packed counter words per lane
constexpr int HIST_PARTIAL = HIST_MONO * 32;   // per workgroup: [monomial][position]
static_assert(HIST_CHUNK <= 15 && HIST_CHUNK * HIST_WIDEN_PER_PASS <= 255, "counter widths");

typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;

__global__ void __launch_bounds__(HIST_THREADS)
code_histogram_kernel(const uint8_t *__restrict__ codes, int64_t nblk, uint32_t *__restrict__ partial) {
  __shared__ __attribute__((aligned(16))) uint32_t lds[HIST_WORDS][HIST_THREADS];   // byte counters of every lane

  const int tid = threadIdx.x;
  const int64_t lanes = (int64_t)gridDim.x * HIST_THREADS;
  const int64_t per_lane = (nblk + lanes - 1) / lanes;                // uniform trip count
  const int ngroup = (int)((per_lane + HIST_GROUP - 1) / HIST_GROUP);
  // the workgroup's blocks are one contiguous span: [wg_first, wg_end)
  const int64_t wg_first = (int64_t)blockIdx.x * per_lane * HIST_THREADS;
  const int64_t wg_end = (wg_first + per_lane * HIST_THREADS < nblk) ? wg_first + per_lane * HIST_THREADS : nblk;
  const int voff = tid * 16;
  constexpr int ROW_BYTES = HIST_THREADS * 16;                        // one block per lane
  constexpr uint32_t K1 = 0x11111111u, KB = 0x0F0F0F0Fu;

  // Group g = the blocks wg_first + (HIST_GROUP g + i) * 256 + lane, i < HIST_GROUP: consecutive lanes
  // read consecutive 16-byte blocks.  The buffer resource starts at the group's first block and
  // ends at the end of the span, so a block past the end reads as zeros.
  auto load_group = [&](u32x4 (&v)[HIST_GROUP], int g) {
    const int64_t first = wg_first + (int64_t)g * HIST_GROUP * HIST_THREADS, left = (wg_end - first) * 16;
    const uint32_t records = left <= 0 ? 0u : (left > 0xFFFFFFFFll ? 0xFFFFFFFFu : (uint32_t)left);
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(codes) + (left <= 0 ? 0 : first * 16), 0, (int)records, 0x00020000);
#pragma unroll
    for (int i = 0; i < HIST_GROUP; ++i) v[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, i * ROW_BYTES, 0);
  };

  uint32_t nib[HIST_MONO][4], bytes[HIST_WORDS];
  auto count_group = [&](const u32x4 (&v)[HIST_GROUP]) {
#pragma unroll
    for (int i = 0; i < HIST_GROUP; ++i)
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t x = v[i][w], y = x >> 1, z = x >> 2;
        const uint32_t m0 = x & K1, m1 = y & K1, m2 = z & K1;
        const uint32_t m01 = m0 & y, m02 = m0 & z, m12 = m1 & z, m012 = m01 & z;
        nib[0][w] += m0;
        nib[1][w] += m1;
        nib[2][w] += m2;
        nib[3][w] += m01;
        nib[4][w] += m02;
        nib[5][w] += m12;
        nib[6][w] += m012;
      }
  };

  // totals of two byte positions of one byte-counter word (see the workgroup sum below)
  uint32_t tot_lo = 0, tot_hi = 0;
#pragma unroll
  for (int i = 0; i < HIST_WORDS; ++i) bytes[i] = 0;

  u32x4 v0[HIST_GROUP], v1[HIST_GROUP], v2[HIST_GROUP];   // two groups in flight beyond the one being counted
  load_group(v0, 0);
  load_group(v1, 1);
  int widened = 0;
  for (int g = 0; g < ngroup; g += 3) {
#pragma unroll
    for (int m = 0; m < HIST_MONO; ++m)
#pragma unroll
      for (int w = 0; w < 4; ++w) nib[m][w] = 0;
    load_group(v2, g + 2);
    count_group(v0);
    load_group(v0, g + 3);
    if (g + 1 < ngroup) count_group(v1);
    load_group(v1, g + 4);
    if (g + 2 < ngroup) count_group(v2);
    // 15 blocks at most: nibble counters -> byte counters, word 2 a = the even nibbles, 2 a + 1 the odd
#pragma unroll
    for (int m = 0; m < HIST_MONO; ++m)
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        bytes[2 * (m * 4 + w)] += nib[m][w] & KB;
        bytes[2 * (m * 4 + w) + 1] += (nib[m][w] >> 4) & KB;
      }
    ++widened;
    if (widened < HIST_WIDEN_PER_PASS && g + 3 < ngroup) continue;
    widened = 0;

    // workgroup sum of the byte counters, two 16-bit fields at a time (256 x 255 < 65536): thread
    // t < 224 adds bytes (h, h + 2) of word r over the lanes 128 g .. 128 g + 127, t = 4 r + 2 h + g,
    // and the two lane halves meet in a neighbour exchange
#pragma unroll
    for (int i = 0; i < HIST_WORDS; ++i) {
      lds[i][tid] = bytes[i];
      bytes[i] = 0;
    }
    __syncthreads();
    {
      const int r = (tid >> 2) % HIST_WORDS, shift = 8 * ((tid >> 1) & 1), l0 = 128 * (tid & 1);
      uint32_t acc = 0;
#pragma unroll 4
      for (int j = 0; j < 32; ++j) {
        // four lanes per read; staggered so that the lanes of a wave spread over the banks
        const u32x4 q = *reinterpret_cast<const u32x4 *>(&lds[r][l0 + 4 * ((j + tid) & 31)]);
        acc += ((q[0] >> shift) & 0x00FF00FFu) + ((q[1] >> shift) & 0x00FF00FFu) +
               ((q[2] >> shift) & 0x00FF00FFu) + ((q[3] >> shift) & 0x00FF00FFu);
      }
      acc += __shfl_xor(acc, 1);
      tot_lo += acc & 0xFFFFu;
      tot_hi += acc >> 16;
    }
    __syncthreads();
  }

  if (tid < HIST_PARTIAL && (tid & 1) == 0) {
    // word r = 2 (m * 4 + w) + odd; byte s of it counts nibble 2 s + odd of dword w: position
    // k = 8 w + 2 s + odd.  This thread holds s = h (tot_lo) and s = h + 2 (tot_hi).  The partial
    // sums are stored counter-major, [counter][workgroup], for the final kernel's coalesced reads.
    const int r = tid >> 2, odd = r & 1, a = r >> 1, m = a >> 2, w = a & 3, h = (tid >> 1) & 1;
    const int k = 8 * w + odd + 2 * h;
    partial[(size_t)(m * 32 + k) * HIST_MAX_WG + blockIdx.x] = tot_lo;
    partial[(size_t)(m * 32 + k + 4) * HIST_MAX_WG + blockIdx.x] = tot_hi;
  }
}

// Workgroup k of 32, 1024 threads: thread (monomial m = t / 128, slice = t % 128) adds the partial
// sums of the workgroups slice, slice + 128, ... (at most 8 of them, all loads in flight at once),
// the 128 slices are added through LDS in a fixed order, and eight threads turn
// (N, s0, s1, s2, s01, s02, s12, s012) into the eight codeword counts of position k by
// inclusion-exclusion.
__global__ void __launch_bounds__(1024)
code_histogram_final_kernel(const uint32_t *__restrict__ partial, int n_partial, uint64_t nblk,
                            uint64_t *__restrict__ counts) {
  __shared__ uint64_t part[8][128];
  __shared__ uint64_t s[8];
  const int tid = threadIdx.x, k = blockIdx.x, m = tid >> 7, slice = tid & 127;
  uint64_t acc = 0;
  if (m < HIST_MONO) {
    const uint32_t *src = partial + (size_t)(m * 32 + k) * HIST_MAX_WG;
    uint32_t v[HIST_MAX_WG / 128];
#pragma unroll
    for (int i = 0; i < HIST_MAX_WG / 128; ++i) v[i] = (slice + 128 * i < n_partial) ? src[slice + 128 * i] : 0u;
#pragma unroll
    for (int i = 0; i < HIST_MAX_WG / 128; ++i) acc += v[i];
  }
  part[m][slice] = acc;
  __syncthreads();
  if (tid < HIST_MONO) {
    uint64_t t = 0;
    for (int i = 0; i < 128; ++i) t += part[tid][i];
    s[tid] = t;
  }
  __syncthreads();
  if (tid < 8) {
    const uint64_t s0 = s[0], s1 = s[1], s2 = s[2], s01 = s[3], s02 = s[4], s12 = s[5], s012 = s[6];
    uint64_t c;
    switch (tid) {   // codeword j = b0 + 2 b1 + 4 b2
      case 0: c = nblk - s0 - s1 - s2 + s01 + s02 + s12 - s012; break;
      case 1: c = s0 - s01 - s02 + s012; break;
      case 2: c = s1 - s01 - s12 + s012; break;
      case 3: c = s01 - s012; break;
      case 4: c = s2 - s02 - s12 + s012; break;
      case 5: c = s02 - s012; break;
      case 6: c = s12 - s012; break;
      default: c = s012; break;
    }
    counts[k * 8 + tid] = c;
  }
}

size_t code_histogram_workspace_bytes() { return (size_t)HIST_MAX_WG * HIST_PARTIAL * sizeof(uint32_t); }

// nblk >= 0 blocks of 16 bytes (none: all counts zero); counts: 256 uint64 on the device; workspace as above
hipError_t launch_code_histogram(const uint8_t *codes, int64_t nblk, uint64_t *counts, void *workspace,
                                 hipStream_t stream) {
  // a workgroup per 256 * 15 blocks (one chunk per lane) while that leaves CUs free; beyond, all
  // the workgroups that can be resident at once, each with a longer span
  int64_t want = (nblk + (int64_t)HIST_THREADS * HIST_CHUNK - 1) / ((int64_t)HIST_THREADS * HIST_CHUNK);
  const int n_wg = (int)(want < 1 ? 1 : (want > HIST_MAX_WG ? HIST_MAX_WG : want));
  uint32_t *partial = static_cast<uint32_t *>(workspace);
  hipLaunchKernelGGL(code_histogram_kernel, dim3(n_wg), dim3(HIST_THREADS), 0, stream, codes, nblk, partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(code_histogram_final_kernel, dim3(32), dim3(1024), 0, stream, partial, n_wg, (uint64_t)nblk,
                     counts);
  return hipGetLastError();
}

}  // namespace torq
