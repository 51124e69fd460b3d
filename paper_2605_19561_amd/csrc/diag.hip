// torq_diag_mfma_burn: what the matrix cores of this machine sustain on operands of the
// caller's choice with nothing else running.  Not a step of the paper's method: it exists so
// that the benchmark can put its MFMA-bound kernels next to a ceiling measured on the same
// part, same day, same data -- the published peaks assume the nominal clock, and the part
// lowers its clock under matrix work on non-trivial operands.
//
// 1024 workgroups of 4 waves.  Every lane takes 4 + 4 operand register sets (4 dwords each)
// from the caller's buffer, then issues `iters` rounds of 16 independent MFMAs (a 4 x 4 grid
// of accumulators, the register-level shape of the GEMM's inner loop) and finally writes one
// value per lane so that the work cannot be dropped.
#include "torq_device.h"
#include "torq_internal.h"

namespace torq {

constexpr int BURN_BLOCKS = 1024;

template <int KIND>   // 0: v_mfma_scale_f32_32x32x64_f8f6f4 on e2m1 operands, 1: v_mfma_f32_32x32x16_bf16
__global__ void __launch_bounds__(256)
mfma_burn_kernel(const uint32_t *__restrict__ words, uint32_t n_words, int iters, float *__restrict__ sink) {
  const uint32_t gid = blockIdx.x * 256u + threadIdx.x;
  i32x4 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      a[i][j] = (int)words[(gid * 32u + i * 4 + j) % n_words];
      b[i][j] = (int)words[(gid * 32u + 16 + i * 4 + j) % n_words];
    }
  f32x16 c[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) c[i][j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (KIND == 0) {
          c[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
              i32x8{a[i][0], a[i][1], a[i][2], a[i][3], 0, 0, 0, 0},
              i32x8{b[j][0], b[j][1], b[j][2], b[j][3], 0, 0, 0, 0}, c[i][j], 4, 4, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
        } else {
          c[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]),
                                                            __builtin_bit_cast(bf16x8, b[j]), c[i][j], 0, 0, 0);
        }
      }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) s += c[i][j][0] + c[i][j][15];
  sink[gid] = s;
}

hipError_t launch_mfma_burn(int kind, const uint32_t *words, uint32_t n_words, int iters, float *sink,
                            hipStream_t stream) {
  if (kind == 0)
    hipLaunchKernelGGL(mfma_burn_kernel<0>, dim3(BURN_BLOCKS), dim3(256), 0, stream, words, n_words, iters, sink);
  else
    hipLaunchKernelGGL(mfma_burn_kernel<1>, dim3(BURN_BLOCKS), dim3(256), 0, stream, words, n_words, iters, sink);
  return hipGetLastError();
}

// torq_diag_copy: a plain copy of a known number of bytes (16 per lane and step, grid-stride), so that a
// counter run of any program of this library carries its own scale for the memory-traffic counters.
__global__ void __launch_bounds__(256) diag_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

hipError_t launch_diag_copy(const void *src, void *dst, size_t bytes, hipStream_t stream) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  const size_t want = (n16 + 255) / 256;
  const unsigned grid = (unsigned)(want < 256 * 16 ? want : 256 * 16);
  hipLaunchKernelGGL(diag_copy_kernel, dim3(grid), dim3(256), 0, stream, static_cast<const uint4 *>(src),
                     static_cast<uint4 *>(dst), n16);
  return hipGetLastError();
}

}  // namespace torq
