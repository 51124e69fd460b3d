// torq_quantize_f32: MXFP4 quantisation of fp32 rows (Section 4, Eq. 1;
// Algorithm 3, step 4), and the MXINT4 / NVFP4 variants of Section 6.  HBM-bound: 4 B read +
// 17/32 B (18/32 for NVFP4) written per element.
//
// Four adjacent lanes share one 32-element block: each lane loads 8 consecutive
// floats (two 16-byte loads), the block amax is an in-lane max followed by two
// quad-permute DPP steps, and each lane stores its 8 nibbles as one dword.
#include "torq_device.h"
#include "torq_internal.h"

namespace torq {

__device__ __forceinline__ float quad_max(float v) {
  // max over the 4 lanes of a quad: xor 1 (quad_perm [1,0,3,2]) then xor 2 ([2,3,0,1])
  float o = __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0xB1, 0xF, 0xF, true));
  v = fmaxf(v, o);
  o = __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0x4E, 0xF, 0xF, true));
  return fmaxf(v, o);
}

// FMT: FMT_MXFP4, FMT_MXINT4 (same block and scale, integer elements) or FMT_NVFP4 (16-element
// blocks = lane pairs, an E4M3 scale byte each, on top of the tensor-wide global_scale).
template <int FMT>
__global__ void __launch_bounds__(256) quantize_f32_kernel(const float4 *__restrict__ z, int64_t n8,
                                                           float global_scale, uint32_t *__restrict__ codes,
                                                           uint8_t *__restrict__ scales) {
  // n8 = number of 8-element pieces = 4 * (number of blocks); a multiple of 4, so a quad is
  // never split by the bound and the DPP steps always see four live lanes.
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += stride) {
    float4 a = z[2 * i], b = z[2 * i + 1];
    float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    if constexpr (FMT == FMT_NVFP4) {
      float amax = amax8(v);
      amax = fmaxf(amax, __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(amax), 0xB1, 0xF, 0xF, true)));
      const uint32_t q = nvfp4_scale_code(amax, 6.0f * global_scale);
      codes[i] = pack8_nvfp4(v, e4m3_to_f32(q) * global_scale);
      if ((threadIdx.x & 1) == 0) scales[i >> 1] = (uint8_t)q;
    } else {
      float amax = quad_max(amax8(v));
      uint32_t byte = e8m0_from_amax(amax);
      codes[i] = (FMT == FMT_MXINT4) ? pack8_int4(v, e8m0_inverse_f32(byte)) : pack8_e2m1(v, e8m0_to_f32(byte));
      if ((threadIdx.x & 3) == 0) scales[i >> 2] = (uint8_t)byte;
    }
  }
}

hipError_t launch_quantize_f32(const float *z, int64_t nblk, int format, float global_scale, uint8_t *codes,
                               uint8_t *scales, hipStream_t stream) {
  if (nblk == 0) return hipSuccess;
  const int64_t n8 = nblk * 4;
  int64_t blocks = (n8 + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  const float4 *zz = reinterpret_cast<const float4 *>(z);
  uint32_t *cc = reinterpret_cast<uint32_t *>(codes);
  switch (format) {
    case FMT_MXFP4:
      hipLaunchKernelGGL(quantize_f32_kernel<FMT_MXFP4>, dim3((unsigned)blocks), dim3(256), 0, stream, zz, n8, 1.0f, cc, scales);
      break;
    case FMT_MXINT4:
      hipLaunchKernelGGL(quantize_f32_kernel<FMT_MXINT4>, dim3((unsigned)blocks), dim3(256), 0, stream, zz, n8, 1.0f, cc, scales);
      break;
    case FMT_NVFP4:
      hipLaunchKernelGGL(quantize_f32_kernel<FMT_NVFP4>, dim3((unsigned)blocks), dim3(256), 0, stream, zz, n8, global_scale, cc, scales);
      break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace torq
