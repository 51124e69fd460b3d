// mxfp4_gemm for few activation rows (decode, M <= 64): the W4A4 linear layer of Section 5
// (weight fusion) / Algorithm 3 ("Return"), same arithmetic as mxfp4_gemm.hip:
//
//   out[m][n] = sum_kb 2^(A_s[m][kb] + W_s[n][kb] - 254) * sum_{k<32} val(A[m][32kb+k]) val(W[n][32kb+k])
//
// With so few rows the work is reading the weights once, so the layout of the job follows the
// memory system, not the matrix cores: one workgroup per strip of 16 weight rows (or two strips),
// so that N / 16 workgroups keep every CU streaming; its 8 waves split the k range between them;
// the codes go global -> registers directly in the operand layout of
// v_mfma_scale_f32_16x16x128_f8f6f4 (lane = (row l % 16, microscaling block l / 16), 16 code
// bytes), all loads of a trip in flight at once; the scale bytes of the strip and of the
// activation rows are copied to LDS once per workgroup; and the eight partial 16 x 16 tiles are
// added through LDS at the end.  Activations (at most 64 rows) are re-read by every workgroup
// from the L2.
//
// The first MFMA operand is the weight strip and the second the activations, so an accumulator
// lane holds out[m = l % 16][n = n0 + 4 (l / 16) + 0..3]: four consecutive outputs of one row.
#include "torq_device.h"
#include "torq_internal.h"

namespace torq {

namespace {

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4;
#define LDSP(x) ((__attribute__((address_space(3))) void *)(x))

constexpr int WAVES = 8;              // waves per workgroup = ways the k range is split
constexpr size_t SKINNY_MAX_LDS = 160 * 1024;
constexpr int SKINNY_MIN_GROUPS = 384; // fewer workgroups than this leave CUs without work (256 CUs)

// a voffset that the range check of any buffer used here rejects (the load then delivers zeros)
constexpr int OOB_VOFF = 0x7FFFFFF0;

}  // namespace

// MT = number of 16-row activation tiles (M <= 16 MT); NS = 16-row weight strips per workgroup
// (1 or 2; they share the activation loads); PT = line pairs per wave and trip
template <int MT, int NS, int PT>
__global__ void __launch_bounds__(64 * WAVES)
mxfp4_gemm_skinny_kernel(const uint8_t *__restrict__ A_q, const uint8_t *__restrict__ A_s,
                         const uint8_t *__restrict__ W_q, const uint8_t *__restrict__ W_s,
                         uint16_t *__restrict__ out, int M, int64_t N, int d) {
  // dynamic LDS: scale bytes of the weight strips (16 NS rows) and of the activation rows (16 MT),
  // d / 32 bytes each, every row padded by 4 bytes (the lanes of a k-step read one byte of 16
  // different rows); the partial tiles of waves 1.. are overlaid on it after the k loop
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r16 = lane & 15, q = lane >> 4;
  const int row_bytes = d / 2, srow_bytes = d / 32;
  const int KS = d / 128;                          // k-steps of one MFMA (128 elements, 4 blocks)
  const int KP = (KS + 1) / 2;                     // pairs of k-steps = whole 128-byte lines of a row
  const int64_t n0 = (int64_t)blockIdx.x * 16 * NS;
  const int rows_w = (N - n0 < 16 * NS) ? (int)(N - n0) : 16 * NS;

  // rows past N or M are outside the buffers: their loads deliver zeros
  const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(W_q + n0 * row_bytes, (uint32_t)rows_w * row_bytes);
  const __amdgpu_buffer_rsrc_t ws_rsrc = make_rsrc(W_s + n0 * srow_bytes, (uint32_t)rows_w * srow_bytes);
  const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(A_q, (uint32_t)M * row_bytes);
  const __amdgpu_buffer_rsrc_t as_rsrc = make_rsrc(A_s, (uint32_t)M * srow_bytes);
  const int c_voff = r16 * row_bytes + q * 16;     // codes: + 64 per k-step

  // ---- scales: copied to LDS by buffer loads with an LDS destination (no registers, nothing to
  // wait for before the code loads go out).  Such an instruction writes lane l's dword at
  // (base + 4 l), the global address per lane is free: LDS dword j of a region is (row j / pd,
  // column j % pd) of the padded layout, the pad column and rows past the end load zeros.
  const int sdw = srow_bytes / 4;                  // dwords per scale row
  const int pd = sdw + 1;                          // padded
  const int w_ins = (16 * NS * pd + 63) / 64;      // instructions (256 bytes each) for the weight strips
  const int a_ins = (16 * MT * pd + 63) / 64;      // ... and for the activation rows
  for (int i = wave; i < w_ins + a_ins; i += WAVES) {
    const bool is_w = i < w_ins;
    const int j = (is_w ? i : i - w_ins) * 64 + lane;
    const int row = j / pd, col = j - row * pd;
    const bool ok = col < sdw && row < (is_w ? 16 * NS : 16 * MT);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(is_w ? ws_rsrc : as_rsrc, LDSP(smem + i * 256), 4,
                                             ok ? row * srow_bytes + col * 4 : OOB_VOFF, 0, 0, 0);
  }
  const int ws_off = r16 * pd * 4 + q;             // this lane's scale byte: + 4 per k-step
  const int as_off = w_ins * 256 + r16 * pd * 4 + q;

  f32x4 acc[NS][MT];
#pragma unroll
  for (int n = 0; n < NS; ++n)
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[n][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Wave w takes the line pairs w, w + WAVES, ...; PT pairs (2 PT k-steps) per trip, all of their
  // loads issued before the first MFMA.  Pairs past the end (and the second k-step of the last
  // pair when KS is odd) load zeros through the range check instead of branching.
  bool first = true;
  for (int p0 = wave; p0 < KP; p0 += PT * WAVES) {
    u32x4 wq[2 * PT][NS], aq[2 * PT][MT];
#pragma unroll
    for (int u = 0; u < 2 * PT; ++u) {
      const int ks = 2 * (p0 + (u >> 1) * WAVES) + (u & 1);
      const bool in = ks < KS;
      const int cv = in ? c_voff : OOB_VOFF;
      const int co = in ? ks * 64 : 0;
#pragma unroll
      for (int n = 0; n < NS; ++n)
        wq[u][n] = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, cv, co + (in ? n * 16 * row_bytes : 0), 0);
#pragma unroll
      for (int t = 0; t < MT; ++t)
        aq[u][t] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, cv, co + (in ? t * 16 * row_bytes : 0), 0);
    }
    __builtin_amdgcn_sched_barrier(0);             // every load of the trip is in flight before the first wait
    if (first) {
      __syncthreads();                             // the scales are in LDS
      first = false;
    }
#pragma unroll
    for (int u = 0; u < 2 * PT; ++u) {
      const int ks = 2 * (p0 + (u >> 1) * WAVES) + (u & 1);
      const int sb = (ks < KS ? ks : 0) * 4;
      int asc[MT];
#pragma unroll
      for (int t = 0; t < MT; ++t) asc[t] = smem[as_off + t * 16 * pd * 4 + sb];
#pragma unroll
      for (int n = 0; n < NS; ++n) {
        const int wsc = smem[ws_off + n * 16 * pd * 4 + sb];
#pragma unroll
        for (int t = 0; t < MT; ++t)
          acc[n][t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
              i32x8{(int)wq[u][n][0], (int)wq[u][n][1], (int)wq[u][n][2], (int)wq[u][n][3], 0, 0, 0, 0},
              i32x8{(int)aq[u][t][0], (int)aq[u][t][1], (int)aq[u][t][2], (int)aq[u][t][3], 0, 0, 0, 0},
              acc[n][t], 4, 4, 0, wsc, 0, asc[t]);
      }
    }
  }
  if (first) __syncthreads();                      // a wave without any pair still meets the others

  // ---- add the waves' partial tiles in a fixed order (wave 0 + 1 + ... + 7), round, store
  __syncthreads();                                 // everybody is done with the scales
  float *red = reinterpret_cast<float *>(smem);    // [WAVES - 1][NS][MT][4][64]
  if (wave > 0) {
#pragma unroll
    for (int n = 0; n < NS; ++n)
#pragma unroll
      for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[((((wave - 1) * NS + n) * MT + t) * 4 + r) * 64 + lane] = acc[n][t][r];
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int n = 0; n < NS; ++n) {
      const int64_t nn = n0 + n * 16 + 4 * q;
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        bf16x4 v;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float sum = acc[n][t][r];
#pragma unroll
          for (int w = 0; w < WAVES - 1; ++w) sum += red[(((w * NS + n) * MT + t) * 4 + r) * 64 + lane];
          v[r] = (__bf16)sum;
        }
        const int m = t * 16 + r16;
        if (m < M) {
          uint16_t *dst = out + (int64_t)m * N + nn;
          if ((N & 3) == 0 && nn + 4 <= N) {
            *reinterpret_cast<bf16x4 *>(dst) = v;
          } else {
            const uint64_t bits = __builtin_bit_cast(uint64_t, v);
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (nn + r < N) dst[r] = (uint16_t)(bits >> (16 * r));
          }
        }
      }
    }
  }
}

template <int MT, int NS, int PT>
static hipError_t launch_cfg(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                             void *out, int64_t M, int64_t N, int d, hipStream_t stream) {
  const int64_t groups = (N + 16 * NS - 1) / (16 * NS);
  if (groups > 0x7FFFFFFF) return hipErrorInvalidValue;
  const int pd = d / 128 + 1;                      // padded dwords per scale row
  const size_t scale_bytes = (size_t)((16 * NS * pd + 63) / 64 + (16 * MT * pd + 63) / 64) * 256;
  const size_t red_bytes = (size_t)(WAVES - 1) * NS * MT * 4 * 64 * sizeof(float);
  const size_t lds_bytes = scale_bytes > red_bytes ? scale_bytes : red_bytes;
  if (lds_bytes > SKINNY_MAX_LDS) return hipErrorInvalidValue;
  if (lds_bytes > 64 * 1024) {
    // raise the dynamic LDS limit once per process and kernel variant (the call is slow)
    static bool raised = false;
    if (!raised) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(mxfp4_gemm_skinny_kernel<MT, NS, PT>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)SKINNY_MAX_LDS);
      if (e != hipSuccess) return e;
      raised = true;
    }
  }
  hipLaunchKernelGGL((mxfp4_gemm_skinny_kernel<MT, NS, PT>), dim3((unsigned)groups), dim3(64 * WAVES), lds_bytes,
                     stream, A_q, A_s, W_q, W_s, reinterpret_cast<uint16_t *>(out), (int)M, N, d);
  return hipGetLastError();
}

template <int MT, int NS>
static hipError_t launch_mt_ns(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                               void *out, int64_t M, int64_t N, int d, hipStream_t stream) {
  // trip depth: as deep as the k range of a wave goes, at most 4 line pairs (8 k-steps) in flight
  // (2 when the operand registers of a trip would not leave room for several workgroups per CU)
  const int pairs_per_wave = ((d / 128 + 1) / 2 + WAVES - 1) / WAVES;
  if (pairs_per_wave <= 1) return launch_cfg<MT, NS, 1>(A_q, A_s, W_q, W_s, out, M, N, d, stream);
  if (pairs_per_wave <= 2) return launch_cfg<MT, NS, 2>(A_q, A_s, W_q, W_s, out, M, N, d, stream);
  return launch_cfg<MT, NS, (MT + NS <= 3 ? 4 : 2)>(A_q, A_s, W_q, W_s, out, M, N, d, stream);
}

template <int MT>
static hipError_t launch_mt(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                            void *out, int64_t M, int64_t N, int d, hipStream_t stream) {
  // Two strips per workgroup share the activation loads.  That pays when the activations are
  // real traffic (not a row or two) and there are still enough workgroups to keep every CU
  // streaming; deeper sharing costs more in registers (fewer loads in flight) than it saves.
  const int64_t strips = (N + 15) / 16;
  if (MT <= 2 && M >= 8 && strips >= 2 * SKINNY_MIN_GROUPS)
    return launch_mt_ns<MT, (MT <= 2 ? 2 : 1)>(A_q, A_s, W_q, W_s, out, M, N, d, stream);
  return launch_mt_ns<MT, 1>(A_q, A_s, W_q, W_s, out, M, N, d, stream);
}

// Whether the scale rows of (up to two) strips and of the activations fit the LDS.
bool mxfp4_gemm_skinny_fits(int64_t M, int d) {
  const int MT = (int)((M + 15) / 16), NS = MT <= 2 ? 2 : 1;
  const int pd = d / 128 + 1;
  return M >= 1 && M <= 64 &&
         (size_t)((16 * NS * pd + 63) / 64 + (16 * MT * pd + 63) / 64) * 256 <= SKINNY_MAX_LDS;
}

// 1 <= M <= 64; d a multiple of 128 with 64 rows of d / 2 bytes addressable in 32 bits (the caller
// checks both) and mxfp4_gemm_skinny_fits(M, d).
hipError_t launch_mxfp4_gemm_skinny(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q,
                                    const uint8_t *W_s, void *out, int64_t M, int64_t N, int d,
                                    hipStream_t stream) {
  switch ((M + 15) / 16) {
    case 1: return launch_mt<1>(A_q, A_s, W_q, W_s, out, M, N, d, stream);
    case 2: return launch_mt<2>(A_q, A_s, W_q, W_s, out, M, N, d, stream);
    case 3: return launch_mt<3>(A_q, A_s, W_q, W_s, out, M, N, d, stream);
    case 4: return launch_mt<4>(A_q, A_s, W_q, W_s, out, M, N, d, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace torq
