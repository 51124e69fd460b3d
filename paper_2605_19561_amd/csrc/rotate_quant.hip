// torq_rotate_quantize / torq_rotate: Algorithm 3 steps 1-4 (Appendix A.3) as one
// gfx950 kernel.
//
// A "token-group" is one run of G consecutive microscaling blocks of one token
// row: G*32 contiguous bf16 values.  Because rows are contiguous too, the whole
// input is a flat array of M*(d/32)/G token-groups, and so are all outputs.
//
// Per token-group, with X the G x 32 view (Section 4, "Notations"):
//   step 2   Y^T[k][b]  = sum_b' X^T[k][b'] * R_inter^T[b'][b]     (32 x G) = (32 x G)(G x G)
//   step 3   Z^T[k][b]  = sum_k' R_intra^T[k][k'] * Y^T[k'][b]     (32 x G) = (32 x 32)(32 x G)
// Both are dense contractions and run on v_mfma_f32_16x16x32_bf16.  The
// transposed formulation makes the accumulator of step 2 (rows k' in registers,
// column b across lanes) directly the B operand of step 3, and leaves, after
// step 3, eight consecutive k of one block b in each lane, so that the block
// amax is an in-lane max plus two cross-lane steps and the eight e2m1 nibbles
// of a lane are one aligned dword of the output.
//
// Precision: X is exact in bf16.  R_inter and R_intra are fp32, so each is split
// into a bf16 high part and a bf16 remainder (two MFMA passes over step 2); the
// fp32 result Y is split the same way for step 3 (three passes: Yhi*Rhi,
// Ylo*Rhi, Yhi*Rlo).  The dropped terms are of relative size 2^-17.
//
// Work split: a workgroup has G/16/NT waves; wave w owns NT tiles of 16 output
// blocks b and keeps the matching slices of R_inter^T (hi and lo) and all of
// R_intra^T in registers for the whole kernel.  All waves read the same X from
// LDS: the workgroup streams batches of TB token-groups global -> registers ->
// LDS (double-buffered, one barrier per batch) and each wave fetches its A
// operands with ds_read_b64_tr_b16, which performs the (k, b') transpose that
// the row-major input needs.
#include "torq_device.h"
#include "torq_internal.h"

namespace torq {

typedef __attribute__((address_space(3))) i16x4 lds_i16x4;

template <int KS>
struct RotCfg {
  static constexpr int TB = (KS <= 4) ? 4 : 2;          // token-groups per batch
  static constexpr int TG_LDS_BYTES = KS * 32 * 64;     // one token-group in LDS, padded to KS*32 rows
  static constexpr int STAGE_BYTES = TB * TG_LDS_BYTES;
};

// One A operand of step 2 (16 positions k x 32 blocks b') out of LDS.  Each
// ds_read_b64_tr_b16 hands lane (i = l%16, q = l/16) the four values
// X[b' = row0 + e][k = col0 + i], e = 0..3, when lane (s = l%16, q) points at
// X[row0 + s/4][col0 + 4*(s%4)].
__device__ __forceinline__ bf16x8 load_xT_frag(const char *tg_base, int ks, int mt, int lane) {
  const int q = lane >> 4, s = lane & 15;
  const int row = 32 * ks + 8 * q + (s >> 2);
  const int col = 16 * mt + 4 * (s & 3);
  const char *p = tg_base + (row * 32 + col) * 2;
  union { bf16x8 v; i16x4 h[2]; } u;
  u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4 *)(p));
  u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4 *)(p + 4 * 64));   // rows + 4
  return u.v;
}

__device__ __forceinline__ uint32_t pack_bf16_rne(float a, float b) {
  bf16x2 v;
  v[0] = (__bf16)a;
  v[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, v);
}

template <int KS, int NT, bool QUANT>
__global__ void __launch_bounds__(64 * ((2 * KS) / NT > 16 ? 16 : (2 * KS) / NT))
rotate_kernel(const uint4 *__restrict__ x, int64_t TG, int G,
              const uint16_t *__restrict__ inter_hi, const uint16_t *__restrict__ inter_lo,
              const uint4 *__restrict__ intra_hi_frag, const uint4 *__restrict__ intra_lo_frag,
              uint32_t *__restrict__ codes, uint8_t *__restrict__ scales, float *__restrict__ z_out) {
  using Cfg = RotCfg<KS>;
  constexpr int TB = Cfg::TB;
  extern __shared__ __attribute__((aligned(16))) char lds[];

  const int tid = threadIdx.x;
  const int nthr = blockDim.x;                 // = 64 * G/16/NT = 4G/NT
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int q = lane >> 4, col = lane & 15;

  // ---- resident operands --------------------------------------------------
  // step 2 B operand: lane (n = b, q) slot j holds R_inter[b][32 ks + 8 q + j]
  bf16x8 Bh[KS][NT], Bl[KS][NT];
#pragma unroll
  for (int i = 0; i < NT; ++i) {
    const int b = 16 * (wave * NT + i) + col;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const size_t off = (size_t)b * (KS * 32) + 32 * ks + 8 * q;
      Bh[ks][i] = *reinterpret_cast<const bf16x8 *>(inter_hi + off);
      Bl[ks][i] = *reinterpret_cast<const bf16x8 *>(inter_lo + off);
    }
  }
  // step 3 A operand (R_intra^T, rows permuted), already in fragment order
  bf16x8 Ah[2], Al[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    Ah[t] = __builtin_bit_cast(bf16x8, intra_hi_frag[t * 64 + lane]);
    Al[t] = __builtin_bit_cast(bf16x8, intra_lo_frag[t * 64 + lane]);
  }

  // ---- LDS: zero once so that the padded rows (b' >= G) read as 0 ------------
  for (int i = tid; i < 2 * Cfg::STAGE_BYTES / 16; i += nthr)
    reinterpret_cast<uint4 *>(lds)[i] = make_uint4(0, 0, 0, 0);
  __syncthreads();

  const int64_t nbatch = (TG + TB - 1) / TB;
  const int64_t chunks_per_tg = (int64_t)nthr * NT;    // 16-byte chunks in one token-group (= 4G)

  uint4 stage_regs[TB][NT];
  auto load_batch = [&](int64_t batch) {
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      const int64_t tg = batch * TB + j;
#pragma unroll
      for (int i = 0; i < NT; ++i) {
        if (tg < TG) stage_regs[j][i] = x[tg * chunks_per_tg + tid + i * nthr];
        else stage_regs[j][i] = make_uint4(0, 0, 0, 0);
      }
    }
  };
  auto store_batch = [&](int buf) {
    char *base = lds + buf * Cfg::STAGE_BYTES;
#pragma unroll
    for (int j = 0; j < TB; ++j)
#pragma unroll
      for (int i = 0; i < NT; ++i)
        *reinterpret_cast<uint4 *>(base + j * Cfg::TG_LDS_BYTES + (tid + i * nthr) * 16) = stage_regs[j][i];
  };

  int64_t batch = blockIdx.x;
  if (batch < nbatch) {
    load_batch(batch);
    store_batch(0);
  }
  __syncthreads();

  int buf = 0;
  for (; batch < nbatch; batch += gridDim.x, buf ^= 1) {
    const int64_t next = batch + gridDim.x;
    const bool have_next = next < nbatch;
    if (have_next) load_batch(next);

    const char *stage = lds + buf * Cfg::STAGE_BYTES;
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      const int64_t tg = batch * TB + j;
      if (tg >= TG) break;                                  // uniform over the workgroup
      const char *tg_base = stage + j * Cfg::TG_LDS_BYTES;

      // ---- step 2: Y^T = X^T R_inter^T --------------------------------------
      f32x4 acc[2][NT];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int i = 0; i < NT; ++i) acc[mt][i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
          const bf16x8 xa = load_xT_frag(tg_base, ks, mt, lane);
#pragma unroll
          for (int i = 0; i < NT; ++i) {
            acc[mt][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, Bh[ks][i], acc[mt][i], 0, 0, 0);
            acc[mt][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, Bl[ks][i], acc[mt][i], 0, 0, 0);
          }
        }
      }

#pragma unroll
      for (int i = 0; i < NT; ++i) {
        // ---- step 3: Z^T = R_intra^T Y^T, Y split into bf16 hi + lo -----------
        // B operand slot j <-> k' = 4q + j (acc[0]), slot 4+j <-> k' = 16 + 4q + j (acc[1])
        float y[8] = {acc[0][i][0], acc[0][i][1], acc[0][i][2], acc[0][i][3],
                      acc[1][i][0], acc[1][i][1], acc[1][i][2], acc[1][i][3]};
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          hi[p] = pack_bf16_rne(y[2 * p], y[2 * p + 1]);
          const float r0 = y[2 * p] - __uint_as_float(hi[p] << 16);
          const float r1 = y[2 * p + 1] - __uint_as_float(hi[p] & 0xFFFF0000u);
          lo[p] = pack_bf16_rne(r0, r1);
        }
        const bf16x8 yh = __builtin_bit_cast(bf16x8, i32x4{(int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]});
        const bf16x8 yl = __builtin_bit_cast(bf16x8, i32x4{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3]});
        f32x4 zacc[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          zacc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
          zacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Al[t], yh, zacc[t], 0, 0, 0);
          zacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Ah[t], yl, zacc[t], 0, 0, 0);
          zacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Ah[t], yh, zacc[t], 0, 0, 0);
        }
        // lane (b = col, q) now holds Z[b][8q + 4t + r] in zacc[t][r]
        const float zz[8] = {zacc[0][0], zacc[0][1], zacc[0][2], zacc[0][3],
                             zacc[1][0], zacc[1][1], zacc[1][2], zacc[1][3]};
        const int64_t blk = tg * G + 16 * (wave * NT + i) + col;   // global block index
        if constexpr (QUANT) {
          // ---- step 4: MXFP4 (Section 4, Eq. 1) ------------------------------
          float amax = amax8(zz);
          amax = fmaxf(amax, __shfl_xor(amax, 16));
          amax = fmaxf(amax, __shfl_xor(amax, 32));
          const uint32_t byte = e8m0_from_amax(amax);
          codes[blk * 4 + q] = pack8_e2m1(zz, e8m0_to_f32(byte));
          if (q == 0) scales[blk] = (uint8_t)byte;
        } else {
          float4 *o = reinterpret_cast<float4 *>(z_out + blk * 32 + 8 * q);
          o[0] = make_float4(zz[0], zz[1], zz[2], zz[3]);
          o[1] = make_float4(zz[4], zz[5], zz[6], zz[7]);
        }
      }
    }

    if (have_next) store_batch(buf ^ 1);
    __syncthreads();
  }
}

template <int KS, int NT>
static hipError_t launch_cfg(const torq_rotation *r, const void *x, int64_t TG, uint8_t *codes,
                             uint8_t *scales, float *z_out, hipStream_t stream) {
  using Cfg = RotCfg<KS>;
  const int nw = r->G / 16 / NT;
  const int64_t nbatch = (TG + Cfg::TB - 1) / Cfg::TB;
  const size_t lds_bytes = 2 * (size_t)Cfg::STAGE_BYTES;
  int64_t grid = 2 * 256;                 // two resident workgroups per CU at most
  if (grid > nbatch) grid = nbatch;
  const uint4 *ih = reinterpret_cast<const uint4 *>(r->intra_hi);
  const uint4 *il = reinterpret_cast<const uint4 *>(r->intra_lo);
  if (z_out)
    hipLaunchKernelGGL((rotate_kernel<KS, NT, false>), dim3((unsigned)grid), dim3(64 * nw), lds_bytes, stream,
                       reinterpret_cast<const uint4 *>(x), TG, r->G, r->inter_hi, r->inter_lo, ih, il,
                       nullptr, nullptr, z_out);
  else
    hipLaunchKernelGGL((rotate_kernel<KS, NT, true>), dim3((unsigned)grid), dim3(64 * nw), lds_bytes, stream,
                       reinterpret_cast<const uint4 *>(x), TG, r->G, r->inter_hi, r->inter_lo, ih, il,
                       reinterpret_cast<uint32_t *>(codes), scales, nullptr);
  return hipGetLastError();
}

hipError_t launch_rotate(const torq_rotation *r, const void *x_bf16, int64_t M, uint8_t *codes,
                         uint8_t *scales, float *z_out, hipStream_t stream) {
  const int64_t TG = M * (int64_t)(r->d / 32 / r->G);
  if (TG == 0) return hipSuccess;
  const int tiles = r->G / 16;
  // two tiles of 16 blocks per wave when that keeps the workgroup at >= 4 waves
  const bool nt2 = (tiles % 2 == 0) && (tiles / 2 >= 4);
  switch (r->KS) {
#define TORQ_CASE(KS_)                                                                          \
  case KS_:                                                                                     \
    return nt2 ? launch_cfg<KS_, 2>(r, x_bf16, TG, codes, scales, z_out, stream)                \
               : launch_cfg<KS_, 1>(r, x_bf16, TG, codes, scales, z_out, stream);
    TORQ_CASE(1) TORQ_CASE(2) TORQ_CASE(3) TORQ_CASE(4)
    TORQ_CASE(5) TORQ_CASE(6) TORQ_CASE(7) TORQ_CASE(8)
#undef TORQ_CASE
  }
  return hipErrorInvalidValue;
}

}  // namespace torq
