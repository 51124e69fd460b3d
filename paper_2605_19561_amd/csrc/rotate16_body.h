// Steps 1-4 of Algorithm 3 on v_mfma_f32_16x16x32_bf16 for one workgroup of 4 G / NT lanes: the body
// of rotate_kernel (rotate_quant.hip, G = 16 and 48), as a device function.  The workgroup takes the
// batches first_batch, first_batch + batch_stride, ... of TB token-groups; `lds` is
// 2 * TB * RotCfg<KS>::TG_LDS_BYTES bytes of dynamic LDS, 16-byte aligned; every lane of the workgroup
// must call it (barriers inside).
// TB: token-groups per batch (RotCfg<KS>::TB for throughput, 1 for the shortest path through one
// token-group).
// The two helpers at the top (the LDS pointer type of the transposing read, pack_bf16_rne) also serve
// rotate32_resident.h.
#pragma once
#include "torq_device.h"

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

// FMT: FMT_NONE writes the rotated fp32 values, else the 4-bit format of step 4 (torq_device.h)
template <int KS, int NT, int FMT, int TB = RotCfg<KS>::TB>
__device__ __forceinline__ void rotate16_body(const uint4 *__restrict__ x, int64_t TG, int G,
                                              const uint16_t *__restrict__ inter_hi, const uint16_t *__restrict__ inter_lo,
                                              const uint4 *__restrict__ intra_hi_frag, const uint4 *__restrict__ intra_lo_frag,
                                              uint32_t *__restrict__ codes, uint8_t *__restrict__ scales,
                                              float *__restrict__ z_out, float global_scale, char *lds,
                                              int64_t first_batch, int64_t batch_stride) {
  using Cfg = RotCfg<KS>;
  constexpr int STAGE_BYTES = TB * Cfg::TG_LDS_BYTES;

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
  for (int i = tid; i < 2 * STAGE_BYTES / 16; i += nthr)
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
    char *base = lds + buf * STAGE_BYTES;
#pragma unroll
    for (int j = 0; j < TB; ++j)
#pragma unroll
      for (int i = 0; i < NT; ++i)
        *reinterpret_cast<uint4 *>(base + j * Cfg::TG_LDS_BYTES + (tid + i * nthr) * 16) = stage_regs[j][i];
  };

  int64_t batch = first_batch;
  if (batch < nbatch) {
    load_batch(batch);
    store_batch(0);
  }
  __syncthreads();

  int buf = 0;
  for (; batch < nbatch; batch += batch_stride, buf ^= 1) {
    const int64_t next = batch + batch_stride;
    const bool have_next = next < nbatch;
    if (have_next) load_batch(next);

    const char *stage = lds + buf * STAGE_BYTES;
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
        if constexpr (FMT == FMT_NVFP4) {
          // ---- step 4 for 16-element blocks: lanes q and q ^ 1 share one, E4M3 scale byte each
          float amax = amax8(zz);
          amax = fmaxf(amax, __shfl_xor(amax, 16));
          const uint32_t sc = nvfp4_scale_code(amax, 6.0f * global_scale);
          codes[blk * 4 + q] = pack8_nvfp4(zz, e4m3_to_f32(sc) * global_scale);
          if ((q & 1) == 0) scales[blk * 2 + (q >> 1)] = (uint8_t)sc;
        } else if constexpr (FMT != FMT_NONE) {
          // ---- step 4: MXFP4 (Section 4, Eq. 1), or MXINT4 on the same scale -----
          float amax = amax8(zz);
          amax = fmaxf(amax, __shfl_xor(amax, 16));
          amax = fmaxf(amax, __shfl_xor(amax, 32));
          const uint32_t byte = e8m0_from_amax(amax);
          const uint32_t packed = (FMT == FMT_MXINT4) ? pack8_int4(zz, e8m0_inverse_f32(byte)) : pack8_e2m1(zz, e8m0_to_f32(byte));
          codes[blk * 4 + q] = packed;
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

}  // namespace torq
