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

// FMT: FMT_NONE writes the rotated fp32 values, else the 4-bit format of step 4 (torq_device.h)
template <int KS, int NT, int FMT>
__global__ void __launch_bounds__(64 * ((2 * KS) / NT > 16 ? 16 : (2 * KS) / NT))
rotate_kernel(const uint4 *__restrict__ x, int64_t TG, int G,
              const uint16_t *__restrict__ inter_hi, const uint16_t *__restrict__ inter_lo,
              const uint4 *__restrict__ intra_hi_frag, const uint4 *__restrict__ intra_lo_frag,
              uint32_t *__restrict__ codes, uint8_t *__restrict__ scales, float *__restrict__ z_out,
              float global_scale) {
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
        if constexpr (FMT == FMT_NVFP4) {
          // ---- step 4 for 16-element blocks: lanes q and q ^ 1 share one, E4M3 scale byte each
          float amax = amax8(zz);
          amax = fmaxf(amax, __shfl_xor(amax, 16));
          const uint32_t sc = e4m3_from_f32(__fdiv_rn(amax, 6.0f * global_scale));
          codes[blk * 4 + q] = pack8_nvfp4(zz, e4m3_to_f32(sc) * global_scale);
          if ((q & 1) == 0) scales[blk * 2 + (q >> 1)] = (uint8_t)sc;
        } else if constexpr (FMT != FMT_NONE) {
          // ---- step 4: MXFP4 (Section 4, Eq. 1), or MXINT4 on the same scale -----
          float amax = amax8(zz);
          amax = fmaxf(amax, __shfl_xor(amax, 16));
          amax = fmaxf(amax, __shfl_xor(amax, 32));
          const uint32_t byte = e8m0_from_amax(amax);
          codes[blk * 4 + q] = (FMT == FMT_MXINT4) ? pack8_int4(zz, e8m0_inverse_f32(byte)) : pack8_e2m1(zz, e8m0_to_f32(byte));
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

// ---------------------------------------------------------------------------
// Variant for G a multiple of 32, on v_mfma_f32_32x32x16_bf16 (which sustains a higher rate than
// the 16x16x32 form).  Same formulation; wave w owns the 32 output blocks b = 32 w .. 32 w + 31
// and there are G/32 waves.  Two token-groups are processed together so that every MFMA has an
// independent neighbour.  After step 3 a lane holds sixteen consecutive k of one block: two
// lanes per block, one cross-lane step for the amax, 8 bytes of codes per lane.
//
// Layouts (lane l: n = l%32, h = l/32):
//   step 2  A = X^T      lane (k = l%32, h), slot j:  X[b' = 16 s + 8 h + j][k]        (LDS, transposing read)
//           B = R_inter^T lane (b = l%32, h), slot j:  R_inter[b][16 s + 8 h + j]
//           D             lane (b, h), reg r:          Y^T[k' = 8 (r/4) + 4 h + r%4][b]
//   step 3  B = Y^T       k-step t uses regs 8t..8t+7: slot jj <-> k' = 16 t + 8 (jj/4) + 4 h + jj%4
//           A = R_intra^T lane (m, h), slot jj:        R_intra[that k'][kout(m)],
//                         kout(m) = 16 ((m/4)%2) + 4 (m/8) + m%4
//           D             lane (b, h), reg r:          Z[b][16 h + r]
// Input staging.  G <= 64: global -> registers -> LDS, the next batch's loads in flight during the
// current batch.  G >= 96: global -> LDS directly (buffer_load ... lds), issued once the wave has
// read its step-2 operands of the current batch and landing during steps 3 and 4; without the
// staging registers three waves fit a SIMD up to G = 128 (160 registers), which is worth 5 - 15 %
// there and a few per cent beyond; at G <= 64 the register path measured faster.
// TB: token-groups per batch, processed together (2: every MFMA has an independent neighbour; 1 for a
// handful of token-groups, where the shortest path through one token-group counts).
template <int KS16, int TB, int FMT>
__global__ void __launch_bounds__(64 * (KS16 / 2), (KS16 >= 6 && KS16 <= 8) ? 3 : 2)   // waves per SIMD
rotate_kernel32(const uint4 *__restrict__ x, int64_t TG, int G,
                const uint16_t *__restrict__ inter_hi, const uint16_t *__restrict__ inter_lo,
                const uint4 *__restrict__ intra_hi_frag, const uint4 *__restrict__ intra_lo_frag,
                uint2 *__restrict__ codes, uint8_t *__restrict__ scales, float *__restrict__ z_out,
                float global_scale) {
  constexpr int TG_BYTES = KS16 * 16 * 64;           // one token-group: G rows of 64 bytes
  constexpr int STAGE_BYTES = TB * TG_BYTES;
  constexpr int NTHR = 64 * (KS16 / 2);
  constexpr int CH = TG_BYTES / 16 / NTHR;           // 16-byte chunks per thread per token-group (= 2)
  constexpr bool DMA = KS16 >= 6;
  extern __shared__ __attribute__((aligned(16))) char lds[];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, h = lane >> 5;

  // ---- resident operands
  bf16x8 Bh[KS16], Bl[KS16];
  {
    const int b = 32 * wave + col;
#pragma unroll
    for (int ks = 0; ks < KS16; ++ks) {
      const size_t off = (size_t)b * (KS16 * 16) + 16 * ks + 8 * h;
      Bh[ks] = *reinterpret_cast<const bf16x8 *>(inter_hi + off);
      Bl[ks] = *reinterpret_cast<const bf16x8 *>(inter_lo + off);
    }
  }
  bf16x8 Ah[2], Al[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    Ah[t] = __builtin_bit_cast(bf16x8, intra_hi_frag[t * 64 + lane]);
    Al[t] = __builtin_bit_cast(bf16x8, intra_lo_frag[t * 64 + lane]);
  }

  // transposing-read address of this lane inside a token-group (k-step 0, first half)
  const int blk = lane >> 4, s16 = lane & 15;
  const int tr_off = ((8 * (blk >> 1) + (s16 >> 2)) * 32 + 16 * (blk & 1) + 4 * (s16 & 3)) * 2;

  const int64_t nbatch = (TG + TB - 1) / TB;
  uint4 stage_regs[TB][CH];
  auto load_batch = [&](int64_t batch) {
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      const int64_t tg = batch * TB + j;
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        if (tg < TG) stage_regs[j][i] = x[tg * (TG_BYTES / 16) + tid + i * NTHR];
        else stage_regs[j][i] = make_uint4(0, 0, 0, 0);
      }
    }
  };
  auto store_batch = [&](int buf) {
    char *base = lds + buf * STAGE_BYTES;
#pragma unroll
    for (int j = 0; j < TB; ++j)
#pragma unroll
      for (int i = 0; i < CH; ++i)
        *reinterpret_cast<uint4 *>(base + j * TG_BYTES + (tid + i * NTHR) * 16) = stage_regs[j][i];
  };

  // the direct form: lane l of wave w fills LDS chunk 64 w + l (+ NTHR i) of a token-group, which is
  // the chunk of the same index in global memory; a token-group past the end reads as zeros through
  // an empty descriptor
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  auto dma_batch = [&](int64_t b_, int buf_) {
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      const int64_t tg = b_ * TB + j;
      const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<char *>(reinterpret_cast<const char *>(x) + (tg < TG ? tg : 0) * (int64_t)TG_BYTES), 0,
          tg < TG ? TG_BYTES : 0, 0x00020000);
#pragma unroll
      for (int i = 0; i < CH; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rs, (__attribute__((address_space(3))) void *)(lds + buf_ * STAGE_BYTES + j * TG_BYTES + (wave_u * 64 + i * NTHR) * 16),
            16, tid * 16, i * NTHR * 16, 0, 0);
    }
  };

  int64_t batch = blockIdx.x;
  if (batch < nbatch) {
    if constexpr (DMA) {
      dma_batch(batch, 0);
    } else {
      load_batch(batch);
      store_batch(0);
    }
  }
  if constexpr (!DMA) __syncthreads();

  int buf = 0;
  for (; batch < nbatch; batch += gridDim.x, buf ^= 1) {
    const int64_t next = batch + gridDim.x;
    const bool have_next = next < nbatch;
    if constexpr (DMA) {
      // this wave's part of the batch has landed (vmcnt(0)), then everybody's; the barrier also says
      // that every wave is done reading the other buffer
      __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();
    } else {
      if (have_next) load_batch(next);
    }

    const char *stage = lds + buf * STAGE_BYTES + tr_off;
    // ---- step 2: Y^T = X^T R_inter^T for both token-groups
    f32x16 acc[TB];
#pragma unroll
    for (int j = 0; j < TB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS16; ++ks) {
      bf16x8 xa[TB];
#pragma unroll
      for (int j = 0; j < TB; ++j) {
        const char *p = stage + j * TG_BYTES + ks * 16 * 64;
        union { bf16x8 v; i16x4 q[2]; } u;
        u.q[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4 *)(p));
        u.q[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4 *)(p + 4 * 64));
        xa[j] = u.v;
      }
#pragma unroll
      for (int j = 0; j < TB; ++j)
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[j], Bh[ks], acc[j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < TB; ++j)
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[j], Bl[ks], acc[j], 0, 0, 0);
    }

    if constexpr (DMA) {
      // this wave's LDS reads of the batch are done (the MFMAs consumed them); no LDS read follows
      // in this iteration, so the compiler's rule "LDS reads wait for loads into LDS" costs nothing
      __builtin_amdgcn_sched_barrier(0);
      if (have_next) dma_batch(next, buf ^ 1);
      __builtin_amdgcn_sched_barrier(0);
    }

    // ---- step 3: Z^T = R_intra^T Y^T with Y split into bf16 hi + lo; then step 4
    f32x16 zacc[TB];
    bf16x8 yh[TB][2], yl[TB][2];
#pragma unroll
    for (int j = 0; j < TB; ++j) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const float y0 = acc[j][8 * t + 2 * p], y1 = acc[j][8 * t + 2 * p + 1];
          hi[p] = pack_bf16_rne(y0, y1);
          lo[p] = pack_bf16_rne(y0 - __uint_as_float(hi[p] << 16), y1 - __uint_as_float(hi[p] & 0xFFFF0000u));
        }
        yh[j][t] = __builtin_bit_cast(bf16x8, i32x4{(int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]});
        yl[j][t] = __builtin_bit_cast(bf16x8, i32x4{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3]});
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) zacc[j][r] = 0.f;
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int j = 0; j < TB; ++j) zacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Al[t], yh[j][t], zacc[j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < TB; ++j) zacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ah[t], yl[j][t], zacc[j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < TB; ++j) zacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ah[t], yh[j][t], zacc[j], 0, 0, 0);
    }

#pragma unroll
    for (int j = 0; j < TB; ++j) {
      const int64_t tg = batch * TB + j;
      if (tg < TG) {                                            // uniform over the workgroup
        const int64_t blkidx = tg * G + 32 * wave + col;        // global block index
        float zz[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) zz[r] = zacc[j][r];
        if constexpr (FMT == FMT_NVFP4) {
          // the lane's sixteen values are one 16-element block: no cross-lane step
          const float amax = fmaxf(amax8(zz), amax8(zz + 8));
          const uint32_t sc = e4m3_from_f32(__fdiv_rn(amax, 6.0f * global_scale));
          const float S = e4m3_to_f32(sc) * global_scale;
          codes[blkidx * 2 + h] = make_uint2(pack8_nvfp4(zz, S), pack8_nvfp4(zz + 8, S));
          scales[blkidx * 2 + h] = (uint8_t)sc;
        } else if constexpr (FMT != FMT_NONE) {
          float amax = fmaxf(amax8(zz), amax8(zz + 8));
          // max with the other half-wave (lane ^ 32): swap the upper half of one copy with the
          // lower half of the other, then every lane holds both partners' values
          const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(amax), __float_as_uint(amax), false, false);
          amax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
          const uint32_t byte = e8m0_from_amax(amax);
          if constexpr (FMT == FMT_MXINT4) {
            const float inv = e8m0_inverse_f32(byte);
            codes[blkidx * 2 + h] = make_uint2(pack8_int4(zz, inv), pack8_int4(zz + 8, inv));
          } else {
            const float sc = e8m0_to_f32(byte);
            codes[blkidx * 2 + h] = make_uint2(pack8_e2m1(zz, sc), pack8_e2m1(zz + 8, sc));
          }
          if (h == 0) scales[blkidx] = (uint8_t)byte;
        } else {
          float4 *o = reinterpret_cast<float4 *>(z_out + blkidx * 32 + 16 * h);
#pragma unroll
          for (int q = 0; q < 4; ++q) o[q] = make_float4(zz[4 * q], zz[4 * q + 1], zz[4 * q + 2], zz[4 * q + 3]);
        }
      }
    }

    if constexpr (!DMA) {
      if (have_next) store_batch(buf ^ 1);
      __syncthreads();
    }
  }
}

// launch KERNEL_<..., FMT> for the runtime format (FMT_NONE when the fp32 output is asked for)
#define TORQ_LAUNCH_FMT(KERNEL_, CODES_T_, ...)                                                                  \
  switch (z_out ? FMT_NONE : format) {                                                                          \
    case FMT_NONE:                                                                                              \
      hipLaunchKernelGGL((KERNEL_<__VA_ARGS__, FMT_NONE>), dim3((unsigned)grid), dim3(64 * nw), lds_bytes, stream, \
                         reinterpret_cast<const uint4 *>(x), TG, r->G, r->inter_hi, r->inter_lo, ih, il,        \
                         (CODES_T_ *)nullptr, (uint8_t *)nullptr, z_out, 1.0f);                                 \
      break;                                                                                                    \
    case FMT_MXFP4:                                                                                             \
      hipLaunchKernelGGL((KERNEL_<__VA_ARGS__, FMT_MXFP4>), dim3((unsigned)grid), dim3(64 * nw), lds_bytes, stream, \
                         reinterpret_cast<const uint4 *>(x), TG, r->G, r->inter_hi, r->inter_lo, ih, il,        \
                         reinterpret_cast<CODES_T_ *>(codes), scales, (float *)nullptr, 1.0f);                  \
      break;                                                                                                    \
    case FMT_MXINT4:                                                                                            \
      hipLaunchKernelGGL((KERNEL_<__VA_ARGS__, FMT_MXINT4>), dim3((unsigned)grid), dim3(64 * nw), lds_bytes, stream, \
                         reinterpret_cast<const uint4 *>(x), TG, r->G, r->inter_hi, r->inter_lo, ih, il,        \
                         reinterpret_cast<CODES_T_ *>(codes), scales, (float *)nullptr, 1.0f);                  \
      break;                                                                                                    \
    case FMT_NVFP4:                                                                                             \
      hipLaunchKernelGGL((KERNEL_<__VA_ARGS__, FMT_NVFP4>), dim3((unsigned)grid), dim3(64 * nw), lds_bytes, stream, \
                         reinterpret_cast<const uint4 *>(x), TG, r->G, r->inter_hi, r->inter_lo, ih, il,        \
                         reinterpret_cast<CODES_T_ *>(codes), scales, (float *)nullptr, global_scale);          \
      break;                                                                                                    \
    default: return hipErrorInvalidValue;                                                                       \
  }                                                                                                             \
  return hipGetLastError();

template <int KS16, int TB = 2>
static hipError_t launch_cfg32(const torq_rotation *r, const void *x, int64_t TG, int format, float global_scale,
                               uint8_t *codes, uint8_t *scales, float *z_out, hipStream_t stream) {
  const int nw = KS16 / 2;                               // = G / 32
  const int64_t nbatch = (TG + TB - 1) / TB;
  const size_t lds_bytes = 2 * (size_t)TB * KS16 * 16 * 64;
  // resident workgroups per CU: limited by LDS (160 KiB) and by the waves per SIMD that the register
  // count admits (three for G = 96 and 128, two otherwise)
  const int waves_per_cu = (KS16 >= 6 && KS16 <= 8) ? 12 : 8;
  int per_cu = (int)((160 * 1024) / lds_bytes);
  if (per_cu * nw > waves_per_cu) per_cu = waves_per_cu / nw;
  if (per_cu < 1) per_cu = 1;
  int64_t grid = (int64_t)per_cu * 256;
  if (grid > nbatch) grid = nbatch;
  const uint4 *ih = reinterpret_cast<const uint4 *>(r->intra32_hi);
  const uint4 *il = reinterpret_cast<const uint4 *>(r->intra32_lo);
  TORQ_LAUNCH_FMT(rotate_kernel32, uint2, KS16, TB)
}

template <int KS, int NT>
static hipError_t launch_cfg(const torq_rotation *r, const void *x, int64_t TG, int format, float global_scale,
                             uint8_t *codes, uint8_t *scales, float *z_out, hipStream_t stream) {
  using Cfg = RotCfg<KS>;
  const int nw = r->G / 16 / NT;
  const int64_t nbatch = (TG + Cfg::TB - 1) / Cfg::TB;
  const size_t lds_bytes = 2 * (size_t)Cfg::STAGE_BYTES;
  // Resident workgroups per CU (measured on X [16384, d]): two for 4 to 8 waves per workgroup, one
  // beyond (two would not fit 16 waves per CU at these register counts); a small G has few waves
  // per workgroup and needs as many workgroups as LDS and 16 waves allow to keep the CU busy
  // (G = 16: 1.4 -> 2.7 TB/s, G = 48: 3.2 -> 3.8 TB/s against two workgroups).
  int per_cu = nw >= 9 ? 1 : 2;
  if (nw <= 3) {
    per_cu = (int)((160 * 1024) / lds_bytes);
    if (per_cu * nw > 16) per_cu = 16 / nw;
  }
  int64_t grid = (int64_t)per_cu * 256;
  if (grid > nbatch) grid = nbatch;
  const uint4 *ih = reinterpret_cast<const uint4 *>(r->intra_hi);
  const uint4 *il = reinterpret_cast<const uint4 *>(r->intra_lo);
  TORQ_LAUNCH_FMT(rotate_kernel, uint32_t, KS, NT)
}
#undef TORQ_LAUNCH_FMT

// Exactly one of (codes, scales) / z_out is used; `format` (FMT_*) picks step 4's block format.
hipError_t launch_rotate(const torq_rotation *r, const void *x_bf16, int64_t M, int format, float global_scale,
                         uint8_t *codes, uint8_t *scales, float *z_out, hipStream_t stream) {
  const int64_t TG = M * (int64_t)(r->d / 32 / r->G);
  if (TG == 0) return hipSuccess;
  // a handful of token-groups at G = 128 (decode): one per workgroup
  if (r->G == 128 && TG <= 128) return launch_cfg32<8, 1>(r, x_bf16, TG, format, global_scale, codes, scales, z_out, stream);
  if (r->G % 32 == 0) {
    switch (r->G / 16) {
#define TORQ_CASE32(K16_) \
  case K16_: return launch_cfg32<K16_>(r, x_bf16, TG, format, global_scale, codes, scales, z_out, stream);
      TORQ_CASE32(2) TORQ_CASE32(4) TORQ_CASE32(6) TORQ_CASE32(8)
      TORQ_CASE32(10) TORQ_CASE32(12) TORQ_CASE32(14) TORQ_CASE32(16)
#undef TORQ_CASE32
    }
  }
  // G = 16 * odd: the 16x16x32 kernel, one tile of 16 blocks per wave
  switch (r->KS) {
#define TORQ_CASE(KS_) \
  case KS_: return launch_cfg<KS_, 1>(r, x_bf16, TG, format, global_scale, codes, scales, z_out, stream);
    TORQ_CASE(1) TORQ_CASE(2) TORQ_CASE(3) TORQ_CASE(4)
    TORQ_CASE(5) TORQ_CASE(6) TORQ_CASE(7) TORQ_CASE(8)
#undef TORQ_CASE
  }
  return hipErrorInvalidValue;
}

}  // namespace torq
