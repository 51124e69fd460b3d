// Steps 1-4 of Algorithm 3 for at most four token-groups of G = 112 or 128 blocks inside a workgroup of
// exactly 512 lanes, MXFP4 results handed to a functor instead of stored: the rotation of
// torq_linear_local_kernel (mxfp4_gemm_skinny.hip), which keeps the packed activations in LDS.
//
// The arithmetic is that of rotate_kernel32<G / 16, 1, FMT_MXFP4> (rotate_quant.hip), operation for
// operation -- the same MFMAs on the same operands in the same order, the same split of Y, the same
// step 4 -- so that the codes and scale bytes are the ones torq_rotate_quantize produces for the same
// rows, bit for bit (the parity tests compare them).  Layouts as documented there; R_inter comes from the
// handle's table in lane order ([tile][k-step][lane][8], zero past G).  G = 112 runs the eight k-steps of
// G = 128: the last one multiplies the table's zero padding (columns 112 .. 127) with zero rows in LDS
// and adds exact zeros to sums that started at +0.
//
// Wave w takes the 32 block rows 32 (w % 4) .. and the token-groups w / 4 and w / 4 + 2.  Every read
// from memory is issued first; then after_loads() runs (a place for loads that may return later:
// vector-memory reads return in order, so what the rotation waits for is requested before them); then
// the token-groups go to LDS, one barrier, steps 2-4, results to sink, one barrier.
//   sink(block index, h, the lane's sixteen codes of positions 16 h .. 16 h + 15, the block's scale byte)
//   lds: 4 * 8192 bytes.
#pragma once
#include "rotate16_body.h"     // lds_i16x4, pack_bf16_rne
#include "torq_device.h"

namespace torq {

template <class Sink, class Hook>
__device__ __forceinline__ void rotate32_resident(const uint4 *__restrict__ x, int TG, int G,
                                                  const uint4 *__restrict__ inter_hi_frag, const uint4 *__restrict__ inter_lo_frag,
                                                  const uint4 *__restrict__ intra32_hi_frag,
                                                  const uint4 *__restrict__ intra32_lo_frag, char *lds, const Sink sink,
                                                  Hook after_loads) {
  constexpr int KS16 = 8, NW = 4;                    // G = 112 or 128: four waves of 32 block rows
  const int TG_BYTES = G * 64;                       // one token-group: G rows of 64 bytes
  constexpr int TG_STRIDE = 8192;                    // its place in LDS: 512 chunks of 16 bytes
  typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned u32x4_t;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int tile = wave & (NW - 1), first_tg = wave >> 2;
  const int col = lane & 31, h = lane >> 5;

  // ---- resident operands (every wave uses them below outside any condition: operands that were only
  // used under one would have their loads moved there by the compiler, behind those of after_loads())
  // (R_inter from the table in lane order: one load of a wave is 1 KiB of consecutive bytes; from the
  // row-major table it would touch 32 cache lines)
  bf16x8 Bh[KS16], Bl[KS16];
#pragma unroll
  for (int ks = 0; ks < KS16; ++ks) {
    Bh[ks] = __builtin_bit_cast(bf16x8, inter_hi_frag[(tile * KS16 + ks) * 64 + lane]);
    Bl[ks] = __builtin_bit_cast(bf16x8, inter_lo_frag[(tile * KS16 + ks) * 64 + lane]);
  }
  bf16x8 Ah[2], Al[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    Ah[t] = __builtin_bit_cast(bf16x8, intra32_hi_frag[t * 64 + lane]);
    Al[t] = __builtin_bit_cast(bf16x8, intra32_lo_frag[t * 64 + lane]);
  }

  // ---- step 1: lane t brings 16-byte chunk t of each token-group (buffer loads: chunks past the end of
  // a token-group and token-groups that do not exist read as zeros without a branch, so that the compiler
  // counts the loads that after_loads() adds exactly and waits for these four only)
  const __amdgpu_buffer_rsrc_t x_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4 *>(x), 0, TG * TG_BYTES, 0x00020000);
  const unsigned x_voff = tid * 16 < TG_BYTES ? (unsigned)tid * 16u : 0x7FFFFFF0u;   // (the range check covers this offset only)
  u32x4_t st[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) st[j] = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, (int)(x_voff + (unsigned)(j * TG_BYTES)), 0, 0);
  after_loads();
  // (all four places are written, zeros where there is no token-group: a store under a condition would
  // take its load with it, behind those of after_loads())
#pragma unroll
  for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4_t *>(lds + j * TG_STRIDE + tid * 16) = st[j];
  __syncthreads();

  // transposing-read address of this lane inside a token-group (k-step 0, first half)
  const int blk = lane >> 4, s16 = lane & 15;
  const int tr_off = ((8 * (blk >> 1) + (s16 >> 2)) * 32 + 16 * (blk & 1) + 4 * (s16 & 3)) * 2;

  auto token_group = [&](int tg) {
    const char *stage = lds + tg * TG_STRIDE + tr_off;
    // ---- step 2: Y^T = X^T R_inter^T
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS16; ++ks) {
      const char *p = stage + ks * 16 * 64;
      union { bf16x8 v; i16x4 q[2]; } u;
      u.q[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4 *)(p));
      u.q[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4 *)(p + 4 * 64));
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u.v, Bh[ks], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u.v, Bl[ks], acc, 0, 0, 0);
    }
    // ---- step 3: Z^T = R_intra^T Y^T with Y split into bf16 hi + lo
    bf16x8 yh[2], yl[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      uint32_t hi[4], lo[4];
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const float y0 = acc[8 * t + 2 * p], y1 = acc[8 * t + 2 * p + 1];
        hi[p] = pack_bf16_rne(y0, y1);
        lo[p] = pack_bf16_rne(y0 - __uint_as_float(hi[p] << 16), y1 - __uint_as_float(hi[p] & 0xFFFF0000u));
      }
      yh[t] = __builtin_bit_cast(bf16x8, i32x4{(int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]});
      yl[t] = __builtin_bit_cast(bf16x8, i32x4{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3]});
    }
    f32x16 zacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) zacc[r] = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      zacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Al[t], yh[t], zacc, 0, 0, 0);
      zacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ah[t], yl[t], zacc, 0, 0, 0);
      zacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ah[t], yh[t], zacc, 0, 0, 0);
    }
    // ---- step 4 (Section 4, Eq. 1): lane (b, h) holds Z[b][16 h .. 16 h + 15]
    float zz[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) zz[r] = zacc[r];
    float amax = fmaxf(amax8(zz), amax8(zz + 8));
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(amax), __float_as_uint(amax), false, false);
    amax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    const uint32_t byte = e8m0_from_amax(amax);
    const float sc = e8m0_to_f32(byte);
    const bool live = 32 * tile + col < G && tg < TG;   // a block row, and a token-group, that exists
    if (live) sink((int64_t)tg * G + 32 * tile + col, h, make_uint2(pack8_e2m1(zz, sc), pack8_e2m1(zz + 8, sc)), byte);
  };
  token_group(first_tg);                       // outside any condition (see above); dropped if there is none
  if (first_tg + 2 < TG) token_group(first_tg + 2);
  __syncthreads();
}

}  // namespace torq
