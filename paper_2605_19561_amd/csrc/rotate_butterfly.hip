// Rotate + quantise for an inter-block rotation that is a BUTTERFLY of plane rotations
// (torq_equalize_inter_butterfly: log2 G rounds, round t turning the G/2 independent pairs of block
// rows (p, p + G / 2^(t+1))), i.e. Algorithm 3's Y = R_inter X without the dense G x G contraction:
// one fused multiply-add per element and round (log2 G + 1 in all) instead of 2 G per element, twice,
// on the matrix cores (Section 5.1 asks for an efficient implementation of R_inter; Appendix A.7
// counts O(B^2 K) for the dense form).  Up to G = 64 the kernel then moves data as fast as a copy.
//
// The two rotations commute (R_inter mixes blocks, R_intra mixes positions), so the kernel applies
// R_intra FIRST: X is exact in bf16, which makes the intra rotation two MFMA passes (R_intra split
// into bf16 hi + lo) and leaves the result in fp32 registers in the layout the butterfly wants.
//
// One wave = one token-group (G blocks of 32) at a time; workgroups are persistent.
//   * global -> LDS directly (buffer_load ... lds, 16 bytes per lane; the LDS side is lane-linear, so
//     the lane picks the global chunk that belongs at its LDS place: 16-byte chunks of a 64-byte row
//     XOR-swizzled with (row >> 1) & 3).  The wave's LDS region is free as soon as the MFMA operands
//     of the current token-group have been read, so the next token-group's loads are issued right
//     there and land while the butterfly and step 4 run: no staging registers, no second buffer;
//   * Z'^T = R_intra^T X^T per tile of 32 blocks on v_mfma_f32_32x32x16_bf16: B operand = two 8-byte
//     LDS reads of row b per k-step; afterwards lane (n = l % 32, h = l / 32) holds
//     v[j][r] = Z'[32 j + b0][16 h + r], j < G / 32, r < 16 (which block row b0 a lane holds: below);
//   * butterfly over the block index b = 32 j + b0 with the cosines deferred: a row carries
//     u = (true value) / sigma, sigma = the product of the cosines of the pairs it has been in, and
//         p' = c (p + t q)  becomes  u_p' = u_p + (t sigma_q / sigma_p) u_q,
//         q' = c (q - t p)  becomes  u_q' = u_q - (t sigma_p / sigma_q) u_p      (t = tan theta),
//     one FMA per value and round with a per-row coefficient from a host-built table; the final
//     sigma multiplies once at the end.  Rounds with stride >= 32 pair registers of the same lane,
//     rounds with stride 16 .. 1 pair lanes.  Block row b0 of a tile sits in lane
//         n = 16 b0[4] ^ 15 b0[3] ^ 7 b0[2] ^ 2 b0[1] ^ b0[0]
//     so that the partners of strides 8, 4, 2, 1 are the lanes n ^ 15, n ^ 7, n ^ 2, n ^ 1: DPP
//     row_mirror, row_half_mirror and two quad permutes, each fused into its multiply-add
//     (v_fmac_f32_dpp, one instruction per value and round); stride 16 is a ds_swizzle;
//   * step 4 as in rotate_kernel32: a lane holds sixteen consecutive positions of one block.
#include "torq_device.h"
#include "torq_internal.h"

namespace torq {

namespace {

template <int PATTERN>
__device__ __forceinline__ float swizzle_f32(float v) {
  return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), PATTERN));
}

// v[r] += t * (v[r] of the lane that the DPP control CTRL_ names), r < 16, in place.  The compiler does
// not fold a DPP move into a fused multiply-add on this target, hence the assembly.  The leading wait
// covers the DPP read-after-VALU-write and EXEC-write hazards that are not tracked across the
// boundary of an asm statement; inside it no instruction reads a register the one before wrote.
#define TORQ_FMAC16_DPP(V_, T_, CTRL_)                                                              \
  asm volatile("s_nop 4\n"                                                                          \
      "v_fmac_f32_dpp %0, %0, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                           \
      "v_fmac_f32_dpp %1, %1, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                           \
      "v_fmac_f32_dpp %2, %2, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                           \
      "v_fmac_f32_dpp %3, %3, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                           \
      "v_fmac_f32_dpp %4, %4, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                           \
      "v_fmac_f32_dpp %5, %5, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                           \
      "v_fmac_f32_dpp %6, %6, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                           \
      "v_fmac_f32_dpp %7, %7, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                           \
      "v_fmac_f32_dpp %8, %8, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                           \
      "v_fmac_f32_dpp %9, %9, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                           \
      "v_fmac_f32_dpp %10, %10, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                         \
      "v_fmac_f32_dpp %11, %11, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                         \
      "v_fmac_f32_dpp %12, %12, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                         \
      "v_fmac_f32_dpp %13, %13, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                         \
      "v_fmac_f32_dpp %14, %14, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                         \
      "v_fmac_f32_dpp %15, %15, %16 " CTRL_ " row_mask:0xf bank_mask:0xf\n"                         \
      : "+v"(V_[0]), "+v"(V_[1]), "+v"(V_[2]), "+v"(V_[3]), "+v"(V_[4]), "+v"(V_[5]), "+v"(V_[6]),  \
        "+v"(V_[7]), "+v"(V_[8]), "+v"(V_[9]), "+v"(V_[10]), "+v"(V_[11]), "+v"(V_[12]),            \
        "+v"(V_[13]), "+v"(V_[14]), "+v"(V_[15])                                                    \
      : "v"(T_))

}  // namespace

// coefficient table, [NC][32] floats, the lane that holds block row b0 reads column b0 (row 32 j + b0
// of the butterfly):
//   round t = 0 .. log2 G - 1, entry t NJ + j:  the row's coefficient of that round (signed: + on the
//                                               row with the stride bit clear, - on its partner)
//   entry (log2 G) NJ + j:                      the row's final sigma
// G <= 64 keeps the lane's coefficients in registers; G >= 128 (32 and 72 of them, next to 64 / 128
// accumulators) reads them from a copy of the table in LDS where they are used.  Workgroups per CU
// that the register counts admit: 8, 5, 4, 2 for G = 32, 64, 128, 256.
template <int NJ, int FMT>
__global__ void __launch_bounds__(256, NJ == 1 ? 8 : NJ == 2 ? 5 : NJ == 4 ? 4 : 2)
rotate_butterfly_kernel(const uint4 *__restrict__ x, int64_t TG, const float *__restrict__ coef,
                        const uint4 *__restrict__ intra_hi_frag, const uint4 *__restrict__ intra_lo_frag,
                        uint2 *__restrict__ codes, uint8_t *__restrict__ scales, float *__restrict__ z_out,
                        float global_scale) {
  constexpr int G = 32 * NJ;
  constexpr int LJ = NJ == 1 ? 0 : NJ == 2 ? 1 : NJ == 4 ? 2 : 3;     // rounds inside a lane
  constexpr int NC = (LJ + 6) * NJ;
  constexpr int TG_BYTES = G * 64;
  constexpr int CH = TG_BYTES / 16 / 64;                               // 16-byte chunks per lane (= 2 NJ)
  extern __shared__ __attribute__((aligned(16))) char lds[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int h = lane >> 5;
  // the block row of the tile that this lane holds (the inverse of the lane map above)
  const int b0 = ((lane & 24) | ((lane ^ (lane >> 1)) & 4) | ((lane ^ (lane >> 1)) & 2) | ((lane ^ (lane >> 2)) & 1)) & 31;
  char *const my = lds + wave * TG_BYTES;                              // this wave's token-group

  constexpr bool CF_LDS = NJ >= 4;
  float cf_reg[CF_LDS ? 1 : NC];
  const float *const cf_lds = reinterpret_cast<const float *>(lds + 4 * TG_BYTES) + b0;
  if constexpr (CF_LDS) {
    float *t = reinterpret_cast<float *>(lds + 4 * TG_BYTES);
    for (int i = threadIdx.x; i < NC * 32; i += 256) t[i] = coef[i];
    __syncthreads();                                         // before the loop: every wave arrives
  } else {
#pragma unroll
    for (int c = 0; c < NC; ++c) cf_reg[c] = coef[c * 32 + b0];
  }
#define cf(I_) (CF_LDS ? cf_lds[(I_) * 32] : cf_reg[CF_LDS ? 0 : (I_)])
  bf16x8 Ah[2], Al[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    Ah[t] = __builtin_bit_cast(bf16x8, intra_hi_frag[t * 64 + lane]);
    Al[t] = __builtin_bit_cast(bf16x8, intra_lo_frag[t * 64 + lane]);
  }

  // LDS place P = 64 i + lane (16-byte units) holds row P / 4, part (P % 4) ^ ((row >> 1) & 3) of the
  // token-group; (row >> 1) & 3 = (lane >> 3) & 3 for every i
  const int ld_voff = ((lane & ~3) | ((lane & 3) ^ ((lane >> 3) & 3))) * 16;
  // B operand of k-step t, tile j: the 8-byte pieces at positions 16 t + 4 h and 16 t + 8 + 4 h of
  // row 32 j + b0, i.e. 16-byte part 2 t (+ 1), half h; (row >> 1) & 3 does not depend on j
  int rd_off[2][2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int u = 0; u < 2; ++u) rd_off[t][u] = b0 * 64 + (((2 * t + u) ^ ((b0 >> 1) & 3)) * 16) + 8 * h;

  const int64_t wave_id = (int64_t)blockIdx.x * 4 + wave, nwave = (int64_t)gridDim.x * 4;
  // loads of token-group TG_: CH instructions of 1 KB each; the range of the descriptor is the
  // token-group itself
#define TORQ_LOAD_TG(TG_)                                                                           \
  {                                                                                                 \
    const __amdgpu_buffer_rsrc_t rs_ = __builtin_amdgcn_make_buffer_rsrc(                           \
        const_cast<char *>(reinterpret_cast<const char *>(x) + (TG_) * (int64_t)TG_BYTES), 0, TG_BYTES, 0x00020000); \
    _Pragma("unroll") for (int i = 0; i < CH; ++i)                                                  \
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_, (__attribute__((address_space(3))) void *)(my + i * 1024), 16, \
                                                 ld_voff, i * 1024, 0, 0);                          \
  }

  int64_t tg = wave_id;
  if (tg < TG) TORQ_LOAD_TG(tg)
  for (; tg < TG; tg += nwave) {
    // the loads of this token-group have landed (vmcnt(0); lgkmcnt and expcnt left alone)
    __builtin_amdgcn_s_waitcnt(0x0F70);
    asm volatile("" ::: "memory");

    // ---- intra-block rotation: Z'^T = R_intra^T X^T, two passes (R_intra hi, lo)
    float v[NJ][16];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const uint2 lo8 = *reinterpret_cast<const uint2 *>(my + j * 32 * 64 + rd_off[t][0]);
        const uint2 hi8 = *reinterpret_cast<const uint2 *>(my + j * 32 * 64 + rd_off[t][1]);
        const bf16x8 xb = __builtin_bit_cast(bf16x8, make_uint4(lo8.x, lo8.y, hi8.x, hi8.y));
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Al[t], xb, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ah[t], xb, acc, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) v[j][r] = acc[r];
    }

    // every LDS read of this token-group has returned (the MFMAs consumed them) and nothing moves
    // across this point: the region can be overwritten
    __builtin_amdgcn_sched_barrier(0);
    if (tg + nwave < TG) TORQ_LOAD_TG(tg + nwave)
    __builtin_amdgcn_sched_barrier(0);

    // ---- inter-block rotation: the butterfly over b = 32 j + b0 (all indices are literals after
    // unrolling).  Round k's NJ coefficients are c[k % 2]; those of round k + 1 are fetched (from LDS when
    // G >= 128) BEFORE round k's arithmetic and nothing moves across the fences, so the read's latency
    // passes behind 16 NJ multiply-adds instead of in front of every 16.
#define TORQ_CF_FETCH(ROUND_)                                                                       \
  _Pragma("unroll") for (int j = 0; j < NJ; ++j) c[(ROUND_) & 1][j] = cf((ROUND_) * NJ + j);         \
  __builtin_amdgcn_sched_barrier(0);
    // (MXINT4 and NVFP4 at G = 128 have no four registers to spare at 128 per lane: they fetch a round's
    // coefficients where the round starts)
    constexpr bool AHEAD = !(NJ == 4 && (FMT == FMT_MXINT4 || FMT == FMT_NVFP4));
#define TORQ_CF_ROUND(K_) if constexpr (AHEAD) { TORQ_CF_FETCH((K_) + 1) } else { TORQ_CF_FETCH(K_) }
    float c[2][NJ];
    if constexpr (AHEAD) { TORQ_CF_FETCH(0) }
#pragma unroll
    for (int m = 0; m < LJ; ++m) {                             // strides 32 hj: pairs of tiles
      const int hj = NJ >> (m + 1);
      TORQ_CF_ROUND(m)
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        if ((j & hj) == 0) {
          const float tp = c[m & 1][j], tq = c[m & 1][j + hj];
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float p = v[j][r], q = v[j + hj][r];
            v[j][r] = fmaf(tp, q, p);
            v[j + hj][r] = fmaf(tq, p, q);
          }
        }
      __builtin_amdgcn_sched_barrier(0);
    }
    TORQ_CF_ROUND(LJ)
#pragma unroll
    for (int j = 0; j < NJ; ++j) {                             // stride 16: lane n ^ 16
      const float t = c[LJ & 1][j];
#pragma unroll
      for (int r = 0; r < 16; ++r) v[j][r] = fmaf(t, swizzle_f32<0x401F>(v[j][r]), v[j][r]);
    }
    __builtin_amdgcn_sched_barrier(0);
    TORQ_CF_ROUND(LJ + 1)
#pragma unroll
    for (int j = 0; j < NJ; ++j) TORQ_FMAC16_DPP(v[j], c[(LJ + 1) & 1][j], "row_mirror");               // stride 8
    __builtin_amdgcn_sched_barrier(0);
    TORQ_CF_ROUND(LJ + 2)
#pragma unroll
    for (int j = 0; j < NJ; ++j) TORQ_FMAC16_DPP(v[j], c[(LJ + 2) & 1][j], "row_half_mirror");          // stride 4
    __builtin_amdgcn_sched_barrier(0);
    TORQ_CF_ROUND(LJ + 3)
#pragma unroll
    for (int j = 0; j < NJ; ++j) TORQ_FMAC16_DPP(v[j], c[(LJ + 3) & 1][j], "quad_perm:[2,3,0,1]");      // stride 2
    __builtin_amdgcn_sched_barrier(0);
    TORQ_CF_ROUND(LJ + 4)
#pragma unroll
    for (int j = 0; j < NJ; ++j) TORQ_FMAC16_DPP(v[j], c[(LJ + 4) & 1][j], "quad_perm:[1,0,3,2]");      // stride 1
    __builtin_amdgcn_sched_barrier(0);
#undef TORQ_CF_ROUND
#undef TORQ_CF_FETCH

    // ---- the rows' sigma, then step 4
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const float rs = AHEAD ? c[(LJ + 5) & 1][j] : cf((LJ + 5) * NJ + j);
      float zz[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) zz[r] = v[j][r] * rs;
      const int64_t blkidx = tg * G + 32 * j + b0;              // global block index
      if constexpr (FMT == FMT_NVFP4) {
        const float amax = fmaxf(amax8(zz), amax8(zz + 8));
        const uint32_t sc = nvfp4_scale_code(amax, 6.0f * global_scale);
        const float S = e4m3_to_f32(sc) * global_scale;
        codes[blkidx * 2 + h] = make_uint2(pack8_nvfp4(zz, S), pack8_nvfp4(zz + 8, S));
        scales[blkidx * 2 + h] = (uint8_t)sc;
      } else if constexpr (FMT != FMT_NONE) {
        float amax = fmaxf(amax8(zz), amax8(zz + 8));
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
}

#undef TORQ_LOAD_TG
#undef cf
#undef TORQ_FMAC16_DPP

int butterfly_coef_count(int G) {
  const int NJ = G / 32, LJ = NJ == 1 ? 0 : NJ == 2 ? 1 : NJ == 4 ? 2 : 3;
  return (LJ + 6) * NJ;
}

template <int NJ>
static hipError_t launch_nj(const torq_rotation *r, const void *x, int64_t TG, int format, float global_scale,
                            uint8_t *codes, uint8_t *scales, float *z_out, hipStream_t stream) {
  const size_t lds_bytes = 4 * (size_t)NJ * 32 * 64 + (NJ >= 4 ? (size_t)butterfly_coef_count(32 * NJ) * 32 * 4 : 0);
  // resident workgroups of 4 waves: what the kernel's register count (and LDS) admits per CU
  int64_t grid = (NJ == 1 ? 8 : NJ == 2 ? 5 : NJ == 4 ? 4 : 2) * 256;
  if (grid * 4 > TG) grid = (TG + 3) / 4;
  const uint4 *ih = reinterpret_cast<const uint4 *>(r->intra32_hi);
  const uint4 *il = reinterpret_cast<const uint4 *>(r->intra32_lo);
  const uint4 *xx = reinterpret_cast<const uint4 *>(x);
  uint2 *cc = reinterpret_cast<uint2 *>(codes);
  switch (z_out ? FMT_NONE : format) {
#define TORQ_BF_CASE(F_, GS_)                                                                                  \
  case F_:                                                                                                     \
    hipLaunchKernelGGL((rotate_butterfly_kernel<NJ, F_>), dim3((unsigned)grid), dim3(256), lds_bytes, stream, xx, TG, \
                       r->butterfly, ih, il, cc, scales, z_out, GS_);                                          \
    break;
    TORQ_BF_CASE(FMT_NONE, 1.0f) TORQ_BF_CASE(FMT_MXFP4, 1.0f) TORQ_BF_CASE(FMT_MXINT4, 1.0f)
    TORQ_BF_CASE(FMT_NVFP4, global_scale)
#undef TORQ_BF_CASE
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// r->butterfly holds the coefficient table; G in {32, 64, 128, 256}
hipError_t launch_rotate_butterfly(const torq_rotation *r, const void *x_bf16, int64_t M, int format,
                                   float global_scale, uint8_t *codes, uint8_t *scales, float *z_out,
                                   hipStream_t stream) {
  const int64_t TG = M * (int64_t)(r->d / 32 / r->G);
  if (TG == 0) return hipSuccess;
  switch (r->G / 32) {
    case 1: return launch_nj<1>(r, x_bf16, TG, format, global_scale, codes, scales, z_out, stream);
    case 2: return launch_nj<2>(r, x_bf16, TG, format, global_scale, codes, scales, z_out, stream);
    case 4: return launch_nj<4>(r, x_bf16, TG, format, global_scale, codes, scales, z_out, stream);
    case 8: return launch_nj<8>(r, x_bf16, TG, format, global_scale, codes, scales, z_out, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace torq
