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
#include <utility>

#include "rotate16_body.h"
#include "torq_device.h"
#include "torq_internal.h"

namespace torq {

// FMT: FMT_NONE writes the rotated fp32 values, else the 4-bit format of step 4 (torq_device.h)
template <int KS, int NT, int FMT>
__global__ void __launch_bounds__(64 * ((2 * KS) / NT > 16 ? 16 : (2 * KS) / NT))
rotate_kernel(const uint4 *__restrict__ x, int64_t TG, int G,
              const uint16_t *__restrict__ inter_hi, const uint16_t *__restrict__ inter_lo,
              const uint4 *__restrict__ intra_hi_frag, const uint4 *__restrict__ intra_lo_frag,
              uint32_t *__restrict__ codes, uint8_t *__restrict__ scales, float *__restrict__ z_out,
              float global_scale) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  rotate16_body<KS, NT, FMT>(x, TG, G, inter_hi, inter_lo, intra_hi_frag, intra_lo_frag, codes, scales, z_out,
                             global_scale, lds, blockIdx.x, gridDim.x);
}

// ---------------------------------------------------------------------------
// Variant on v_mfma_f32_32x32x16_bf16 (which sustains a higher rate than the 16x16x32 form): every G
// that is a multiple of 32, and G = 16 * odd from 80 up (80 and 112 are the Qwen3-32B and LLaMA3-8B
// down-projection widths), where the last wave's tile is half empty; the 16x16x32 kernel above
// keeps G = 16 and 48.  Same formulation; wave w owns the 32 output blocks b = 32 w .. 32 w + 31
// and there are ceil(G/32) waves.  Two token-groups are processed together so that every MFMA has an
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
// Input staging.  G <= 80: global -> registers -> LDS, the next batch's loads in flight during the
// current batch.  G >= 96: global -> LDS directly (buffer_load ... lds), issued once the wave has
// read its step-2 operands of the current batch and landing during steps 3 and 4; without the
// staging registers three waves fit a SIMD up to G = 128 (160 registers), which is worth 5 - 15 %
// there and a few per cent beyond; at G <= 80 the register path measured faster (and fits three
// waves per SIMD from G = 64 up as it is).
// TB: token-groups per batch, processed together (2: every MFMA has an independent neighbour; 1 for a
// handful of token-groups, where the shortest path through one token-group counts).
template <int KS16, int TB, int FMT>
__global__ void __launch_bounds__(64 * ((KS16 + 1) / 2), (KS16 >= 4 && KS16 <= 8) ? 3 : 2)   // waves per SIMD
rotate_kernel32(const uint4 *__restrict__ x, int64_t TG, int G,
                const uint16_t *__restrict__ inter_hi, const uint16_t *__restrict__ inter_lo,
                const uint4 *__restrict__ intra_hi_frag, const uint4 *__restrict__ intra_lo_frag,
                uint2 *__restrict__ codes, uint8_t *__restrict__ scales, float *__restrict__ z_out,
                float global_scale) {
  // G = 16 KS16 blocks; one wave per 32 of them.  KS16 odd (G = 80, 112, ...): the last wave's tile is
  // half empty -- its upper 16 block rows read R_inter as zeros and store nothing -- and a token-group
  // is not a whole number of 16-byte chunks per thread, so its LDS place is padded to one
  // (TG_STRIDE); the chunks past its end load as zeros into the pad.
  constexpr int NW = (KS16 + 1) / 2;
  constexpr bool ODD = (KS16 & 1) != 0;
  constexpr int TG_BYTES = KS16 * 16 * 64;           // one token-group: G rows of 64 bytes
  constexpr int NTHR = 64 * NW;
  constexpr int CHUNKS = TG_BYTES / 16;
  constexpr int CH = (CHUNKS + NTHR - 1) / NTHR;     // 16-byte chunks per thread per token-group (= 2)
  constexpr int TG_STRIDE = CH * NTHR * 16;          // = TG_BYTES unless KS16 is odd
  constexpr int STAGE_BYTES = TB * TG_STRIDE;
  constexpr bool DMA = KS16 >= 6;
  extern __shared__ __attribute__((aligned(16))) char lds[];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, h = lane >> 5;

  // ---- resident operands: R_inter from the handle's table in lane order ([tile][k-step 2 NW][lane][8],
  // zeros for the block rows and columns past G), one load of a wave = 1 KiB of consecutive bytes
  bf16x8 Bh[KS16], Bl[KS16];
  {
    const uint4 *fh = reinterpret_cast<const uint4 *>(inter_hi), *fl = reinterpret_cast<const uint4 *>(inter_lo);
#pragma unroll
    for (int ks = 0; ks < KS16; ++ks) {
      Bh[ks] = __builtin_bit_cast(bf16x8, fh[(wave * 2 * NW + ks) * 64 + lane]);
      Bl[ks] = __builtin_bit_cast(bf16x8, fl[(wave * 2 * NW + ks) * 64 + lane]);
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
        if (tg < TG && (!ODD || tid + i * NTHR < CHUNKS)) stage_regs[j][i] = x[tg * (TG_BYTES / 16) + tid + i * NTHR];
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
        *reinterpret_cast<uint4 *>(base + j * TG_STRIDE + (tid + i * NTHR) * 16) = stage_regs[j][i];
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
            rs, (__attribute__((address_space(3))) void *)(lds + buf_ * STAGE_BYTES + j * TG_STRIDE + (wave_u * 64 + i * NTHR) * 16),
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
        const char *p = stage + j * TG_STRIDE + ks * 16 * 64;
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
        const bool live = !ODD || 32 * wave + col < 16 * KS16;  // a block row that exists
        float zz[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) zz[r] = zacc[j][r];
        if constexpr (FMT == FMT_NVFP4) {
          // the lane's sixteen values are one 16-element block: no cross-lane step
          const float amax = fmaxf(amax8(zz), amax8(zz + 8));
          const uint32_t sc = nvfp4_scale_code(amax, 6.0f * global_scale);
          const float S = e4m3_to_f32(sc) * global_scale;
          if (live) {
            codes[blkidx * 2 + h] = make_uint2(pack8_nvfp4(zz, S), pack8_nvfp4(zz + 8, S));
            scales[blkidx * 2 + h] = (uint8_t)sc;
          }
        } else if constexpr (FMT != FMT_NONE) {
          float amax = fmaxf(amax8(zz), amax8(zz + 8));
          // max with the other half-wave (lane ^ 32): swap the upper half of one copy with the
          // lower half of the other, then every lane holds both partners' values
          const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(amax), __float_as_uint(amax), false, false);
          amax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
          const uint32_t byte = e8m0_from_amax(amax);
          if constexpr (FMT == FMT_MXINT4) {
            const float inv = e8m0_inverse_f32(byte);
            if (live) codes[blkidx * 2 + h] = make_uint2(pack8_int4(zz, inv), pack8_int4(zz + 8, inv));
          } else {
            const float sc = e8m0_to_f32(byte);
            if (live) codes[blkidx * 2 + h] = make_uint2(pack8_e2m1(zz, sc), pack8_e2m1(zz + 8, sc));
          }
          if (h == 0 && live) scales[blkidx] = (uint8_t)byte;
        } else {
          float4 *o = reinterpret_cast<float4 *>(z_out + blkidx * 32 + 16 * h);
          if (live) {
#pragma unroll
            for (int q = 0; q < 4; ++q) o[q] = make_float4(zz[4 * q], zz[4 * q + 1], zz[4 * q + 2], zz[4 * q + 3]);
          }
        }
      }
    }

    if constexpr (!DMA) {
      if (have_next) store_batch(buf ^ 1);
      __syncthreads();
    }
  }
}

// ---------------------------------------------------------------------------
// The same kernel for G = 80, 96, 112, 128 with THREE LDS buffers, filled two batches ahead (quantising
// formats only; the fp32 output of torq_rotate stays with rotate_kernel32).  With two buffers the next
// batch can only be requested once every wave has read the current one, which leaves the request about a
// third of an iteration to land; with three it is requested a whole iteration earlier, at the top of the
// iteration before.  Measured against the two-buffer form, same machine: 3 - 5 % (51.5 -> 49.0 us at
// X [8192, 8192], 311 -> 301 us at [16384, 28672]) -- the kernel runs at the board's power limit, so
// removing stalls buys little; it is kept because it costs nothing else.
//
// Two things are issued from assembly because of how the compiler orders LDS traffic: it places every LDS
// read it recognises behind ALL outstanding loads into LDS (vmcnt(0)), which would undo the ring.  So
// the loads into LDS (dma16) and the transposing reads (lds_tr_read) are invisible to it, and the waits
// are written by hand:
//   * LDS reads: lds_wait4 (lgkmcnt(0)) in front of the MFMAs that consume them; the next k-step's four
//     reads are issued right after it and have the MFMAs of this k-step to land.
//   * loads into LDS: every wave issues exactly PER_ITER_LD = TB * CH of them at the top of an iteration
//     and exactly PER_ITER_ST = 2 * TB buffer stores at its end, whatever the batch (a token-group past
//     the end gets empty descriptors: its loads return zeros, its stores are dropped; lanes without a
//     block store to an out-of-range offset).  Vector-memory operations of a wave complete in order, so
//     "at most PER_ITER_LD + 2 * PER_ITER_ST operations outstanding" means the batch requested two
//     iterations ago has landed.  No other vector-memory instruction may appear in the loop: the build
//     test tests/test_kernel_isa.py counts them in the compiled code.
// SKIP (diagnostic builds only, torq_diag_rotate_ablation): work left out to measure what it costs --
// 1: the R_inter low-part pass, 2: the hi/lo split of Y on the vector ALU (raw register pairs are fed
// instead), 4: the amax and the conversion of step 4 (bit patterns are stored instead), 8: two of the
// three R_intra passes.  The output is then meaningless.  SKIP = 0 is the product.
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

template <int OFF>
__device__ __forceinline__ i16x4 lds_tr_read(uint32_t addr) {
  i16x4 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
}
__device__ __forceinline__ void lds_wait4(i16x4 &a, i16x4 &b, i16x4 &c, i16x4 &d) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}
// 16 bytes per lane from a buffer straight into LDS at lds_addr + 16 * lane (lds_addr wave-uniform)
__device__ __forceinline__ void dma16(i32x4 rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
}
typedef __attribute__((__vector_size__(2 * sizeof(unsigned)))) unsigned u32x2;

template <int KS16, int FMT, int SKIP = 0>
__global__ void __launch_bounds__(64 * ((KS16 + 1) / 2), 3)
rotate_ring_kernel32(const uint4 *__restrict__ x, int64_t TG, int G,
                     const uint16_t *__restrict__ inter_hi, const uint16_t *__restrict__ inter_lo,
                     const uint4 *__restrict__ intra_hi_frag, const uint4 *__restrict__ intra_lo_frag,
                     uint8_t *__restrict__ codes, uint8_t *__restrict__ scales, float global_scale) {
  static_assert(FMT != FMT_NONE, "quantising formats only");
  constexpr int TB = 2;
  constexpr int NW = (KS16 + 1) / 2;
  constexpr bool ODD = (KS16 & 1) != 0;
  constexpr int TG_BYTES = KS16 * 16 * 64;
  constexpr int NTHR = 64 * NW;
  constexpr int CHUNKS = TG_BYTES / 16;
  constexpr int CH = (CHUNKS + NTHR - 1) / NTHR;
  constexpr int TG_STRIDE = CH * NTHR * 16;          // a token-group's place in LDS (= TG_BYTES unless KS16 is odd)
  constexpr int STAGE_BYTES = TB * TG_STRIDE;
  constexpr int OOB = 0x7FFFFFF0;                    // beyond every descriptor: loads give zero, stores are dropped
  // three separate arrays: the stages are distinct objects
  __shared__ __attribute__((aligned(16))) char stage0[STAGE_BYTES];
  __shared__ __attribute__((aligned(16))) char stage1[STAGE_BYTES];
  __shared__ __attribute__((aligned(16))) char stage2[STAGE_BYTES];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, h = lane >> 5;
  const int b = 32 * wave + col;                     // this lane's block row inside a token-group
  const bool live = !ODD || b < 16 * KS16;

  // R_inter from the handle's table in lane order (zeros for the block rows past G)
  bf16x8 Bh[KS16], Bl[KS16];
  {
    const uint4 *fh = reinterpret_cast<const uint4 *>(inter_hi), *fl = reinterpret_cast<const uint4 *>(inter_lo);
#pragma unroll
    for (int ks = 0; ks < KS16; ++ks) {
      Bh[ks] = __builtin_bit_cast(bf16x8, fh[(wave * 2 * NW + ks) * 64 + lane]);
      Bl[ks] = __builtin_bit_cast(bf16x8, fl[(wave * 2 * NW + ks) * 64 + lane]);
    }
  }
  bf16x8 Ah[2], Al[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    Ah[t] = __builtin_bit_cast(bf16x8, intra_hi_frag[t * 64 + lane]);
    Al[t] = __builtin_bit_cast(bf16x8, intra_lo_frag[t * 64 + lane]);
  }
  const int blk = lane >> 4, s16 = lane & 15;
  const int tr_off = ((8 * (blk >> 1) + (s16 >> 2)) * 32 + 16 * (blk & 1) + 4 * (s16 & 3)) * 2;
  const int64_t nbatch = (TG + TB - 1) / TB;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  // bytes of scales per token-group, and where this lane's scale byte goes in them
  constexpr int SC_PER_BLK = FMT == FMT_NVFP4 ? 2 : 1;
  const int sc_off = FMT == FMT_NVFP4 ? (live ? b * 2 + h : OOB) : ((live && h == 0) ? b : OOB);
  const int cd_off = live ? (b * 2 + h) * 8 : OOB;

  auto dma = [&](int64_t b_, char *dst) {
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      const int64_t tg = b_ * TB + j;
      const bool ok = b_ < nbatch && tg < TG;
      const uint64_t base = reinterpret_cast<uint64_t>(x) + (uint64_t)((ok ? tg : 0) * (int64_t)TG_BYTES);
      const i32x4 rs = i32x4{(int)(uint32_t)base, (int)((uint32_t)(base >> 32) & 0xFFFFu), ok ? TG_BYTES : 0, 0x00020000};
      const uint32_t la = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)(dst) + j * TG_STRIDE + wave_u * 64 * 16;
#pragma unroll
      for (int i = 0; i < CH; ++i) dma16(rs, la + i * NTHR * 16, tid * 16, i * NTHR * 16);
    }
  };

  auto compute = [&](int64_t batch, const char *stage_base) {
    // ---- step 2
    f32x16 acc[TB];
#pragma unroll
    for (int j = 0; j < TB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    const uint32_t sa = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char *)(stage_base) + tr_off;
    i16x4 q[2][4];
    q[0][0] = lds_tr_read<0>(sa);
    q[0][1] = lds_tr_read<256>(sa);
    q[0][2] = lds_tr_read<TG_STRIDE>(sa);
    q[0][3] = lds_tr_read<TG_STRIDE + 256>(sa);
    static_for<KS16>([&](auto ks_c) {
      constexpr int ks = decltype(ks_c)::value;
      constexpr int cur = ks & 1, nxt = cur ^ 1;
      lds_wait4(q[cur][0], q[cur][1], q[cur][2], q[cur][3]);
      if constexpr (ks + 1 < KS16) {
        q[nxt][0] = lds_tr_read<(ks + 1) * 1024>(sa);
        q[nxt][1] = lds_tr_read<(ks + 1) * 1024 + 256>(sa);
        q[nxt][2] = lds_tr_read<TG_STRIDE + (ks + 1) * 1024>(sa);
        q[nxt][3] = lds_tr_read<TG_STRIDE + (ks + 1) * 1024 + 256>(sa);
      }
      bf16x8 xa[TB];
#pragma unroll
      for (int j = 0; j < TB; ++j) {
        union { bf16x8 v; i16x4 h2[2]; } u;
        u.h2[0] = q[cur][2 * j];
        u.h2[1] = q[cur][2 * j + 1];
        xa[j] = u.v;
      }
#pragma unroll
      for (int j = 0; j < TB; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[j], Bh[ks], acc[j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < TB; ++j)
        if constexpr (!(SKIP & 1)) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[j], Bl[ks], acc[j], 0, 0, 0);
    });

    // ---- step 3
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
          if constexpr ((SKIP & 2) != 0) {
            hi[p] = __float_as_uint(y0);
            lo[p] = __float_as_uint(y1);
          } else {
            hi[p] = pack_bf16_rne(y0, y1);
            lo[p] = pack_bf16_rne(y0 - __uint_as_float(hi[p] << 16), y1 - __uint_as_float(hi[p] & 0xFFFF0000u));
          }
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
      for (int j = 0; j < TB; ++j)
        if constexpr (!(SKIP & 8)) zacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Al[t], yh[j][t], zacc[j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < TB; ++j) zacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ah[t], yl[j][t], zacc[j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < TB; ++j)
        if constexpr (!(SKIP & 8)) zacc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ah[t], yh[j][t], zacc[j], 0, 0, 0);
    }

    // ---- step 4 and the two stores of each token-group
#pragma unroll
    for (int j = 0; j < TB; ++j) {
      const int64_t tg = batch * TB + j;
      const bool ok = tg < TG;
      float zz[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) zz[r] = zacc[j][r];
      u32x2 c;
      uint32_t byte;
      if constexpr ((SKIP & 4) != 0) {
        uint32_t c0 = 0, c1 = 0;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          c0 ^= __float_as_uint(zz[r]);
          c1 ^= __float_as_uint(zz[8 + r]);
        }
        c = u32x2{c0, c1};
        byte = c0 >> 23;
      } else if constexpr (FMT == FMT_NVFP4) {
        const float amax = fmaxf(amax8(zz), amax8(zz + 8));
        byte = nvfp4_scale_code(amax, 6.0f * global_scale);
        const float S = e4m3_to_f32(byte) * global_scale;
        c = u32x2{pack8_nvfp4(zz, S), pack8_nvfp4(zz + 8, S)};
      } else {
        float amax = fmaxf(amax8(zz), amax8(zz + 8));
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(amax), __float_as_uint(amax), false, false);
        amax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        byte = e8m0_from_amax(amax);
        if constexpr (FMT == FMT_MXINT4) {
          const float inv = e8m0_inverse_f32(byte);
          c = u32x2{pack8_int4(zz, inv), pack8_int4(zz + 8, inv)};
        } else {
          const float sc = e8m0_to_f32(byte);
          c = u32x2{pack8_e2m1(zz, sc), pack8_e2m1(zz + 8, sc)};
        }
      }
      const __amdgpu_buffer_rsrc_t crs = __builtin_amdgcn_make_buffer_rsrc(
          codes + (ok ? tg : 0) * (int64_t)(G * 16), 0, ok ? G * 16 : 0, 0x00020000);
      const __amdgpu_buffer_rsrc_t srs = __builtin_amdgcn_make_buffer_rsrc(
          scales + (ok ? tg : 0) * (int64_t)(G * SC_PER_BLK), 0, ok ? G * SC_PER_BLK : 0, 0x00020000);
      __builtin_amdgcn_raw_buffer_store_b64(c, crs, cd_off, 0, 0);
      __builtin_amdgcn_raw_buffer_store_b8((unsigned char)byte, srs, sc_off, 0, 0);
    }
  };

  const int64_t stride = gridDim.x;
  int64_t batch = blockIdx.x;
  if (batch >= nbatch) return;                       // uniform over the workgroup; before any barrier
  dma(batch, stage0);
  dma(batch + stride, stage1);
  // The resident operands above are ordinary loads; waiting for them here, once, leaves the compiler
  // nothing to wait for inside the loop (its own wait would come out as vmcnt(0): it does not see the
  // requests above, which are younger).  The first two batches land with them.
  __builtin_amdgcn_s_waitcnt(0x0F70);
  constexpr int PER_ITER_LD = TB * CH, PER_ITER_ST = 2 * TB;
  static_assert(PER_ITER_LD + 2 * PER_ITER_ST <= 15, "the wait below encodes its count in four bits");
  int it = 0;
  // s_waitcnt with vmcnt = N (low four bits), no wait on the other counters
#define TORQ_RING_ITER(CUR_, FREE_)                                                                 \
  {                                                                                                 \
    if (it == 0) __builtin_amdgcn_s_waitcnt(0x0F70 | PER_ITER_LD);                                  \
    else if (it == 1) __builtin_amdgcn_s_waitcnt(0x0F70 | (PER_ITER_LD + PER_ITER_ST));             \
    else __builtin_amdgcn_s_waitcnt(0x0F70 | (PER_ITER_LD + 2 * PER_ITER_ST));                      \
    __syncthreads();           /* everybody's part of this batch has landed; FREE_ has been read */ \
    dma(batch + 2 * stride, FREE_);                                                                 \
    compute(batch, CUR_);                                                                           \
    batch += stride;                                                                                \
    ++it;                                                                                           \
    if (batch >= nbatch) break;                                                                     \
  }
  for (;;) {
    TORQ_RING_ITER(stage0, stage2)
    TORQ_RING_ITER(stage1, stage0)
    TORQ_RING_ITER(stage2, stage1)
  }
#undef TORQ_RING_ITER
  __builtin_amdgcn_s_waitcnt(0x0F70);                // nothing of this wave's is in flight when it ends
}

// launch KERNEL_<..., FMT> for the runtime format (FMT_NONE when the fp32 output is asked for)
#define TORQ_LAUNCH_FMT(KERNEL_, CODES_T_, ...)                                                                  \
  switch (z_out ? FMT_NONE : format) {                                                                          \
    case FMT_NONE:                                                                                              \
      hipLaunchKernelGGL((KERNEL_<__VA_ARGS__, FMT_NONE>), dim3((unsigned)grid), dim3(64 * nw), lds_bytes, stream, \
                         reinterpret_cast<const uint4 *>(x), TG, r->G, ri_hi, ri_lo, ih, il,                    \
                         (CODES_T_ *)nullptr, (uint8_t *)nullptr, z_out, 1.0f);                                 \
      break;                                                                                                    \
    case FMT_MXFP4:                                                                                             \
      hipLaunchKernelGGL((KERNEL_<__VA_ARGS__, FMT_MXFP4>), dim3((unsigned)grid), dim3(64 * nw), lds_bytes, stream, \
                         reinterpret_cast<const uint4 *>(x), TG, r->G, ri_hi, ri_lo, ih, il,                    \
                         reinterpret_cast<CODES_T_ *>(codes), scales, (float *)nullptr, 1.0f);                  \
      break;                                                                                                    \
    case FMT_MXINT4:                                                                                            \
      hipLaunchKernelGGL((KERNEL_<__VA_ARGS__, FMT_MXINT4>), dim3((unsigned)grid), dim3(64 * nw), lds_bytes, stream, \
                         reinterpret_cast<const uint4 *>(x), TG, r->G, ri_hi, ri_lo, ih, il,                    \
                         reinterpret_cast<CODES_T_ *>(codes), scales, (float *)nullptr, 1.0f);                  \
      break;                                                                                                    \
    case FMT_NVFP4:                                                                                             \
      hipLaunchKernelGGL((KERNEL_<__VA_ARGS__, FMT_NVFP4>), dim3((unsigned)grid), dim3(64 * nw), lds_bytes, stream, \
                         reinterpret_cast<const uint4 *>(x), TG, r->G, ri_hi, ri_lo, ih, il,                    \
                         reinterpret_cast<CODES_T_ *>(codes), scales, (float *)nullptr, global_scale);          \
      break;                                                                                                    \
    default: return hipErrorInvalidValue;                                                                       \
  }                                                                                                             \
  return hipGetLastError();

// Persistent workgroups: `per_cu` of them on each of the 256 CUs; with fewer than a few rounds of
// batches the grid is cut to ceil(nbatch / rounds) so that every workgroup gets the same number.
static int64_t balanced_grid(int64_t nbatch, int per_cu) {
  const int64_t slots = (int64_t)per_cu * 256;
  if (nbatch <= slots) return nbatch;
  const int64_t rounds = (nbatch + slots - 1) / slots;
  return (nbatch + rounds - 1) / rounds;
}

template <int KS16, int TB = 2>
static hipError_t launch_cfg32(const torq_rotation *r, const void *x, int64_t TG, int format, float global_scale,
                               uint8_t *codes, uint8_t *scales, float *z_out, hipStream_t stream) {
  const int nw = (KS16 + 1) / 2;                         // = ceil(G / 32)
  const int64_t nbatch = (TG + TB - 1) / TB;
  // a token-group's place in LDS: a whole number of 16-byte chunks per thread (padded when KS16 is odd)
  const size_t tg_stride = (size_t)((KS16 * 64 + 64 * nw - 1) / (64 * nw)) * (64 * nw) * 16;
  const size_t lds_bytes = 2 * (size_t)TB * tg_stride;
  // resident workgroups per CU: limited by LDS (160 KiB) and by the waves per SIMD that the register
  // count admits (three for G = 64 ... 128, two otherwise)
  const int waves_per_cu = (KS16 >= 4 && KS16 <= 8) ? 12 : 8;
  int per_cu = (int)((160 * 1024) / lds_bytes);
  if (per_cu * nw > waves_per_cu) per_cu = waves_per_cu / nw;
  if (per_cu < 1) per_cu = 1;
  const int64_t grid = balanced_grid(nbatch, per_cu);
  const uint4 *ih = reinterpret_cast<const uint4 *>(r->intra32_hi);
  const uint4 *il = reinterpret_cast<const uint4 *>(r->intra32_lo);
  const uint16_t *ri_hi = r->inter32f_hi, *ri_lo = r->inter32f_lo;      // the table in lane order
  TORQ_LAUNCH_FMT(rotate_kernel32, uint2, KS16, TB)
}

template <int KS16>
static hipError_t launch_ring32(const torq_rotation *r, const void *x, int64_t TG, int format, float global_scale,
                                uint8_t *codes, uint8_t *scales, hipStream_t stream) {
  const int nw = (KS16 + 1) / 2;
  const int64_t nbatch = (TG + 1) / 2;
  // 3 x <= 48 KiB of LDS, 12 waves of <= 160 registers (G = 80: 4 x 36 KiB, 12 waves of three per workgroup)
  const int64_t grid = balanced_grid(nbatch, KS16 == 5 ? 4 : 3);
  const uint4 *ih = reinterpret_cast<const uint4 *>(r->intra32_hi);
  const uint4 *il = reinterpret_cast<const uint4 *>(r->intra32_lo);
#define TORQ_RING_LAUNCH(FMT_, GS_)                                                                                  \
  hipLaunchKernelGGL((rotate_ring_kernel32<KS16, FMT_>), dim3((unsigned)grid), dim3(64 * nw), 0, stream,               \
                     reinterpret_cast<const uint4 *>(x), TG, r->G, r->inter32f_hi, r->inter32f_lo, ih, il, codes, scales, GS_)
  switch (format) {
    case FMT_MXFP4: TORQ_RING_LAUNCH(FMT_MXFP4, 1.0f); break;
    case FMT_MXINT4: TORQ_RING_LAUNCH(FMT_MXINT4, 1.0f); break;
    case FMT_NVFP4: TORQ_RING_LAUNCH(FMT_NVFP4, global_scale); break;
    default: return hipErrorInvalidValue;
  }
#undef TORQ_RING_LAUNCH
  return hipGetLastError();
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
  const uint16_t *ri_hi = r->inter_hi, *ri_lo = r->inter_lo;            // the row-major table
  TORQ_LAUNCH_FMT(rotate_kernel, uint32_t, KS, NT)
}
#undef TORQ_LAUNCH_FMT

// Exactly one of (codes, scales) / z_out is used; `format` (FMT_*) picks step 4's block format.
hipError_t launch_rotate(const torq_rotation *r, const void *x_bf16, int64_t M, int format, float global_scale,
                         uint8_t *codes, uint8_t *scales, float *z_out, hipStream_t stream) {
  const int64_t TG = M * (int64_t)(r->d / 32 / r->G);
  if (TG == 0) return hipSuccess;
  constexpr int64_t RING_MIN_TG = 2 * 8 * 3 * 256;       // eight batches for each of the ring's 768 workgroups
  // quantising, G = 80 ... 128, large inputs: the three-buffer form of the 32x32x16 kernel.  Below eight
  // batches per workgroup the two batches requested ahead of the loop cost more than the ring saves (same
  // machine, ring against two buffers of two token-groups: X [4096, 4096] 18.7 against 17.3 us,
  // [1024, 4096] 8.8 against 8.2, [2048, 14336] 27.1 against 25.5, [4096, 5120] 18.2 against 17.3; equal at
  // [8192, 4096]; from [16384, 4096] on the ring wins, 45.7 against 49.6 us there)
  if (!z_out && TG >= RING_MIN_TG) {
    if (r->G == 128) return launch_ring32<8>(r, x_bf16, TG, format, global_scale, codes, scales, stream);
    if (r->G == 112) return launch_ring32<7>(r, x_bf16, TG, format, global_scale, codes, scales, stream);
    if (r->G == 96) return launch_ring32<6>(r, x_bf16, TG, format, global_scale, codes, scales, stream);
    if (r->G == 80) return launch_ring32<5>(r, x_bf16, TG, format, global_scale, codes, scales, stream);
  }
  // Below that, batches of ONE token-group instead of two for G = 128, 112 and 80 (a) up to 256 token-groups
  // (they spread over twice as many workgroups) and (b) from 3072 on (three or more batches of two per
  // workgroup: as batches of one the same share leaves in smaller steps).  Between, two per batch, on fewer
  // workgroups: each loads its slice of R_inter, 64 KB, first.  HIP-graph replays over rotating input copies,
  // one per batch against two, same machine: X [256, 4096] 3.7 against 4.3 us, [512, 4096] 4.7 / 4.6,
  // [1536, 4096] 8.25 / 7.97, [2048, 4096] 10.4 / 9.9, [1024, 8192] 10.3 / 9.9, [3072, 4096] 12.8 / 12.9,
  // [4096, 4096] 15.7 / 16.2, [4096, 5120] (G = 80) 17.8 / 19.7; plain launch loops agree from [4096, 4096] on
  // ([8192, 4096] 27.2 / 28.0, [2048, 8192] 16.9 / 18.2) and are bound by the host below.  G = 64 gains 3 % from
  // 3072 to 16384 token-groups; G = 96 and G = 32 lose 0 - 5 % and keep two.  (The fp32 output keeps batches of
  // two but for a handful of token-groups at G = 128 and 112, the decode case.)
  const bool one_per_batch = !z_out ? (TG <= 256 || TG >= 3072) : TG <= 128;
  if (one_per_batch) {
    if (r->G == 128) return launch_cfg32<8, 1>(r, x_bf16, TG, format, global_scale, codes, scales, z_out, stream);
    if (r->G == 112) return launch_cfg32<7, 1>(r, x_bf16, TG, format, global_scale, codes, scales, z_out, stream);
    if (r->G == 80 && !z_out) return launch_cfg32<5, 1>(r, x_bf16, TG, format, global_scale, codes, scales, z_out, stream);
    if (r->G == 64 && !z_out && TG >= 3072 && TG <= 16384)
      return launch_cfg32<4, 1>(r, x_bf16, TG, format, global_scale, codes, scales, z_out, stream);
  }
  // G a multiple of 32, or 16 * odd from 80 up: the 32x32x16 kernel (with a half-empty last tile).
  // Measured on X [16384, d] against the 16x16x32 kernel: G = 112 gains 7 - 9 %, G = 80 3 - 7 % (at
  // three waves per SIMD; at two it lost 3 - 4 %).
  if (r->G % 32 == 0 || r->G >= 80) {
    switch (r->G / 16) {
#define TORQ_CASE32(K16_) \
  case K16_: return launch_cfg32<K16_>(r, x_bf16, TG, format, global_scale, codes, scales, z_out, stream);
      TORQ_CASE32(2) TORQ_CASE32(4) TORQ_CASE32(5) TORQ_CASE32(6) TORQ_CASE32(7) TORQ_CASE32(8)
      TORQ_CASE32(9) TORQ_CASE32(10) TORQ_CASE32(11) TORQ_CASE32(12) TORQ_CASE32(13) TORQ_CASE32(14)
      TORQ_CASE32(15) TORQ_CASE32(16)
#undef TORQ_CASE32
    }
  }
  // G = 16 and 48: the 16x16x32 kernel, one tile of 16 blocks per wave
  switch (r->KS) {
#define TORQ_CASE(KS_) \
  case KS_: return launch_cfg<KS_, 1>(r, x_bf16, TG, format, global_scale, codes, scales, z_out, stream);
    TORQ_CASE(1) TORQ_CASE(2)
#undef TORQ_CASE
  }
  return hipErrorInvalidValue;
}

// torq_diag_rotate_ablation: rotate_ring_kernel32<8, MXFP4> (G = 128) with work left out (see SKIP there),
// in the launch shape of the product.
hipError_t launch_rotate_ablated(const torq_rotation *r, const void *x, int64_t M, uint8_t *codes, uint8_t *scales,
                                 int skip, hipStream_t stream) {
  if (r->G != 128 || r->butterfly) return hipErrorInvalidValue;
  const int64_t TG = M * (int64_t)(r->d / 32 / 128);
  if (TG == 0) return hipSuccess;
  const int64_t grid = balanced_grid((TG + 1) / 2, 3);
  const uint4 *ih = reinterpret_cast<const uint4 *>(r->intra32_hi), *il = reinterpret_cast<const uint4 *>(r->intra32_lo);
  switch (skip) {
#define TORQ_ABLATE(S_)                                                                                             \
  case S_:                                                                                                          \
    hipLaunchKernelGGL((rotate_ring_kernel32<8, FMT_MXFP4, S_>), dim3((unsigned)grid), dim3(256), 0, stream,         \
                       reinterpret_cast<const uint4 *>(x), TG, 128, r->inter32f_hi, r->inter32f_lo, ih, il, codes, scales, \
                       1.0f);                                                                                       \
    break;
    TORQ_ABLATE(0) TORQ_ABLATE(1) TORQ_ABLATE(2) TORQ_ABLATE(4) TORQ_ABLATE(6) TORQ_ABLATE(8) TORQ_ABLATE(9) TORQ_ABLATE(15)
#undef TORQ_ABLATE
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace torq
