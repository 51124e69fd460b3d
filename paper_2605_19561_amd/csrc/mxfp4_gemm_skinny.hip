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
#include "rotate16_body.h"
#include "rotate32_resident.h"
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
constexpr int LOCAL_MAX_TG = 4;       // token-groups that torq_linear_local_kernel rotates in every workgroup
constexpr int SKINNY_MIN_GROUPS = 384; // fewer workgroups than this leave CUs without work (256 CUs)

// a voffset that the range check of any buffer used here rejects (the load then delivers zeros)
constexpr int OOB_VOFF = 0x7FFFFFF0;

// what the decode form of torq_linear needs on top of the GEMM's arguments
struct DecodeArgs {
  const uint4 *x;
  int64_t TG;
  const uint4 *inter_hi, *inter_lo;            // R_inter in lane order, R_intra as the 32x32x16 operand
  const uint4 *intra_hi_frag, *intra_lo_frag;
  uint8_t *A_q, *A_s;          // written by the first P workgroups, read by the others
  int P;
  unsigned *ctr;
  int spin_limit;              // polls of the "ready" word before a waiting workgroup gives up
  int raise_ready;             // 0: the producers never raise "ready" (host-driven test of the give-up path)
};

}  // namespace

// The end of both kernels: add the waves' partial tiles through LDS and store.  Every wave's partial
// tiles go through LDS (red_mem: WAVES NS MT KiB) and the NS MT output tiles are shared out over the
// waves (tile k to wave k % WAVES), each added in the same fixed order, wave 0 + 1 + ... + 7: the same
// bits whichever wave does it (one wave adding up to eight tiles took a microsecond while seven waited).
template <int MT, int NS>
__device__ __forceinline__ void skinny_reduce_store(f32x4 (&acc)[NS][MT], unsigned char *red_mem, uint16_t *__restrict__ out,
                                                    int M, int64_t N, int64_t n0, int wave, int lane) {
  const int r16 = lane & 15, q = lane >> 4;
  __syncthreads();                                 // everybody is done with the scales
  float *red = reinterpret_cast<float *>(red_mem); // [WAVES][NS][MT][4][64]
#pragma unroll
  for (int n = 0; n < NS; ++n)
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) red[(((wave * NS + n) * MT + t) * 4 + r) * 64 + lane] = acc[n][t][r];
  __syncthreads();
#pragma unroll
  for (int n = 0; n < NS; ++n) {
    const int64_t nn = n0 + n * 16 + 4 * q;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      if ((n * MT + t) % WAVES != wave) continue;  // uniform over the wave
      bf16x4 v;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float sum = red[((n * MT + t) * 4 + r) * 64 + lane];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) sum += red[(((w * NS + n) * MT + t) * 4 + r) * 64 + lane];
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

// MT = number of 16-row activation tiles (M <= 16 MT); NS = 16-row weight strips per workgroup
// (1 or 2; they share the activation loads); PT = line pairs per wave and trip.
// PERSIST: a workgroup takes the strip groups blockIdx.x, blockIdx.x + gridDim.x, ... and loads the
// activations' codes (and scale bytes) ONCE, keeping the codes in registers across its groups; only
// when one trip covers the k range (d / 256 <= PT * WAVES line pairs), where those registers are the
// trip's own.  Every workgroup otherwise re-reads all activation rows from the L2, which at 8 - 16 rows
// is half as many bytes again as the weights it streams.  Same arithmetic in the same order: the
// outputs are bit-identical.
template <int MT, int NS, int PT, bool PERSIST = false>
__global__ void __launch_bounds__(64 * WAVES)
mxfp4_gemm_skinny_kernel(const uint8_t *__restrict__ A_q, const uint8_t *__restrict__ A_s,
                         const uint8_t *__restrict__ W_q, const uint8_t *__restrict__ W_s,
                         uint16_t *__restrict__ out, int M, int64_t N, int d) {
  // dynamic LDS: scale bytes of the weight strips (16 NS rows) and of the activation rows (16 MT),
  // d / 32 bytes each, every row padded by 4 bytes (the lanes of a k-step read one byte of 16
  // different rows); the waves' partial tiles are overlaid on it after the k loop
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r16 = lane & 15, q = lane >> 4;
  const int row_bytes = d / 2, srow_bytes = d / 32;
  const int KS = d / 128;                          // k-steps of one MFMA (128 elements, 4 blocks)
  const int KP = (KS + 1) / 2;                     // pairs of k-steps = whole 128-byte lines of a row
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
  const int ws_off = r16 * pd * 4 + q;             // this lane's scale byte: + 4 per k-step
  const int as_off = w_ins * 256 + r16 * pd * 4 + q;
  // the waves' partial tiles: over the scales (one group per workgroup), behind them (PERSIST:
  // the activations' scale bytes stay)
  unsigned char *const red_mem = PERSIST ? smem + (w_ins + a_ins) * 256 : smem;

  auto load_scales = [&](int i0, int i1, const __amdgpu_buffer_rsrc_t ws_rs) {
    for (int i = i0 + wave; i < i1; i += WAVES) {
      const bool is_w = i < w_ins;
      const int j = (is_w ? i : i - w_ins) * 64 + lane;
      const int row = j / pd, col = j - row * pd;
      const bool ok = col < sdw && row < (is_w ? 16 * NS : 16 * MT);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(is_w ? ws_rs : as_rsrc, LDSP(smem + i * 256), 4,
                                               ok ? row * srow_bytes + col * 4 : OOB_VOFF, 0, 0, 0);
    }
  };
  // the activation codes of the k-steps of the trip that starts at line pair p0_
#define TORQ_LOAD_A(DST_, P0_)                                                                    \
  _Pragma("unroll") for (int u = 0; u < 2 * PT; ++u) {                                            \
    const int ks = 2 * ((P0_) + (u >> 1) * WAVES) + (u & 1);                                      \
    const bool in = ks < KS;                                                                      \
    _Pragma("unroll") for (int t = 0; t < MT; ++t)                                                \
        DST_[u][t] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, in ? c_voff : OOB_VOFF,        \
                                                           in ? ks * 64 + t * 16 * row_bytes : 0, 0); \
  }
  u32x4 aq_keep[PERSIST ? 2 * PT : 1][MT];
  if constexpr (PERSIST) {
    load_scales(w_ins, w_ins + a_ins, as_rsrc);
    TORQ_LOAD_A(aq_keep, wave)
  }

  const int64_t groups = (N + 16 * NS - 1) / (16 * NS);
  for (int64_t grp = blockIdx.x; grp < groups; grp += gridDim.x) {   // one group unless PERSIST
    const int64_t n0 = grp * 16 * NS;
    const int rows_w = (N - n0 < 16 * NS) ? (int)(N - n0) : 16 * NS;
    // rows past N or M are outside the buffers: their loads deliver zeros
    const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(W_q + n0 * row_bytes, (uint32_t)rows_w * row_bytes);
    const __amdgpu_buffer_rsrc_t ws_rsrc = make_rsrc(W_s + n0 * srow_bytes, (uint32_t)rows_w * srow_bytes);
    load_scales(0, PERSIST ? w_ins : w_ins + a_ins, ws_rsrc);

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
      u32x4 wq[2 * PT][NS], aq_trip[PERSIST ? 1 : 2 * PT][MT];
#pragma unroll
      for (int u = 0; u < 2 * PT; ++u) {
        const int ks = 2 * (p0 + (u >> 1) * WAVES) + (u & 1);
        const bool in = ks < KS;
        const int cv = in ? c_voff : OOB_VOFF;
        const int co = in ? ks * 64 : 0;
#pragma unroll
        for (int n = 0; n < NS; ++n)
          wq[u][n] = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, cv, co + (in ? n * 16 * row_bytes : 0), 0);
      }
      if constexpr (!PERSIST) { TORQ_LOAD_A(aq_trip, p0) }
      __builtin_amdgcn_sched_barrier(0);           // every load of the trip is in flight before the first wait
      if (first) {
        __syncthreads();                           // the scales are in LDS
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
          for (int t = 0; t < MT; ++t) {
            const u32x4 av = PERSIST ? aq_keep[PERSIST ? u : 0][t] : aq_trip[PERSIST ? 0 : u][t];
            acc[n][t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                i32x8{(int)wq[u][n][0], (int)wq[u][n][1], (int)wq[u][n][2], (int)wq[u][n][3], 0, 0, 0, 0},
                i32x8{(int)av[0], (int)av[1], (int)av[2], (int)av[3], 0, 0, 0, 0},
                acc[n][t], 4, 4, 0, wsc, 0, asc[t]);
          }
        }
      }
    }
    if (first) __syncthreads();                    // a wave without any pair still meets the others

    skinny_reduce_store<MT, NS>(acc, red_mem, out, M, N, n0, wave, lane);
    // PERSIST: the next group's scale bytes replace this group's, which every wave has read (first
    // barrier of the reduction); its partial tiles replace these once the adding waves have
    // arrived at the next group's barrier
  }
#undef TORQ_LOAD_A
}

// One lane of a consumer workgroup that is done with ctr[0] (see torq_linear_decode_kernel).
__device__ __forceinline__ void decode_consumer_done(unsigned *ctr, int gid, int groups) {
  const int stripes = groups < 64 ? groups : 64;
  const int s = gid % stripes;
  const unsigned quota = (unsigned)((groups - s + stripes - 1) / stripes);    // workgroups with gid % stripes == s
  const unsigned mine = __hip_atomic_fetch_add(&ctr[32 * (1 + s)], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (mine != quota - 1u) return;
  const unsigned full = __hip_atomic_fetch_add(&ctr[32 * 65], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (full != (unsigned)stripes - 1u) return;
  __hip_atomic_store(&ctr[0], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (int i = 0; i < stripes; ++i) __hip_atomic_store(&ctr[32 * (1 + i)], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(&ctr[32 * 65], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (int i = 0; i < 64; ++i) __hip_atomic_store(&ctr[32 * (66 + i)], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---------------------------------------------------------------------------------------------
// torq_linear_single_launch: torq_linear for decode sizes in ONE launch (Algorithm 3, steps 1-4 and
// "Return").  With a few
// rows, rotate + quantise is a latency of 4-5 us in front of a GEMM of 4-30 us; here it runs in the
// first P workgroups of the GEMM's own launch (rotate32_resident, one token-group each: the codes are
// torq_rotate_quantize's, bit for bit) while
// the others, one per weight strip as in mxfp4_gemm_skinny_kernel, already have their scale bytes and
// the first trip of their weight codes on the way.  The two meet at counters in device memory
// (DECODE_CTR_WORDS words, one counter per 128-byte line: read-modify-writes of one address from
// the whole device take about 80 ns each, one after the other):
//   ctr[0]                   producers done: each adds 1 once its codes and scales (stored through to
//                            device-coherent memory) have been acknowledged; the last one raises
//   ctr[32 (66 + s)], s < 64  "ready", 64 copies: consumer g polls copy g % 64, so that no address is
//                            polled by more than 1/64 of the workgroups (thousands of polls on one
//                            address delay the producers' own updates of it);
//   ctr[32 (1 + s)], s < 64   consumers finished, striped the same way; a complete stripe adds 1 to
//   ctr[32 * 65]             stripes complete; the workgroup that completes the last one sets every
//                            counter back to 0, so that the next launch (and every replay of a
//                            captured one) starts from the same state;
//   ctr[DECODE_ERR]          "a workgroup gave up": set by a consumer whose bounded wait ran out, never
//                            cleared by a launch.  Such a consumer does not count itself as finished, so
//                            the counters are not set back either (late producers may still be adding to
//                            them); every consumer of every later launch sees the word first and writes
//                            NaN instead of multiplying whatever the stale counters would let through,
//                            until decode_ctr_reset_kernel has cleared all words.
// The consumers read the activations with device-coherent loads (sc1), so neither side needs a
// cache write-back or invalidate.
// Workgroups are dispatched in index order and the producers come first, so a waiting consumer can
// never keep a producer off the machine; the wait is bounded all the same (a consumer that gives
// up writes NaN to its outputs and raises the sticky error word).  Launches that share a handle's
// counters must not overlap.
template <int MT, int NS, int PT>
__global__ void __launch_bounds__(64 * WAVES, 4)
torq_linear_decode_kernel(const uint4 *__restrict__ x, int64_t TG, const uint4 *__restrict__ inter_hi,
                          const uint4 *__restrict__ inter_lo, const uint4 *__restrict__ intra_hi_frag,
                          const uint4 *__restrict__ intra_lo_frag, uint8_t *__restrict__ A_q,
                          uint8_t *__restrict__ A_s, const uint8_t *__restrict__ W_q,
                          const uint8_t *__restrict__ W_s, uint16_t *__restrict__ out, int M, int64_t N, int d,
                          int P, int groups, unsigned *__restrict__ ctr, int spin_limit, int raise_ready) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  if ((int)blockIdx.x < P) {
    {
      // codes and scale bytes are stored through to device-coherent memory (what an atomic store of device
      // scope does), for the readers in the other workgroups of this launch
      struct CoherentSink {
        unsigned long long *codes;
        uint8_t *scales;
        int64_t first_block;
        __device__ __forceinline__ void operator()(int64_t blk, int h, uint2 packed, uint32_t byte) const {
          const int64_t b = first_block + blk;
          __hip_atomic_store(&codes[b * 2 + h], ((unsigned long long)packed.y << 32) | packed.x, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
          if (h == 0) __hip_atomic_store(&scales[b], (uint8_t)byte, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      } sink{reinterpret_cast<unsigned long long *>(A_q), A_s, (int64_t)blockIdx.x * 128};
      rotate32_resident(x + (int64_t)blockIdx.x * 512, 1, 128, inter_hi, inter_lo, intra_hi_frag, intra_lo_frag,
                        reinterpret_cast<char *>(smem), sink, []() {});
    }
    __builtin_amdgcn_s_waitcnt(0);                 // this lane's stores have been acknowledged
    __syncthreads();
    if (tid == 0) {
      const unsigned before = __hip_atomic_fetch_add(&ctr[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (before == (unsigned)P - 1u && raise_ready)   // every producer's stores were complete before its own add
        for (int s = 0; s < 64; ++s) __hip_atomic_store(&ctr[32 * (66 + s)], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return;
  }
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r16 = lane & 15, q = lane >> 4;
  const int row_bytes = d / 2, srow_bytes = d / 32;
  const int KS = d / 128;
  const int KP = (KS + 1) / 2;
  const int64_t n0 = (int64_t)((int)blockIdx.x - P) * 16 * NS;
  const int rows_w = (N - n0 < 16 * NS) ? (int)(N - n0) : 16 * NS;
  const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(W_q + n0 * row_bytes, (uint32_t)rows_w * row_bytes);
  const __amdgpu_buffer_rsrc_t ws_rsrc = make_rsrc(W_s + n0 * srow_bytes, (uint32_t)rows_w * srow_bytes);
  const __amdgpu_buffer_rsrc_t a_rsrc = make_rsrc(A_q, (uint32_t)M * row_bytes);
  const __amdgpu_buffer_rsrc_t as_rsrc = make_rsrc(A_s, (uint32_t)M * srow_bytes);
  const int c_voff = r16 * row_bytes + q * 16;
  const int sdw = srow_bytes / 4, pd = sdw + 1;
  const int w_ins = (16 * NS * pd + 63) / 64, a_ins = (16 * MT * pd + 63) / 64;
  const int ws_off = r16 * pd * 4 + q;
  const int as_off = w_ins * 256 + r16 * pd * 4 + q;

  // ---- the weight side goes out first: scale bytes to LDS, the first trip's codes to registers
  for (int i = wave; i < w_ins; i += WAVES) {
    const int j = i * 64 + lane;
    const int row = j / pd, col = j - row * pd;
    const bool ok = col < sdw && row < 16 * NS;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(ws_rsrc, LDSP(smem + i * 256), 4, ok ? row * srow_bytes + col * 4 : OOB_VOFF, 0, 0, 0);
  }
  u32x4 wq[2 * PT][NS], aq[2 * PT][MT];
  // AUX_: cache policy of the load; 16 = sc1, a device-coherent read
#define TORQ_LOAD_TRIP(DST_, RSRC_, CNT_, P0_, AUX_)                                             \
  _Pragma("unroll") for (int u = 0; u < 2 * PT; ++u) {                                           \
    const int ks = 2 * ((P0_) + (u >> 1) * WAVES) + (u & 1);                                     \
    const bool in = ks < KS;                                                                     \
    _Pragma("unroll") for (int n = 0; n < CNT_; ++n)                                             \
        DST_[u][n] = __builtin_amdgcn_raw_buffer_load_b128(RSRC_, in ? c_voff : OOB_VOFF,        \
                                                           in ? ks * 64 + n * 16 * row_bytes : 0, AUX_); \
  }
  int p0 = wave;
  if (p0 < KP) { TORQ_LOAD_TRIP(wq, w_rsrc, NS, p0, 0) }
  __builtin_amdgcn_sched_barrier(0);

  // ---- wait for the activations' codes and scales
  if (tid == 0) {
    const unsigned *flag = &ctr[32 * (66 + (((int)blockIdx.x - P) & 63))];
    // an earlier launch on these counters gave up: they are stale, nothing they say can be trusted
    const unsigned err = __hip_atomic_load(&ctr[DECODE_ERR], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned seen = 0;
    if (!err) {
      for (int spin = 0; spin < spin_limit; ++spin) {
        seen = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (seen) break;
        __builtin_amdgcn_s_sleep(8);
      }
      if (!seen) __hip_atomic_store(&ctr[DECODE_ERR], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    reinterpret_cast<volatile unsigned *>(smem)[(w_ins + a_ins) * 64] = seen;
  }
  __syncthreads();
  const bool ready = reinterpret_cast<volatile unsigned *>(smem)[(w_ins + a_ins) * 64] != 0;
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("" ::: "memory");                   // nothing below is moved above the wait
  if (!ready) {                                    // uniform over the workgroup
    __builtin_amdgcn_s_waitcnt(0);                 // the loads already issued land before the workgroup's LDS and registers go
    // gave up (or the counters are stale): mark this strip's outputs as NaN rather than leave what the
    // buffer held; the workgroup does not count as finished, so no launch sets the counters back
    for (int e = tid; e < M * 16 * NS; e += 64 * WAVES) {
      const int m = e / (16 * NS);
      const int64_t n = n0 + e % (16 * NS);
      if (n < N) out[(int64_t)m * N + n] = 0x7FC0;
    }
    return;
  }

  for (int i = w_ins + wave; i < w_ins + a_ins; i += WAVES) {
    const int j = (i - w_ins) * 64 + lane;
    const int row = j / pd, col = j - row * pd;
    const bool ok = col < sdw && row < 16 * MT;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(as_rsrc, LDSP(smem + i * 256), 4, ok ? row * srow_bytes + col * 4 : OOB_VOFF, 0, 0, 16);
  }

  f32x4 acc[NS][MT];
#pragma unroll
  for (int n = 0; n < NS; ++n)
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[n][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  bool first = true;
  for (; p0 < KP; p0 += PT * WAVES) {
    if (!first) { TORQ_LOAD_TRIP(wq, w_rsrc, NS, p0, 0) }
    TORQ_LOAD_TRIP(aq, a_rsrc, MT, p0, 16)
    __builtin_amdgcn_sched_barrier(0);
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
#undef TORQ_LOAD_TRIP
  if (first) __syncthreads();                      // a wave without any pair still meets the others

  skinny_reduce_store<MT, NS>(acc, smem, out, M, N, n0, wave, lane);
  if (tid == 0) decode_consumer_done(ctr, (int)blockIdx.x - P, groups);
}

// ---------------------------------------------------------------------------------------------
// torq_linear for a few token-groups (one to four rows of a decode step) with the packed activations
// never leaving the chip: Algorithm 3, steps 1-4 and "Return", in one launch and without any hand-off
// between workgroups.  Every workgroup rotates and quantises ALL token-groups itself (rotate32_resident
// on its 8 waves, G = 112 or 128: 2.9 MFLOP per token-group, well under a microsecond) into its own LDS while the
// scale bytes and the first trip of weight codes of its first strips are on the way, and then
// streams its share of the weight strips as mxfp4_gemm_skinny_kernel<1, NS, PT, true> does, with the
// activation operand read from LDS instead of from memory.  Workgroups are persistent (the rotation is
// paid once per workgroup, not once per strip).  Workgroup 0 also stores the codes and scale bytes to
// A_q / A_s (the caller's workspace, same layout as torq_rotate_quantize), which nothing in the launch
// reads: they are what was multiplied, for the caller to inspect.
//
// One trip of a wave holds 2 PT k-steps of NS strips in registers (32 PT NS bytes per lane); the launcher
// picks NS and PT so that, where 128 registers allow, one trip is the workgroup's whole share: then every
// weight byte of the launch is requested before the rotation starts, and the rotation's latency (two
// dependent reads from memory and a chain of 22 MFMAs) hides behind the stream.
//
// LDS: [weight-strip scales | activation scales (16 rows, zero beyond M) | codes, M rows of d / 2 + 16
// bytes (the pad spreads the rows over the banks) | the token-groups' bf16 values (8 KiB each), later
// the partial tiles of the reduction (8 NS KiB)].
namespace {
struct LocalSink {
  unsigned char *a_c, *s_a;
  int a_stride, s_stride, bpr;        // bytes per code row / scale row in LDS; blocks per activation row
  uint2 *codes_g;                     // workgroup 0: the copy in device memory, else nullptr
  uint8_t *scales_g;
  __device__ __forceinline__ void operator()(int64_t blk, int h, uint2 packed, uint32_t byte) const {
    const int b = (int)blk, row = b / bpr, bk = b - row * bpr;
    *reinterpret_cast<uint2 *>(a_c + row * a_stride + bk * 16 + h * 8) = packed;
    if (h == 0) s_a[row * s_stride + bk] = (unsigned char)byte;
    if (codes_g) {
      codes_g[blk * 2 + h] = packed;
      if (h == 0) scales_g[blk] = (uint8_t)byte;
    }
  }
};
}  // namespace

// The end of torq_linear_local_kernel: as skinny_reduce_store for one activation tile, but with wave n
// adding strip n (every wave's partial tile goes through LDS, red_mem = 8 NS KiB): with up to four
// strips per workgroup one wave would add 112 values per lane while seven wait.  Same order of additions
// (wave 0 + 1 + ... + 7): the same bits.
template <int NS>
__device__ __forceinline__ void local_reduce_store(f32x4 (&acc)[NS][1], unsigned char *red_mem, uint16_t *__restrict__ out,
                                                   int M, int64_t N, int64_t n0, int wave, int lane) {
  const int r16 = lane & 15, q = lane >> 4;
  __syncthreads();                                 // everybody is done with the scales and the codes
  float *red = reinterpret_cast<float *>(red_mem); // [WAVES][NS][4][64]
#pragma unroll
  for (int n = 0; n < NS; ++n)
#pragma unroll
    for (int r = 0; r < 4; ++r) red[((wave * NS + n) * 4 + r) * 64 + lane] = acc[n][0][r];
  __syncthreads();
  if (wave < NS) {
    const int n = wave;
    const int64_t nn = n0 + n * 16 + 4 * q;
    bf16x4 v;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float sum = red[(n * 4 + r) * 64 + lane];
#pragma unroll
      for (int w = 1; w < WAVES; ++w) sum += red[((w * NS + n) * 4 + r) * 64 + lane];
      v[r] = (__bf16)sum;
    }
    if (r16 < M) {
      uint16_t *dst = out + (int64_t)r16 * N + nn;
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

// EXACT: d / 256 == PT * WAVES, one trip is the k range with no k-step past the end: its loads then need
// no range predicate, compile to straight-line code, and the compiler's count of them is exact.
template <int NS, int PT, bool EXACT>
__global__ void __launch_bounds__(64 * WAVES, 2)
torq_linear_local_kernel(const uint4 *__restrict__ x, int TG, int G, const uint4 *__restrict__ inter_hi,
                         const uint4 *__restrict__ inter_lo, const uint4 *__restrict__ intra_hi_frag,
                         const uint4 *__restrict__ intra_lo_frag, uint8_t *__restrict__ A_q,
                         uint8_t *__restrict__ A_s, const uint8_t *__restrict__ W_q,
                         const uint8_t *__restrict__ W_s, uint16_t *__restrict__ out, int M, int64_t N, int d) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r16 = lane & 15, q = lane >> 4;
  const int row_bytes = d / 2, srow_bytes = d / 32;
  const int KS = d / 128;
  const int KP = (KS + 1) / 2;
  const int c_voff = r16 * row_bytes + q * 16;
  const int sdw = srow_bytes / 4, pd = sdw + 1;
  const int w_ins = (16 * NS * pd + 63) / 64, a_ins = (16 * pd + 63) / 64;
  const int ws_off = r16 * pd * 4 + q;
  const int as_off = w_ins * 256 + r16 * pd * 4 + q;
  const int a_stride = row_bytes + 16;
  unsigned char *const s_a = smem + w_ins * 256;
  unsigned char *const a_c = smem + (w_ins + a_ins) * 256;
  unsigned char *const xs = a_c + (M * a_stride + 255) / 256 * 256;     // TG token-groups, then partial tiles

  const int64_t groups = (N + 16 * NS - 1) / (16 * NS);
  auto load_w_scales = [&](const __amdgpu_buffer_rsrc_t ws_rs) {
    for (int i = wave; i < w_ins; i += WAVES) {
      const int j = i * 64 + lane;
      const int row = j / pd, col = j - row * pd;
      const bool ok = col < sdw && row < 16 * NS;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(ws_rs, LDSP(smem + i * 256), 4, ok ? row * srow_bytes + col * 4 : OOB_VOFF, 0, 0, 0);
    }
  };
  u32x4 wq[2 * PT][NS];
#define TORQ_LOAD_W(RSRC_, P0_)                                                                   \
  _Pragma("unroll") for (int u = 0; u < 2 * PT; ++u) {                                            \
    const int ks = 2 * ((P0_) + (u >> 1) * WAVES) + (u & 1);                                      \
    const bool in = EXACT || ks < KS;                                                             \
    _Pragma("unroll") for (int n = 0; n < NS; ++n)                                                \
        wq[u][n] = __builtin_amdgcn_raw_buffer_load_b128(RSRC_, in ? c_voff : OOB_VOFF,           \
                                                         in ? ks * 64 + n * 16 * row_bytes : 0, 0); \
  }

  // ---- steps 1-4 into LDS.  The rotation's own reads from memory are requested first and the first
  // trip's weight codes right behind them (reads return in order: the rotation must not queue behind
  // the weights); the scale bytes of the rows past M are zeros
  for (int i = tid; i < a_ins * 64; i += 64 * WAVES) reinterpret_cast<uint32_t *>(s_a)[i] = 0u;
  {
    LocalSink sink;
    sink.a_c = a_c;
    sink.s_a = s_a;
    sink.a_stride = a_stride;
    sink.s_stride = pd * 4;
    sink.bpr = srow_bytes;
    sink.codes_g = blockIdx.x == 0 ? reinterpret_cast<uint2 *>(A_q) : nullptr;
    sink.scales_g = A_s;
    const int64_t n0 = (int64_t)blockIdx.x * 16 * NS;
    const int rows_w = (N - n0 < 16 * NS) ? (int)(N - n0) : 16 * NS;
    load_w_scales(make_rsrc(W_s + n0 * srow_bytes, (uint32_t)rows_w * srow_bytes));   // few bytes, ahead of everything
    const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(W_q + n0 * row_bytes, (uint32_t)rows_w * row_bytes);
    auto weights_first_trip = [&]() {
      // The waves meet (nothing is waited for) so that every wave's rotation reads are in the CU's
      // memory pipeline before any wave's weight reads: the pipeline takes requests in order, and a
      // later wave's 5 KB for the rotation would otherwise queue behind 16 KB of weights per earlier wave.
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      if (EXACT || wave < KP) { TORQ_LOAD_W(w_rsrc, wave) }
      __builtin_amdgcn_sched_barrier(0);
    };
    // (two barriers inside: the first also orders the clearing above before any scale byte, the second
    // makes the results visible)
    rotate32_resident(x, TG, G, inter_hi, inter_lo, intra_hi_frag, intra_lo_frag, reinterpret_cast<char *>(xs), sink,
                      weights_first_trip);
  }

  // ---- the strip groups of this workgroup
  bool preloaded = true;
  for (int64_t grp = blockIdx.x; grp < groups; grp += gridDim.x) {
    const int64_t n0 = grp * 16 * NS;
    const int rows_w = (N - n0 < 16 * NS) ? (int)(N - n0) : 16 * NS;
    const __amdgpu_buffer_rsrc_t w_rsrc = make_rsrc(W_q + n0 * row_bytes, (uint32_t)rows_w * row_bytes);
    if (!preloaded) load_w_scales(make_rsrc(W_s + n0 * srow_bytes, (uint32_t)rows_w * srow_bytes));

    f32x4 acc[NS][1];
#pragma unroll
    for (int n = 0; n < NS; ++n) acc[n][0] = f32x4{0.f, 0.f, 0.f, 0.f};

    bool first = true;
    for (int p0 = wave; p0 < KP; p0 += PT * WAVES) {
      if (!(preloaded && first)) { TORQ_LOAD_W(w_rsrc, p0) }
      u32x4 aq[2 * PT];
#pragma unroll
      for (int u = 0; u < 2 * PT; ++u) {
        const int ks = 2 * (p0 + (u >> 1) * WAVES) + (u & 1);
        aq[u] = ((EXACT || ks < KS) && r16 < M) ? *reinterpret_cast<const u32x4 *>(a_c + r16 * a_stride + ks * 64 + q * 16)
                                     : u32x4{0u, 0u, 0u, 0u};
      }
      __builtin_amdgcn_sched_barrier(0);
      if (first) {
        __syncthreads();                           // the strip's scale bytes are in LDS
        first = false;
      }
#pragma unroll
      for (int u = 0; u < 2 * PT; ++u) {
        const int ks = 2 * (p0 + (u >> 1) * WAVES) + (u & 1);
        const int sb = ((EXACT || ks < KS) ? ks : 0) * 4;
        const int asc = smem[as_off + sb];
#pragma unroll
        for (int n = 0; n < NS; ++n) {
          const int wsc = smem[ws_off + n * 16 * pd * 4 + sb];
          acc[n][0] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
              i32x8{(int)wq[u][n][0], (int)wq[u][n][1], (int)wq[u][n][2], (int)wq[u][n][3], 0, 0, 0, 0},
              i32x8{(int)aq[u][0], (int)aq[u][1], (int)aq[u][2], (int)aq[u][3], 0, 0, 0, 0},
              acc[n][0], 4, 4, 0, wsc, 0, asc);
        }
      }
    }
    if (first) __syncthreads();                    // a wave without any pair still meets the others
    preloaded = false;

    // the partial tiles go where the rotation staged its input; the next group's scale bytes replace
    // this group's once every wave has read them (first barrier of the reduction), and its partial tiles
    // these once the adding waves have arrived at the next group's barrier
    local_reduce_store<NS>(acc, xs, out, M, N, n0, wave, lane);
  }
#undef TORQ_LOAD_W
}

template <int MT, int NS, int PT>
static hipError_t launch_cfg(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                             void *out, int64_t M, int64_t N, int d, hipStream_t stream, const DecodeArgs *fused) {
  const int64_t groups = (N + 16 * NS - 1) / (16 * NS);
  if (groups > 0x7FFFFFF0) return hipErrorInvalidValue;
  const int pd = d / 128 + 1;                      // padded dwords per scale row
  const size_t scale_bytes = (size_t)((16 * NS * pd + 63) / 64 + (16 * MT * pd + 63) / 64) * 256;
  const size_t red_bytes = (size_t)WAVES * NS * MT * 4 * 64 * sizeof(float);
  size_t lds_bytes = scale_bytes > red_bytes ? scale_bytes : red_bytes;
  if (fused) {
    // + the "ready" word behind the scales; at least the rotation's four token-group places
    lds_bytes = lds_bytes > scale_bytes + 16 ? lds_bytes : scale_bytes + 16;
    const size_t rot_bytes = 4 * (size_t)RotCfg<4>::TG_LDS_BYTES;
    lds_bytes = lds_bytes > rot_bytes ? lds_bytes : rot_bytes;
    if (lds_bytes > SKINNY_MAX_LDS) return hipErrorInvalidValue;
    if (lds_bytes > 64 * 1024) {
      static bool raised_fused = false;
      if (!raised_fused) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(torq_linear_decode_kernel<MT, NS, PT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)SKINNY_MAX_LDS);
        if (e != hipSuccess) return e;
        raised_fused = true;
      }
    }
    hipLaunchKernelGGL((torq_linear_decode_kernel<MT, NS, PT>), dim3((unsigned)(groups + fused->P)), dim3(64 * WAVES),
                       lds_bytes, stream, fused->x, fused->TG, fused->inter_hi, fused->inter_lo, fused->intra_hi_frag,
                       fused->intra_lo_frag, fused->A_q, fused->A_s, W_q, W_s, reinterpret_cast<uint16_t *>(out), (int)M,
                       N, d, fused->P, (int)groups, fused->ctr, fused->spin_limit, fused->raise_ready);
    return hipGetLastError();
  }
  // The persistent form (activation codes loaded once per workgroup and kept in registers): 8 - 16 rows,
  // one trip over the k range, and weights enough for the re-reads to cost more than the parallelism
  // given up (measured: [16, 8192] x 28672 34.2 -> 28.4 us, [8, 8192] x 28672 32.2 -> 27.4,
  // [16, 8192] x 8192 10.7 -> 9.7, [16, 4096] x 14336 9.2 -> 9.0; below 24 MB of weights it loses).  Each
  // workgroup takes `per` groups, the smallest power of two that leaves at most 256 workgroups (one per CU,
  // evenly loaded: 3 or 7 groups per workgroup measured 15 - 20 % slower than 4, and half as many
  // workgroups as CUs 30 % slower than one each).
  const int KP = (d / 128 + 1) / 2;
  const size_t p_bytes = scale_bytes + red_bytes;
  if (MT == 1 && M >= 8 && KP <= PT * WAVES && (double)N * (double)d * 0.53125 >= 24e6 && p_bytes <= 64 * 1024) {
    int64_t per = 1;
    while ((groups + per - 1) / per > 256) per *= 2;
    if (per > 1) {
      const int64_t grid = (groups + per - 1) / per;
      hipLaunchKernelGGL((mxfp4_gemm_skinny_kernel<MT, NS, PT, true>), dim3((unsigned)grid), dim3(64 * WAVES), p_bytes,
                         stream, A_q, A_s, W_q, W_s, reinterpret_cast<uint16_t *>(out), (int)M, N, d);
      return hipGetLastError();
    }
  }
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
                               void *out, int64_t M, int64_t N, int d, hipStream_t stream, const DecodeArgs *fused) {
  // trip depth: as deep as the k range of a wave goes, at most 4 line pairs (8 k-steps) in flight
  // (2 when the operand registers of a trip would not leave room for several workgroups per CU)
  const int pairs_per_wave = ((d / 128 + 1) / 2 + WAVES - 1) / WAVES;
  if (pairs_per_wave <= 1) return launch_cfg<MT, NS, 1>(A_q, A_s, W_q, W_s, out, M, N, d, stream, fused);
  if (pairs_per_wave <= 2) return launch_cfg<MT, NS, 2>(A_q, A_s, W_q, W_s, out, M, N, d, stream, fused);
  return launch_cfg<MT, NS, (MT + NS <= 3 ? 4 : 2)>(A_q, A_s, W_q, W_s, out, M, N, d, stream, fused);
}

template <int MT>
static hipError_t launch_mt(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                            void *out, int64_t M, int64_t N, int d, hipStream_t stream, const DecodeArgs *fused) {
  // Two strips per workgroup share the activation loads.  That pays when the activations are
  // real traffic (not a row or two) and there are still enough workgroups to keep every CU
  // streaming; deeper sharing costs more in registers (fewer loads in flight) than it saves.
  const int64_t strips = (N + 15) / 16;
  if (MT <= 2 && M >= 8 && strips >= 2 * SKINNY_MIN_GROUPS)
    return launch_mt_ns<MT, (MT <= 2 ? 2 : 1)>(A_q, A_s, W_q, W_s, out, M, N, d, stream, fused);
  return launch_mt_ns<MT, 1>(A_q, A_s, W_q, W_s, out, M, N, d, stream, fused);
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
static hipError_t launch_by_rows(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                                 void *out, int64_t M, int64_t N, int d, hipStream_t stream, const DecodeArgs *fused) {
  switch ((M + 15) / 16) {
    case 1: return launch_mt<1>(A_q, A_s, W_q, W_s, out, M, N, d, stream, fused);
    case 2: return launch_mt<2>(A_q, A_s, W_q, W_s, out, M, N, d, stream, fused);
    case 3: return launch_mt<3>(A_q, A_s, W_q, W_s, out, M, N, d, stream, fused);
    case 4: return launch_mt<4>(A_q, A_s, W_q, W_s, out, M, N, d, stream, fused);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_mxfp4_gemm_skinny(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q,
                                    const uint8_t *W_s, void *out, int64_t M, int64_t N, int d,
                                    hipStream_t stream) {
  return launch_by_rows(A_q, A_s, W_q, W_s, out, M, N, d, stream, nullptr);
}

// torq_linear in one launch (torq_linear_single_launch); the caller has checked G = 128, a dense R_inter,
// 1 <= M <= 64, mxfp4_gemm_skinny_fits(M, r->d) and N > 0.  A_q / A_s: the workspace's code and scale areas.
hipError_t launch_torq_linear_decode(const torq_rotation *r, const void *x_bf16, uint8_t *A_q, uint8_t *A_s,
                                     const uint8_t *W_q, const uint8_t *W_s, void *out, int64_t M, int64_t N,
                                     int spin_limit, int raise_ready, hipStream_t stream) {
  DecodeArgs fz;
  fz.x = reinterpret_cast<const uint4 *>(x_bf16);
  fz.TG = M * (int64_t)(r->d / 32 / r->G);
  fz.inter_hi = reinterpret_cast<const uint4 *>(r->inter32f_hi);
  fz.inter_lo = reinterpret_cast<const uint4 *>(r->inter32f_lo);
  fz.intra_hi_frag = reinterpret_cast<const uint4 *>(r->intra32_hi);
  fz.intra_lo_frag = reinterpret_cast<const uint4 *>(r->intra32_lo);
  fz.A_q = A_q;
  fz.A_s = A_s;
  fz.P = (int)fz.TG;                               // one token-group per rotating workgroup
  fz.ctr = r->decode_ctr;
  fz.spin_limit = spin_limit;
  fz.raise_ready = raise_ready;
  return launch_by_rows(A_q, A_s, W_q, W_s, out, M, N, r->d, stream, &fz);
}

// torq_linear with the activations rotated and quantised inside every workgroup (torq_linear_local_kernel).
// Preconditions (torq_linear_local_fits): dense R_inter with 96 < G <= 128, at most LOCAL_MAX_TG
// token-groups in all, d a multiple of 128, and LDS for one strip per workgroup.
static size_t local_lds_bytes(int64_t M, int d, int NS) {
  const int pd = d / 128 + 1;
  const size_t red = (size_t)WAVES * NS * 4 * 64 * sizeof(float), rot = LOCAL_MAX_TG * (size_t)RotCfg<4>::TG_LDS_BYTES;
  return (size_t)((16 * NS * pd + 63) / 64 + (16 * pd + 63) / 64) * 256 + ((size_t)M * (d / 2 + 16) + 255) / 256 * 256 +
         (red > rot ? red : rot);
}

bool torq_linear_local_fits(const torq_rotation *r, int64_t M) {
  if (r->butterfly || r->G <= 96 || r->G > 128 || r->G % 16 != 0 || r->d % 128 != 0) return false;
  if (M < 1 || M > 16) return false;
  if (M * (int64_t)(r->d / 32 / r->G) > LOCAL_MAX_TG) return false;
  return (r->d / 128 + 1) / 2 <= 8 * WAVES * 4 && local_lds_bytes(M, r->d, 1) <= 64 * 1024;
}

// Where the one-launch form is the faster way through torq_linear, measured against rotate + quantise
// followed by the GEMM as HIP-graph replays over weight copies of 600 MB in all (weights from HBM, as in a
// model; with six copies of a 31 MB layer the 256 MB Infinity Cache held them, and the form seemed to pay up
// to 48 MB): one or two token-groups up to 20 MB of packed weights, three or four up to 16 MB.  One launch
// against two, us: [1, 4096] x 1024 5.9 / 7.3, x 4096 6.2 / 7.7, x 8192 8.3 / 9.0, x 11008 11.2 / 10.2,
// x 14336 11.4 / 11.6; [1, 8192] x 4096 8.6 / 9.6, x 8192 12.1 / 12.1; [4, 4096] x 4096 7.9 / 8.0, x 6144
// 9.1 / 9.3, x 8192 10.0 / 9.4, x 14336 12.8 / 12.2; [2, 8192] x 2048 8.7 / 9.1, x 4096 10.1 / 9.7;
// [1, 14336] x 2048 (G = 112) 10.7 / 11.9, x 4096 12.4 / 12.6; [1, 8192] x 28672 (125 MB): 30.1 / 28.7.
bool torq_linear_local_pays(const torq_rotation *r, int64_t M, int64_t N) {
  if (!torq_linear_local_fits(r, M) || N <= 0) return false;
  const int64_t token_groups = M * (int64_t)(r->d / 32 / r->G);
  return (double)N * (double)r->d * 0.53125 <= (token_groups <= 2 ? 20e6 : 16e6);
}

template <int NS, int PT>
static hipError_t launch_local_cfg(const torq_rotation *r, const void *x_bf16, uint8_t *A_q, uint8_t *A_s,
                                   const uint8_t *W_q, const uint8_t *W_s, void *out, int64_t M, int64_t N,
                                   hipStream_t stream) {
  const int d = r->d;
  const int64_t groups = (N + 16 * NS - 1) / (16 * NS);
  // as for the persistent GEMM: the smallest power of two of groups per workgroup that leaves at most
  // 256 workgroups, so that every workgroup has the same share
  int64_t per = 1;
  while ((groups + per - 1) / per > 256) per *= 2;
  const int64_t grid = (groups + per - 1) / per;
  const bool exact = d % 256 == 0 && d / 256 == PT * WAVES;
  auto kernel = exact ? torq_linear_local_kernel<NS, PT, true> : torq_linear_local_kernel<NS, PT, false>;
  hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(64 * WAVES), local_lds_bytes(M, d, NS), stream,
                     reinterpret_cast<const uint4 *>(x_bf16), (int)(M * (int64_t)(d / 32 / r->G)), r->G,
                     reinterpret_cast<const uint4 *>(r->inter32f_hi), reinterpret_cast<const uint4 *>(r->inter32f_lo),
                     reinterpret_cast<const uint4 *>(r->intra32_hi),
                     reinterpret_cast<const uint4 *>(r->intra32_lo), A_q, A_s, W_q, W_s,
                     reinterpret_cast<uint16_t *>(out), (int)M, N, d);
  return hipGetLastError();
}

hipError_t launch_torq_linear_local(const torq_rotation *r, const void *x_bf16, uint8_t *A_q, uint8_t *A_s,
                                    const uint8_t *W_q, const uint8_t *W_s, void *out, int64_t M, int64_t N,
                                    hipStream_t stream) {
  if (!torq_linear_local_fits(r, M) || N <= 0) return hipErrorInvalidValue;
  // PT: the line pairs of a wave, so that one trip covers the k range (at most 8); NS: as many strips per
  // workgroup as leave every CU a workgroup, within the registers (NS PT <= 8: 128 for the weight codes
  // of a trip) and the LDS
  const int pairs_per_wave = ((r->d / 128 + 1) / 2 + WAVES - 1) / WAVES;
  const int PT = pairs_per_wave <= 8 ? pairs_per_wave : 8;
  const int64_t strips = (N + 15) / 16;
  int NS = 1;
  while (NS < 4 && strips > 256 * NS && 2 * NS * PT <= 8 && local_lds_bytes(M, r->d, 2 * NS) <= 64 * 1024) NS *= 2;
#define TORQ_LOCAL_CASE(NS_, PT_) \
  if (NS == NS_ && PT == PT_) return launch_local_cfg<NS_, PT_>(r, x_bf16, A_q, A_s, W_q, W_s, out, M, N, stream);
  TORQ_LOCAL_CASE(1, 1) TORQ_LOCAL_CASE(1, 2) TORQ_LOCAL_CASE(1, 3) TORQ_LOCAL_CASE(1, 4)
  TORQ_LOCAL_CASE(1, 5) TORQ_LOCAL_CASE(1, 6) TORQ_LOCAL_CASE(1, 7) TORQ_LOCAL_CASE(1, 8)
  TORQ_LOCAL_CASE(2, 1) TORQ_LOCAL_CASE(2, 2) TORQ_LOCAL_CASE(2, 3) TORQ_LOCAL_CASE(2, 4)
  TORQ_LOCAL_CASE(4, 1) TORQ_LOCAL_CASE(4, 2)
#undef TORQ_LOCAL_CASE
  return hipErrorInvalidValue;
}

// every counter of a handle back to zero, the error word included (a fill kernel rather than a
// memset node, so that the call may sit in a captured graph)
__global__ void __launch_bounds__(256) decode_ctr_reset_kernel(unsigned *__restrict__ ctr) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < DECODE_CTR_WORDS) ctr[i] = 0u;
}

hipError_t launch_decode_ctr_reset(const torq_rotation *r, hipStream_t stream) {
  hipLaunchKernelGGL(decode_ctr_reset_kernel, dim3((DECODE_CTR_WORDS + 255) / 256), dim3(256), 0, stream, r->decode_ctr);
  return hipGetLastError();
}

}  // namespace torq
