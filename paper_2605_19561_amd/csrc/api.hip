// C-ABI entry points of libtorq: argument validation, the rotation handle, and
// dispatch to the kernel launchers.  The online path computes nothing on the host; the calibration
// entry points that are documented as host routines do.
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "torq_internal.h"

// Scratch of torq_linear_static: the packed activations between its two kernels.  One copy per GPU
// the library runs on, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels get the address that call returns for the current device.
static __device__ __align__(256) unsigned char scratch[TORQ_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::atomic<unsigned char *> g_scratch_ptr[MAX_DEVICES];
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device, looked up once per device.
hipError_t scratch_of_current_device(unsigned char **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  unsigned char *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
    if (!p) {
      void *sym = nullptr;
      e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
      if (e != hipSuccess) return e;
      if (!sym) return hipErrorInvalidSymbol;
      p = static_cast<unsigned char *>(sym);
      g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
  }
  *out = p;
  return hipSuccess;
}

inline bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// fp32 -> bf16 pattern, round to nearest even (host side, for the operand tables)
inline uint16_t to_bf16(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
inline float from_bf16(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}
// v = hi + lo + O(2^-17 |v|) with hi, lo both bf16
inline void split_bf16(float v, uint16_t *hi, uint16_t *lo) {
  *hi = to_bf16(v);
  *lo = to_bf16(v - from_bf16(*hi));
}

template <class T>
hipError_t upload(T **dst, const std::vector<T> &src) {
  hipError_t e = hipMalloc(reinterpret_cast<void **>(dst), src.size() * sizeof(T));
  if (e != hipSuccess) return e;
  return hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice);
}

thread_local char g_hip_msg[256] = "";

int hip_fail(hipError_t e) {
  std::snprintf(g_hip_msg, sizeof g_hip_msg, "HIP runtime error: %s", hipGetErrorString(e));
  return TORQ_EHIP;
}

// Host routines allocate with std::vector; no exception may cross the C boundary.
template <class F>
int guarded(F &&body) noexcept {
  try {
    return body();
  } catch (const std::bad_alloc &) {
    return TORQ_ENOMEM;
  } catch (...) {
    return TORQ_EINVAL;
  }
}

// the dense-matrix kernels, or the butterfly kernel for a handle made by torq_rotation_create_butterfly
hipError_t rotate_any(const torq_rotation *r, const void *x_bf16, int64_t M, int format, float global_scale,
                      uint8_t *codes, uint8_t *scales, float *z_out, hipStream_t stream) {
  return r->butterfly ? torq::launch_rotate_butterfly(r, x_bf16, M, format, global_scale, codes, scales, z_out, stream)
                      : torq::launch_rotate(r, x_bf16, M, format, global_scale, codes, scales, z_out, stream);
}

}  // namespace

extern "C" {

const char *torq_status_string(int status) {
  switch (status) {
    case TORQ_OK: return "ok";
    case TORQ_EINVAL: return "invalid argument (null pointer, negative size, or a dimension the library does not support)";
    case TORQ_EALIGN: return "device pointer not 16-byte aligned";
    case TORQ_EWORKSPACE: return "workspace too small";
    case TORQ_EHIP: return g_hip_msg[0] ? g_hip_msg : "HIP runtime error";
    case TORQ_ENODEVICE: return "no gfx950 device is current";
    case TORQ_ECONVERGE: return "variance equalisation did not converge (Sigma not symmetric, or eps too small)";
    case TORQ_ENOMEM: return "host memory allocation failed";
    case TORQ_ETOOBIG: return "packed activations exceed the library's built-in scratch (TORQ_STATIC_SCRATCH_BYTES); use torq_linear with a workspace";
    default: return "unknown status";
  }
}

static int torq_rotation_create_impl(torq_rotation_t **out, int d, int G, const float *R_inter_host,
                         const float *R_intra_host) {
  if (!out) return TORQ_EINVAL;
  *out = nullptr;
  if (!R_inter_host || !R_intra_host) return TORQ_EINVAL;
  if (d <= 0 || d % TORQ_BLOCK != 0) return TORQ_EINVAL;
  if (G <= 0 || G % 16 != 0 || G > TORQ_MAX_G) return TORQ_EINVAL;
  if ((d / TORQ_BLOCK) % G != 0) return TORQ_EINVAL;

  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return TORQ_ENODEVICE;
  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, dev);
  if (e != hipSuccess) return TORQ_ENODEVICE;
  if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return TORQ_ENODEVICE;

  // R_inter, bf16 hi/lo, [G][KS*32] with zero padding: row b is the B operand
  // "column" b of R_inter^T (Algorithm 3 step 2: Y[b] = sum_b' R_inter[b][b'] X[b']).
  const int KS = (G + 31) / 32;
  const int ld = KS * 32;
  std::vector<uint16_t> ih((size_t)G * ld, 0), il((size_t)G * ld, 0);
  for (int b = 0; b < G; ++b)
    for (int bp = 0; bp < G; ++bp)
      split_bf16(R_inter_host[(size_t)b * G + bp], &ih[(size_t)b * ld + bp], &il[(size_t)b * ld + bp]);

  // R_intra^T as the A operand of v_mfma_f32_16x16x32_bf16 for the two output
  // tiles t: lane (m = l%16, q = l/16), slot j<4 holds R_intra[4q+j][kout] and
  // slot 4+j holds R_intra[16+4q+j][kout] (the k' order in which step 2 leaves Y
  // in its accumulators), with kout = 8*(m/4) + 4t + m%4 so that after step 3 a
  // lane holds eight consecutive output positions.
  std::vector<uint16_t> ah(2 * 64 * 8), al(2 * 64 * 8);
  for (int t = 0; t < 2; ++t)
    for (int l = 0; l < 64; ++l) {
      const int m = l % 16, q = l / 16;
      const int kout = 8 * (m / 4) + 4 * t + (m % 4);
      for (int j = 0; j < 8; ++j) {
        const int kin = (j < 4) ? (4 * q + j) : (16 + 4 * q + (j - 4));
        split_bf16(R_intra_host[kin * 32 + kout], &ah[(t * 64 + l) * 8 + j], &al[(t * 64 + l) * 8 + j]);
      }
    }

  // The same for v_mfma_f32_32x32x16_bf16, k-step t = 0, 1: lane (m = l%32, h = l/32), slot jj
  // holds R_intra[16t + 8(jj/4) + 4h + jj%4][kout] with kout = 16((m/4)%2) + 4(m/8) + m%4, so that
  // after step 3 lane (b, h) holds Z[b][16h .. 16h + 15] in register order.
  std::vector<uint16_t> a32h(2 * 64 * 8), a32l(2 * 64 * 8);
  for (int t = 0; t < 2; ++t)
    for (int l = 0; l < 64; ++l) {
      const int m = l % 32, h = l / 32;
      const int kout = 16 * ((m / 4) % 2) + 4 * (m / 8) + (m % 4);
      for (int jj = 0; jj < 8; ++jj) {
        const int kin = 16 * t + 8 * (jj / 4) + 4 * h + (jj % 4);
        split_bf16(R_intra_host[kin * 32 + kout], &a32h[(t * 64 + l) * 8 + jj], &a32l[(t * 64 + l) * 8 + jj]);
      }
    }

  // R_inter as the B operand of v_mfma_f32_32x32x16_bf16 in lane order: tile w < NW = ceil(G / 32),
  // k-step ks < 2 NW, lane (col = l%32, h = l/32), slot j holds R_inter[32 w + col][16 ks + 8 h + j],
  // zero past G
  const int NW = KS;
  std::vector<uint16_t> fh((size_t)NW * 2 * NW * 64 * 8, 0), fl((size_t)NW * 2 * NW * 64 * 8, 0);
  for (int w = 0; w < NW; ++w)
    for (int ks = 0; ks < 2 * NW; ++ks)
      for (int l = 0; l < 64; ++l)
        for (int j = 0; j < 8; ++j) {
          const int b = 32 * w + l % 32, bp = 16 * ks + 8 * (l / 32) + j;
          if (b < G && bp < G) {
            const size_t at = (((size_t)w * 2 * NW + ks) * 64 + l) * 8 + j;
            split_bf16(R_inter_host[(size_t)b * G + bp], &fh[at], &fl[at]);
          }
        }

  const std::vector<unsigned> zero_ctr(DECODE_CTR_WORDS, 0u);

  // every host table exists: from here on nothing throws
  torq_rotation *r = new (std::nothrow) torq_rotation();
  if (!r) return TORQ_ENOMEM;
  r->d = d;
  r->G = G;
  r->KS = KS;
  r->device = dev;
  r->inter_hi = r->inter_lo = r->intra_hi = r->intra_lo = r->intra32_hi = r->intra32_lo = nullptr;
  r->inter32f_hi = r->inter32f_lo = nullptr;
  r->butterfly = nullptr;
  r->decode_ctr = nullptr;

  e = upload(&r->inter_hi, ih);
  if (e == hipSuccess) e = upload(&r->inter_lo, il);
  if (e == hipSuccess) e = upload(&r->intra_hi, ah);
  if (e == hipSuccess) e = upload(&r->intra_lo, al);
  if (e == hipSuccess) e = upload(&r->intra32_hi, a32h);
  if (e == hipSuccess) e = upload(&r->intra32_lo, a32l);
  if (e == hipSuccess) e = upload(&r->inter32f_hi, fh);
  if (e == hipSuccess) e = upload(&r->inter32f_lo, fl);
  if (e == hipSuccess) e = upload(&r->decode_ctr, zero_ctr);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    torq_rotation_destroy(r);
    return hip_fail(e);
  }
  *out = r;
  return TORQ_OK;
}

void torq_rotation_destroy(torq_rotation_t *r) {
  if (!r) return;
  if (r->inter_hi) (void)hipFree(r->inter_hi);
  if (r->inter_lo) (void)hipFree(r->inter_lo);
  if (r->intra_hi) (void)hipFree(r->intra_hi);
  if (r->intra_lo) (void)hipFree(r->intra_lo);
  if (r->intra32_hi) (void)hipFree(r->intra32_hi);
  if (r->intra32_lo) (void)hipFree(r->intra32_lo);
  if (r->inter32f_hi) (void)hipFree(r->inter32f_hi);
  if (r->inter32f_lo) (void)hipFree(r->inter32f_lo);
  if (r->butterfly) (void)hipFree(r->butterfly);
  if (r->decode_ctr) (void)hipFree(r->decode_ctr);
  delete r;
}

// ---- R_inter as a butterfly of plane rotations -------------------------------------------------
namespace {

inline bool butterfly_size(int G) { return G == 32 || G == 64 || G == 128 || G == 256; }
inline int log2i(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }
// position of the pair that holds row p in a round of stride h, pairs counted in increasing p
inline int pair_index(int p, int h) { return ((p / (2 * h)) * h) + (p % h); }

// R = J_last ... J_first in double; round t turns rows (p, p + G / 2^(t+1)) by atan(tan[t][pair])
void butterfly_dense(const float *tangents, int G, std::vector<double> &R) {
  R.assign((size_t)G * G, 0.0);
  for (int i = 0; i < G; ++i) R[(size_t)i * G + i] = 1.0;
  int t = 0;
  for (int h = G / 2; h >= 1; h /= 2, ++t)
    for (int p = 0; p < G; ++p) {
      if (p & h) continue;
      const double tn = tangents[t * (G / 2) + pair_index(p, h)];
      const double cs = 1.0 / std::sqrt(1.0 + tn * tn), sn = tn * cs;
      double *rp = &R[(size_t)p * G], *rq = &R[(size_t)(p + h) * G];
      for (int k = 0; k < G; ++k) {
        const double a = rp[k], b = rq[k];
        rp[k] = cs * a + sn * b;
        rq[k] = -sn * a + cs * b;
      }
    }
}

}  // namespace

// The output condition of Algorithm 1 reached with a butterfly: round t makes the two diagonal
// entries of every pair (p, p + G / 2^(t+1)) equal,
//   (a - b) cos 2 theta + 2 g sin 2 theta = 0,  theta = atan((b - a) / (2 g)) / 2 in (-pi/4, pi/4)
// (g = 0: pi/4 unless a = b), so that after round t the diagonal is constant on the residue classes of
// the row index modulo the stride, and after the last round constant.
static int torq_equalize_inter_butterfly_impl(const double *Sigma_host, int G, float *R_inter_host, float *tangents_host) {
  if (!Sigma_host || !tangents_host || !butterfly_size(G)) return TORQ_EINVAL;
  const size_t n = (size_t)G;
  for (size_t i = 0; i < n * n; ++i)
    if (!std::isfinite(Sigma_host[i])) return TORQ_EINVAL;
  std::vector<double> S(Sigma_host, Sigma_host + n * n);
  int t = 0;
  for (int h = G / 2; h >= 1; h /= 2, ++t) {
    // the pairs of a round are disjoint: angles first, then all rows, then all columns
    std::vector<double> cs((size_t)G / 2), sn((size_t)G / 2);
    for (int p = 0; p < G; ++p) {
      if (p & h) continue;
      const int q = p + h, i = pair_index(p, h);
      const double a = S[p * n + p], b = S[q * n + q], g = S[p * n + q];
      const double theta = g != 0.0 ? 0.5 * std::atan((b - a) / (2.0 * g)) : (a != b ? 0.78539816339744830962 : 0.0);
      cs[i] = std::cos(theta);
      sn[i] = std::sin(theta);
      tangents_host[(size_t)t * (G / 2) + i] = (float)std::tan(theta);
    }
    for (int p = 0; p < G; ++p) {
      if (p & h) continue;
      const int i = pair_index(p, h);
      double *rp = &S[p * n], *rq = &S[(size_t)(p + h) * n];
      for (size_t k = 0; k < n; ++k) {
        const double u = rp[k], v = rq[k];
        rp[k] = cs[i] * u + sn[i] * v;
        rq[k] = -sn[i] * u + cs[i] * v;
      }
    }
    for (size_t k = 0; k < n; ++k) {
      double *row = &S[k * n];
      for (int p = 0; p < G; ++p) {
        if (p & h) continue;
        const int i = pair_index(p, h);
        const double u = row[p], v = row[p + h];
        row[p] = cs[i] * u + sn[i] * v;
        row[p + h] = -sn[i] * u + cs[i] * v;
      }
    }
  }
  if (R_inter_host) {
    // the dense matrix of the tangents as handed back (fp32), which is what the handle applies
    std::vector<double> R;
    butterfly_dense(tangents_host, G, R);
    for (size_t i = 0; i < n * n; ++i) R_inter_host[i] = (float)R[i];
  }
  return TORQ_OK;
}

static int torq_rotation_create_butterfly_impl(torq_rotation_t **out, int d, int G, const float *tangents_host,
                                   const float *R_intra_host) {
  if (!out) return TORQ_EINVAL;
  *out = nullptr;
  if (!tangents_host || !R_intra_host || !butterfly_size(G)) return TORQ_EINVAL;
  const int L = log2i(G), NJ = G / 32;
  for (int i = 0; i < L * (G / 2); ++i)
    if (!(std::fabs(tangents_host[i]) <= TORQ_BUTTERFLY_MAX_TAN)) return TORQ_EINVAL;   // NaN fails too
  std::vector<double> Rd;
  butterfly_dense(tangents_host, G, Rd);
  std::vector<float> Rf(Rd.begin(), Rd.end());
  const int status = torq_rotation_create_impl(out, d, G, Rf.data(), R_intra_host);
  if (status != TORQ_OK) return status;

  // per-row coefficients (rotate_butterfly.hip): the kernel carries u = value / sigma, sigma = the
  // product of the cosines the row has met, so round t's update of row p with partner q = p ^ h is
  // u_p += (+-tan theta) (sigma_q / sigma_p) u_q; lane b0 owns the rows 32 j + b0
  const int NC = torq::butterfly_coef_count(G);
  std::vector<float> coef((size_t)NC * 32, 0.f);
  std::vector<double> sigma((size_t)G, 1.0), cosine((size_t)G);
  int t = 0;
  for (int h = G / 2; h >= 1; h /= 2, ++t) {
    for (int p = 0; p < G; ++p) {
      const bool low = (p & h) == 0;
      const double tn = tangents_host[t * (G / 2) + pair_index(low ? p : p - h, h)];
      coef[(size_t)(t * NJ + p / 32) * 32 + p % 32] = (float)((low ? tn : -tn) * sigma[p ^ h] / sigma[p]);
      cosine[p] = 1.0 / std::sqrt(1.0 + tn * tn);
    }
    for (int p = 0; p < G; ++p) sigma[p] *= cosine[p];
  }
  for (int p = 0; p < G; ++p) coef[(size_t)(L * NJ + p / 32) * 32 + p % 32] = (float)sigma[p];
  // within the tangent limit every entry is a finite fp32 value (and sigma a normal one); checked all
  // the same, because the kernel divides by nothing but multiplies by all of them
  bool usable = true;
  for (float c : coef) usable = usable && std::isfinite(c);
  for (int p = 0; p < G; ++p) usable = usable && std::fpclassify((float)sigma[p]) == FP_NORMAL;
  if (!usable) {
    torq_rotation_destroy(*out);
    *out = nullptr;
    return TORQ_EINVAL;
  }
  hipError_t e = upload(&(*out)->butterfly, coef);
  if (e != hipSuccess) {
    torq_rotation_destroy(*out);
    *out = nullptr;
    return hip_fail(e);
  }
  return TORQ_OK;
}

int torq_rotation_d(const torq_rotation_t *r) { return r ? r->d : TORQ_EINVAL; }
int torq_rotation_G(const torq_rotation_t *r) { return r ? r->G : TORQ_EINVAL; }

int torq_rotate_quantize(const torq_rotation_t *r, const void *x_bf16, int64_t M, uint8_t *codes,
                         uint8_t *scales, void *stream) {
  if (!r || M < 0) return TORQ_EINVAL;
  if (M == 0) return TORQ_OK;
  if (!x_bf16 || !codes || !scales) return TORQ_EINVAL;
  if (misaligned(x_bf16) || misaligned(codes) || misaligned(scales)) return TORQ_EALIGN;
  hipError_t e = rotate_any(r, x_bf16, M, TORQ_FMT_MXFP4, 1.0f, codes, scales, nullptr, (hipStream_t)stream);
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

int torq_rotate(const torq_rotation_t *r, const void *x_bf16, int64_t M, float *z_f32, void *stream) {
  if (!r || M < 0) return TORQ_EINVAL;
  if (M == 0) return TORQ_OK;
  if (!x_bf16 || !z_f32) return TORQ_EINVAL;
  if (misaligned(x_bf16) || misaligned(z_f32)) return TORQ_EALIGN;
  hipError_t e = rotate_any(r, x_bf16, M, TORQ_FMT_MXFP4, 1.0f, nullptr, nullptr, z_f32, (hipStream_t)stream);
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

int torq_quantize_f32(const float *z_f32, int64_t M, int d, uint8_t *codes, uint8_t *scales,
                      void *stream) {
  if (M < 0 || d <= 0 || d % TORQ_BLOCK != 0) return TORQ_EINVAL;
  if (M == 0) return TORQ_OK;
  if (!z_f32 || !codes || !scales) return TORQ_EINVAL;
  if (misaligned(z_f32) || misaligned(codes) || misaligned(scales)) return TORQ_EALIGN;
  hipError_t e = torq::launch_quantize_f32(z_f32, M * (int64_t)(d / TORQ_BLOCK), TORQ_FMT_MXFP4, 1.0f, codes, scales,
                                           (hipStream_t)stream);
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

int mxfp4_gemm(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
               void *out_bf16, int64_t M, int64_t N, int d, void *stream) {
  if (M < 0 || N < 0 || d <= 0 || d % 128 != 0) return TORQ_EINVAL;
  if (M == 0 || N == 0) return TORQ_OK;
  if (!A_q || !A_s || !W_q || !W_s || !out_bf16) return TORQ_EINVAL;
  if (misaligned(A_q) || misaligned(W_q) || misaligned(out_bf16)) return TORQ_EALIGN;
  if ((reinterpret_cast<uintptr_t>(A_s) & 3u) || (reinterpret_cast<uintptr_t>(W_s) & 3u)) return TORQ_EALIGN;
  hipError_t e = torq::launch_mxfp4_gemm(A_q, A_s, W_q, W_s, out_bf16, M, N, d, nullptr, 0, (hipStream_t)stream);
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

static bool valid_format(int format, float global_scale) {
  if (format == TORQ_FMT_MXFP4 || format == TORQ_FMT_MXINT4) return true;
  return format == TORQ_FMT_NVFP4 && std::isfinite(global_scale) && global_scale > 0.0f;
}

int torq_rotate_quantize_fmt(const torq_rotation_t *r, const void *x_bf16, int64_t M, int format, float global_scale,
                             uint8_t *codes, uint8_t *scales, void *stream) {
  if (!r || M < 0 || !valid_format(format, global_scale)) return TORQ_EINVAL;
  if (M == 0) return TORQ_OK;
  if (!x_bf16 || !codes || !scales) return TORQ_EINVAL;
  if (misaligned(x_bf16) || misaligned(codes) || misaligned(scales)) return TORQ_EALIGN;
  hipError_t e = rotate_any(r, x_bf16, M, format, global_scale, codes, scales, nullptr, (hipStream_t)stream);
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

int torq_quantize_f32_fmt(const float *z_f32, int64_t M, int d, int format, float global_scale, uint8_t *codes,
                          uint8_t *scales, void *stream) {
  if (M < 0 || d <= 0 || d % TORQ_BLOCK != 0 || !valid_format(format, global_scale)) return TORQ_EINVAL;
  if (M == 0) return TORQ_OK;
  if (!z_f32 || !codes || !scales) return TORQ_EINVAL;
  if (misaligned(z_f32) || misaligned(codes) || misaligned(scales)) return TORQ_EALIGN;
  hipError_t e = torq::launch_quantize_f32(z_f32, M * (int64_t)(d / TORQ_BLOCK), format, global_scale, codes, scales,
                                           (hipStream_t)stream);
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

size_t mxfp4_gemm_workspace_bytes(int64_t M, int64_t N, int d) {
  if (M <= 0 || N <= 0 || d <= 0 || d % 128 != 0) return 0;
  return torq::mxfp4_gemm_workspace_bytes(M, N, d);
}

int mxfp4_gemm_plan(int64_t M, int64_t N, int d, size_t workspace_bytes, int *weight_streaming, int *tile_m,
                    int *tile_n, int *k_pieces) {
  if (M <= 0 || N <= 0 || d <= 0 || d % 128 != 0) return TORQ_EINVAL;
  if (!weight_streaming || !tile_m || !tile_n || !k_pieces) return TORQ_EINVAL;
  torq::mxfp4_gemm_plan(M, N, d, workspace_bytes, weight_streaming, tile_m, tile_n, k_pieces);
  return TORQ_OK;
}

int64_t mxfp4_gemm_main_columns(int64_t M, int64_t N, int d, size_t workspace_bytes) {
  if (M <= 0 || N <= 0 || d <= 0 || d % 128 != 0) return 0;
  return torq::mxfp4_gemm_main_columns(M, N, d, workspace_bytes);
}

int mxfp4_gemm_ws(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                  void *out_bf16, int64_t M, int64_t N, int d, void *workspace, size_t workspace_bytes,
                  void *stream) {
  if (M < 0 || N < 0 || d <= 0 || d % 128 != 0) return TORQ_EINVAL;
  if (M == 0 || N == 0) return TORQ_OK;
  if (!A_q || !A_s || !W_q || !W_s || !out_bf16) return TORQ_EINVAL;
  if (misaligned(A_q) || misaligned(W_q) || misaligned(out_bf16) || misaligned(workspace)) return TORQ_EALIGN;
  if ((reinterpret_cast<uintptr_t>(A_s) & 3u) || (reinterpret_cast<uintptr_t>(W_s) & 3u)) return TORQ_EALIGN;
  hipError_t e = torq::launch_mxfp4_gemm(A_q, A_s, W_q, W_s, out_bf16, M, N, d, workspace,
                                         workspace ? workspace_bytes : 0, (hipStream_t)stream);
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

size_t torq_linear_workspace_bytes(int64_t M, int d) {
  if (M <= 0 || d <= 0 || d % TORQ_BLOCK != 0) return 0;
  const size_t codes = ((size_t)M * (size_t)(d / 2) + 255) & ~(size_t)255;
  const size_t scales = ((size_t)M * (size_t)(d / TORQ_BLOCK) + 255) & ~(size_t)255;
  return codes + scales;
}

int torq_linear(const torq_rotation_t *r, const void *x_bf16, const uint8_t *W_q, const uint8_t *W_s,
                void *out_bf16, int64_t M, int64_t N, void *workspace, size_t workspace_bytes,
                void *stream) {
  if (!r || M < 0 || N < 0) return TORQ_EINVAL;
  if (r->d % 128 != 0) return TORQ_EINVAL;
  if (M == 0 || N == 0) return TORQ_OK;
  if (!x_bf16 || !W_q || !W_s || !out_bf16 || !workspace) return TORQ_EINVAL;
  if (misaligned(x_bf16) || misaligned(W_q) || misaligned(out_bf16) || misaligned(workspace)) return TORQ_EALIGN;
  if (reinterpret_cast<uintptr_t>(W_s) & 3u) return TORQ_EALIGN;
  if (workspace_bytes < torq_linear_workspace_bytes(M, r->d)) return TORQ_EWORKSPACE;
  uint8_t *codes = static_cast<uint8_t *>(workspace);
  uint8_t *scales = codes + (((size_t)M * (size_t)(r->d / 2) + 255) & ~(size_t)255);
  // a row or two of a decode step: one launch, every workgroup rotates the rows itself (same bits out)
  if (torq::torq_linear_local_pays(r, M, N) && (int64_t)r->d * 128 < 0x7FFFFFFF) {
    hipError_t el = torq::launch_torq_linear_local(r, x_bf16, codes, scales, W_q, W_s, out_bf16, M, N, (hipStream_t)stream);
    return el == hipSuccess ? TORQ_OK : hip_fail(el);
  }
  hipError_t e = rotate_any(r, x_bf16, M, TORQ_FMT_MXFP4, 1.0f, codes, scales, nullptr, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e);
  // whatever the caller gave beyond the packed activations serves the GEMM's split-k pieces
  const size_t used = torq_linear_workspace_bytes(M, r->d);
  e = torq::launch_mxfp4_gemm(codes, scales, W_q, W_s, out_bf16, M, N, r->d, static_cast<char *>(workspace) + used,
                              workspace_bytes - used, (hipStream_t)stream);
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

int torq_linear_static(const torq_rotation_t *r, const void *x_bf16, const uint8_t *W_q, const uint8_t *W_s,
                       void *out_bf16, int64_t M, int64_t N, void *stream) {
  if (!r || M < 0 || N < 0) return TORQ_EINVAL;
  if (r->d % 128 != 0) return TORQ_EINVAL;
  if (M == 0 || N == 0) return TORQ_OK;
  if (!x_bf16 || !W_q || !W_s || !out_bf16) return TORQ_EINVAL;
  if (misaligned(x_bf16) || misaligned(W_q) || misaligned(out_bf16)) return TORQ_EALIGN;
  if (reinterpret_cast<uintptr_t>(W_s) & 3u) return TORQ_EALIGN;
  // M * d / 2 cannot overflow: both factors are checked against the limit first
  if (M > (int64_t)TORQ_STATIC_SCRATCH_BYTES || torq_linear_workspace_bytes(M, r->d) > TORQ_STATIC_SCRATCH_BYTES)
    return TORQ_ETOOBIG;
  unsigned char *ws = nullptr;
  hipError_t e = scratch_of_current_device(&ws);
  if (e != hipSuccess) return hip_fail(e);
  uint8_t *codes = ws;
  uint8_t *scales = codes + (((size_t)M * (size_t)(r->d / 2) + 255) & ~(size_t)255);
  if (torq::torq_linear_local_pays(r, M, N) && (int64_t)r->d * 128 < 0x7FFFFFFF) {      // as torq_linear
    e = torq::launch_torq_linear_local(r, x_bf16, codes, scales, W_q, W_s, out_bf16, M, N, (hipStream_t)stream);
    return e == hipSuccess ? TORQ_OK : hip_fail(e);
  }
  e = rotate_any(r, x_bf16, M, TORQ_FMT_MXFP4, 1.0f, codes, scales, nullptr, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e);
  e = torq::launch_mxfp4_gemm(codes, scales, W_q, W_s, out_bf16, M, N, r->d, nullptr, 0, (hipStream_t)stream);
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

int torq_linear_single_launch_probe(const torq_rotation_t *r, const void *x_bf16, const uint8_t *W_q,
                                    const uint8_t *W_s, void *out_bf16, int64_t M, int64_t N, void *workspace,
                                    size_t workspace_bytes, int spin_limit, int withhold_ready, void *stream) {
  if (!r || M < 0 || N < 0 || spin_limit < 1 || spin_limit > (1 << 18)) return TORQ_EINVAL;
  if (r->G != 128 || r->butterfly || r->d % 128 != 0 || M > 64) return TORQ_EINVAL;
  if ((int64_t)r->d * 128 >= 0x7FFFFFFF || (M > 0 && !torq::mxfp4_gemm_skinny_fits(M, r->d))) return TORQ_EINVAL;
  if (M == 0 || N == 0) return TORQ_OK;
  if (!x_bf16 || !W_q || !W_s || !out_bf16 || !workspace) return TORQ_EINVAL;
  if (misaligned(x_bf16) || misaligned(W_q) || misaligned(out_bf16) || misaligned(workspace)) return TORQ_EALIGN;
  if (reinterpret_cast<uintptr_t>(W_s) & 3u) return TORQ_EALIGN;
  if (workspace_bytes < torq_linear_workspace_bytes(M, r->d)) return TORQ_EWORKSPACE;
  uint8_t *codes = static_cast<uint8_t *>(workspace);
  uint8_t *scales = codes + (((size_t)M * (size_t)(r->d / 2) + 255) & ~(size_t)255);
  hipError_t e = torq::launch_torq_linear_decode(r, x_bf16, codes, scales, W_q, W_s, out_bf16, M, N, spin_limit,
                                                 withhold_ready ? 0 : 1, (hipStream_t)stream);
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

int torq_linear_single_launch(const torq_rotation_t *r, const void *x_bf16, const uint8_t *W_q, const uint8_t *W_s,
                              void *out_bf16, int64_t M, int64_t N, void *workspace, size_t workspace_bytes,
                              void *stream) {
  // a few token-groups: every workgroup rotates them itself, nothing is handed over between workgroups
  // (and the handle's counters, the give-up word included, are neither read nor written)
  if (r && M >= 1 && N >= 1 && torq::torq_linear_local_fits(r, M) && (int64_t)r->d * 128 < 0x7FFFFFFF) {
    if (!x_bf16 || !W_q || !W_s || !out_bf16 || !workspace) return TORQ_EINVAL;
    if (misaligned(x_bf16) || misaligned(W_q) || misaligned(out_bf16) || misaligned(workspace)) return TORQ_EALIGN;
    if (reinterpret_cast<uintptr_t>(W_s) & 3u) return TORQ_EALIGN;
    if (workspace_bytes < torq_linear_workspace_bytes(M, r->d)) return TORQ_EWORKSPACE;
    uint8_t *codes = static_cast<uint8_t *>(workspace);
    uint8_t *scales = codes + (((size_t)M * (size_t)(r->d / 2) + 255) & ~(size_t)255);
    hipError_t e = torq::launch_torq_linear_local(r, x_bf16, codes, scales, W_q, W_s, out_bf16, M, N, (hipStream_t)stream);
    return e == hipSuccess ? TORQ_OK : hip_fail(e);
  }
  return torq_linear_single_launch_probe(r, x_bf16, W_q, W_s, out_bf16, M, N, workspace, workspace_bytes, 1 << 18, 0,
                                         stream);
}

int torq_linear_single_launch_reset(const torq_rotation_t *r, void *stream) {
  if (!r) return TORQ_EINVAL;
  hipError_t e = torq::launch_decode_ctr_reset(r, (hipStream_t)stream);
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

int torq_linear_single_launch_gave_up(const torq_rotation_t *r, int *gave_up) {
  if (!r || !gave_up) return TORQ_EINVAL;
  unsigned word = 0;
  hipError_t e = hipMemcpy(&word, r->decode_ctr + DECODE_ERR, sizeof word, hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hip_fail(e);
  *gave_up = word != 0;
  return TORQ_OK;
}

size_t torq_linear_workspace_bytes_n(int64_t M, int64_t N, int d) {
  const size_t base = torq_linear_workspace_bytes(M, d);
  if (base == 0 || N <= 0 || d % 128 != 0) return base;
  return base + torq::mxfp4_gemm_workspace_bytes(M, N, d);
}

size_t torq_block_gram_workspace_bytes(int G) {
  if (G <= 0 || G % 16 != 0 || G > TORQ_MAX_G) return 0;
  return torq::block_gram_workspace_bytes(G);
}

int torq_block_gram(const void *x_bf16, int64_t M, int d, int G, double *Sigma, void *workspace,
                    size_t workspace_bytes, void *stream) {
  if (M <= 0 || d <= 0 || d % TORQ_BLOCK != 0) return TORQ_EINVAL;
  if (G <= 0 || G % 16 != 0 || G > TORQ_MAX_G || (d / TORQ_BLOCK) % G != 0) return TORQ_EINVAL;
  if (!x_bf16 || !Sigma || !workspace) return TORQ_EINVAL;
  if (misaligned(x_bf16) || misaligned(workspace) || (reinterpret_cast<uintptr_t>(Sigma) & 7u)) return TORQ_EALIGN;
  if (workspace_bytes < torq::block_gram_workspace_bytes(G)) return TORQ_EWORKSPACE;
  const int64_t TG = M * (int64_t)(d / TORQ_BLOCK / G);
  hipError_t e = torq::launch_block_gram(x_bf16, TG, G, -1, Sigma, workspace, (hipStream_t)stream);
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

int torq_block_gram_positions(const void *x_bf16, int64_t M, int d, int G, double *Sigma_pos, void *workspace,
                              size_t workspace_bytes, void *stream) {
  if (M <= 0 || d <= 0 || d % TORQ_BLOCK != 0) return TORQ_EINVAL;
  if (G <= 0 || G % 16 != 0 || G > TORQ_MAX_G || (d / TORQ_BLOCK) % G != 0) return TORQ_EINVAL;
  if (!x_bf16 || !Sigma_pos || !workspace) return TORQ_EINVAL;
  if (misaligned(x_bf16) || misaligned(workspace) || (reinterpret_cast<uintptr_t>(Sigma_pos) & 7u)) return TORQ_EALIGN;
  if (workspace_bytes < torq::block_gram_workspace_bytes(G)) return TORQ_EWORKSPACE;
  const int64_t TG = M * (int64_t)(d / TORQ_BLOCK / G);
  // one pass per position: the partial sums in the workspace are reused in stream order
  for (int k = 0; k < TORQ_BLOCK; ++k) {
    hipError_t e = torq::launch_block_gram(x_bf16, TG, G, k, Sigma_pos + (size_t)k * G * G, workspace, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e);
  }
  return TORQ_OK;
}

// Algorithm 1 (Section 5.1) with the equalising angle.  One step takes the block p furthest above
// the target c and the block n furthest below it and turns the (p, n) plane by theta with
//   c = cos^2 a + 2 sin cos g + sin^2 b      (a = S_pp, b = S_nn, g = S_pn),
// i.e. t = tan theta solves (b - c) t^2 + 2 g t + (a - c) = 0; (a - c)(b - c) < 0 makes the
// discriminant positive, and the root of smaller magnitude is t = -(a - c) / (g + sgn(g) D).
// After the step S_pp = c exactly and S_nn = a + b - c (the trace is conserved), so at most G - 1
// steps are needed.
static int torq_equalize_inter_impl(const double *Sigma_host, int G, double eps, float *R_inter_host, int *steps_out) {
  if (!Sigma_host || !R_inter_host || G < 1 || G > 4096 || !(eps >= 0.0)) return TORQ_EINVAL;
  const size_t n = (size_t)G;
  // NaN compares false with everything: the search below would find no deviation and hand back R = I
  for (size_t i = 0; i < n * n; ++i)
    if (!std::isfinite(Sigma_host[i])) return TORQ_EINVAL;
  std::vector<double> S(Sigma_host, Sigma_host + n * n), R(n * n, 0.0);
  for (size_t i = 0; i < n; ++i) R[i * n + i] = 1.0;
  double trace = 0.0;
  for (size_t i = 0; i < n; ++i) trace += S[i * n + i];
  const double c = trace / (double)G;

  int steps = 0;
  for (;;) {
    int p = -1, q = -1;
    double above = 0.0, below = 0.0, worst = 0.0;
    for (int i = 0; i < G; ++i) {
      const double dev = S[(size_t)i * n + i] - c;
      worst = std::fmax(worst, std::fabs(dev));
      if (dev > above) { above = dev; p = i; }
      if (dev < below) { below = dev; q = i; }
    }
    if (worst <= eps) break;
    if (p < 0 || q < 0 || steps >= 4 * G) return TORQ_ECONVERGE;

    const double a = S[(size_t)p * n + p], b = S[(size_t)q * n + q], g = S[(size_t)p * n + q];
    const double disc = std::sqrt(g * g - (a - c) * (b - c));
    const double t = -(a - c) / (g + (g >= 0.0 ? disc : -disc));
    const double cs = 1.0 / std::sqrt(1.0 + t * t), sn = t * cs;
    // S <- J S J^T, R <- J R with J = the plane rotation of rows p and q
    auto rotate_rows = [&](std::vector<double> &A) {
      double *rp = &A[(size_t)p * n], *rq = &A[(size_t)q * n];
      for (size_t j = 0; j < n; ++j) {
        const double u = rp[j], v = rq[j];
        rp[j] = cs * u + sn * v;
        rq[j] = cs * v - sn * u;
      }
    };
    rotate_rows(S);
    rotate_rows(R);
    for (size_t i = 0; i < n; ++i) {
      const double u = S[i * n + p], v = S[i * n + q];
      S[i * n + p] = cs * u + sn * v;
      S[i * n + q] = cs * v - sn * u;
    }
    ++steps;
  }
  for (size_t i = 0; i < n * n; ++i) R_inter_host[i] = (float)R[i];
  if (steps_out) *steps_out = steps;
  return TORQ_OK;
}

size_t torq_code_histogram_workspace_bytes(void) { return torq::code_histogram_workspace_bytes(); }

int torq_code_histogram(const uint8_t *codes, int64_t M, int d, uint64_t *counts, void *workspace,
                        size_t workspace_bytes, void *stream) {
  if (M < 0 || d <= 0 || d % TORQ_BLOCK != 0 || !counts || !workspace) return TORQ_EINVAL;
  if (M > 0 && !codes) return TORQ_EINVAL;
  if (misaligned(codes) || misaligned(workspace) || (reinterpret_cast<uintptr_t>(counts) & 7u)) return TORQ_EALIGN;
  if (workspace_bytes < torq::code_histogram_workspace_bytes()) return TORQ_EWORKSPACE;
  // M = 0 launches the same kernels over no blocks: every count comes out zero
  hipError_t e = torq::launch_code_histogram(codes, M * (int64_t)(d / TORQ_BLOCK), counts, workspace,
                                             (hipStream_t)stream);
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

int torq_intra_pair_scores(const uint64_t *counts_host, double lambda, double *h_host, double *H_host) {
  if (!counts_host || !h_host || !H_host || !(lambda >= 0.0)) return TORQ_EINVAL;
  torq::intra_pair_scores(counts_host, lambda, h_host, H_host);
  return TORQ_OK;
}

static int torq_intra_best_angle_impl(const double *u_host, const double *v_host, int64_t n, const uint64_t *rest_host,
                          double *theta, double *loss, int64_t *critical) {
  if (n < 0 || n > TORQ_INTRA_MAX_SAMPLE || !rest_host || !theta || !loss) return TORQ_EINVAL;
  if (n > 0 && (!u_host || !v_host)) return TORQ_EINVAL;
  for (int64_t b = 0; b < n; ++b)
    if (!std::isfinite(u_host[b]) || !std::isfinite(v_host[b])) return TORQ_EINVAL;
  const int64_t k = torq::intra_best_angle(u_host, v_host, n, rest_host, theta, loss);
  if (critical) *critical = k;
  return TORQ_OK;
}

static int torq_calibrate_intra_impl(const float *X_host, int64_t n, int max_iter, int k_top, int P, double lambda,
                         double eps, float *R_intra_host, double *losses_host, int *n_eval) {
  if (!X_host || !R_intra_host || !losses_host || !n_eval) return TORQ_EINVAL;
  if (n < 1 || n > TORQ_INTRA_MAX_SAMPLE || max_iter < 0 || max_iter > 1000) return TORQ_EINVAL;
  if (k_top < 1 || k_top > TORQ_BLOCK || P < 1 || P > TORQ_BLOCK / 2) return TORQ_EINVAL;
  if (!(lambda >= 0.0) || !(eps >= 0.0)) return TORQ_EINVAL;
  for (int64_t i = 0; i < n * TORQ_BLOCK; ++i)
    if (!std::isfinite(X_host[i])) return TORQ_EINVAL;
  double R[TORQ_BLOCK * TORQ_BLOCK];
  torq::intra_rotation(X_host, n, max_iter, k_top, P, lambda, eps, R, losses_host, n_eval);
  for (int i = 0; i < TORQ_BLOCK * TORQ_BLOCK; ++i) R_intra_host[i] = (float)R[i];
  return TORQ_OK;
}

int torq_diag_mfma_burn(int kind, const void *operands, size_t n_bytes, int iters, float *sink,
                        void *stream) {
  if ((kind != TORQ_DIAG_FP4 && kind != TORQ_DIAG_BF16) || !operands || !sink || n_bytes < 128 || iters <= 0)
    return TORQ_EINVAL;
  if ((reinterpret_cast<uintptr_t>(operands) & 3u) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return TORQ_EALIGN;
  const size_t n_words = n_bytes / 4 > 0x40000000u ? 0x40000000u : n_bytes / 4;
  hipError_t e = torq::launch_mfma_burn(kind, static_cast<const uint32_t *>(operands), (uint32_t)n_words, iters,
                                        sink, (hipStream_t)stream);
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

int torq_diag_gemm_ablation(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                            void *out_bf16, int64_t M, int64_t N, int d, int skip, void *stream) {
  if (M <= 0 || N <= 0 || d <= 0 || d % 512 != 0 || skip < 0) return TORQ_EINVAL;
  if (!A_q || !A_s || !W_q || !W_s || !out_bf16) return TORQ_EINVAL;
  if (misaligned(A_q) || misaligned(W_q) || misaligned(out_bf16) || misaligned(A_s) || misaligned(W_s)) return TORQ_EALIGN;
  hipError_t e = torq::launch_mxfp4_gemm_ablated(A_q, A_s, W_q, W_s, out_bf16, M, N, d, skip, (hipStream_t)stream);
  if (e == hipErrorInvalidValue) return TORQ_EINVAL;
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

int torq_diag_gemm_persistent(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                              void *out_bf16, int64_t M, int64_t N, int d, int tile, int workgroups, void *stream) {
  if (M <= 0 || N <= 0 || d <= 0 || d % 1024 != 0 || (tile != 0 && tile != 1) || workgroups < 1 || workgroups > 65536)
    return TORQ_EINVAL;
  if (!A_q || !A_s || !W_q || !W_s || !out_bf16) return TORQ_EINVAL;
  if (misaligned(A_q) || misaligned(W_q) || misaligned(out_bf16) || misaligned(A_s) || misaligned(W_s)) return TORQ_EALIGN;
  hipError_t e = torq::launch_mxfp4_gemm_persistent(A_q, A_s, W_q, W_s, out_bf16, M, N, d, tile, workgroups,
                                                    (hipStream_t)stream);
  if (e == hipErrorInvalidValue) return TORQ_EINVAL;
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

int torq_diag_gemm_plan(const uint8_t *A_q, const uint8_t *A_s, const uint8_t *W_q, const uint8_t *W_s,
                        void *out_bf16, int64_t M, int64_t N, int d, int tile, int k_pieces, int deep,
                        void *workspace, size_t workspace_bytes, void *stream) {
  if (M <= 0 || N <= 0 || d <= 0 || d % 128 != 0 || tile < 0 || tile > 3 || k_pieces < 1 || k_pieces > 64)
    return TORQ_EINVAL;
  if (!A_q || !A_s || !W_q || !W_s || !out_bf16) return TORQ_EINVAL;
  if (misaligned(A_q) || misaligned(W_q) || misaligned(out_bf16) || misaligned(workspace)) return TORQ_EALIGN;
  hipError_t e = torq::launch_mxfp4_gemm_forced(A_q, A_s, W_q, W_s, out_bf16, M, N, d, tile, k_pieces, deep, workspace,
                                                workspace_bytes, (hipStream_t)stream);
  if (e == hipErrorInvalidValue) return TORQ_EINVAL;
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

int torq_diag_rotate_ablation(const torq_rotation_t *r, const void *x_bf16, int64_t M, uint8_t *codes,
                              uint8_t *scales, int skip, void *stream) {
  if (!r || M < 0 || skip < 0) return TORQ_EINVAL;
  if (M == 0) return TORQ_OK;
  if (!x_bf16 || !codes || !scales) return TORQ_EINVAL;
  if (misaligned(x_bf16) || misaligned(codes) || misaligned(scales)) return TORQ_EALIGN;
  hipError_t e = torq::launch_rotate_ablated(r, x_bf16, M, codes, scales, skip, (hipStream_t)stream);
  if (e == hipErrorInvalidValue) return TORQ_EINVAL;
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

int torq_diag_copy(const void *src, void *dst, size_t n_bytes, void *stream) {
  if (!src || !dst || n_bytes % 16 != 0) return TORQ_EINVAL;
  if (misaligned(src) || misaligned(dst)) return TORQ_EALIGN;
  hipError_t e = torq::launch_diag_copy(src, dst, n_bytes, (hipStream_t)stream);
  return e == hipSuccess ? TORQ_OK : hip_fail(e);
}

// The host routines above behind a guard: an allocation failure comes back as TORQ_ENOMEM.
int torq_rotation_create(torq_rotation_t **out, int d, int G, const float *R_inter_host, const float *R_intra_host) {
  return guarded([&] { return torq_rotation_create_impl(out, d, G, R_inter_host, R_intra_host); });
}

int torq_equalize_inter_butterfly(const double *Sigma_host, int G, float *R_inter_host, float *tangents_host) {
  return guarded([&] { return torq_equalize_inter_butterfly_impl(Sigma_host, G, R_inter_host, tangents_host); });
}

int torq_rotation_create_butterfly(torq_rotation_t **out, int d, int G, const float *tangents_host, const float *R_intra_host) {
  return guarded([&] { return torq_rotation_create_butterfly_impl(out, d, G, tangents_host, R_intra_host); });
}

int torq_equalize_inter(const double *Sigma_host, int G, double eps, float *R_inter_host, int *steps_out) {
  return guarded([&] { return torq_equalize_inter_impl(Sigma_host, G, eps, R_inter_host, steps_out); });
}

int torq_intra_best_angle(const double *u_host, const double *v_host, int64_t n, const uint64_t *rest_host, double *theta, double *loss, int64_t *critical) {
  return guarded([&] { return torq_intra_best_angle_impl(u_host, v_host, n, rest_host, theta, loss, critical); });
}

int torq_calibrate_intra(const float *X_host, int64_t n, int max_iter, int k_top, int P, double lambda, double eps, float *R_intra_host, double *losses_host, int *n_eval) {
  return guarded([&] { return torq_calibrate_intra_impl(X_host, n, max_iter, k_top, P, lambda, eps, R_intra_host, losses_host, n_eval); });
}

}  // extern "C"
