// Host side of the intra-block calibration (Section 5.2, Algorithm 2): pair scores (Appendix A.5),
// the exact angle solver (Appendix A.4) and the alternating S-step / R-step loop, all in double on a
// sample of blocks.  Nothing here runs on the GPU; the full-data statistic (the codeword histogram
// of the quantiser's output) is code_histogram.hip.
//
// The angle solver is a sweep: every critical angle is an event (sample, axis); events are sorted
// once, the occupancy is counted in full for the interval that wraps around 2 pi, and crossing a
// critical angle re-reads only the samples that have an event there (or just before it).
// O(|T| log |T|) for the sort and O(|T|) for the sweep, against O(|T| n) for counting every
// interval afresh.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "torq_internal.h"

#pragma clang fp contract(off)

namespace torq {

namespace {

constexpr int K = TORQ_BLOCK;   // 32 positions
constexpr int J = 8;            // magnitude codewords
constexpr double kPi = 3.14159265358979323846;
constexpr double kBound[7] = {0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0};

// interval of |a| between the e2m1 decision boundaries; a boundary value goes where round-to-
// nearest-even sends it (boundaries 0, 2, 4, 6 belong to the interval below, 1, 3, 5 to the one above)
inline int interval_of(double a) {
  const double m = std::fabs(a);
  int j = 0;
  while (j < 7 && (m > kBound[j] || (m == kBound[j] && (j & 1)))) ++j;
  return j;
}

typedef unsigned __int128 u128;

inline u128 sum_squares(const uint64_t n[J]) {
  u128 t = 0;
  for (int j = 0; j < J; ++j) t += (u128)n[j] * n[j];
  return t;
}

inline double occupancy_loss(const uint64_t n[J]) {
  double total = 0.0, loss = 0.0;
  for (int j = 0; j < J; ++j) total += (double)n[j];
  if (total == 0.0) return 0.0;
  for (int j = 0; j < J; ++j) {
    const double dev = (double)n[j] / total - 1.0 / J;
    loss += dev * dev;
  }
  return loss;
}

struct Event {
  double tau;
  uint32_t sample;
  uint32_t axis;
};

}  // namespace

void intra_pair_scores(const uint64_t *counts, double lambda, double *h, double *H) {
  double dev[K][J];
  for (int k = 0; k < K; ++k) {
    double total = 0.0;
    for (int j = 0; j < J; ++j) total += (double)counts[k * J + j];
    h[k] = 0.0;
    for (int j = 0; j < J; ++j) {
      dev[k][j] = (total > 0.0 ? (double)counts[k * J + j] / total : 0.0) - 1.0 / J;
      h[k] += dev[k][j] * dev[k][j];
    }
  }
  for (int k = 0; k < K; ++k)
    for (int l = 0; l < K; ++l) {
      double c = 0.0;
      for (int j = 0; j < J; ++j) c -= dev[k][j] * dev[l][j];
      H[k * K + l] = h[k] + h[l] + lambda * c;
    }
}

// Returns the number of distinct critical angles.  theta in [0, 2 pi); the pair becomes
// (u cos + v sin, -u sin + v cos).
int64_t intra_best_angle(const double *u, const double *v, int64_t n, const uint64_t rest[J], double *theta,
                         double *loss) {
  const double two_pi = 2.0 * kPi;
  std::vector<Event> ev;
  ev.reserve((size_t)n * 16);
  for (int64_t b = 0; b < n; ++b) {
    const double r = std::sqrt(u[b] * u[b] + v[b] * v[b]);
    const double phi = std::atan2(v[b], u[b]);
    for (int j = 0; j < 7; ++j) {
      if (r < kBound[j]) break;
      const double alpha = std::acos(kBound[j] / r);
      for (uint32_t axis = 0; axis < 2; ++axis) {
        const double base = phi - (axis ? kPi / 2.0 : 0.0);
        const double cand[4] = {base - alpha, base + alpha, base - alpha + kPi, base + alpha + kPi};
        for (double a : cand) {
          a = std::fmod(a, two_pi);
          if (a < 0.0) a += two_pi;
          if (a >= two_pi) a -= two_pi;
          ev.push_back(Event{a, (uint32_t)b, axis});
        }
      }
    }
  }

  // codes of both axes of every sample at one angle
  std::vector<uint8_t> code((size_t)n * 2);
  uint64_t cnt[J];
  auto count_all = [&](double th) {
    const double c = std::cos(th), s = std::sin(th);
    for (int j = 0; j < J; ++j) cnt[j] = rest[j];
    for (int64_t b = 0; b < n; ++b) {
      const int j0 = interval_of(u[b] * c + v[b] * s), j1 = interval_of(-u[b] * s + v[b] * c);
      code[2 * b] = (uint8_t)j0;
      code[2 * b + 1] = (uint8_t)j1;
      cnt[j0] += 1;
      cnt[j1] += 1;
    }
  };

  if (ev.empty()) {
    count_all(0.0);
    *theta = 0.0;
    *loss = occupancy_loss(cnt);
    return 0;
  }
  std::sort(ev.begin(), ev.end(), [](const Event &a, const Event &b) { return a.tau < b.tau; });

  // the interval from the last critical angle round to the first
  double mid = 0.5 * (ev.back().tau + ev.front().tau + two_pi);
  if (mid >= two_pi) mid -= two_pi;
  count_all(mid);
  u128 best_key = sum_squares(cnt);
  double best_theta = mid;
  uint64_t best_cnt[J];
  std::memcpy(best_cnt, cnt, sizeof(cnt));

  // A critical angle is computed with rounding, so the sample's code, as evaluated at a midpoint,
  // may flip a few ulps away from it.  When neighbouring critical angles are that close, one
  // re-reading right after the event could come too early; therefore every interval re-reads all
  // events of the last kSlack radians, not only those of the angle just crossed.
  constexpr double kSlack = 1e-9;
  int64_t distinct = 1;
  size_t i = 0, lo = 0;
  const size_t ne = ev.size();
  while (i < ne) {
    size_t e = i;
    while (e < ne && ev[e].tau == ev[i].tau) ++e;     // all events at this critical angle
    if (e == ne) break;                               // past the last one lies the wrapping interval again
    ++distinct;
    mid = 0.5 * (ev[i].tau + ev[e].tau);
    const double c = std::cos(mid), s = std::sin(mid);
    while (ev[lo].tau < ev[i].tau - kSlack) ++lo;
    for (size_t t = lo; t < e; ++t) {
      const uint32_t b = ev[t].sample, axis = ev[t].axis;
      const int now = axis ? interval_of(-u[b] * s + v[b] * c) : interval_of(u[b] * c + v[b] * s);
      uint8_t &was = code[2 * (size_t)b + axis];
      cnt[was] -= 1;
      cnt[now] += 1;
      was = (uint8_t)now;
    }
    const u128 key = sum_squares(cnt);
    if (key < best_key || (key == best_key && mid < best_theta)) {
      best_key = key;
      best_theta = mid;
      std::memcpy(best_cnt, cnt, sizeof(cnt));
    }
    i = e;
  }
  *theta = best_theta;
  *loss = occupancy_loss(best_cnt);
  return distinct;
}

// Algorithm 2 on n sample blocks (X: [n][32] floats).  Evaluation = S-step (scale of a block from
// the maximum of Z = X R, the quantiser's rule) + histograms + loss of Z / s; stop when the loss
// fell by no more than eps since the previous evaluation or after max_iter R-steps; an R-step turns
// the P best-scoring disjoint pairs of the k_top most imbalanced columns by their exact angles, each
// pair seeing the occupancy as the earlier turns left it.  R_out = the rotation of the evaluation
// with the smallest loss (the earliest among equals); losses[i] = loss of evaluation i.
void intra_rotation(const float *X, int64_t n, int max_iter, int k_top, int P, double lambda, double eps,
                    double *R_out, double *losses, int *n_eval) {
  std::vector<double> R((size_t)K * K, 0.0), best_R, Z((size_t)n * K), u((size_t)n), v((size_t)n);
  for (int i = 0; i < K; ++i) R[(size_t)i * K + i] = 1.0;
  best_R = R;
  double h[K], H[K * K], best_loss = 0.0;
  uint64_t counts[K * J], total[J];
  *n_eval = 0;
  for (int iter = 0;; ++iter) {
    for (int64_t b = 0; b < n; ++b) {
      const float *x = X + b * K;
      double *z = &Z[(size_t)b * K];
      double amax = 0.0;
      for (int k = 0; k < K; ++k) {
        double acc = 0.0;
        for (int i = 0; i < K; ++i) acc += (double)x[i] * R[(size_t)i * K + k];
        z[k] = acc;
        amax = std::fmax(amax, std::fabs(acc));
      }
      // E8M0 byte of the block: exponent field of the fp32 maximum minus 2, not below 0
      const float af = (float)amax;
      uint32_t bits;
      std::memcpy(&bits, &af, 4);
      int byte = (int)((bits >> 23) & 0xFFu) - 2;
      if (byte < 0) byte = 0;
      const double inv = std::ldexp(1.0, 127 - byte);
      for (int k = 0; k < K; ++k) z[k] *= inv;
    }
    std::memset(counts, 0, sizeof(counts));
    for (int64_t b = 0; b < n; ++b)
      for (int k = 0; k < K; ++k) counts[k * J + interval_of(Z[(size_t)b * K + k])] += 1;
    for (int j = 0; j < J; ++j) {
      total[j] = 0;
      for (int k = 0; k < K; ++k) total[j] += counts[k * J + j];
    }
    const double loss = occupancy_loss(total);
    losses[*n_eval] = loss;
    if (*n_eval == 0 || loss < best_loss) {
      best_loss = loss;
      best_R = R;
    }
    *n_eval += 1;
    if (iter >= max_iter) break;
    if (iter > 0 && !(losses[iter - 1] - loss > eps)) break;

    intra_pair_scores(counts, lambda, h, H);
    // pool: the k_top largest h, the lower index first among equals
    int order[K];
    for (int k = 0; k < K; ++k) order[k] = k;
    std::stable_sort(order, order + K, [&](int a, int b) { return h[a] > h[b]; });
    bool in_pool[K] = {}, used[K] = {};
    for (int t = 0; t < k_top && t < K; ++t) in_pool[order[t]] = true;
    // candidate pairs by score, the lexicographically first among equals
    struct Pair { double score; int p, q; };
    std::vector<Pair> pairs;
    for (int p = 0; p < K; ++p)
      for (int q = p + 1; q < K; ++q)
        if (in_pool[p] && in_pool[q]) pairs.push_back(Pair{H[p * K + q], p, q});
    std::stable_sort(pairs.begin(), pairs.end(), [](const Pair &a, const Pair &b) { return a.score > b.score; });
    int taken = 0;
    for (const Pair &pr : pairs) {
      if (taken >= P) break;
      if (used[pr.p] || used[pr.q]) continue;
      used[pr.p] = used[pr.q] = true;
      ++taken;
      const int p = pr.p, q = pr.q;
      uint64_t rest[J];
      for (int j = 0; j < J; ++j) rest[j] = total[j] - counts[p * J + j] - counts[q * J + j];
      for (int64_t b = 0; b < n; ++b) {
        u[(size_t)b] = Z[(size_t)b * K + p];
        v[(size_t)b] = Z[(size_t)b * K + q];
      }
      double theta, pair_loss;
      intra_best_angle(u.data(), v.data(), n, rest, &theta, &pair_loss);
      const double c = std::cos(theta), s = std::sin(theta);
      for (int i = 0; i < K; ++i) {
        const double rp = R[(size_t)i * K + p], rq = R[(size_t)i * K + q];
        R[(size_t)i * K + p] = rp * c + rq * s;
        R[(size_t)i * K + q] = -rp * s + rq * c;
      }
      for (int j = 0; j < J; ++j) counts[p * J + j] = counts[q * J + j] = 0;
      for (int64_t b = 0; b < n; ++b) {
        const double zp = u[(size_t)b] * c + v[(size_t)b] * s, zq = -u[(size_t)b] * s + v[(size_t)b] * c;
        Z[(size_t)b * K + p] = zp;
        Z[(size_t)b * K + q] = zq;
        counts[p * J + interval_of(zp)] += 1;
        counts[q * J + interval_of(zq)] += 1;
      }
      for (int j = 0; j < J; ++j) total[j] = rest[j] + counts[p * J + j] + counts[q * J + j];
    }
  }
  std::memcpy(R_out, best_R.data(), sizeof(double) * K * K);
}

}  // namespace torq
