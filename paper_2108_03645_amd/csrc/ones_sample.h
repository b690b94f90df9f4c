// Probability sampling of the remaining work (ONES, arXiv 2108.03645, Alg. 1 and Eq. 7): once
// per generation the progress rho_j of every job is drawn from Be(alpha_j, beta_j) and the pool
// is scored with Y_j = Y_processed_j (1/rho_j - 1).  A few thousand slots at most, so this is
// latency, not throughput: sixteen lanes share a slot's two gamma draws.
//
// Every floating-point step below is a plain IEEE double operation in the order written (the
// library is built without contraction), square root and division are the correctly rounded
// ones, and the logarithm is spelled out, so the draw is a function of (seed, slot, generation)
// that any implementation of the same steps reproduces bit for bit.
//
// Device code shared by the kernel of ones_sample.hip, which draws a run of generations ahead,
// and by the single-launch kernel, whose drawing workgroups keep ahead of its generations
// (ones_fused.hip).
#pragma once

#include "ones_device.h"

namespace ones {
namespace {

constexpr double kMaxParam = 1e100;                  // cap of the ratio 1/rho - 1 and of Y
constexpr int kGammaAttempts = 64;

// ln x for a positive normal x: x = m 2^e with m in [sqrt(1/2), sqrt(2)), ln m = 2 artanh(s),
// s = (m - 1)/(m + 1), by the series s + s^3/3 + ... + s^23/23; ln 2 split into a 32-bit head
// (its product with e is exact) and a tail.
__device__ inline double series_log(double x) {
  const uint64_t bits = static_cast<uint64_t>(__double_as_longlong(x));
  int e = static_cast<int>((bits >> 52) & 0x7FFu) - 1023;
  double m = __longlong_as_double(static_cast<long long>((bits & 0x000FFFFFFFFFFFFFull) | 0x3FF0000000000000ull));
  if (m > 1.4142135623730951) { m = m * 0.5; e = e + 1; }
  const double f = m - 1.0;
  const double s = f / (2.0 + f);
  const double z = s * s;
  double p = 1.0 / 23.0;
#pragma unroll
  for (int k = 21; k >= 3; k -= 2) p = p * z + 1.0 / static_cast<double>(k);
  const double s2 = 2.0 * s;
  const double lm = s2 + s2 * (z * p);
  const double ef = static_cast<double>(e);
  return ef * 0.6931471803691238 + (ef * 1.9082149292705877e-10 + lm);
}

// Gamma(shape, 1), shape >= 1 (Marsaglia and Tsang, ACM TOMS 26, 2000): d = shape - 1/3,
// c = 1/sqrt(9 d); x ~ N(0,1) by the polar method, v = (1 + c x)^3; d v is accepted when v > 0
// and ln u < x^2/2 + d - d v + d ln v.  Candidate n reads Philox counter (n, slot, t, which):
// words 0, 1 the point in the square, words 2, 3 a 52-bit uniform.  The draw is the first
// accepted candidate in the order n = 0, 1, ...; after kGammaAttempts rejected ones it is d.
//
// One candidate: returns whether it is accepted and its value.
__device__ inline bool gamma_candidate(uint32_t key0, uint32_t key1, uint32_t n, uint32_t j, uint32_t t, uint32_t which,
                                double d, double c, double &value) {
  const Words w = philox4x32_10(n, j, t, which, key0, key1);
  const double u1 = (static_cast<double>(w.w[0]) + 0.5) * (1.0 / 2147483648.0) - 1.0;
  const double u2 = (static_cast<double>(w.w[1]) + 0.5) * (1.0 / 2147483648.0) - 1.0;
  const double s = u1 * u1 + u2 * u2;
  if (s >= 1.0) return false;
  const double x = u1 * sqrt((-2.0 * series_log(s)) / s);
  const double t1 = 1.0 + c * x;
  if (t1 <= 0.0) return false;
  const double v = (t1 * t1) * t1;
  const uint64_t k = (static_cast<uint64_t>(w.w[2]) << 20) | static_cast<uint64_t>(w.w[3] >> 12);
  const double u = (static_cast<double>(k) + 0.5) * (1.0 / 4503599627370496.0);
  const double bound = ((0.5 * (x * x) + d) - d * v) + d * series_log(v);
  value = d * v;
  return series_log(u) < bound;
}

// A team of kTeam consecutive lanes makes one gamma draw: the lanes try kTeam candidates at
// once, the first accepted one in candidate order is the draw (so the result is the one a
// single thread trying them one after the other would get); almost always the first round
// decides.  Sixteen lanes serve a job slot: lanes 0-7 its first gamma, lanes 8-15 the second.
constexpr int kTeam = 8;
constexpr int kLanesPerSlot = 2 * kTeam;

// The draw of slot j for generation t: Y_j = processed_j (1/rho_j - 1), rho_j ~ Be(alpha_j, beta_j)
// (0 for a slot at or beyond Jn).  Called by whole waves with all lanes active, the kLanesPerSlot
// lanes of a slot next to each other and aligned (lane % kLanesPerSlot = position in the slot's
// team); every lane of the slot gets the value.
__device__ inline double draw_remaining(const Progress &pr, uint32_t Jn, uint32_t key0, uint32_t key1, uint32_t t,
                                        uint32_t j) {
  const uint32_t lane = threadIdx.x & (kLanes - 1);
  const uint32_t in_slot = lane % kLanesPerSlot, which = in_slot / kTeam + 1, member = in_slot % kTeam;
  const bool real = j < Jn;
  const double shape = real ? (which == 1 ? pr.alpha[j] : pr.beta[j]) : 1.0;
  const double d = shape - 1.0 / 3.0;
  const double c = 1.0 / sqrt(9.0 * d);
  double draw = d;                                           // what is left when every candidate fails
  bool done = false;
  for (uint32_t first = 0; first < static_cast<uint32_t>(kGammaAttempts); first += kTeam) {
    double value = 0.0;
    const bool ok = !done && gamma_candidate(key0, key1, first + member, j, t, which, d, c, value);
    // the team's accepted candidates as a bit mask, lowest candidate number first
    const uint64_t all = __ballot(ok);
    const uint32_t mine = static_cast<uint32_t>(all >> (lane - member)) & ((1u << kTeam) - 1u);
    const int winner = mine != 0 ? static_cast<int>(lane - member) + __ffs(static_cast<int>(mine)) - 1
                                 : static_cast<int>(lane);
    const double won = __shfl(value, winner, kLanes);
    if (!done && mine != 0) {
      draw = won;
      done = true;
    }
    if (__ballot(!done) == 0) break;
  }
  // lanes 0 and kTeam of the slot now hold its two gamma draws
  const double ga = __shfl(draw, static_cast<int>(lane - in_slot), kLanes);
  const double gb = __shfl(draw, static_cast<int>(lane - in_slot + kTeam), kLanes);
  double Y = 0.0;
  if (real) {
    const double rho = ga / (ga + gb);
    double ratio = 1.0 / rho - 1.0;
    if (ratio > kMaxParam) ratio = kMaxParam;
    Y = pr.processed[j] * ratio;
    if (Y > kMaxParam) Y = kMaxParam;
  }
  return Y;
}

// thread: position among the Jp * kLanesPerSlot threads that serve the Jp slots (whole waves,
// all lanes active).  Writes tab.Y[j] and the slot's entries of tab.terms for generation t.
__device__ inline void sample_remaining_slot(const Progress &pr, const JobTable &tab, uint32_t Jn, uint32_t key0,
                                             uint32_t key1, uint32_t t, uint32_t thread) {
  const uint32_t j = thread / kLanesPerSlot;                 // grid covers Jp slots exactly
  const uint32_t in_slot = (threadIdx.x & (kLanes - 1)) % kLanesPerSlot;
  const double Y = draw_remaining(pr, Jn, key0, key1, t, j);
  if (in_slot == 0) tab.Y[j] = Y;
  // the slot's column of the term table, its entries dealt to the slot's lanes
  const uint32_t E = tab.term_E, col = j % kLanes, row = j / kLanes;
  const uint32_t blexp = info_blexp(tab.info[j]);
  const double abl = tab.abl[j], cc = tab.cc[j], dd = tab.d[j];
  for (uint32_t e = in_slot; e < E; e += kLanesPerSlot)
    tab.terms[(row * E + e) * kLanes + col] = term_of(abl, cc, dd, Y, blexp, e);
}

}  // namespace
}  // namespace ones
