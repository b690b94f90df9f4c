// Evolve kernel of the ONES search (arXiv 2108.03645, Section 3.2.2) for gfx950.
//
// One wave64 owns one pool slot (a crossover wave owns the two children of a pair): the
// job columns lie across the 64 lanes, the rows of a column in a lane's registers.  The
// wave composes the candidate from the survivors of the previous generation (refresh copy,
// uniform crossover, uniform mutation), repairs it to the cluster capacity (refresh + fill
// under Eq. 4), scores it (Eq. 3 with T = Y/X, Eq. 5) and writes genome and score.
#include "ones_device.h"

#include <utility>

#pragma clang fp contract(off)   // every fp64 product and sum is rounded on its own

namespace ones {
namespace {

// ------------------------------------------------------------------ RNG ------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11).
struct Words { uint32_t w[4]; };

__device__ __forceinline__ Words philox4x32_10(uint32_t x0, uint32_t x1, uint32_t x2, uint32_t x3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint64_t pa = static_cast<uint64_t>(x0) * 0xD2511F53ull;
    const uint64_t pb = static_cast<uint64_t>(x2) * 0xCD9E8D57ull;
    const uint32_t n0 = static_cast<uint32_t>(pb >> 32) ^ x1 ^ k0;
    const uint32_t n2 = static_cast<uint32_t>(pa >> 32) ^ x3 ^ k1;
    x1 = static_cast<uint32_t>(pb);
    x3 = static_cast<uint32_t>(pa);
    x0 = n0;
    x2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Words{{x0, x1, x2, x3}};
}

__device__ __forceinline__ uint32_t bounded(uint32_t w, uint32_t n) { return __umulhi(w, n); }

// Per-candidate draw: ranks of the two parents among the K survivors and the rotation of
// the repair order.  Counter block 0xFFFFFFFF is reserved for it.
struct Draw { uint32_t ra, rb, r; };

__device__ __forceinline__ Draw candidate_draw(const EvolveArgs &a, uint32_t p) {
  const Words w = philox4x32_10(0xFFFFFFFFu, p, a.t, 0u, a.key0, a.key1);
  Draw d;
  d.ra = __builtin_amdgcn_readfirstlane(bounded(w.w[0], a.K));
  d.rb = __builtin_amdgcn_readfirstlane(bounded(w.w[1], a.K));
  d.r  = __builtin_amdgcn_readfirstlane(bounded(w.w[2], a.Jp));
  return d;
}

// One 32-bit word per gene: the lane's rows 4q..4q+3 share Philox block q*64 + lane.
template <int R>
__device__ __forceinline__ void gene_words(const EvolveArgs &a, uint32_t p, int lane, uint32_t (&w)[R]) {
#pragma unroll
  for (int q = 0; q < (R + 3) / 4; ++q) {
    const Words x = philox4x32_10(static_cast<uint32_t>(q * kLanes + lane), p, a.t, 0u, a.key0, a.key1);
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (4 * q + k < R) w[4 * q + k] = x.w[k];
  }
}

// --------------------------------------------------------- wave primitives ---------
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v, int lane) {
#pragma unroll
  for (int d = 1; d < kLanes; d <<= 1) {
    const uint32_t up = __shfl_up(v, d, kLanes);
    if (lane >= d) v += up;
  }
  return v;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, kLanes);
  return v;
}

// ------------------------------------------------------------- per-lane state ------
template <int R>
struct Lane {
  uint32_t cstart[R], cmax[R], info[R];
};

template <int R>
__device__ __forceinline__ void load_lane(const JobTable &tab, int lane, Lane<R> &L) {
#pragma unroll
  for (int i = 0; i < R; ++i) {
    const int j = lane + kLanes * i;
    L.cstart[i] = tab.cstart[j];
    L.cmax[i] = tab.cmax[j];
    L.info[i] = tab.info[j];
  }
}

// Global batch -> GPU count after clamp to the window and the free lift: a running job
// holds clamp(B >> mu, cstart, cmax) GPUs; an empty slot has cstart = cmax = 0.
__device__ __forceinline__ uint32_t gpus_from_batch(uint32_t B, uint32_t info, uint32_t cstart, uint32_t cmax) {
  const uint32_t c = min(max(B >> info_mu(info), cstart), cmax);
  return B ? c : 0u;
}

// Redraw of a gene from k in [0, n): 0 = the job is pre-empted, else 2^(lo + k - 1).
__device__ __forceinline__ uint32_t batch_from_draw(uint32_t k, uint32_t info) {
  return k ? (1u << (info_lo(info) + k - 1u)) : 0u;
}

// Accept the longest prefix, in the rotated visiting order, of the asks v whose running
// sum stays within limit.  Visiting order: column-major (a lane's rows are consecutive),
// starting at lane lr, row ir, wrapping.  ok bit i is set iff row i's prefix fits; a row
// with v = 0 does not matter.  Returns the sum of the accepted asks (wave-uniform).
template <int R>
__device__ __forceinline__ uint32_t accept_prefix(const uint32_t (&v)[R], uint32_t limit, uint32_t lr,
                                                  uint32_t ir, int lane, uint32_t &ok) {
  uint32_t run = 0, pre = 0;
#pragma unroll
  for (int i = 0; i < R; ++i) {
    pre = (static_cast<uint32_t>(i) == ir) ? run : pre;   // sum of the lane's rows above ir
    run += v[i];
  }
  const uint32_t incl = wave_inclusive_scan(run, lane);
  const uint32_t excl = incl - run;
  const uint32_t total = __builtin_amdgcn_readlane(incl, kLanes - 1);
  const uint32_t base = __builtin_amdgcn_readlane(excl + pre, lr);   // asks visited "last" (before the start)
  const uint32_t off_hi = excl - base;            // rows at or after the start
  const uint32_t off_lo = excl + (total - base);  // rows before the start: visited after the wrap
  const uint32_t irow = static_cast<uint32_t>(lane) > lr ? 0u : (static_cast<uint32_t>(lane) < lr ? R : ir);
  uint32_t acc = 0;
  run = 0;
  ok = 0;
#pragma unroll
  for (int i = 0; i < R; ++i) {
    run += v[i];
    const uint32_t q = run + (static_cast<uint32_t>(i) >= irow ? off_hi : off_lo);
    const bool fits = q <= limit;
    ok |= fits ? (1u << i) : 0u;
    acc += fits ? v[i] : 0u;
  }
  return __builtin_amdgcn_readfirstlane(wave_sum(acc));
}

// Refresh + fill (Section 3.2.2) on GPU counts c[]; clamp and lift already applied.
template <int R>
__device__ __forceinline__ void repair(uint32_t (&c)[R], const Lane<R> &L, uint32_t G, uint32_t r, int lane) {
  const uint32_t lr = r / R, ir = r % R;
  uint32_t ok;
  // admit: jobs beyond the capacity in visiting order wait (Eq. 4)
  uint32_t used = accept_prefix<R>(c, G, lr, ir, lane, ok);
#pragma unroll
  for (int i = 0; i < R; ++i) c[i] = (ok >> i) & 1u ? c[i] : 0u;
  // fill: a waiting job asks for cstart GPUs, a running one below its limit asks to double
  // Every round accepts at least its first ask, and a job doubles at most 20 times, so
  // kMaxRows * 64 * 21 rounds always suffice; the bound and the got == 0 exit only make the
  // loop end whatever happens.
  uint32_t idle = G - used;
  for (int round = 0; round < kMaxRows * kLanes * 21 && idle > 0; ++round) {
    uint32_t v[R];
    uint32_t any = 0;
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const uint32_t cost = max(c[i], L.cstart[i]);
      v[i] = (c[i] < L.cmax[i] && cost <= idle) ? cost : 0u;
      any |= v[i];
    }
    if (__ballot(any != 0) == 0) break;
    const uint32_t got = accept_prefix<R>(v, idle, lr, ir, lane, ok);
#pragma unroll
    for (int i = 0; i < R; ++i) c[i] += (ok >> i) & 1u ? v[i] : 0u;
    if (got == 0) break;
    idle -= got;
  }
}

// Eq. 3: sum over running jobs of T_j c_j = Y_j t_j / (local batch), t = a b + c log2(g) + d.
// Summation order: a lane's rows top to bottom, then a xor butterfly 32,16,..,1 over lanes.
template <int R>
__device__ __forceinline__ double score(const uint32_t (&c)[R], const Lane<R> &L, const JobTable &tab, int lane) {
  double acc = 0.0;
#pragma unroll
  for (int i = 0; i < R; ++i) {
    const int j = lane + kLanes * i;
    const uint32_t ci = c[i];
    const double lg = static_cast<double>(31 - __clz(static_cast<int>(ci | 1u)));
    const double inv_bl = __hiloint2double(static_cast<int>((1023u - info_blexp(L.info[i])) << 20), 0);
    const double t = (tab.abl[j] + tab.cc[j] * lg) + tab.d[j];
    const double term = (tab.Y[j] * t) * inv_bl;
    acc = acc + (ci ? term : 0.0);
  }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) acc = acc + __shfl_xor(acc, s, kLanes);
  return acc;
}

template <int R>
__device__ __forceinline__ void finish(const EvolveArgs &a, const Lane<R> &L, uint32_t p, uint32_t r,
                                       uint32_t (&c)[R], int lane) {
  repair<R>(c, L, a.G, r, lane);
  const double f = score<R>(c, L, a.tab, lane);
  int32_t *row = a.genes_new + static_cast<size_t>(p) * a.Jp;
#pragma unroll
  for (int i = 0; i < R; ++i) row[lane + kLanes * i] = static_cast<int32_t>(c[i] << info_blexp(L.info[i]));
  if (lane == 0) a.fit[p] = f;
}

template <int R>
__device__ __forceinline__ void load_genes(const int32_t *row, int lane, uint32_t (&B)[R]) {
#pragma unroll
  for (int i = 0; i < R; ++i) B[i] = static_cast<uint32_t>(row[lane + kLanes * i]);
}

// ----------------------------------------------------------------- kernels ---------
constexpr int kWavesPerBlock = 4;

// Initial population G_0: every gene uniform over {waiting, bmin..bmax}.
template <int R>
__global__ __launch_bounds__(kWavesPerBlock * kLanes) void init_kernel(EvolveArgs a) {
  const int lane = threadIdx.x & (kLanes - 1);
  const uint32_t p = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
  if (p >= a.P) return;
  Lane<R> L;
  load_lane<R>(a.tab, lane, L);
  const Draw dr = candidate_draw(a, p);
  uint32_t w[R], c[R];
  gene_words<R>(a, p, lane, w);
#pragma unroll
  for (int i = 0; i < R; ++i) {
    const uint32_t B = info_active(L.info[i]) ? batch_from_draw(bounded(w[i], info_n(L.info[i])), L.info[i]) : 0u;
    c[i] = gpus_from_batch(B, L.info[i], L.cstart[i], L.cmax[i]);
  }
  finish<R>(a, L, p, dr.r, c, lane);
}

// One generation.  Work items: K crossover pairs, K mutants, K refreshed survivors.
template <int R>
__global__ __launch_bounds__(kWavesPerBlock * kLanes) void evolve_kernel(EvolveArgs a) {
  const int lane = threadIdx.x & (kLanes - 1);
  const uint32_t item = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
  const uint32_t K = a.K;
  if (item >= 3 * K) return;
  Lane<R> L;
  load_lane<R>(a.tab, lane, L);
  uint32_t c[R];
  if (item < K) {
    // uniform crossover: per gene the children swap their parents' genes with rate chi
    const uint32_t p0 = K + 2 * item;
    const Draw d0 = candidate_draw(a, p0);
    const Draw d1 = candidate_draw(a, p0 + 1);
    uint32_t A[R], B[R], w[R];
    load_genes<R>(a.genes_old + static_cast<size_t>(a.sel[d0.ra]) * a.Jp, lane, A);
    load_genes<R>(a.genes_old + static_cast<size_t>(a.sel[d0.rb]) * a.Jp, lane, B);
    gene_words<R>(a, p0, lane, w);
#pragma unroll
    for (int i = 0; i < R; ++i)
      c[i] = gpus_from_batch(w[i] < a.T_x ? B[i] : A[i], L.info[i], L.cstart[i], L.cmax[i]);
    finish<R>(a, L, p0, d0.r, c, lane);
#pragma unroll
    for (int i = 0; i < R; ++i)
      c[i] = gpus_from_batch(w[i] < a.T_x ? A[i] : B[i], L.info[i], L.cstart[i], L.cmax[i]);
    finish<R>(a, L, p0 + 1, d1.r, c, lane);
  } else if (item < 2 * K) {
    // uniform mutation: each job redrawn with rate theta (k = 0 pre-empts it)
    const uint32_t p = 3 * K + (item - K);
    const Draw d = candidate_draw(a, p);
    uint32_t A[R], w[R];
    load_genes<R>(a.genes_old + static_cast<size_t>(a.sel[d.ra]) * a.Jp, lane, A);
    gene_words<R>(a, p, lane, w);
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const uint32_t k = ((w[i] & 0xFFFFu) * info_n(L.info[i])) >> 16;
      const uint32_t redrawn = info_active(L.info[i]) ? batch_from_draw(k, L.info[i]) : 0u;
      c[i] = gpus_from_batch(w[i] < a.T_mut ? redrawn : A[i], L.info[i], L.cstart[i], L.cmax[i]);
    }
    finish<R>(a, L, p, d.r, c, lane);
  } else {
    // refresh: the survivor of rank p, projected onto the current job table
    const uint32_t p = item - 2 * K;
    const Draw d = candidate_draw(a, p);
    uint32_t A[R];
    load_genes<R>(a.genes_old + static_cast<size_t>(a.sel[p]) * a.Jp, lane, A);
#pragma unroll
    for (int i = 0; i < R; ++i) c[i] = gpus_from_batch(A[i], L.info[i], L.cstart[i], L.cmax[i]);
    finish<R>(a, L, p, d.r, c, lane);
  }
}

template <int R>
hipError_t launch_rows(const EvolveArgs &a, hipStream_t s) {
  const uint32_t items = a.t == 0 ? a.P : 3 * a.K;
  const uint32_t blocks = (items + kWavesPerBlock - 1) / kWavesPerBlock;
  if (a.t == 0)
    hipLaunchKernelGGL(init_kernel<R>, dim3(blocks), dim3(kWavesPerBlock * kLanes), 0, s, a);
  else
    hipLaunchKernelGGL(evolve_kernel<R>, dim3(blocks), dim3(kWavesPerBlock * kLanes), 0, s, a);
  return hipGetLastError();
}

template <int... Rs>
hipError_t dispatch_rows(const EvolveArgs &a, int rows, hipStream_t s, std::integer_sequence<int, Rs...>) {
  hipError_t rc = hipErrorInvalidValue;
  (void)((rows == Rs + 1 ? (rc = launch_rows<Rs + 1>(a, s), true) : false) || ...);
  return rc;
}

}  // namespace

hipError_t launch_evolve(const EvolveArgs &a, int rows, hipStream_t s) {
  return dispatch_rows(a, rows, s, std::make_integer_sequence<int, kMaxRows>{});
}

}  // namespace ones
