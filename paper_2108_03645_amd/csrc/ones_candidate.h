// Device code that composes, repairs and scores one candidate schedule of the ONES search
// (arXiv 2108.03645, Section 3.2.2) on gfx950: one wave64 per candidate, the job columns across
// the 64 lanes, the rows of a column in the lane's registers.  Shared by the kernels of
// ones_evolve.hip (a generation of a large pool) and ones_fused.hip (all generations of a small
// pool in one launch).
#pragma once

#include "ones_device.h"

#include <algorithm>

#pragma clang fp contract(off)   // every fp64 product and sum is rounded on its own

namespace ones {
namespace {

constexpr size_t kLdsBudget = 160 * 1024;             // LDS of one gfx950 compute unit

// Keeps the instruction scheduler from interleaving two phases of a work item, or too many
// rows of one loop, which would keep all their registers live at once.
__device__ __forceinline__ void phase_fence() {
  asm volatile("" ::: "memory");        // loads stay on their side of the fence in the optimiser
  __builtin_amdgcn_sched_barrier(0);    // ... and in the instruction scheduler
}
__device__ __forceinline__ void fence_every(int i, int n) { if (i % n == n - 1) phase_fence(); }
// Forces x to be computed before the following fence (its producers cannot sink below it).
template <typename T> __device__ __forceinline__ void pin(T &x) { asm volatile("" : "+v"(x)); }
// The lane number, re-materialised so that nothing derived from it (LDS addresses, the first
// Philox round) is hoisted out of the work-item loop and kept live, or spilled, across it.
__device__ __forceinline__ int opaque(int v) { asm volatile("" : "+v"(v)); return v; }

// ------------------------------------------------------------------ RNG ------------
__device__ __forceinline__ uint32_t bounded(uint32_t w, uint32_t n) { return __umulhi(w, n); }

// Per-candidate draw: ranks of the two parents among the K survivors and the rotation of
// the repair order.  Counter block 0xFFFFFFFF is reserved for it.
struct Draw { uint32_t ra, rb, r; };

// t: the generation the draw is for.
__device__ __forceinline__ Draw candidate_draw(const EvolveArgs &a, uint32_t t, uint32_t p) {
  const Words w = philox4x32_10(0xFFFFFFFFu, p, t, 0u, a.key0, a.key1);
  Draw d;
  d.ra = __builtin_amdgcn_readfirstlane(bounded(w.w[0], a.K));
  d.rb = __builtin_amdgcn_readfirstlane(bounded(w.w[1], a.K));
  d.r  = __builtin_amdgcn_readfirstlane(bounded(w.w[2], a.Jp));
  return d;
}

// One 32-bit word per gene: the lane's rows 4q..4q+3 share Philox block q*64 + lane.
template <int R>
__device__ __forceinline__ void gene_words(const EvolveArgs &a, uint32_t t, uint32_t p, int lane, uint32_t (&w)[R]) {
#pragma unroll
  for (int q = 0; q < (R + 3) / 4; ++q) {
    const Words x = philox4x32_10(static_cast<uint32_t>(q * kLanes + lane), p, t, 0u, a.key0, a.key1);
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (4 * q + k < R) w[4 * q + k] = x.w[k];
    fence_every(q, 2);
  }
}

// --------------------------------------------------------- wave primitives ---------
// DPP controls (gfx9): row_shr:n shifts within a row of 16 lanes, row_bcast:15 / :31 copy the
// last lane of a row / of the lower half-wave into the following row(s).
constexpr int kRowShr = 0x110, kRowBcast15 = 0x142, kRowBcast31 = 0x143;

template <int Ctrl, int RowMask, bool Bound>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v) {
  return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), Ctrl, RowMask, 0xF, Bound));
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  v += dpp_or_zero<kRowShr + 1, 0xF, true>(v);
  v += dpp_or_zero<kRowShr + 2, 0xF, true>(v);
  v += dpp_or_zero<kRowShr + 4, 0xF, true>(v);
  v += dpp_or_zero<kRowShr + 8, 0xF, true>(v);
  v += dpp_or_zero<kRowBcast15, 0xA, false>(v);
  v += dpp_or_zero<kRowBcast31, 0xC, false>(v);
  return v;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
  return __builtin_amdgcn_readlane(wave_inclusive_scan(v), kLanes - 1);
}

// ------------------------------------------------------------- job table in LDS ----
struct Smem {
  uint2    *cc2;     // [Jp] {cstart, cmax}: GPUs a waiting job resumes with / at the limit R_j
  uint32_t *info;    // [Jp]
  double   *abl, *cc, *d, *Y;   // [Jp] model parameters (when the term table does not fit)
  double   *terms;   // [E][R][64] T_j c_j of job (row, lane) at GPU-count code E-1-e, or null
  uint64_t *split;   // [kMaxBuckets] bucket splitters, then [1] the K-th survivor's score bits
  uint8_t  *stash;   // [waves][stash_stride] second crossover child while the first is repaired; before
                     //                       that, the coins of a crossover over the GPUs
  uint32_t *free_in_group; // [groups] free rows in each group of kRowGroupWords bitmap words
  uint32_t *rows;          // [4 * kRound] rows of the slots this workgroup fills in the current round
  uint32_t *next_item;     // [1] the next work item of the round that no wave has taken yet
};

// E = entries per job of the term table kept in LDS, 0 = keep the four model parameters.
constexpr uint32_t kRound = 256;                     // survivors' ranks a workgroup covers between two barriers

inline uint32_t row_groups(uint32_t rows) {
  return ((rows + 31) / 32 + kRowGroupWords - 1) / kRowGroupWords;
}

// LDS scratch per wave: a byte per job, or the 256 coin words with their running counts
inline uint32_t stash_stride(uint32_t Jp, bool per_gpu) {
  return per_gpu ? std::max<uint32_t>(Jp, kMaxCoinGpus / 32 * 8) : Jp;
}

inline size_t smem_bytes(uint32_t Jp, int waves, uint32_t E, uint32_t rows, uint32_t stride) {
  return static_cast<size_t>(Jp) * (8 + 4 + (E ? 8 * E : 32)) + (kMaxBuckets + 1) * 8 +
         static_cast<size_t>(waves) * stride + static_cast<size_t>(row_groups(rows)) * 4 + 4 * kRound * 4 + 16;
}

__device__ __forceinline__ Smem carve(unsigned char *base, uint32_t Jp, uint32_t E, uint32_t waves, uint32_t stride) {
  Smem s;
  s.abl = reinterpret_cast<double *>(base);
  s.cc = s.abl + Jp;
  s.d = s.cc + Jp;
  s.Y = s.d + Jp;
  s.terms = E ? s.abl : nullptr;
  s.split = reinterpret_cast<uint64_t *>(s.abl + static_cast<size_t>(Jp) * (E ? E : 4));
  s.cc2 = reinterpret_cast<uint2 *>(s.split + kMaxBuckets + 1);
  s.info = reinterpret_cast<uint32_t *>(s.cc2 + Jp);
  s.stash = reinterpret_cast<uint8_t *>(s.info + Jp);
  s.rows = reinterpret_cast<uint32_t *>(s.stash + static_cast<size_t>(waves) * stride);   // a multiple of 64
  s.next_item = s.rows + 4 * kRound;
  s.free_in_group = s.next_item + 4;
  return s;
}

// Stages the job table into LDS, the work dealt to the `threads` threads (whole waves) that call it
// with tid = 0 .. threads - 1.  No barrier at the end: the caller places one before the first use.
constexpr int kStageBatch = 3;
template <int R>
__device__ __forceinline__ void stage_table(const JobTable &tab, const BucketArgs &bk, const Smem &s, uint32_t Jp,
                                            uint32_t E, uint32_t tid, uint32_t threads) {
  if (bk.nb != 0) {
    for (uint32_t q = tid; q <= kMaxBuckets; q += threads)
      s.split[q] = q < kMaxBuckets ? bk.split[q] : *bk.thresh;
  }
  for (uint32_t j = tid; j < Jp; j += threads) {
    s.cc2[j] = make_uint2(tab.cstart[j], tab.cmax[j]);
    s.info[j] = tab.info[j];
    if (E == 0) {
      s.abl[j] = tab.abl[j];
      s.cc[j] = tab.cc[j];
      s.d[j] = tab.d[j];
      s.Y[j] = tab.Y[j];
    }
  }
  if (E != 0)
    // global memory holds the table row-major ([row][code][lane]); here the code is the slowest
    // index, so that a row's part of the LDS address is a compile-time offset, and the codes
    // run backwards, so that the index follows the count of leading zeros of the GPU count
    // (tiles of 64 entries; a batch of loads in flight per wave before the first LDS store waits for one)
    for (uint32_t first = tid / kLanes; first < E * R; first += kStageBatch * (threads / kLanes)) {
      const uint32_t l = tid % kLanes;
      double v[kStageBatch];
#pragma unroll
      for (int u = 0; u < kStageBatch; ++u) {
        const uint32_t tile = first + u * (threads / kLanes), e = tile / R, row = tile % R;
        if (tile < E * R) v[u] = tab.terms[(row * E + e) * kLanes + l];
      }
#pragma unroll
      for (int u = 0; u < kStageBatch; ++u) {
        const uint32_t tile = first + u * (threads / kLanes), e = tile / R, row = tile % R;
        if (tile < E * R) s.terms[((E - 1 - e) * R + row) * kLanes + l] = v[u];
      }
    }
}

// ------------------------------------------------------------------ free rows ----
// Bits of bitmap word w that stand for free rows (rows beyond P + K count as taken).
__device__ __forceinline__ uint32_t free_bits(const uint32_t *occupied, uint32_t w, uint32_t rows) {
  const uint32_t words = (rows + 31) / 32;
  if (w >= words) return 0u;
  uint32_t f = ~occupied[w];
  if (w == words - 1 && rows % 32 != 0) f &= (1u << (rows % 32)) - 1u;
  return f;
}

// Every workgroup builds the same small index: the number of free rows in each group of
// kRowGroupWords bitmap words.  The first bitmap loads are issued ahead of the rest.
constexpr int kIndexAhead = 4;                       // groups per wave whose words are loaded ahead

struct IndexLoads { uint32_t bits[kIndexAhead]; };

__device__ __forceinline__ IndexLoads index_free_rows_begin(const EvolveArgs &a, int lane) {
  const uint32_t rows = a.P + a.K;
  const uint32_t wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
  IndexLoads ld;
#pragma unroll
  for (int k = 0; k < kIndexAhead; ++k) ld.bits[k] = free_bits(a.occupied, (wave + k * waves) * kRowGroupWords + lane, rows);
  return ld;
}

// Also clears this workgroup's share of the other bitmap.  Ends with a barrier.
__device__ __forceinline__ void index_free_rows_end(const EvolveArgs &a, const Smem &s, const IndexLoads &ld, int lane) {
  const uint32_t rows = a.P + a.K, words = (rows + 31) / 32;
  const uint32_t groups = (words + kRowGroupWords - 1) / kRowGroupWords;
  const uint32_t wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
#pragma unroll
  for (int k = 0; k < kIndexAhead; ++k) {
    const uint32_t n = wave_sum(__popc(ld.bits[k]));
    if (lane == 0 && wave + k * waves < groups) s.free_in_group[wave + k * waves] = n;
  }
  for (uint32_t g = wave + kIndexAhead * waves; g < groups; g += waves) {
    const uint32_t n = wave_sum(__popc(free_bits(a.occupied, g * kRowGroupWords + lane, rows)));
    if (lane == 0) s.free_in_group[g] = n;
  }
  for (uint32_t w = blockIdx.x * blockDim.x + threadIdx.x; w < words; w += gridDim.x * blockDim.x)
    a.occupied_other[w] = 0;
  __syncthreads();
}

// One wave lists the free rows number q0 .. q0 + count - 1 (in ascending order; all below the
// number of free rows) into dst.
__device__ __forceinline__ void list_free_rows(const EvolveArgs &a, const Smem &s, uint32_t q0, uint32_t count,
                                               uint32_t *dst, int lane) {
  const uint32_t rows = a.P + a.K;
  const uint32_t groups = ((rows + 31) / 32 + kRowGroupWords - 1) / kRowGroupWords;
  // the group that holds free row q0, and the free rows before that group
  uint32_t g = groups, before = 0;
  for (uint32_t g0 = 0; g0 < groups; g0 += kLanes) {
    const uint32_t n = g0 + lane < groups ? s.free_in_group[g0 + lane] : 0u;
    const uint32_t incl = wave_inclusive_scan(n);
    const uint64_t beyond = __ballot(before + incl > q0);
    if (beyond != 0) {
      const int l = __builtin_amdgcn_readfirstlane(__ffsll(static_cast<long long>(beyond)) - 1);
      g = g0 + static_cast<uint32_t>(l);
      before += __builtin_amdgcn_readlane(incl - n, l);
      break;
    }
    before += __builtin_amdgcn_readlane(incl, kLanes - 1);
  }
  // position in dst of the first free row of the group being read
  int32_t base = -static_cast<int32_t>(q0 - before);
  for (; g < groups && base < static_cast<int32_t>(count); ++g) {
    const uint32_t w = g * kRowGroupWords + lane;
    uint32_t bits = free_bits(a.occupied, w, rows);
    const uint32_t n = __popc(bits);
    const uint32_t incl = wave_inclusive_scan(n);
    int32_t pos = base + static_cast<int32_t>(incl - n);
    while (bits) {
      if (pos >= 0 && pos < static_cast<int32_t>(count)) dst[pos] = w * 32 + (__ffs(static_cast<int>(bits)) - 1);
      bits &= bits - 1;
      ++pos;
    }
    base += static_cast<int32_t>(__builtin_amdgcn_readlane(incl, kLanes - 1));
  }
}

// The kernel's own argument block, for values that only a rare path needs: read there, at the
// point of use, they are not carried (and spilled) through every work item.  Valid in kernels
// whose argument block starts with one EvolveArgs passed by value, which every kernel that
// includes this header must take (each of them says so at its signature).
using KernelArgs = const __attribute__((address_space(4))) EvolveArgs;
__device__ __forceinline__ KernelArgs *kernel_args() {
  KernelArgs *ka = (KernelArgs *)__builtin_amdgcn_kernarg_segment_ptr();
  asm volatile("" : "+s"(ka));
  return ka;
}

// A row index is kept inside the genome array whatever the free-row list holds, so that a mistake
// in it cannot turn into a stray access; but such a mistake must not pass unnoticed either.
// Every entry of a round's list passes through checked_row once, when the kernel records the
// rows of the round's slots: a clamp that changes a value is noted in LDS (s.next_item[1]) and
// the workgroup raises the context's fault word, which ones_export reports, when it ends.
__device__ __forceinline__ uint32_t checked_row(const Smem &s, uint32_t row, uint32_t n_rows) {
  if (row >= n_rows) s.next_item[1] = 1;
  return min(row, n_rows - 1);
}

// Row listed at position i of the current round (wave-uniform); never outside the genome array.
// (No note here: this sits in the work-item loop, whose register allocation has no room to spare,
// and reads the entries that checked_row has seen.)
__device__ __forceinline__ uint32_t row_at(const Smem &s, uint32_t i, const EvolveArgs &a) {
  return min(static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(s.rows[i])), a.P + a.K - 1);
}

// Global batch -> GPU count.  In general: clamp to the window and lift for free to the
// per-GPU max batch, i.e. clamp(B >> mu, cstart, cmax) for a running job.  A gene written by
// this kernel under the same job table is already of the form c << bl_exp.
template <int R, bool kSameTable>
__device__ __forceinline__ void gpus_from_batches(const Smem &s, int lane, uint32_t (&c)[R]) {
#pragma unroll
  for (int i = 0; i < R; ++i) {
    const int j = lane + kLanes * i;
    const uint32_t w = s.info[j];
    if (kSameTable) {
      c[i] = c[i] >> info_blexp(w);
    } else {
      const uint2 k = s.cc2[j];
      const uint32_t g = min(max(c[i] >> info_mu(w), k.x), k.y);
      c[i] = c[i] ? g : 0u;
    }
    fence_every(i, 8);
  }
}

// Accept the longest prefix, in the rotated visiting order, of the asks v whose running sum
// stays within limit.  Visiting order: column-major (a lane's rows are consecutive), starting
// at lane lr, row ir, wrapping.  On return v[i] is unchanged if accepted, else 0; returns the
// accepted sum (wave-uniform).
template <int R>
__device__ __forceinline__ uint32_t accept_prefix(uint32_t (&v)[R], uint32_t limit, uint32_t lr, uint32_t ir,
                                                  int lane) {
  // first pass: lane totals, with the running sum noted after every eighth row
  constexpr int kBlocks = (R + 7) / 8;
  uint32_t run = 0, snap[kBlocks];
#pragma unroll
  for (int i = 0; i < R; ++i) {
    run += v[i];
    if (i % 8 == 7 || i == R - 1) snap[i / 8] = run;
  }
  const uint32_t incl = wave_inclusive_scan(run);
  const uint32_t total = __builtin_amdgcn_readlane(incl, kLanes - 1);
  if (total <= limit) return total;                // everything fits: no second pass
  const uint32_t excl = incl - run;
  // pre = sum of the lane's rows above ir (only lane lr's value is used): the snapshot of the
  // blocks before ir's block plus the rows of that block above ir.  ir is wave-uniform.
  uint32_t pre = 0;
#pragma unroll
  for (int k = 0; k < kBlocks; ++k) {
    if (ir / 8 == static_cast<uint32_t>(k)) {
      if (k > 0) pre = snap[k - 1];
#pragma unroll
      for (int t = 0; t < 7; ++t)
        if (8 * k + t < R && static_cast<uint32_t>(t) < ir % 8) pre += v[8 * k + t];
    }
  }
  const uint32_t base = __builtin_amdgcn_readlane(excl + pre, lr);   // asks visited after the wrap
  // A row's prefix is run_i + off; it fits iff run_i <= limit - off (0 when off exceeds the
  // limit: then only rows without an ask "fit", which changes nothing).
  const uint32_t off_hi = excl - base;             // rows at or after the start
  const uint32_t off_lo = excl + (total - base);   // rows before the start, visited after the wrap
  const bool at = static_cast<uint32_t>(lane) == lr;
  // off_hi of lane lr is -pre (mod 2^32): add pre to the threshold instead
  const uint32_t thr_hi = at ? limit + pre : (off_hi <= limit ? limit - off_hi : 0u);
  const uint32_t thr_lo = off_lo <= limit ? limit - off_lo : 0u;
  // first row of the lane that is visited before the wrap (a per-lane value on purpose, so
  // that the row test below is one vector compare instead of a scalar mask per row)
  const uint32_t first_hi = static_cast<uint32_t>(lane) > lr ? 0u : (at ? ir : static_cast<uint32_t>(R));
  uint32_t acc = 0;
  run = 0;
#pragma unroll
  for (int i = 0; i < R; ++i) {
    run += v[i];
    const uint32_t thr = static_cast<uint32_t>(i) >= first_hi ? thr_hi : thr_lo;
    v[i] = run <= thr ? v[i] : 0u;
    acc += v[i];
  }
  return wave_sum(acc);
}

// Refresh + fill (Section 3.2.2) on GPU counts c[]; clamp and lift already applied.
// new_first (only in the generation after a table change): the jobs that arrived with the table
// are served first (refresh (3)): each starts on cstart GPUs while the capacity lasts, in
// visiting order, and the others are admitted to what is left: in visiting order too, or, with
// time_rank (position of every job in ascending order of executed time), least executed time
// first, so that the room is taken from the jobs with the largest T_processed.
template <int R>
__device__ __forceinline__ void repair(uint32_t (&c)[R], const Smem &s, uint32_t G, uint32_t r, int lane,
                                       bool new_first, const uint32_t *time_rank = nullptr) {
  const uint32_t lr = r / R, ir = r % R;
  uint32_t used;
  if (new_first) {
    uint32_t v[R];
#pragma unroll
    for (int i = 0; i < R; ++i) v[i] = info_new(s.info[lane + kLanes * i]) ? s.cc2[lane + kLanes * i].x : 0u;
    const uint32_t taken = accept_prefix<R>(v, G, lr, ir, lane);
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const bool is_new = info_new(s.info[lane + kLanes * i]) != 0;
      c[i] = is_new ? v[i] : c[i];
      v[i] = is_new ? 0u : c[i];
    }
    phase_fence();
    if (time_rank) {
      // The running sum over the ranks never decreases, so the admitted jobs are the ranks below
      // some bound: the largest n whose first n ranks ask for no more than what is left.
      const uint32_t cap = G - taken;
      uint32_t rk[R];
#pragma unroll
      for (int i = 0; i < R; ++i) rk[i] = time_rank[lane + kLanes * i];
      uint32_t lo = 0, hi = static_cast<uint32_t>(R * kLanes), fits = 0;   // the first lo ranks fit (sum fits)
      while (lo < hi) {                                                    // at most log2(R * 64) + 1 steps
        const uint32_t mid = (lo + hi + 1) / 2;
        uint32_t sum = 0;
#pragma unroll
        for (int i = 0; i < R; ++i) sum += rk[i] < mid ? v[i] : 0u;
        sum = wave_sum(sum);
        if (sum <= cap) { lo = mid; fits = sum; } else { hi = mid - 1; }
      }
#pragma unroll
      for (int i = 0; i < R; ++i) v[i] = rk[i] < lo ? v[i] : 0u;
      used = taken + fits;
    } else {
      used = taken + accept_prefix<R>(v, G - taken, lr, ir, lane);
    }
#pragma unroll
    for (int i = 0; i < R; ++i) c[i] = info_new(s.info[lane + kLanes * i]) ? c[i] : v[i];
  } else {
    // admit: jobs beyond the capacity in visiting order wait (Eq. 4)
    used = accept_prefix<R>(c, G, lr, ir, lane);
  }
  // fill: a waiting job asks for cstart GPUs, a running one below its limit asks to double.
  // Every round accepts at least its first ask (got == 0: nobody could ask), and a job doubles
  // at most 20 times, so kMaxRows * 64 * 21 rounds always suffice; the bound only makes the
  // loop end whatever happens.
  uint32_t idle = G - used;
  for (int round = 0; round < kMaxRows * kLanes * 21 && idle > 0; ++round) {
    uint32_t v[R];
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const uint2 k = s.cc2[lane + kLanes * i];
      const uint32_t cost = max(c[i], k.x);
      v[i] = (c[i] < k.y && cost <= idle) ? cost : 0u;
      if (i % 8 == 7) { pin(v[i]); phase_fence(); }
    }
    const uint32_t got = accept_prefix<R>(v, idle, lr, ir, lane);
#pragma unroll
    for (int i = 0; i < R; ++i) c[i] += v[i];
    if (got == 0) break;
    idle -= got;
  }
}

// Eq. 3: sum over running jobs of T_j c_j = Y_j t_j / (local batch), t = a b + c log2(g) + d.
// Summation order: a lane's rows top to bottom, then a xor butterfly 32,16,..,1 over lanes.
template <int R>
__device__ __forceinline__ double score(const uint32_t (&c)[R], const Smem &s, uint32_t E, int lane) {
  double acc = 0.0;
  if (E != 0) {
    // the job's term only depends on its GPU count c = 2^(code-1) (code 0: waiting), and the
    // table holds exactly the value the formula below produces
    // code = 32 - z with z the leading zeros of c (32 for a waiting job); the table is stored
    // with the codes backwards, entry E-1-code = z - (33 - E)
    // (column itself lies before the table; every address formed from it lies inside: z >= 33 - E)
    const double *column = s.terms + lane + (static_cast<int>(E) - 33) * (R * kLanes);
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const int z = __clz(static_cast<int>(c[i]));
      acc = acc + (column + z * (R * kLanes))[i * kLanes];
      if (i % 8 == 7) { pin(acc); phase_fence(); }
    }
  } else
#pragma unroll
  for (int i = 0; i < R; ++i) {
    const int j = lane + kLanes * i;
    const uint32_t ci = c[i];
    const double lg = static_cast<double>(31 - __clz(static_cast<int>(ci | 1u)));
    const double inv_bl = __hiloint2double(static_cast<int>((1023u - info_blexp(s.info[j])) << 20), 0);
    const double t = (s.abl[j] + s.cc[j] * lg) + s.d[j];
    const double term = (s.Y[j] * t) * inv_bl;
    acc = acc + (ci ? term : 0.0);
    if (i % 4 == 3) { pin(acc); phase_fence(); }
  }
#pragma unroll
  for (int sft = 32; sft >= 1; sft >>= 1) acc = acc + __shfl_xor(acc, sft, kLanes);
  return acc;
}

// The score of pool slot p, for a general selection that follows (the pointer is read from the
// kernel's argument block at the point of use, like the bucket storage below).
__device__ __forceinline__ void note_slot_score(uint32_t p, double f, int lane) {
  if (lane == 0) kernel_args()->slot_score[p] = f;
}

// A child or mutant that beats the K-th survivor joins the bucket of the survivors it falls
// between: bucket = number of splitters <= its score.  Scores at or above the threshold
// cannot be among the best K (the K survivors themselves are in the pool, in smaller slots).
__device__ __forceinline__ void drop_in_bucket(const EvolveArgs &a, const Smem &s, uint32_t p, double f, int lane) {
  const uint64_t raw = static_cast<uint64_t>(__double_as_longlong(f));
  // the butterfly leaves the same sum in every lane; make that visible to the compiler
  // (the builtin returns a signed int: widen through uint32_t, not by sign extension)
  const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(raw >> 32)));
  const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(raw)));
  const uint64_t bits = (static_cast<uint64_t>(hi) << 32) | lo;
  if (bits >= s.split[kMaxBuckets]) return;
  uint32_t b = 0;
  for (uint32_t q = 0; q * kLanes + 1 < a.bk.nb; ++q)      // splitters 0 .. nb-2, the rest is +inf
    b += static_cast<uint32_t>(__popcll(__ballot(s.split[q * kLanes + lane] <= bits)));
  if (lane == 0) {
    // The pointers of the bucket storage are read from the kernel's argument block here, where
    // the few candidates that get this far need them, instead of being carried (and spilled)
    // through every work item.
    KernelArgs *ka = kernel_args();
    uint32_t *count = ka->bk.count;
    const uint32_t seg = ka->bk.seg;
    const uint32_t slot = atomicAdd(&count[b], 1u);
    if (slot < seg) {
      const size_t at = static_cast<size_t>(b) * seg + slot;
      ka->bk.keys[at] = bits;
      ka->bk.idx[at] = p;
    } else {                                               // bucket full: shared spill list
      const uint32_t at = atomicAdd(&count[kSpillCounter], 1u);
      ka->bk.spill_keys[at] = bits;
      ka->bk.spill_idx[at] = p;
      ka->bk.spill_bucket[at] = b;
    }
  }
}

template <int R>
__device__ __forceinline__ double finish(const EvolveArgs &a, const Smem &s, uint32_t dst_row, uint32_t r,
                                         uint32_t (&c)[R], int lane, bool new_first = false) {
  repair<R>(c, s, a.G, r, lane, new_first, a.time_rank);
  phase_fence();
  const double f = score<R>(c, s, a.term_lds, lane);
  phase_fence();
  int32_t *row = a.genes + static_cast<size_t>(dst_row) * a.Jp;
#pragma unroll
  for (int i = 0; i < R; ++i)
    __builtin_nontemporal_store(static_cast<int32_t>(c[i] << info_blexp(s.info[lane + kLanes * i])),
                                &row[lane + kLanes * i]);
  if (lane == 0) a.fit_row[dst_row] = f;
  return f;
}

template <int R>
__device__ __forceinline__ void load_genes(const int32_t *row, int lane, uint32_t (&B)[R]) {
#pragma unroll
  for (int i = 0; i < R; ++i) B[i] = static_cast<uint32_t>(row[lane + kLanes * i]);
}

// Uniform crossover over the GPUs (Section 3.2.2 on the encoding of Eq. 1).  Both parents are
// laid out as the reorder operator leaves them: the jobs in slot order on consecutive GPUs, cA
// resp. cB GPUs each, GPUs beyond the cluster do not exist.  Every GPU has a fair coin: heads,
// the first parent's job on it goes to the first child and the second parent's to the second
// child; tails, the other way round.  A child then runs each job on the largest power of two
// among the GPUs it inherited for it, inside the job's window.  On return cA holds the first
// child and cB the second.
// Coin of GPU i: bit i mod 32 of word (i mod 128) div 32 of Philox block (i div 128, p0, t, 3);
// lane l draws the coins of GPUs 128 l .. 128 l + 127.  coins: this wave's kMaxCoinGpus / 32
// entries of LDS, each a coin word and, above it, the number of heads on the GPUs before it.
// kFeasible: both parents are known to fit the cluster (they were repaired under the current
// job table), so no GPU position needs to be cut off at the cluster's size.
template <int R, bool kFeasible>
__device__ __forceinline__ void crossover_over_gpus(const EvolveArgs &a, uint32_t t, const Smem &s, uint64_t *coins, uint32_t p0,
                                                    int lane, uint32_t (&cA)[R], uint32_t (&cB)[R]) {
  {
    const Words w = philox4x32_10(static_cast<uint32_t>(lane), p0, t, 3u, a.key0, a.key1);
    const uint32_t heads = __popc(w.w[0]) + __popc(w.w[1]) + __popc(w.w[2]) + __popc(w.w[3]);
    uint32_t before = wave_inclusive_scan(heads) - heads;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      coins[4 * lane + k] = (static_cast<uint64_t>(before) << 32) | w.w[k];
      before += __popc(w.w[k]);
    }
  }
  // the lanes read each other's entries: one wave, whose LDS operations complete in order
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  phase_fence();
  // heads among the GPUs below x, x <= G <= kMaxCoinGpus
  auto heads_below = [&](uint32_t x) {
    const uint32_t word = min(x >> 5, static_cast<uint32_t>(kMaxCoinGpus / 32 - 1));
    const uint32_t bits = x - (word << 5);                       // 0 .. 32
    const uint64_t e = coins[word];
    const uint32_t mask = bits >= 32u ? 0xFFFFFFFFu : (1u << bits) - 1u;
    return static_cast<uint32_t>(e >> 32) + static_cast<uint32_t>(__popc(static_cast<uint32_t>(e) & mask));
  };
  // A job's first GPU is the GPU after its predecessor's last one (slot order: the lane to the left,
  // or the last lane of the row above), so the heads below a job's range are looked up once, at
  // its end, and its start takes the predecessor's value.
  uint32_t carry_a = 0, carry_b = 0;                             // GPUs of the rows above (wave-uniform)
  uint32_t above_a = 0, above_b = 0;                             // heads below the first GPU of the row (wave-uniform)
#pragma unroll
  for (int i = 0; i < R; ++i) {
    const uint32_t incl_a = wave_inclusive_scan(cA[i]), incl_b = wave_inclusive_scan(cB[i]);
    uint32_t end_a = carry_a + incl_a, start_a = end_a - cA[i];
    uint32_t end_b = carry_b + incl_b, start_b = end_b - cB[i];
    if (!kFeasible) {
      end_a = min(end_a, a.G); start_a = min(start_a, a.G);
      end_b = min(end_b, a.G); start_b = min(start_b, a.G);
    }
    carry_a += __builtin_amdgcn_readlane(incl_a, kLanes - 1);
    carry_b += __builtin_amdgcn_readlane(incl_b, kLanes - 1);
    const uint32_t at_end_a = heads_below(end_a), at_end_b = heads_below(end_b);
    const uint32_t left_a = __shfl_up(at_end_a, 1, kLanes), left_b = __shfl_up(at_end_b, 1, kLanes);
    const uint32_t heads_a = at_end_a - (lane == 0 ? above_a : left_a);
    const uint32_t heads_b = at_end_b - (lane == 0 ? above_b : left_b);
    above_a = __builtin_amdgcn_readlane(at_end_a, kLanes - 1);
    above_b = __builtin_amdgcn_readlane(at_end_b, kLanes - 1);
    const uint32_t n1 = heads_a + ((end_b - start_b) - heads_b);
    const uint32_t n2 = ((end_a - start_a) - heads_a) + heads_b;
    const uint2 k = s.cc2[lane + kLanes * i];
    cA[i] = n1 ? min(max(0x80000000u >> __clz(static_cast<int>(n1)), k.x), k.y) : 0u;
    cB[i] = n2 ? min(max(0x80000000u >> __clz(static_cast<int>(n2)), k.x), k.y) : 0u;
    fence_every(i, 4);
  }
}

// Redraw of a gene from k in [0, n): 0 = the job is pre-empted, else 2^(lo + k - 1).
__device__ __forceinline__ uint32_t batch_from_draw(uint32_t k, uint32_t info) {
  const uint32_t b = (info_active(info) << (info_lo(info) + k)) >> 1;   // k = 0 or empty slot -> 0
  return k ? b : 0u;
}

}  // namespace
}  // namespace ones
