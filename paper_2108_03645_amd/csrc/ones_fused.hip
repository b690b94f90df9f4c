// All generations of one ones_generation call in a single launch (ONES, arXiv 2108.03645,
// Section 3.2.2), for the pools the paper itself schedules with (population = cluster size,
// Section 3.2.2 "Initialization"; 64 GPUs in Section 4.1): at most 64 job slots and
// kFusedMaxPool candidates.
//
// Two launches per generation cost more than the generation itself at this size, so here a
// co-resident grid stays on the chip for the whole call.  Per generation every wave composes,
// repairs and scores its share of the 3K children (4K candidates after a table change) and
// publishes genome and score; every workgroup then collects all scores and ranks the pool by
// itself in its LDS: the survivors' scores, rows and the list of free rows are kept there
// redundantly, so the only data that cross workgroups are the genomes and one score per
// candidate.  While the job table stays the same the K survivors reappear with the scores they
// had, already in order, so the ranking is a merge of the few children that beat the K-th
// survivor into that order; when there are many of them, or after a table change, every
// workgroup ranks a share of the pool by counting and the ranks are exchanged like the scores.
//
// Exchange.  Data written by one workgroup and read by another inside the launch (genomes,
// scores, ranks) go through relaxed atomic stores and loads at device scope, which the hardware
// performs at the device's point of coherence instead of in the caches of one XCD.  There is no
// barrier: a published score carries a tag (its sign bit, which a score never uses, alternating
// with every reuse of the exchange buffer; ranks carry the generation number), a reader polls
// until every entry shows the tag of the current generation, and a wave publishes its score only
// after its genome stores have been acknowledged.  Seeing all scores of a generation therefore
// means that every wave has finished reading that generation's parents and writing its
// children, which is all the ordering the rows need.  Every poll is bounded: a workgroup that
// gives up sets an error word and leaves, and so, in time, do all others.
#include "ones_candidate.h"
#include "ones_sample.h"
#include "ones_sort.h"

#include <cstddef>
#include <cstdlib>

namespace ones {
namespace {

#ifndef ONES_FUSED_WAVES
#define ONES_FUSED_WAVES 8
#endif
#ifndef ONES_FUSED_WORKGROUPS
#define ONES_FUSED_WORKGROUPS 192
#endif
constexpr int kFusedWaves = ONES_FUSED_WAVES;          // waves per workgroup
constexpr int kFusedThreads = kFusedWaves * kLanes;
constexpr uint32_t kFusedMaxWorkgroups = ONES_FUSED_WORKGROUPS;
#ifndef ONES_FUSED_SAMPLED_WORKGROUPS
#define ONES_FUSED_SAMPLED_WORKGROUPS 248
#endif
constexpr uint32_t kFusedMaxSampledWorkgroups = ONES_FUSED_SAMPLED_WORKGROUPS;   // plus the drawing ones: one per compute unit at most
constexpr uint32_t kFusedUnits = 4;          // most units (candidates) one wave computes per generation
constexpr uint32_t kMergeMax = 128;          // children beating the K-th survivor that are still merged locally
constexpr int kGatherPer = (kFusedMaxPool + kFusedThreads - 1) / kFusedThreads;   // entries per thread when a workgroup collects P values

template <typename T>
__device__ __forceinline__ T shared_load(const T *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ void shared_store(T *p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Tag of the n-th use (n = 0, 1, ..) of a pair of exchange buffers that start out zeroed: use n
// goes to buffer n & 1 and flips the tag that buffer's entries carried before.
__device__ __forceinline__ uint64_t use_tag(uint32_t n) { return static_cast<uint64_t>(((n >> 1) & 1u) ^ 1u) << 63; }
constexpr uint64_t kTagBit = 1ull << 63;
// The draws of the remaining work are published two generations ahead, so they rotate through
// four buffers instead of two.
constexpr uint32_t kDrawBuffers = 4;
constexpr uint32_t kDrawGroups = (kLanes / 4 + kFusedWaves - 1) / kFusedWaves;   // workgroups that only draw: a wave per four slots
static_assert(kDrawGroups * kFusedWaves == kLanes / 4, "the drawing workgroups have exactly one wave per four job slots");
__device__ __forceinline__ uint64_t draw_tag(uint32_t n) { return static_cast<uint64_t>(((n / kDrawBuffers) & 1u) ^ 1u) << 63; }

// Per-workgroup copy of the search state between two generations, plus scratch of the ranking.
struct Ranks {
  uint64_t *skeys;     // [2][K] score bits of the survivors, best first (two generations alternate)
  uint16_t *srows;     // [2][K] their genome rows
  uint32_t K;
  // (pointer arithmetic instead of an array of pointers: a runtime index into such an array would
  // put this struct into scratch memory)
  __device__ __forceinline__ uint64_t *skey(int which) const { return skeys + static_cast<uint32_t>(which) * K; }
  __device__ __forceinline__ uint16_t *srow(int which) const { return srows + static_cast<uint32_t>(which) * K; }
  uint16_t *nsel;      // [K] pool slot each new survivor had in the generation just ranked
  uint16_t *frow;      // [P] the free rows in ascending order: unit u of a generation writes row frow[u]
  uint64_t *ckey;      // [P] score bits by pool slot
  uint64_t *mkey;      // [3K] children that beat the K-th survivor
  uint32_t *mslot;     // [3K]
  uint64_t *okey;      // [kMergeMax] ... in order
  uint32_t *oslot;     // [kMergeMax]
  uint32_t *below;     // [kMergeMax] counters of the rankings by counting
  uint32_t *occ;       // bitmap over the P + K rows: the survivors' rows
  uint32_t *wfree;     // free rows before each word of the bitmap
  uint32_t *misc;      // [0] number of children that beat the K-th survivor, [1] whether there is one
  uint32_t *draws;     // [waves][kFusedUnits][4] per unit: ranks of the parents, rotation (drawn ahead)
  uint32_t *words;     // [waves][kFusedUnits][64] per unit: the gene words (drawn ahead)
  uint64_t *ukeys;     // [waves][kFusedUnits] per unit: the score, until the wave publishes it
  double   *ydraw;     // [64] remaining work of every slot as drawn for the generation being computed (Alg. 1)
  double   *model;     // [3][64] the slots' a * local batch, c and d, from which a draw gives the term table
};

inline size_t ranks_bytes(uint32_t P) {
  const size_t K = P / 4;
  return 2 * K * 8 + 2 * K * 2 + K * 2 + P * 2 + P * 8 + 3 * K * 8 + 3 * K * 4 + kMergeMax * (8 + 4 + 4) +
         ((P + K + 31) / 32) * 8 + 16 + kFusedWaves * kFusedUnits * ((4 + kLanes) * 4 + 8) + 4 * kLanes * 8 + 64;
}

__device__ __forceinline__ Ranks carve_ranks(unsigned char *base, uint32_t P) {
  const uint32_t K = P / 4;
  Ranks r;
  r.K = K;
  r.ydraw = reinterpret_cast<double *>(base);
  r.model = r.ydraw + kLanes;
  r.ukeys = reinterpret_cast<uint64_t *>(r.model + 3 * kLanes);
  r.skeys = r.ukeys + kFusedWaves * kFusedUnits;
  r.ckey = r.skeys + 2 * K;
  r.mkey = r.ckey + P;
  r.okey = r.mkey + 3 * K;
  r.mslot = reinterpret_cast<uint32_t *>(r.okey + kMergeMax);
  r.oslot = r.mslot + 3 * K;
  r.below = r.oslot + kMergeMax;
  r.occ = r.below + kMergeMax;
  r.wfree = r.occ + (P + K + 31) / 32;
  r.misc = r.wfree + (P + K + 31) / 32;
  r.draws = r.misc + 4;
  r.words = r.draws + kFusedWaves * kFusedUnits * 4;
  r.srows = reinterpret_cast<uint16_t *>(r.words + kFusedWaves * kFusedUnits * kLanes);
  r.nsel = r.srows + 2 * K;
  r.frow = r.nsel + K;
  return r;
}

// The survivors' rows (rows[0..K)) as a bitmap, and from it the free rows in ascending order.
// from_bitmap: the bitmap is there already.  Whole workgroup; ends with a barrier.
__device__ __forceinline__ void list_free_rows(const Ranks &rk, const uint16_t *rows, uint32_t P, bool from_bitmap) {
  const uint32_t K = P / 4, n_rows = P + K, words = (n_rows + 31) / 32;   // at most 80 words
  if (!from_bitmap) {
    for (uint32_t w = threadIdx.x; w < words; w += blockDim.x) rk.occ[w] = 0;
    __syncthreads();
    for (uint32_t g = threadIdx.x; g < K; g += blockDim.x) atomicOr(&rk.occ[rows[g] >> 5], 1u << (rows[g] & 31u));
    __syncthreads();
  }
  // free rows before each bitmap word (one wave scans the words' counts), ...
  if (threadIdx.x < kLanes) {
    uint32_t carry = 0;
    for (uint32_t base = 0; base < words; base += kLanes) {
      const uint32_t w = base + threadIdx.x;
      const uint32_t n = w < words ? __popc(~rk.occ[w]) : 0u;   // bits beyond the last row are never looked at
      const uint32_t incl = wave_inclusive_scan(n);
      if (w < words) rk.wfree[w] = carry + incl - n;
      carry += __builtin_amdgcn_readlane(incl, kLanes - 1);
    }
  }
  __syncthreads();
  // ... then every row finds its own place in the list
  for (uint32_t row = threadIdx.x; row < n_rows; row += blockDim.x) {
    const uint32_t free_bits = ~rk.occ[row >> 5], bit = row & 31u;
    if ((free_bits >> bit) & 1u) {
      const uint32_t pos = rk.wfree[row >> 5] + __popc(free_bits & ((1u << bit) - 1u));
      if (pos < P) rk.frow[pos] = static_cast<uint16_t>(row);
    }
  }
  __syncthreads();
}

// Row of pool slot p in the generation just computed.
__device__ __forceinline__ uint32_t row_of_slot(const Ranks &rk, int cur, uint32_t p, uint32_t K, bool changed) {
  if (p >= K) return rk.frow[p - K];
  return changed ? rk.frow[3 * K + p] : rk.srow(cur)[p];
}

// Collects published 64-bit entries from two arrays at once (n2 may be 0): thread t takes entries
// t, t + threads, ... of each, polls until every one is ready and hands it to the array's take.
// False when the polls ran out.
template <typename Ready1, typename Take1, typename Ready2, typename Take2>
__device__ __forceinline__ bool gather2(const uint64_t *src1, uint32_t n1, Ready1 ready1, Take1 take1,
                                        const uint64_t *src2, uint32_t n2, Ready2 ready2, Take2 take2,
                                        uint32_t spin_limit) {
  uint32_t pending1 = 0, pending2 = 0;
#pragma unroll
  for (int k = 0; k < kGatherPer; ++k) {
    if (threadIdx.x + k * kFusedThreads < n1) pending1 |= 1u << k;
    if (threadIdx.x + k * kFusedThreads < n2) pending2 |= 1u << k;
  }
  for (uint32_t spins = 0; (pending1 | pending2) != 0; ++spins) {
    if (spins >= spin_limit) return false;
    uint64_t v1[kGatherPer], v2[kGatherPer];
#pragma unroll
    for (int k = 0; k < kGatherPer; ++k) {
      if ((pending1 >> k) & 1u) v1[k] = shared_load(src1 + threadIdx.x + k * kFusedThreads);
      if ((pending2 >> k) & 1u) v2[k] = shared_load(src2 + threadIdx.x + k * kFusedThreads);
    }
#pragma unroll
    for (int k = 0; k < kGatherPer; ++k) {
      if (((pending1 >> k) & 1u) && ready1(v1[k])) {
        take1(threadIdx.x + k * kFusedThreads, v1[k]);
        pending1 &= ~(1u << k);
      }
      if (((pending2 >> k) & 1u) && ready2(v2[k])) {
        take2(threadIdx.x + k * kFusedThreads, v2[k]);
        pending2 &= ~(1u << k);
      }
    }
  }
  return true;
}

// The same for one array.
template <typename Ready, typename Take>
__device__ __forceinline__ bool gather(const uint64_t *src, uint32_t n, uint32_t spin_limit, Ready ready, Take take) {
  return gather2(src, n, ready, take, src, 0u, ready, take, spin_limit);
}

// What a child or mutant draws before it needs anything of its parents: the parents' ranks and
// the rotation of its repair (draw_parents), its word per gene (draw_words).  Both depend on
// (seed, generation, slot) only, so a wave draws for the coming generation while the scores of
// the current generation are still arriving.
__device__ __forceinline__ void draw_parents(const EvolveArgs &a, uint32_t t, uint32_t u, int lane, uint32_t *draws) {
  const uint32_t K = a.K;
  Draw d;
  if (u < 2 * K) {                                   // child of a pair: both share the pair's parents
    const uint32_t p0 = K + (u & ~1u);
    d = candidate_draw(a, t, p0);
    if (u & 1u) d.r = candidate_draw(a, t, p0 + 1).r;
  } else {
    d = candidate_draw(a, t, K + u);
  }
  if (lane == 0) { draws[0] = d.ra; draws[1] = d.rb; draws[2] = d.r; }
}

template <bool kOverGpus>
__device__ __forceinline__ void draw_words(const EvolveArgs &a, uint32_t t, uint32_t u, int lane, uint32_t *words) {
  const uint32_t K = a.K;
  uint32_t w[1] = {0u};
  if (u >= 2 * K) gene_words<1>(a, t, K + u, lane, w);
  else if (!kOverGpus) gene_words<1>(a, t, K + (u & ~1u), lane, w);   // both children share the pair's words
  words[lane] = w[0];
}

// One candidate of generation t: unit u < 2K is a child of pair u / 2, u < 3K a mutant, u >= 3K
// (only after a table change) the survivor of rank u - 3K to refresh.  srow: rows of the
// survivors by rank.  Returns the score; the repaired GPU counts are left in c.
template <bool kSameTable, bool kOverGpus>
__device__ __forceinline__ double compose_unit(const EvolveArgs &a, uint32_t t, const Smem &s, const uint16_t *srow,
                                               uint32_t u, bool new_first, uint8_t *stash, const uint32_t *draws,
                                               const uint32_t *words, int lane, uint32_t (&c)[1]) {
  const uint32_t K = a.K;
  uint32_t r;
  auto gene_of = [&](uint32_t row) {
    return static_cast<uint32_t>(shared_load(a.genes + static_cast<size_t>(row) * kLanes + lane));
  };
  if (u < 3 * K) {
    const uint32_t ra = __builtin_amdgcn_readfirstlane(draws[0]), rb = __builtin_amdgcn_readfirstlane(draws[1]);
    r = __builtin_amdgcn_readfirstlane(draws[2]);
    const uint32_t w = words[lane];
    if (u < 2 * K) {
      const uint32_t side = u & 1u;
      uint32_t B[1];
      c[0] = gene_of(srow[ra]);
      B[0] = gene_of(srow[rb]);
      gpus_from_batches<1, kSameTable>(s, lane, c);
      gpus_from_batches<1, kSameTable>(s, lane, B);
      if (kOverGpus) {
        crossover_over_gpus<1, kSameTable>(a, t, s, reinterpret_cast<uint64_t *>(stash), K + (u & ~1u), lane, c, B);
        c[0] = side ? B[0] : c[0];
      } else {
        const bool swap = w < a.T_x;                 // the first child takes the second parent's gene
        c[0] = (swap != (side != 0)) ? B[0] : c[0];
      }
    } else {
      c[0] = gene_of(srow[ra]);
      const uint32_t word = s.info[lane];
      const uint32_t k = ((w & 0xFFFFu) * info_n(word)) >> 16;
      c[0] = w < a.T_mut ? batch_from_draw(k, word) : c[0];
      gpus_from_batches<1, false>(s, lane, c);
    }
  } else {
    const uint32_t p = u - 3 * K;
    r = candidate_draw(a, t, p).r;
    c[0] = gene_of(srow[p]);
    gpus_from_batches<1, false>(s, lane, c);
  }
  repair<1>(c, s, a.G, r, lane, new_first, a.time_rank);
  return score<1>(c, s, a.term_lds, lane);
}

// (Argument block: FusedArgs by value, which starts with its EvolveArgs, see kernel_args.)
static_assert(offsetof(FusedArgs, ev) == 0, "kernel_args() reads the EvolveArgs at the start of the argument block");
// kSampled: the remaining work is drawn anew for every generation (Alg. 1, Eq. 7) and the whole
// pool, survivors included, is scored with the draw.
template <bool kOverGpus, bool kSampled>
__global__ __launch_bounds__(kFusedThreads) void fused_kernel(FusedArgs fa) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const EvolveArgs &a = fa.ev;
  const uint32_t P = a.P, K = a.K, tid = threadIdx.x;
  const Smem s = carve(smem_raw, kLanes, a.term_lds, kFusedWaves, a.stash_stride);
  const Ranks rk = carve_ranks(smem_raw + fa.table_lds, P);
  const int lane0 = tid & (kLanes - 1);
  const uint32_t wave_in_block = __builtin_amdgcn_readfirstlane(tid >> 6);
  // the first work_groups workgroups compute candidates; under probability sampling kDrawGroups more only draw
  const uint32_t n_groups = fa.work_groups;
  const uint32_t wave = blockIdx.x * kFusedWaves + wave_in_block, n_waves = n_groups * kFusedWaves;
  uint8_t *stash = s.stash + static_cast<size_t>(wave_in_block) * a.stash_stride;
  uint32_t *my_draws = rk.draws + wave_in_block * kFusedUnits * 4;
  uint32_t *my_words = rk.words + wave_in_block * kFusedUnits * kLanes;
  uint64_t *my_keys = rk.ukeys + wave_in_block * kFusedUnits;
  auto draw_unit_parents = [&](uint32_t t) {         // for this wave's children and mutants of generation t
    for (uint32_t k = 0, u = wave; k < kFusedUnits && u < 3 * K; ++k, u += n_waves)
      draw_parents(a, t, u, opaque(lane0), my_draws + 4 * k);
  };
  auto draw_unit_words = [&](uint32_t t) {
    for (uint32_t k = 0, u = wave; k < kFusedUnits && u < 3 * K; ++k, u += n_waves)
      draw_words<kOverGpus>(a, t, u, opaque(lane0), my_words + kLanes * k);
  };
  // Probability sampling.  The draw of a generation takes a long chain of fp64 operations (about
  // 5 us), so it is made two generations ahead, by workgroups that do nothing else (sixteen lanes
  // per job slot, four slots per wave), and published like the scores, tagged; every computing
  // workgroup collects the 64 values and rebuilds its LDS copy of the term table from them between
  // two generations.  n: how many draws these launches have made for the context before.
  auto publish_draw = [&](uint32_t t, uint32_t n) {  // called by the kLanes / 4 waves of the drawing workgroups
    uint64_t *xd = fa.xdraw + static_cast<size_t>(n % kDrawBuffers) * kLanes;
    const uint32_t j = 4 * (wave - n_waves) + static_cast<uint32_t>(lane0) / kLanesPerSlot;
    const double Y = draw_remaining(fa.pr, fa.n_slots, a.key0, a.key1, t, j);
    if (lane0 % kLanesPerSlot == 0) shared_store(xd + j, static_cast<uint64_t>(__double_as_longlong(Y)) | draw_tag(n));
  };
  auto build_terms = [&](uint32_t n) -> bool {       // whole workgroup; false when the polls ran out
    const uint64_t *xd = fa.xdraw + static_cast<size_t>(n % kDrawBuffers) * kLanes;
    const bool got = gather(xd, kLanes, fa.spin_limit, [&](uint64_t v) { return (v & kTagBit) == draw_tag(n); },
                            [&](uint32_t j, uint64_t v) { rk.ydraw[j] = __longlong_as_double(static_cast<long long>(v & ~kTagBit)); });
    if (__syncthreads_or(got ? 0 : 1)) return false;
    const uint32_t E = a.term_lds;
    for (uint32_t q = tid; q < E * kLanes; q += kFusedThreads) {
      const uint32_t e = q / kLanes, j = q % kLanes;
      s.terms[(E - 1 - e) * kLanes + j] =
          term_of(rk.model[j], rk.model[kLanes + j], rk.model[2 * kLanes + j], rk.ydraw[j], info_blexp(s.info[j]), e);
    }
    __syncthreads();
    return true;
  };
  if (kSampled && blockIdx.x >= n_groups) {
    // A drawing workgroup: the draws of the first three generations at once, then the draw of
    // generation g + 2 as soon as all scores of generation g - 1 are out.  By then every workgroup
    // has built its term table of generation g - 1, hence has long read the draw of generation
    // g - 2, whose buffer the new one takes (four rotate).
    for (uint32_t g = 0; g < 3 && g < fa.n_generations; ++g) publish_draw(a.t + g + 1, fa.draws_before + g);
    for (uint32_t g = 1; g + 2 < fa.n_generations; ++g) {
      const uint32_t use = fa.generations_before + g - 1;
      const bool seen = gather(fa.xkeys + static_cast<size_t>(use & 1u) * P + K, 3 * K, fa.spin_limit,
                               [&](uint64_t v) { return (v & kTagBit) == use_tag(use); }, [&](uint32_t, uint64_t) {});
      if (__syncthreads_or(seen ? 0 : 1)) {
        if (tid == 0) shared_store(fa.sync + 1, 1u);
        return;
      }
      publish_draw(a.t + g + 3, fa.draws_before + g + 2);
    }
    return;
  }
  draw_unit_parents(a.t + 1);
  draw_unit_words(a.t + 1);
  stage_table<1>(a.tab, a.bk, s, kLanes, a.term_lds, threadIdx.x, blockDim.x);
  // the state the last selection left: the survivors' rows and scores, the bitmap of their rows
  for (uint32_t e = tid; e < K; e += kFusedThreads) {
    const uint32_t row = fa.parent_rows[e];
    rk.srow(0)[e] = static_cast<uint16_t>(row);
    rk.skey(0)[e] = static_cast<uint64_t>(__double_as_longlong(a.fit_row[row]));
  }
  for (uint32_t w = tid; w < (P + K + 31) / 32; w += kFusedThreads) rk.occ[w] = fa.occupied[w];
  if (tid == 0) rk.misc[0] = rk.misc[1] = 0;
  if (kSampled && tid < kLanes) {
    rk.model[tid] = a.tab.abl[tid];
    rk.model[kLanes + tid] = a.tab.cc[tid];
    rk.model[2 * kLanes + tid] = a.tab.d[tid];
  }
  __syncthreads();
  list_free_rows(rk, nullptr, P, true);
  if (kSampled && !build_terms(fa.draws_before)) {
    if (tid == 0) shared_store(fa.sync + 1, 1u);
    return;
  }

  int cur = 0;
  for (uint32_t g = 0; g < fa.n_generations; ++g) {
    const uint32_t t = a.t + g + 1;
    const uint32_t use = fa.generations_before + g;            // how often the children's exchange buffers have been used
    const bool changed = g == 0 && fa.first_changed != 0;
    const bool new_first = changed && a.new_first != 0;
    const bool last = g + 1 == fa.n_generations;
    const bool all_new = changed || kSampled;                   // every candidate of the pool gets a new score
    const uint32_t units = all_new ? 4 * K : 3 * K;
    const uint32_t surv_use = fa.changes_before + (kSampled ? g : 0u);   // ... uses of the survivors' exchange buffers
    uint64_t *xk = fa.xkeys + static_cast<size_t>(use & 1u) * P;
    uint64_t *xs = fa.xsurv + static_cast<size_t>(surv_use & 1u) * K;
    // ---- compose, repair, score and store this wave's candidates (at most kFusedUnits of them)
    for (uint32_t k = 0, u = wave; u < units; ++k, u += n_waves) {
      const int lane = opaque(lane0);
      uint32_t c[1];
      if (kSampled && !changed && u >= 3 * K) {
        // the survivor of rank u - 3K keeps genome and row; only its score changes with the draw
        const uint32_t row = rk.srow(cur)[u - 3 * K];
        c[0] = static_cast<uint32_t>(shared_load(a.genes + static_cast<size_t>(row) * kLanes + lane));
        gpus_from_batches<1, true>(s, lane, c);
        const uint64_t bits = static_cast<uint64_t>(__double_as_longlong(score<1>(c, s, a.term_lds, lane)));
        if (lane == 0) {
          shared_store(reinterpret_cast<uint64_t *>(a.fit_row) + row, bits);
          my_keys[k] = bits;
        }
        continue;
      }
      const double f = changed ? compose_unit<false, kOverGpus>(a, t, s, rk.srow(cur), u, new_first, stash,
                                                                my_draws + 4 * k, my_words + kLanes * k, lane, c)
                               : compose_unit<true, kOverGpus>(a, t, s, rk.srow(cur), u, false, stash,
                                                               my_draws + 4 * k, my_words + kLanes * k, lane, c);
      const uint32_t row = rk.frow[u];
      shared_store(a.genes + static_cast<size_t>(row) * kLanes + lane,
                   static_cast<int32_t>(c[0] << info_blexp(s.info[lane])));
      if (lane == 0) {
        // (the score kept with the row goes to the point of coherence too: a row is written by
        // different workgroups in different generations, and a plain store could linger in one
        // XCD's cache and be written back over a later one)
        const uint64_t bits = static_cast<uint64_t>(__double_as_longlong(f));
        shared_store(reinterpret_cast<uint64_t *>(a.fit_row) + row, bits);
        my_keys[k] = bits;
      }
    }
    // the genomes have arrived before their scores are published
    __builtin_amdgcn_s_waitcnt(0);
    if (lane0 == 0)
      for (uint32_t k = 0, u = wave; u < units; ++k, u += n_waves) {
        if (u < 3 * K) shared_store(xk + K + u, my_keys[k] | use_tag(use));
        else shared_store(xs + (u - 3 * K), my_keys[k] | use_tag(surv_use));
      }
    if (!last) {                                     // while the others' scores are on their way
      draw_unit_parents(t + 1);
      draw_unit_words(t + 1);
    }

    // ---- collect the scores; a child that beats the K-th survivor raises a flag (an equal score
    // loses to the survivor's smaller slot)
    const uint64_t thresh = all_new ? 0ull : rk.skey(cur)[K - 1];
    bool ok = gather2(xk + K, 3 * K, [&](uint64_t v) { return (v & kTagBit) == use_tag(use); },
                      [&](uint32_t i, uint64_t v) {
                        rk.ckey[K + i] = v & ~kTagBit;
                        if ((v & ~kTagBit) < thresh) rk.misc[1] = 1;
                      },
                      xs, all_new ? K : 0u, [&](uint64_t v) { return (v & kTagBit) == use_tag(surv_use); },
                      [&](uint32_t i, uint64_t v) { rk.ckey[i] = v & ~kTagBit; }, fa.spin_limit);
    if (__syncthreads_or(ok ? 0 : 1)) {              // a poll ran out
      if (tid == 0) shared_store(fa.sync + 1, 1u);
      return;
    }

    // every wave of this workgroup is done with the term table of this generation: the next one's
    if (kSampled && !last && !build_terms(fa.draws_before + g + 1)) {
      if (tid == 0) shared_store(fa.sync + 1, 1u);
      return;
    }

    // ---- rank the pool
    bool moved = true;                               // the set of survivors (hence the free rows) changes
    bool by_counting = all_new;                      // rank the whole pool, a share per workgroup
    if (!all_new && rk.misc[1] == 0) {
      // no child beats the K-th survivor: same survivors, same order, same free rows
      if (last && blockIdx.x != 0) return;
      moved = false;
      if (last) for (uint32_t e = tid; e < K; e += kFusedThreads) rk.nsel[e] = static_cast<uint16_t>(e);
    } else if (!all_new) {
      // list the children that beat the K-th survivor
      for (uint32_t base = 0; base < 3 * K; base += kFusedThreads) {   // whole waves go round together
        const uint32_t i = base + tid;
        const uint64_t key = i < 3 * K ? rk.ckey[K + i] : ~0ull;
        const bool beats = key < thresh;
        const uint64_t mask = __ballot(beats);
        uint32_t at = 0;
        if (lane0 == 0 && mask != 0) at = atomicAdd(&rk.misc[0], static_cast<uint32_t>(__popcll(mask)));
        at = __builtin_amdgcn_readfirstlane(at) + static_cast<uint32_t>(__popcll(mask & ((1ull << lane0) - 1ull)));
        if (beats) { rk.mkey[at] = key; rk.mslot[at] = K + i; }
      }
      __syncthreads();
      const uint32_t M = rk.misc[0];
      // in the last generation only the first workgroup needs the ranking (it writes the state the
      // call leaves); the others stay for their share of a ranking by counting, if there is one
      if (last && blockIdx.x != 0 && M <= kMergeMax) return;
      if (M > kMergeMax) {
        by_counting = true;
        for (uint32_t e = tid; e < K; e += kFusedThreads) rk.ckey[e] = rk.skey(cur)[e];
      } else {
        // rank of each such child among them, the comparisons dealt to all threads
        const uint32_t Mp = pow2_at_least(M), parts = kFusedThreads / Mp, per = (M + parts - 1) / parts;
        if (tid < kMergeMax) rk.below[tid] = 0;
        __syncthreads();
        {
          const uint32_t i = tid % Mp, from = (tid / Mp) * per, to = min(from + per, M);
          if (i < M) {
            const uint64_t key = rk.mkey[i];
            const uint32_t slot = rk.mslot[i];
            uint32_t n = 0;
            for (uint32_t j = from; j < to; ++j) n += key_less(rk.mkey[j], rk.mslot[j], key, slot) ? 1u : 0u;
            if (n) atomicAdd(&rk.below[i], n);
          }
        }
        __syncthreads();
        if (tid < M) { rk.okey[rk.below[tid]] = rk.mkey[tid]; rk.oslot[rk.below[tid]] = rk.mslot[tid]; }
        __syncthreads();
        const int nxt = cur ^ 1;
        // child at position b: new rank = b + survivors with a score <= its own
        if (tid < M) {
          const uint64_t key = rk.okey[tid];
          uint32_t lo = 0, hi = K;
          while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (rk.skey(cur)[mid] <= key) lo = mid + 1; else hi = mid;
          }
          const uint32_t rank = tid + lo;
          if (rank < K) {
            rk.skey(nxt)[rank] = key;
            rk.srow(nxt)[rank] = rk.frow[rk.oslot[tid] - K];
            rk.nsel[rank] = static_cast<uint16_t>(rk.oslot[tid]);
          }
        }
        // survivor e: new rank = e + such children with a strictly smaller score
        for (uint32_t e = tid; e < K; e += kFusedThreads) {
          const uint64_t key = rk.skey(cur)[e];
          uint32_t lo = 0, hi = M;
          while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (rk.okey[mid] < key) lo = mid + 1; else hi = mid;
          }
          const uint32_t rank = e + lo;
          if (rank < K) {
            rk.skey(nxt)[rank] = key;
            rk.srow(nxt)[rank] = rk.srow(cur)[e];
            rk.nsel[rank] = static_cast<uint16_t>(e);
          }
        }
      }
      __syncthreads();
      if (tid == 0) rk.misc[0] = rk.misc[1] = 0;     // for the next generation (read again only after further barriers)
    }
    if (by_counting) {
      // ckey holds the whole pool's scores by slot.  This workgroup ranks its share of the slots
      // (rank = candidates below in (score, slot) order), publishes the ranks, collects all.
      const uint32_t lo = static_cast<uint32_t>(static_cast<uint64_t>(P) * blockIdx.x / n_groups);
      const uint32_t hi = static_cast<uint32_t>(static_cast<uint64_t>(P) * (blockIdx.x + 1) / n_groups);
      const uint32_t ns = hi - lo, parts = ns ? kFusedThreads / ns : 0u;   // 0 < parts: ns <= kMergeMax
      if (tid < kMergeMax) rk.below[tid] = 0;
      __syncthreads();
      if (ns != 0 && tid < parts * ns) {
        // thread (i, part): slot lo + i against the candidates part, part + parts, ...; candidate j is
        // below when its score is smaller, or equal with a smaller slot, i.e. smaller than the
        // score + 1 for j < slot (scores are integers below 2^63 here)
        const uint32_t i = tid % ns, part = tid / ns, slot = lo + i;
        const uint64_t key = rk.ckey[slot];
        uint32_t n = 0;
        uint32_t j = part;
        for (; j + 3 * parts < P; j += 4 * parts) {
          const uint64_t k0 = rk.ckey[j], k1 = rk.ckey[j + parts], k2 = rk.ckey[j + 2 * parts], k3 = rk.ckey[j + 3 * parts];
          n += k0 < key + (j < slot ? 1u : 0u) ? 1u : 0u;
          n += k1 < key + (j + parts < slot ? 1u : 0u) ? 1u : 0u;
          n += k2 < key + (j + 2 * parts < slot ? 1u : 0u) ? 1u : 0u;
          n += k3 < key + (j + 3 * parts < slot ? 1u : 0u) ? 1u : 0u;
        }
        for (; j < P; j += parts) n += rk.ckey[j] < key + (j < slot ? 1u : 0u) ? 1u : 0u;
        if (n) atomicAdd(&rk.below[i], n);
      }
      __syncthreads();
      const uint64_t stamp = static_cast<uint64_t>(use + 1u) << 32;     // no generation has number 0
      if (tid < ns) shared_store(fa.xrank + lo + tid, stamp | rk.below[tid]);
      if (last && blockIdx.x != 0) return;
      const int nxt = cur ^ 1;
      ok = gather(fa.xrank, P, fa.spin_limit, [&](uint64_t v) { return (v >> 32) == (stamp >> 32); },
                  [&](uint32_t p, uint64_t v) {
                    const uint32_t rank = static_cast<uint32_t>(v);
                    if (rank < K) {
                      rk.skey(nxt)[rank] = rk.ckey[p];
                      rk.srow(nxt)[rank] = static_cast<uint16_t>(row_of_slot(rk, cur, p, K, changed));
                      rk.nsel[rank] = static_cast<uint16_t>(p);
                    }
                  });
      if (__syncthreads_or(ok ? 0 : 1)) {
        if (tid == 0) shared_store(fa.sync + 1, 1u);
        return;
      }
    }
    const int nxt = moved ? cur ^ 1 : cur;
    if (last) {
      // the state the next call (of either kind) starts from
      for (uint32_t p = tid; p < P; p += kFusedThreads) fa.row_of_cur[p] = row_of_slot(rk, cur, p, K, changed);
      for (uint32_t e = tid; e < K; e += kFusedThreads) {
        fa.parent_rows[e] = rk.srow(nxt)[e];
        fa.row_of_next[e] = rk.srow(nxt)[e];
        fa.sel[e] = rk.nsel[e];
      }
      const uint32_t words = (P + K + 31) / 32;
      __syncthreads();
      for (uint32_t w = tid; w < words; w += kFusedThreads) rk.occ[w] = 0;
      __syncthreads();
      for (uint32_t e = tid; e < K; e += kFusedThreads)
        atomicOr(&rk.occ[rk.srow(nxt)[e] >> 5], 1u << (rk.srow(nxt)[e] & 31u));
      __syncthreads();
      for (uint32_t w = tid; w < words; w += kFusedThreads) fa.occupied[w] = rk.occ[w];
      if (kSampled && tid < kLanes) fa.y_out[tid] = rk.ydraw[tid];   // the remaining work the last generation was scored with
      return;
    }
    if (moved) list_free_rows(rk, rk.srow(nxt), P, false);
    cur = nxt;
  }
}

size_t table_lds_bytes(const EvolveArgs &ev) {
  return (smem_bytes(kLanes, kFusedWaves, ev.term_lds, ev.P + ev.K, ev.stash_stride) + 15) & ~size_t(15);
}

}  // namespace

uint32_t fused_workgroups(uint32_t P, bool sampled) {
  // one wave per candidate a generation computes: the 3K children, and under probability sampling the K survivors too
  const uint32_t units = (sampled ? 4 : 3) * (P / 4);
  return std::max(1u, std::min(sampled ? kFusedMaxSampledWorkgroups : kFusedMaxWorkgroups, (units + kFusedWaves - 1) / kFusedWaves));
}

uint32_t fused_grid_limit(uint32_t P) {
  return std::max(fused_workgroups(P, false), fused_workgroups(P, true) + kDrawGroups);
}

size_t fused_exchange_bytes(uint32_t P) {             // xkeys [2][P], xsurv [2][K], xrank [P], xdraw [4][64]; zeroed once
  return (static_cast<size_t>(2) * P + 2 * (P / 4) + P + kDrawBuffers * kLanes) * 8;
}

hipError_t launch_fused(const FusedArgs &args, hipStream_t stream) {
  FusedArgs fa = args;
  if (fa.ev.Jp != static_cast<uint32_t>(kLanes) || fa.ev.P > kFusedMaxPool || fa.ev.P < 4 || fa.n_generations == 0)
    return hipErrorInvalidValue;
  const uint32_t n_wg = fused_workgroups(fa.ev.P, fa.sampled != 0);
  // every wave keeps its units of a generation in registers, and a workgroup's share of a ranking by counting fits its counters
  if ((fa.ev.P + n_wg * kFusedWaves - 1) / (n_wg * kFusedWaves) > kFusedUnits || (fa.ev.P + n_wg - 1) / n_wg > kMergeMax)
    return hipErrorInvalidValue;
  fa.ev.bk.nb = 0;
  fa.ev.stash_stride = stash_stride(kLanes, fa.ev.per_gpu != 0);
  fa.ev.term_lds = fa.ev.tab.term_E;                  // 64 job columns: the term table always fits
  fa.table_lds = static_cast<uint32_t>(table_lds_bytes(fa.ev));
  const size_t lds = fa.table_lds + ranks_bytes(fa.ev.P);
  if (lds > kLdsBudget) return hipErrorInvalidValue;
  const void *fn = fa.sampled ? (fa.ev.per_gpu ? reinterpret_cast<const void *>(fused_kernel<true, true>)
                                               : reinterpret_cast<const void *>(fused_kernel<false, true>))
                              : (fa.ev.per_gpu ? reinterpret_cast<const void *>(fused_kernel<true, false>)
                                               : reinterpret_cast<const void *>(fused_kernel<false, false>));
  hipError_t rc = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
  if (rc != hipSuccess) return rc;
  fa.work_groups = n_wg;
  const uint32_t grid = n_wg + (fa.sampled ? kDrawGroups : 0u);
  void *params[] = {&fa};
  // For tools that cannot follow a cooperative launch (rocprofv3's kernel trace ends in a fault when
  // the process exits after one): the same kernel as an ordinary launch.  Its waits stay bounded,
  // but nothing then guarantees that all workgroups are resident at once, so this is not for production.
  static const bool plain = getenv("ONES_FUSED_PLAIN_LAUNCH") != nullptr;
  if (plain) return hipLaunchKernel(fn, dim3(grid), dim3(kFusedThreads), params, lds, stream);
  // cooperative: the runtime refuses the launch unless all workgroups can be resident at once
  return hipLaunchCooperativeKernel(fn, dim3(grid), dim3(kFusedThreads), params, static_cast<unsigned int>(lds), stream);
}

}  // namespace ones
