// Evolve kernel of the ONES search (arXiv 2108.03645, Section 3.2.2) for gfx950.
//
// One wave64 owns one pool slot (a crossover wave owns the two children of a pair): the
// job columns lie across the 64 lanes, the rows of a column in a lane's registers.  The
// wave composes the candidate from the survivors of the previous generation (refresh copy,
// uniform crossover, uniform mutation), repairs it to the cluster capacity (refresh + fill
// under Eq. 4), scores it (Eq. 3 with T = Y/X, Eq. 5) and writes genome and score.
//
// Workgroups are persistent: each owns a contiguous share of the work; two or three of its waves
// list the free genome rows the share will fill while the others stage the job table in LDS;
// then all waves take the share's items one by one from an LDS counter and never wait for each other.
#include "ones_candidate.h"

#include <utility>

#ifndef ONES_ROW_GROUP
#error "compile with -DONES_ROW_GROUP=0..3"
#endif

namespace ones {
namespace {

constexpr int kGroupFirst = 8 * ONES_ROW_GROUP + 1;   // row counts kGroupFirst .. kGroupFirst + 7

// ----------------------------------------------------------------- kernels ---------
#ifndef ONES_WAVES_BIG
#define ONES_WAVES_BIG 16
#endif
template <int R> struct Shape { static constexpr int kWaves = R > 16 ? ONES_WAVES_BIG : (R > 4 ? 8 : 4); };

// Initial population G_0: every gene uniform over {waiting, bmin..bmax}.
// (Argument block: one EvolveArgs by value, see kernel_args.)
template <int R>
__global__ __launch_bounds__(Shape<R>::kWaves *kLanes) void init_kernel(EvolveArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const Smem s = carve(smem_raw, a.Jp, a.term_lds, Shape<R>::kWaves, a.stash_stride);
  stage_table<R>(a.tab, a.bk, s, a.Jp, a.term_lds, threadIdx.x, blockDim.x);
  if (threadIdx.x == 0) *s.next_item = 0;
  __syncthreads();
  const int lane0 = threadIdx.x & (kLanes - 1);
  // The workgroup owns a contiguous share of the slots; its waves take them one by one from an
  // LDS counter (random genomes differ widely in the fill rounds their repair needs).
  const uint32_t first = static_cast<uint32_t>(static_cast<uint64_t>(a.P) * blockIdx.x / gridDim.x);
  const uint32_t last = static_cast<uint32_t>(static_cast<uint64_t>(a.P) * (blockIdx.x + 1) / gridDim.x);
  for (;;) {
    const int lane = opaque(lane0);
    uint32_t taken = 0;
    if (lane == 0) taken = atomicAdd(s.next_item, 1u);
    const uint32_t p = first + static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(taken));
    if (p >= last) break;
    const Draw dr = candidate_draw(a, a.t, p);
    uint32_t c[R];
    gene_words<R>(a, a.t, p, lane, c);
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const uint32_t w = s.info[lane + kLanes * i];
      c[i] = batch_from_draw(bounded(c[i], info_n(w)), w);
    }
    gpus_from_batches<R, false>(s, lane, c);
    const double f = finish<R>(a, s, p, dr.r, c, lane);   // slot p starts in row p
    note_slot_score(p, f, lane);
    if (lane == 0) a.row_of[p] = p;
  }
}

// One generation.  Work items: K crossover pairs, K mutants and, after a table change, the K
// survivors to refresh (or, when only the remaining work changed, to score again).  kSameTable: the job table has not changed since the previous
// generation was repaired and scored, so a survivor is a fixed point of the repair with the
// same score: it stays in its row untouched, and stored genes need no clamp.
// kOverGpus: the uniform crossover scans the GPUs instead of the jobs.
// (Argument block: one EvolveArgs by value, see kernel_args.)
template <int R, bool kSameTable, bool kOverGpus>
__global__ __launch_bounds__(Shape<R>::kWaves *kLanes) void evolve_kernel(EvolveArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const Smem s = carve(smem_raw, a.Jp, a.term_lds, Shape<R>::kWaves, a.stash_stride);
  const int lane0 = threadIdx.x & (kLanes - 1);
  const IndexLoads index_loads = index_free_rows_begin(a, lane0);
  if (threadIdx.x == 0) s.next_item[1] = 0;          // no row index has been out of range (checked_row)
  index_free_rows_end(a, s, index_loads, lane0);
  const uint32_t wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t K = a.K;
  uint8_t *stash = s.stash + static_cast<size_t>(wave_in_block) * a.stash_stride;
  // This workgroup's share of the ranks 0..K-1: for each rank a pair, a mutant and, after a
  // table change, a survivor.  Slot K + q of the new pool takes the q-th free row and the
  // refreshed survivor of rank e the (3K + e)-th, so every share needs three runs of
  // consecutive free rows, which one wave each lists into LDS, a round of kRound ranks at a time.
  const uint32_t first = static_cast<uint32_t>(static_cast<uint64_t>(K) * blockIdx.x / gridDim.x);
  const uint32_t last = static_cast<uint32_t>(static_cast<uint64_t>(K) * (blockIdx.x + 1) / gridDim.x);
  // The first round's rows are listed while the other waves stage the job table.
  constexpr uint32_t kListing = (kSameTable ? 2 : 3) * kLanes;
  auto list_round = [&](uint32_t ra, uint32_t n) {
    if (wave_in_block == 0) list_free_rows(a, s, 2 * ra, 2 * n, s.rows, lane0);
    if (wave_in_block == 1) list_free_rows(a, s, 2 * K + ra, n, s.rows + 2 * n, lane0);
    if (!kSameTable && wave_in_block == 2) list_free_rows(a, s, 3 * K + ra, n, s.rows + 3 * n, lane0);
  };
  if (first < last) list_round(first, min(kRound, last - first));
  if (threadIdx.x >= kListing)
    stage_table<R>(a.tab, a.bk, s, a.Jp, a.term_lds, threadIdx.x - kListing, blockDim.x - kListing);
  for (uint32_t ra = first; ra < last; ra += kRound) {
  const uint32_t n = min(kRound, last - ra);
  if (ra != first) {
    __syncthreads();                                 // the previous round's rows have been used
    list_round(ra, n);
  }
  if (threadIdx.x == blockDim.x - 1) *s.next_item = 0;
  __syncthreads();
  for (uint32_t i = threadIdx.x; i < (kSameTable ? 3 : 4) * n; i += blockDim.x) {
    const uint32_t p = i < 2 * n ? K + 2 * ra + i : i < 3 * n ? 3 * K + ra + (i - 2 * n) : ra + (i - 3 * n);
    a.row_of[p] = checked_row(s, s.rows[i], a.P + a.K);
  }
  const uint32_t kinds = (!kSameTable || a.rescore) ? 3u : 2u;
  const bool new_first = !kSameTable && a.new_first != 0;       // never under an unchanged table
  // The waves take the items one by one (the pairs first: they take twice as long), so that a
  // wave whose items needed many fill rounds does not hold the others up at the end.
  for (;;) {
    const int lane = opaque(lane0);
    uint32_t taken = 0;
    if (lane == 0) taken = atomicAdd(s.next_item, 1u);
    const uint32_t idx = __builtin_amdgcn_readfirstlane(taken);
    if (idx >= kinds * n) break;
    // pairs first, then mutants, then survivors; item as numbered over the whole pool
    const uint32_t item = idx < n ? ra + idx : idx < 2 * n ? K + ra + (idx - n) : 2 * K + ra + (idx - 2 * n);
    uint32_t c[R];
    if (item < K) {
      // uniform crossover: per gene the children swap their parents' genes with rate chi
      const uint32_t p0 = K + 2 * item;
      const Draw d0 = candidate_draw(a, a.t, p0);
      const Draw d1 = candidate_draw(a, a.t, p0 + 1);
      if (kOverGpus) {
        uint32_t B[R];
        load_genes<R>(a.genes + static_cast<size_t>(a.parent_row[d0.ra]) * a.Jp, lane, c);
        load_genes<R>(a.genes + static_cast<size_t>(a.parent_row[d0.rb]) * a.Jp, lane, B);
        gpus_from_batches<R, kSameTable>(s, lane, c);
        gpus_from_batches<R, kSameTable>(s, lane, B);
        phase_fence();
        crossover_over_gpus<R, kSameTable>(a, a.t, s, reinterpret_cast<uint64_t *>(stash), p0, lane, c, B);
        phase_fence();                                   // the coins are no longer needed: their place holds the second child
#pragma unroll
        for (int i = 0; i < R; ++i) stash[lane + kLanes * i] = static_cast<uint8_t>(32 - __clz(static_cast<int>(B[i])));
      } else {
      uint32_t swap = 0;
      {
        uint32_t w[R];
        gene_words<R>(a, a.t, p0, lane, w);
#pragma unroll
        for (int i = 0; i < R; ++i) swap |= (w[i] < a.T_x ? 1u : 0u) << i;
      }
      phase_fence();
      {
        uint32_t B[R];
        load_genes<R>(a.genes + static_cast<size_t>(a.parent_row[d0.ra]) * a.Jp, lane, c);
        load_genes<R>(a.genes + static_cast<size_t>(a.parent_row[d0.rb]) * a.Jp, lane, B);
        gpus_from_batches<R, kSameTable>(s, lane, c);
        gpus_from_batches<R, kSameTable>(s, lane, B);
        // second child goes to LDS as a 5-bit code (0 = waiting, k = 2^(k-1) GPUs)
#pragma unroll
        for (int i = 0; i < R; ++i) {
          const bool sw = (swap >> i) & 1u;
          const uint32_t second = sw ? c[i] : B[i];
          c[i] = sw ? B[i] : c[i];
          stash[lane + kLanes * i] = static_cast<uint8_t>(32 - __clz(static_cast<int>(second)));
        }
      }
      }
      phase_fence();
      const double f0 = finish<R>(a, s, row_at(s, 2 * idx, a), d0.r, c, lane, new_first);
      if (kSameTable && a.bk.nb != 0) drop_in_bucket(a, s, p0, f0, lane); else note_slot_score(p0, f0, lane);
      phase_fence();
#pragma unroll
      for (int i = 0; i < R; ++i) c[i] = (1u << stash[lane + kLanes * i]) >> 1;
      const double f1 = finish<R>(a, s, row_at(s, 2 * idx + 1, a), d1.r, c, lane, new_first);
      if (kSameTable && a.bk.nb != 0) drop_in_bucket(a, s, p0 + 1, f1, lane); else note_slot_score(p0 + 1, f1, lane);
    } else if (item < 2 * K) {
      // uniform mutation: each job redrawn with rate theta (k = 0 pre-empts it)
      const uint32_t p = 3 * K + (item - K);
      const Draw d = candidate_draw(a, a.t, p);
      {
        uint32_t w[R];
        gene_words<R>(a, a.t, p, lane, w);
        phase_fence();
        load_genes<R>(a.genes + static_cast<size_t>(a.parent_row[d.ra]) * a.Jp, lane, c);
#pragma unroll
        for (int i = 0; i < R; ++i) {
          const uint32_t word = s.info[lane + kLanes * i];
          const uint32_t k = ((w[i] & 0xFFFFu) * info_n(word)) >> 16;
          const uint32_t redrawn = batch_from_draw(k, word);
          const uint32_t pick = w[i] < a.T_mut ? 0xFFFFFFFFu : 0u;     // branch-free select
          c[i] = (redrawn & pick) | (c[i] & ~pick);
          fence_every(i, 8);
        }
      }
      phase_fence();
      gpus_from_batches<R, false>(s, lane, c);
      const double f = finish<R>(a, s, row_at(s, idx + n, a), d.r, c, lane, new_first);
      if (kSameTable && a.bk.nb != 0) drop_in_bucket(a, s, p, f, lane); else note_slot_score(p, f, lane);
    } else if (kSameTable) {
      // the remaining work was drawn anew: the survivor of this rank keeps its genome and row
      // and only gets its score under the new draw
      const uint32_t row = a.parent_row[item - 2 * K];
      load_genes<R>(a.genes + static_cast<size_t>(row) * a.Jp, lane, c);
      gpus_from_batches<R, true>(s, lane, c);
      const double f = score<R>(c, s, a.term_lds, lane);
      if (lane == 0) a.fit_row[row] = f;
      note_slot_score(item - 2 * K, f, lane);
    } else {
      // refresh: the survivor of rank p, projected onto the new job table, goes to one of the
      // last K free rows (its old row is still being read as a parent by other waves)
      const uint32_t p = item - 2 * K;
      const Draw d = candidate_draw(a, a.t, p);
      load_genes<R>(a.genes + static_cast<size_t>(a.parent_row[p]) * a.Jp, lane, c);
      gpus_from_batches<R, false>(s, lane, c);
      const double f = finish<R>(a, s, row_at(s, idx + n, a), d.r, c, lane, new_first);
      note_slot_score(p, f, lane);
    }
  }
  }
  __syncthreads();
  if (threadIdx.x == 0 && s.next_item[1] != 0) atomicOr(kernel_args()->fault, 1u);
}

template <typename Kernel>
hipError_t launch_persistent(Kernel k, EvolveArgs a, int waves, uint32_t items, uint32_t max_blocks, int n_cus,
                             hipStream_t s) {
  // the term table goes to LDS when it fits beside the rest
  const uint32_t rows = a.P + a.K;
  a.stash_stride = stash_stride(a.Jp, a.per_gpu != 0);
  a.term_lds = (a.tab.term_E != 0 && smem_bytes(a.Jp, waves, a.tab.term_E, rows, a.stash_stride) <= kLdsBudget)
                   ? a.tab.term_E : 0u;
  const size_t lds = smem_bytes(a.Jp, waves, a.term_lds, rows, a.stash_stride);
  // as many workgroups as can be resident (LDS- and wave-limited), at most one wave per item
  const size_t per_cu = std::max<size_t>(1, std::min<size_t>(kLdsBudget / lds, 32 / waves));
  const uint32_t blocks = std::max<uint32_t>(
      1u, std::min<uint32_t>({(items + waves - 1) / waves, static_cast<uint32_t>(n_cus * per_cu), max_blocks}));
  hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                      static_cast<int>(lds));
  if (rc != hipSuccess) return rc;
  hipLaunchKernelGGL(k, dim3(blocks), dim3(waves * kLanes), lds, s, a);
  return hipGetLastError();
}

template <int R>
hipError_t launch_rows(const EvolveArgs &a, bool same_table, int n_cus, hipStream_t s) {
  constexpr int kWaves = Shape<R>::kWaves;
  if (a.t == 0) return launch_persistent(init_kernel<R>, a, kWaves, a.P, a.P, n_cus, s);
  const uint32_t items = (!same_table || a.rescore ? 3 : 2) * a.K;       // a share of the ranks each
  if (a.per_gpu)
    return same_table ? launch_persistent(evolve_kernel<R, true, true>, a, kWaves, items, a.K, n_cus, s)
                      : launch_persistent(evolve_kernel<R, false, true>, a, kWaves, items, a.K, n_cus, s);
  return same_table ? launch_persistent(evolve_kernel<R, true, false>, a, kWaves, items, a.K, n_cus, s)
                    : launch_persistent(evolve_kernel<R, false, false>, a, kWaves, items, a.K, n_cus, s);
}

template <int... Rs>
hipError_t dispatch_rows(const EvolveArgs &a, int rows, bool same_table, int n_cus, hipStream_t s,
                         std::integer_sequence<int, Rs...>) {
  hipError_t rc = hipErrorInvalidValue;
  (void)((rows == kGroupFirst + Rs ? (rc = launch_rows<kGroupFirst + Rs>(a, same_table, n_cus, s), true) : false) || ...);
  return rc;
}

}  // namespace

// This file is compiled once per group of eight row counts (-DONES_ROW_GROUP=0..3) so that
// the 32 instantiations build in parallel.
#define ONES_CONCAT2(x, y) x##y
#define ONES_CONCAT(x, y) ONES_CONCAT2(x, y)
hipError_t ONES_CONCAT(launch_evolve_group, ONES_ROW_GROUP)(const EvolveArgs &a, int rows, bool same_table,
                                                            int n_cus, hipStream_t s) {
  return dispatch_rows(a, rows, same_table, n_cus, s, std::make_integer_sequence<int, 8>{});
}

}  // namespace ones
