// All generations of one ones_generation call in a single launch (ONES, arXiv 2108.03645,
// Section 3.2.2), for the pools the paper itself schedules with (population = cluster size,
// Section 3.2.2 "Initialization"; 64 GPUs in Section 4.1): at most 64 job slots and
// kFusedMaxPool candidates.
//
// Two launches per generation cost more than the generation itself at this size, so here a
// co-resident grid stays on the chip for the whole call.  Per generation every wave composes,
// repairs and scores its share of the 3K children (4K candidates after a table change) and
// publishes genome and score; then all workgroups meet at a device-wide wait, and each of them
// ranks the pool by itself in its LDS: the survivors' scores, rows and the list of free rows are
// kept there redundantly, so the only data that cross workgroups are the genomes and one score
// per candidate.  While the job table stays the same the K survivors reappear with the scores
// they had, already in order, so the ranking is a merge of the few children that beat the K-th
// survivor into that order; otherwise the pool is sorted.
//
// Data written by one workgroup and read by another inside the launch (genomes, scores, the
// arrival counter) go through relaxed atomic stores and loads at device scope, which the
// hardware performs at the device's point of coherence instead of in the caches of one XCD;
// every wave waits for its stores to be acknowledged before its workgroup arrives, and reads
// others' data only after the wait.  The wait is bounded: a workgroup that gives up sets an
// error word and leaves, and so do all others.
#include "ones_candidate.h"
#include "ones_sort.h"

namespace ones {
namespace {

constexpr int kFusedThreads = kFusedWaves * kLanes;
constexpr uint32_t kFusedMaxWorkgroups = 96;
constexpr uint32_t kMergeMax = 256;          // children beating the K-th survivor that are still ranked by counting

template <typename T>
__device__ __forceinline__ T shared_load(const T *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ void shared_store(T *p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

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
  uint64_t *ckey;      // [pow2(P)] score bits by pool slot; sorted in place when the pool is sorted
  uint32_t *cidx;      // [pow2(P)] payload of that sort: the slot
  uint64_t *mkey;      // [3K] children that beat the K-th survivor, then the same in order
  uint32_t *mslot;     // [3K]
  uint64_t *okey;      // [kMergeMax] ... ordered
  uint32_t *oslot;     // [kMergeMax]
  uint32_t *below;     // [kMergeMax] rank of such a child among them
  uint32_t *occ;       // bitmap over the P + K rows: the survivors' rows
  uint32_t *misc;      // [0] outcome of the wait, [1] number of such children
};

inline size_t ranks_bytes(uint32_t P) {
  const size_t K = P / 4, Ppad = 1u << (32 - __builtin_clz(std::max(P, 2u) - 1));
  return 2 * K * 8 + 2 * K * 2 + K * 2 + P * 2 + Ppad * 8 + Ppad * 4 + 3 * K * 8 + 3 * K * 4 +
         kMergeMax * (8 + 4 + 4) + ((P + K + 31) / 32) * 4 + 16 + 64;
}

__device__ __forceinline__ Ranks carve_ranks(unsigned char *base, uint32_t P) {
  const uint32_t K = P / 4, Ppad = pow2_at_least(P);
  Ranks r;
  r.K = K;
  r.skeys = reinterpret_cast<uint64_t *>(base);
  r.ckey = r.skeys + 2 * K;
  r.mkey = r.ckey + Ppad;
  r.okey = r.mkey + 3 * K;
  r.cidx = reinterpret_cast<uint32_t *>(r.okey + kMergeMax);
  r.mslot = r.cidx + Ppad;
  r.oslot = r.mslot + 3 * K;
  r.below = r.oslot + kMergeMax;
  r.occ = r.below + kMergeMax;
  r.misc = r.occ + (P + K + 31) / 32;
  r.srows = reinterpret_cast<uint16_t *>(r.misc + 4);
  r.nsel = r.srows + 2 * K;
  r.frow = r.nsel + K;
  return r;
}

// The survivors' rows (rows[0..K)) as a bitmap, and from it the free rows in ascending order.
// Whole workgroup; ends with a barrier.
__device__ __forceinline__ void list_free_rows(const Ranks &rk, const uint16_t *rows, uint32_t P, bool from_bitmap) {
  const uint32_t K = P / 4, n_rows = P + K, words = (n_rows + 31) / 32;
  if (!from_bitmap) {
    for (uint32_t w = threadIdx.x; w < words; w += blockDim.x) rk.occ[w] = 0;
    __syncthreads();
    for (uint32_t g = threadIdx.x; g < K; g += blockDim.x) atomicOr(&rk.occ[rows[g] >> 5], 1u << (rows[g] & 31u));
    __syncthreads();
  }
  if (threadIdx.x < kLanes) {
    const uint32_t lane = threadIdx.x;
    uint32_t carry = 0;
    for (uint32_t base = 0; base < words; base += kLanes) {
      const uint32_t w = base + lane;
      uint32_t bits = 0;
      if (w < words) {
        bits = ~rk.occ[w];
        if (w == words - 1 && n_rows % 32 != 0) bits &= (1u << (n_rows % 32)) - 1u;
      }
      const uint32_t n = __popc(bits);
      const uint32_t incl = wave_inclusive_scan(n);
      uint32_t pos = carry + incl - n;
      while (bits) {
        if (pos < P) rk.frow[pos] = static_cast<uint16_t>(w * 32 + (__ffs(static_cast<int>(bits)) - 1));
        bits &= bits - 1;
        ++pos;
      }
      carry += __builtin_amdgcn_readlane(incl, kLanes - 1);
    }
  }
  __syncthreads();
}

// Row of pool slot p in the generation just computed.
__device__ __forceinline__ uint32_t row_of_slot(const Ranks &rk, int cur, uint32_t p, uint32_t K, bool changed) {
  if (p >= K) return rk.frow[p - K];
  return changed ? rk.frow[3 * K + p] : rk.srow(cur)[p];
}

// Ranks the whole pool: ckey[0..P) holds every slot's score bits.  Writes the new survivors
// into the buffers number nxt.  Whole workgroup; ends with a barrier.
__device__ __forceinline__ void rank_by_sorting(const Ranks &rk, int cur, uint32_t P, bool changed) {
  const uint32_t K = P / 4, Ppad = pow2_at_least(P);
  for (uint32_t i = threadIdx.x; i < Ppad; i += blockDim.x) {
    rk.cidx[i] = i < P ? i : 0xFFFFFFFFu;
    if (i >= P) rk.ckey[i] = ~0ull;
  }
  __syncthreads();
  bitonic_sort(rk.ckey, rk.cidx, Ppad);
  const int nxt = cur ^ 1;
  for (uint32_t g = threadIdx.x; g < K; g += blockDim.x) {
    const uint32_t slot = rk.cidx[g];
    rk.skey(nxt)[g] = rk.ckey[g];
    rk.srow(nxt)[g] = static_cast<uint16_t>(row_of_slot(rk, cur, slot, K, changed));
    rk.nsel[g] = static_cast<uint16_t>(slot);
  }
  __syncthreads();
}

// One candidate of generation t: unit u < 2K is a child of pair u / 2, u < 3K a mutant, u >= 3K
// (only after a table change) the survivor of rank u - 3K to refresh.  srow: rows of the
// survivors by rank.  Returns the score; the repaired GPU counts are left in c.
template <bool kSameTable, bool kOverGpus>
__device__ __forceinline__ double compose_unit(const EvolveArgs &a, uint32_t t, const Smem &s, const uint16_t *srow, uint32_t u,
                                               bool new_first, uint8_t *stash, int lane, uint32_t (&c)[1]) {
  const uint32_t K = a.K;
  uint32_t r;
  auto gene_of = [&](uint32_t row) {
    return static_cast<uint32_t>(shared_load(a.genes + static_cast<size_t>(row) * kLanes + lane));
  };
  if (u < 2 * K) {
    const uint32_t p0 = K + (u & ~1u), side = u & 1u;
    const Draw d0 = candidate_draw(a, t, p0);
    r = side ? candidate_draw(a, t, p0 + 1).r : d0.r;
    uint32_t B[1];
    c[0] = gene_of(srow[d0.ra]);
    B[0] = gene_of(srow[d0.rb]);
    gpus_from_batches<1, kSameTable>(s, lane, c);
    gpus_from_batches<1, kSameTable>(s, lane, B);
    if (kOverGpus) {
      crossover_over_gpus<1>(a, t, s, reinterpret_cast<uint64_t *>(stash), p0, lane, c, B);
      c[0] = side ? B[0] : c[0];
    } else {
      uint32_t w[1];
      gene_words<1>(a, t, p0, lane, w);
      const bool swap = w[0] < a.T_x;                      // the first child takes the second parent's gene
      c[0] = (swap != (side != 0)) ? B[0] : c[0];
    }
  } else if (u < 3 * K) {
    const uint32_t p = K + u;
    const Draw d = candidate_draw(a, t, p);
    r = d.r;
    uint32_t w[1];
    gene_words<1>(a, t, p, lane, w);
    c[0] = gene_of(srow[d.ra]);
    const uint32_t word = s.info[lane];
    const uint32_t k = ((w[0] & 0xFFFFu) * info_n(word)) >> 16;
    c[0] = w[0] < a.T_mut ? batch_from_draw(k, word) : c[0];
    gpus_from_batches<1, false>(s, lane, c);
  } else {
    const uint32_t p = u - 3 * K;
    r = candidate_draw(a, t, p).r;
    c[0] = gene_of(srow[p]);
    gpus_from_batches<1, false>(s, lane, c);
  }
  repair<1>(c, s, a.G, r, lane, new_first, a.time_rank);
  return score<1>(c, s, a.term_lds, lane);
}

template <bool kOverGpus>
__global__ __launch_bounds__(kFusedThreads) void fused_kernel(FusedArgs fa) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const uint32_t P = fa.ev.P, K = fa.ev.K, tid = threadIdx.x;
  const Smem s = carve(smem_raw, kLanes, fa.ev.term_lds, kFusedWaves, fa.ev.stash_stride);
  const Ranks rk = carve_ranks(smem_raw + fa.table_lds, P);
  stage_table<1>(fa.ev.tab, fa.ev.bk, s, kLanes, fa.ev.term_lds);
  // the state the last selection left: the survivors' rows and scores, the bitmap of their rows
  for (uint32_t e = tid; e < K; e += kFusedThreads) {
    const uint32_t row = fa.parent_rows[e];
    rk.srow(0)[e] = static_cast<uint16_t>(row);
    rk.skey(0)[e] = static_cast<uint64_t>(__double_as_longlong(fa.ev.fit_row[row]));
  }
  for (uint32_t w = tid; w < (P + K + 31) / 32; w += kFusedThreads) rk.occ[w] = fa.occupied[w];
  __syncthreads();
  list_free_rows(rk, nullptr, P, true);

  const int lane0 = tid & (kLanes - 1);
  const uint32_t wave_in_block = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t wave = blockIdx.x * kFusedWaves + wave_in_block, n_waves = gridDim.x * kFusedWaves;
  uint8_t *stash = s.stash + static_cast<size_t>(wave_in_block) * fa.ev.stash_stride;
  int cur = 0;
  for (uint32_t g = 0; g < fa.n_generations; ++g) {
    const EvolveArgs &a = fa.ev;
    const uint32_t t = fa.ev.t + g + 1;
    const bool changed = g == 0 && fa.first_changed != 0;
    const bool new_first = changed && fa.ev.new_first != 0;
    const bool last = g + 1 == fa.n_generations;
    const uint32_t units = changed ? 4 * K : 3 * K;
    uint64_t *xk = fa.xkeys + static_cast<size_t>(g & 1u) * P;
    for (uint32_t u = wave; u < units; u += n_waves) {
      const int lane = opaque(lane0);
      uint32_t c[1];
      const double f = changed ? compose_unit<false, kOverGpus>(a, t, s, rk.srow(cur), u, new_first, stash, lane, c)
                               : compose_unit<true, kOverGpus>(a, t, s, rk.srow(cur), u, false, stash, lane, c);
      const uint32_t row = rk.frow[u], slot = u < 3 * K ? K + u : u - 3 * K;
      shared_store(a.genes + static_cast<size_t>(row) * kLanes + lane, static_cast<int32_t>(c[0] << info_blexp(s.info[lane])));
      if (lane == 0) {
        // (also the score kept with the row goes to the point of coherence: a row is written by
        // different workgroups in different generations, and a plain store could linger in one
        // XCD's cache and be written back over a later one)
        const uint64_t bits = static_cast<uint64_t>(__double_as_longlong(f));
        shared_store(reinterpret_cast<uint64_t *>(a.fit_row) + row, bits);
        shared_store(xk + slot, bits);
      }
    }
    // every store of this wave has been acknowledged before its workgroup arrives
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (tid == 0) __hip_atomic_fetch_add(fa.sync, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (last && blockIdx.x != 0) return;             // only the first workgroup writes the final state
    if (tid == 0) {
      const uint32_t target = fa.arrivals_before + gridDim.x * (g + 1);
      uint32_t ok = 0;
      for (uint32_t spins = 0; spins < fa.spin_limit; ++spins) {
        if (static_cast<int32_t>(shared_load(fa.sync) - target) >= 0) { ok = 1; break; }
        __builtin_amdgcn_s_sleep(1);
      }
      if (!ok) shared_store(fa.sync + 1, 1u);
      rk.misc[0] = ok;
      rk.misc[1] = 0;
    }
    __syncthreads();
    if (rk.misc[0] == 0) return;                     // the wait gave up: the error word is set

    // ---- rank the pool
    bool moved = true;                               // the set of survivors (hence the free rows) changed
    if (changed) {
      for (uint32_t i = tid; i < P; i += kFusedThreads) rk.ckey[i] = shared_load(xk + i);
      rank_by_sorting(rk, cur, P, true);
    } else {
      // children that beat the K-th survivor (an equal score loses to the survivor's smaller slot)
      const uint64_t thresh = rk.skey(cur)[K - 1];
      for (uint32_t base = 0; base < 3 * K; base += kFusedThreads) {   // whole waves go round together
        const uint32_t i = base + tid;
        const uint64_t key = i < 3 * K ? shared_load(xk + K + i) : ~0ull;
        if (i < 3 * K) rk.ckey[K + i] = key;
        const bool beats = key < thresh;
        const uint64_t mask = __ballot(beats);
        uint32_t at = 0;
        if (lane0 == 0 && mask != 0) at = atomicAdd(&rk.misc[1], static_cast<uint32_t>(__popcll(mask)));
        at = __builtin_amdgcn_readfirstlane(at) + static_cast<uint32_t>(__popcll(mask & ((1ull << lane0) - 1ull)));
        if (beats) { rk.mkey[at] = key; rk.mslot[at] = K + i; }
      }
      __syncthreads();
      const uint32_t M = rk.misc[1];
      if (M == 0) {
        moved = false;                               // same survivors, same order, same free rows
        if (last) for (uint32_t e = tid; e < K; e += kFusedThreads) rk.nsel[e] = static_cast<uint16_t>(e);
      } else if (M > kMergeMax) {
        for (uint32_t e = tid; e < K; e += kFusedThreads) rk.ckey[e] = rk.skey(cur)[e];
        rank_by_sorting(rk, cur, P, false);
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
        __syncthreads();
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

uint32_t fused_workgroups(uint32_t P) {
  const uint32_t units = 3 * (P / 4);                 // one wave per child of an ordinary generation
  return std::max(1u, std::min(kFusedMaxWorkgroups, (units + kFusedWaves - 1) / kFusedWaves));
}

hipError_t launch_fused(const FusedArgs &args, hipStream_t stream) {
  FusedArgs fa = args;
  if (fa.ev.Jp != static_cast<uint32_t>(kLanes) || fa.ev.P > kFusedMaxPool || fa.ev.P < 4 || fa.n_generations == 0)
    return hipErrorInvalidValue;
  fa.ev.bk.nb = 0;
  fa.ev.stash_stride = stash_stride(kLanes, fa.ev.per_gpu != 0);
  fa.ev.term_lds = fa.ev.tab.term_E;                  // 64 job columns: the term table always fits
  fa.table_lds = static_cast<uint32_t>(table_lds_bytes(fa.ev));
  const size_t lds = fa.table_lds + ranks_bytes(fa.ev.P);
  if (lds > kLdsBudget) return hipErrorInvalidValue;
  const void *fn = fa.ev.per_gpu ? reinterpret_cast<const void *>(fused_kernel<true>)
                                 : reinterpret_cast<const void *>(fused_kernel<false>);
  hipError_t rc = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
  if (rc != hipSuccess) return rc;
  void *params[] = {&fa};
  // cooperative: the runtime refuses the launch unless all workgroups can be resident at once
  return hipLaunchCooperativeKernel(fn, dim3(fused_workgroups(fa.ev.P)), dim3(kFusedThreads), params,
                                    static_cast<unsigned int>(lds), stream);
}

}  // namespace ones
