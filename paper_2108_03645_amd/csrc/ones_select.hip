// Selection of the best K candidates (arXiv 2108.03645, Section 3.2.2 "Selection"; Alg. 1:
// the smallest score wins), plus the small table / readout kernels of libones.
//
// Order: ascending (score, pool slot).  A score is a non-negative fp64, so its bit pattern
// read as an unsigned 64-bit integer orders the same way; ties fall to the smaller slot.
#include "ones_device.h"
#include "ones_sort.h"

#pragma clang fp contract(off)

namespace ones {
namespace {

constexpr int kSortThreads = kSortChunk / 2 > 1024 ? 1024 : kSortChunk / 2;

// Value of lane + n within the lane's row of 16 (DPP row_shl:n), or fallback where that row ends.
template <int N>
__device__ __forceinline__ uint32_t from_lane_above(uint32_t fallback, uint32_t v) {
  return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(static_cast<int>(fallback), static_cast<int>(v), 0x100 + N,
                                                           0xF, 0xF, false));
}

// The candidate in genome row `row` takes rank g < K (lanes with valid set): it survives in its row.  Called by whole
// waves.  Neighbouring lanes whose rows share a word of the bitmap hand their bits to the first
// lane of their run (within a row of 16 lanes), which issues one atomic for all of them: the
// rows of a pool that has stopped changing are neighbours, and one atomic per row would queue
// up on the same few words.  Lanes that share a word without being neighbours simply issue
// their own atomics.
__device__ __forceinline__ void keep_rows_at(const RowPlan &rp, bool valid, uint32_t g, uint32_t row) {
  if (valid) {
    rp.parent_next[g] = row;
    rp.row_of_next[g] = row;
  }
  const uint32_t word = valid ? row / 32 : 0xFFFFFFFFu;        // no bitmap has that many words
  uint32_t bits = valid ? 1u << (row % 32) : 0u;
  // after the steps 1, 2, 4, 8 a lane holds the bits of the lanes above it up to the end of its run
  { const uint32_t w = from_lane_above<1>(~word, word), b = from_lane_above<1>(0u, bits); bits |= w == word ? b : 0u; }
  { const uint32_t w = from_lane_above<2>(~word, word), b = from_lane_above<2>(0u, bits); bits |= w == word ? b : 0u; }
  { const uint32_t w = from_lane_above<4>(~word, word), b = from_lane_above<4>(0u, bits); bits |= w == word ? b : 0u; }
  { const uint32_t w = from_lane_above<8>(~word, word), b = from_lane_above<8>(0u, bits); bits |= w == word ? b : 0u; }
  // the lane below (DPP row_shr:1) has another word, or there is none: this lane starts a run
  const uint32_t below = static_cast<uint32_t>(
      __builtin_amdgcn_update_dpp(static_cast<int>(~word), static_cast<int>(word), 0x111, 0xF, 0xF, false));
  if (valid && below != word) atomicOr(&rp.occupied[word], bits);
}

// The same, the row looked up from the slot.
__device__ __forceinline__ void keep_rows(const RowPlan &rp, bool valid, uint32_t g, uint32_t id) {
  uint32_t row = 0;
  if (valid) row = rp.row_of_cur[id];
  keep_rows_at(rp, valid, g, row);
}

// ---------------------------------------------------------------- general path -----
// Pools of at most kRankPoolMax slots: the rank of a candidate is the number of candidates below
// it in (score, slot) order.  Every workgroup loads all scores into LDS and ranks 64 of them:
// lane l of every wave works on element l, each wave over its own sixteenth of the pool (so a
// wave reads one LDS address at a time, a broadcast); ranks below K are survivors.  One launch,
// where the sample sort below takes three; but the comparisons per thread grow with the pool
// (P / 16), and at P = 16384 this takes 75 us where the three launches take 21.
#ifndef ONES_RANK_POOL_MAX
#define ONES_RANK_POOL_MAX 4096
#endif
constexpr uint32_t kRankPoolMax = ONES_RANK_POOL_MAX;
constexpr int kRankPoolPer = 64;
__global__ __launch_bounds__(kSortThreads) void rank_pool_kernel(const double *fit_row, const double *slot_score,
                                                                RowPlan rp, uint32_t P, uint32_t K, int32_t *sel) {
  const uint32_t *row_of = rp.row_of_cur;
  extern __shared__ __align__(16) uint64_t sk[];       // [padded] scores, then [kRankPoolPer] counters
  constexpr uint32_t kTeam = kSortThreads / kRankPoolPer;
  const uint32_t t = threadIdx.x;
  const uint32_t padded = (P + 8 * kTeam - 1) / (8 * kTeam) * (8 * kTeam);     // eight comparisons per step
  uint32_t *below = reinterpret_cast<uint32_t *>(sk + padded);
  constexpr int kAhead = 4;                            // loads in flight per thread
  for (uint32_t base = 0; base < padded; base += kAhead * kSortThreads) {
    uint64_t loaded[kAhead];
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {                 // all loads first
      const uint32_t e = base + t + u * kSortThreads;
      loaded[u] = e < P ? static_cast<uint64_t>(__double_as_longlong(slot_score ? slot_score[e] : fit_row[row_of[e]])) : ~0ull;
    }
#pragma unroll
    for (int u = 0; u < kAhead; ++u)
      if (base + t + u * kSortThreads < padded) sk[base + t + u * kSortThreads] = loaded[u];
  }
  if (t < kRankPoolPer) below[t] = 0;
  __syncthreads();
  const uint32_t mine = blockIdx.x * kRankPoolPer + t % kRankPoolPer;
  const uint32_t part = padded / kTeam, from = (t / kRankPoolPer) * part;
  if (mine < P) {
    const uint64_t key = sk[mine];
    uint32_t n = 0;
    for (uint32_t q = from; q < from + part; q += 8) {
#pragma unroll
      for (int u = 0; u < 8; ++u) n += key_less(sk[q + u], q + u, key, mine) ? 1u : 0u;   // padding is never below
    }
    if (n != 0) atomicAdd(&below[t % kRankPoolPer], n);
  }
  __syncthreads();
  if (t < kRankPoolPer) {                              // one whole wave
    const bool in = mine < P && below[t] < K;
    if (in) sel[below[t]] = static_cast<int32_t>(mine);
    keep_rows(rp, in, below[t], mine);
  }
}

// ----------------------------------------------------------- quantile buckets ------
// While the job table stays the same, the K survivors reappear in the next pool with the same
// scores, already in rank order (slots 0..K-1).  Their scores at ranks r_c = c*K/nb therefore
// split the next pool into nb buckets that each hold K/nb survivors; the evolve kernel drops
// every child or mutant that beats the K-th survivor into its bucket, and one workgroup per
// bucket sorts those few and merges them with its survivors.  Buckets concatenate to the
// global order.

// Boundary rank of bucket c (c = 0..nb); bucket b owns survivor ranks [bound(b), bound(b+1)).
__device__ __forceinline__ uint32_t bucket_bound(uint32_t c, uint32_t K, uint32_t nb) {
  return (c * K) / nb;          // c <= 1024, K <= 2^18: the product fits 32 bits
}

// Records the next generation's splitters when an element lands on a boundary rank.
__device__ __forceinline__ void note_rank(uint32_t g, uint64_t bits, uint32_t K, uint32_t nb, uint64_t *split,
                                          uint64_t *thresh) {
  if (g == K - 1) *thresh = bits;
  const uint32_t c = (g * nb) / K;                   // g < 2^20, nb <= 1024
  if (c >= 1 && bucket_bound(c, K, nb) == g) split[c - 1] = bits;
  if (c + 1 < nb && bucket_bound(c + 1, K, nb) == g) split[c] = bits;
}

constexpr int kBucketThreads = 256;
constexpr int kBucketLds = 2048;      // offspring of one bucket that are sorted in LDS
constexpr int kBucketCount = 512;     // up to here offspring are ranked by counting, not sorted
constexpr int kBucketElites = 1025;   // survivors of one bucket: at most ceil(2^18 / 256) + 1

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, kLanes);
  return v;
}

// Ranks one bucket: offspring in (sk, si)[0..n) (padded with never-smaller keys up to npad, a
// multiple of 8), survivors' score bits in ek[0..ne).  Writes the survivor list entries that
// fall below K and notes the next generation's splitters.
template <bool kElites, int kThreads, typename K64, typename I32>
__device__ __forceinline__ void rank_bucket(K64 *sk, I32 *si, const uint64_t *ek, uint32_t n, uint32_t npad,
                                            uint32_t ne, uint32_t e0, uint32_t off, bool sorted, uint32_t K,
                                            const BucketArgs &bk, const RowPlan &rp, int32_t *sel) {
  const uint32_t tid = threadIdx.x, nb = bk.nb;
  // offspring i: rank = offspring before it + survivors with score <= its score (a survivor
  // wins a tie: smaller slot)
  for (uint32_t base = 0; base < n; base += kThreads) {   // whole waves go round together
    const uint32_t i = base + tid;
    uint32_t g = K, id = 0;
    if (i < n) {
      const uint64_t key = sk[i];
      id = si[i];
      uint32_t below = i;
      if (!sorted) {
        // scores alone decide nearly every comparison: count the smaller and the equal ones, and
        // only an element that shares its score looks at the slots
        uint32_t equal = 0;
        below = 0;                                   // padding keys are never below a real one
        for (uint32_t q = 0; q < npad; q += 8) {
#pragma unroll
          for (int u = 0; u < 8; ++u) {
            const uint64_t other = sk[q + u];
            below += other < key ? 1u : 0u;
            equal += other == key ? 1u : 0u;
          }
        }
        if (equal > 1)
          for (uint32_t q = 0; q < n; ++q) below += (sk[q] == key && si[q] < id) ? 1u : 0u;
      }
      uint32_t lo = 0, hi = ne;
      while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (ek[mid] <= key) lo = mid + 1; else hi = mid;
      }
      g = off + below + lo;
      if (g < K) {
        sel[g] = static_cast<int32_t>(id);
        if (kElites) note_rank(g, key, K, nb, bk.split_next, bk.thresh_next);
      }
    }
    keep_rows(rp, g < K, g, id);
  }
  if (!kElites) return;
  // survivor e: rank = e + offspring with a strictly smaller score.  The threads are taken from
  // the top, so that in a small bucket the survivors' waves are not the offspring's.
  for (uint32_t base = 0; base < ne; base += kThreads) {
    const uint32_t e = base + (kThreads - 1 - tid);
    uint32_t g = K;
    if (e < ne) {
      const uint64_t key = ek[e];
      uint32_t lo = 0;
      if (!sorted) {
        for (uint32_t q = 0; q < npad; q += 8) {
#pragma unroll
          for (int u = 0; u < 8; ++u) lo += sk[q + u] < key ? 1u : 0u;
        }
      } else {
        uint32_t hi = n;
        while (lo < hi) {
          const uint32_t mid = (lo + hi) >> 1;
          if (sk[mid] < key) lo = mid + 1; else hi = mid;
        }
      }
      g = off + e + lo;
      if (g < K) {
        sel[g] = static_cast<int32_t>(e0 + e);
        note_rank(g, key, K, nb, bk.split_next, bk.thresh_next);
      }
    }
    keep_rows(rp, g < K, g, e0 + e);
  }
}

// Gathers the bucket's offspring (own storage, then its share of the spill list) into
// (dk, di)[0..n) and pads up to npad.
template <typename K64, typename I32>
__device__ __forceinline__ void gather_bucket(K64 *dk, I32 *di, const BucketArgs &bk, uint32_t b, uint32_t n,
                                              uint32_t npad, uint32_t *lds_counter) {
  const uint32_t tid = threadIdx.x;
  const uint32_t n_main = n < bk.seg ? n : bk.seg;
  const uint64_t *gk = bk.keys + static_cast<size_t>(b) * bk.seg;
  const uint32_t *gi = bk.idx + static_cast<size_t>(b) * bk.seg;
  for (uint32_t e = tid; e < n_main; e += blockDim.x) { dk[e] = gk[e]; di[e] = gi[e]; }
  for (uint32_t e = n + tid; e < npad; e += blockDim.x) { dk[e] = ~0ull; di[e] = 0xFFFFFFFFu; }
  if (n > n_main) {
    const uint32_t spilled = bk.count[kSpillCounter];
    for (uint32_t q = tid; q < spilled; q += blockDim.x) {
      if (bk.spill_bucket[q] == b) {
        const uint32_t at = n_main + atomicAdd(lds_counter, 1u);
        dk[at] = bk.spill_keys[q];
        di[at] = bk.spill_idx[q];
      }
    }
  }
  __threadfence_block();
  __syncthreads();
}

// kElites: the quantile buckets above, each with its share of the survivors.  Without: the last
// step of the sample sort of the general path below, a bucket holds candidates only (fit_row,
// parent_row, count_next unused) and its first rank is the number of candidates before it.
// kThreads: a bucket of at most that many offspring (nearly all) is ranked straight from registers.
template <bool kElites, int kThreads>
__global__ __launch_bounds__(kThreads) void bucket_select_kernel(const double *fit_row,
                                                                       const uint32_t *parent_row, BucketArgs bk,
                                                                       RowPlan rp, uint32_t K, uint32_t *count_next,
                                                                       int32_t *sel) {
  __shared__ uint64_t sk[kBucketLds];
  __shared__ uint32_t si[kBucketLds];
  __shared__ uint64_t ek[kBucketElites];
  __shared__ uint32_t red[kThreads / kLanes];
  __shared__ uint32_t spill_cursor, pool_base;
  const uint32_t b = blockIdx.x, nb = bk.nb, tid = threadIdx.x;
  // offset of this bucket = its first survivor rank + all offspring of the buckets before it
  uint32_t before = 0;
  for (uint32_t c = tid; c < b; c += kThreads) before += bk.count[c];
  before = wave_sum_u32(before);
  if ((tid & (kLanes - 1)) == 0) red[tid / kLanes] = before;
  const uint32_t e0 = kElites ? bucket_bound(b, K, nb) : 0u, ne = kElites ? bucket_bound(b + 1, K, nb) - e0 : 0u;
  const uint32_t n = bk.count[b];
  // Every global load a small bucket needs is issued here, before anything waits for one: an
  // offspring per thread counted from thread 0 (read before the bucket's count is known: the
  // places beyond it hold whatever an earlier generation left, which is only used as an index
  // when it is one), a survivor per thread counted from the last one, and the rows of both.
  const uint32_t seg = bk.seg;
  uint64_t my_key = ~0ull, elite_key = 0;
  uint32_t my_idx = 0xFFFFFFFFu, my_row = 0, elite_row = 0;
  if (tid < seg) {
    my_key = bk.keys[static_cast<size_t>(b) * seg + tid];
    my_idx = bk.idx[static_cast<size_t>(b) * seg + tid];
  }
  const uint32_t se = kThreads - 1 - tid;
  if (se < ne) elite_row = parent_row[e0 + se];
  if (se < ne) elite_key = static_cast<uint64_t>(__double_as_longlong(fit_row[elite_row]));   // survivors stayed in their rows
  if (my_idx < 4 * K) my_row = rp.row_of_cur[my_idx];
  static_assert(kThreads <= kBucketCount, "a small bucket is ranked by counting");
  const bool small = n <= static_cast<uint32_t>(kThreads) && n <= seg && ne <= static_cast<uint32_t>(kThreads);
  // counting loops run in steps of 8 over padding; the sorting network needs a power of two
  const bool sorted = n > static_cast<uint32_t>(kBucketCount);
  const uint32_t npad = sorted ? pow2_at_least(n) : (n < 8 ? 8u : (n + 7) & ~7u);
  const bool in_lds = npad <= static_cast<uint32_t>(kBucketLds);
  if (small) {
    if (tid < npad) {                                // never sorted: npad <= the threads
      sk[tid] = tid < n ? my_key : ~0ull;
      si[tid] = tid < n ? my_idx : 0xFFFFFFFFu;
    }
    if (se < ne) ek[se] = elite_key;
  } else {
    for (uint32_t e = tid; e < ne; e += kThreads)
      ek[e] = static_cast<uint64_t>(__double_as_longlong(fit_row[parent_row[e0 + e]]));
  }
  if (tid == 0) {
    spill_cursor = 0;
    pool_base = in_lds ? 0u : atomicAdd(&bk.count[kPoolCounter], npad);   // a slice of the scratch pool
  }
  __syncthreads();
  uint32_t off = e0;
#pragma unroll
  for (int w = 0; w < kThreads / kLanes; ++w) off += red[w];
  if (off < K && n + ne != 0) {                      // otherwise nothing of this bucket survives
    if (small) {
      // offspring tid: rank = offspring below it + survivors with score <= its score (a survivor
      // wins a tie: smaller slot)
      {
        uint32_t g = K;
        if (tid < n) {
          uint32_t below = 0, equal = 0;             // padding keys are never below a real one
          for (uint32_t q = 0; q < npad; q += 8) {
#pragma unroll
            for (int v = 0; v < 8; ++v) {
              const uint64_t other = sk[q + v];
              below += other < my_key ? 1u : 0u;
              equal += other == my_key ? 1u : 0u;
            }
          }
          if (equal > 1)                             // shares its score: the slots decide
            for (uint32_t q = 0; q < n; ++q) below += (sk[q] == my_key && si[q] < my_idx) ? 1u : 0u;
          uint32_t lo = 0, hi = ne;
          while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (ek[mid] <= my_key) lo = mid + 1; else hi = mid;
          }
          g = off + below + lo;
          if (g < K) {
            sel[g] = static_cast<int32_t>(my_idx);
            if (kElites) note_rank(g, my_key, K, nb, bk.split_next, bk.thresh_next);
          }
        }
        keep_rows_at(rp, g < K, g, my_row);
      }
      // survivor se: rank = se + offspring with a strictly smaller score
      if (kElites) {
        uint32_t g = K;
        if (se < ne) {
          uint32_t lo = 0;
          for (uint32_t q = 0; q < npad; q += 8) {
#pragma unroll
            for (int v = 0; v < 8; ++v) lo += sk[q + v] < elite_key ? 1u : 0u;
          }
          g = off + se + lo;
          if (g < K) {
            sel[g] = static_cast<int32_t>(e0 + se);
            note_rank(g, elite_key, K, nb, bk.split_next, bk.thresh_next);
          }
        }
        keep_rows_at(rp, g < K, g, elite_row);
      }
    } else if (in_lds) {
      gather_bucket(sk, si, bk, b, n, npad, &spill_cursor);
      if (sorted) bitonic_sort(sk, si, npad);
      rank_bucket<kElites, kThreads>(sk, si, ek, n, npad, ne, e0, off, sorted, K, bk, rp, sel);
    } else {                                         // oversized bucket: same network in global memory
      uint64_t *pk = bk.pool_keys + pool_base;
      uint32_t *pi = bk.pool_idx + pool_base;
      gather_bucket(pk, pi, bk, b, n, npad, &spill_cursor);
      bitonic_sort(pk, pi, npad);
      rank_bucket<kElites, kThreads>(pk, pi, ek, n, npad, ne, e0, off, true, K, bk, rp, sel);
    }
  }
  if (kElites) {                                     // the other counter set, for the next generation
    if (tid == 0) count_next[b] = 0;
    if (b == 0 && tid < 2) count_next[kMaxBuckets + tid] = 0;
  }
}

// ------------------------------------------------- general path, larger pools -----
// Sample sort over the same bucket storage: a ranked sample of the pool's scores gives the
// splitters, every candidate is dropped into its bucket, and one workgroup per bucket ranks its
// share (bucket_select_kernel<false, .>); buckets concatenate to the global (score, slot) order and
// only those that reach below rank K do any work.  The sample only decides how even the buckets
// are, never the result.

// Splitters: `sample` = per * nb scores taken at a fixed stride from the pool; those of rank
// per * (c + 1) - 1 among them become splitter c (per = kOversample sample points per bucket, two
// where that would take more than kSampleMax; a bucket of 64 to 127 candidates on average then
// hardly ever grows beyond the 512 that are ranked straight from registers).  A splitter may be any value, so the low bits of a sample score
// give way to its position in the sample: all sample values differ and one 64-bit comparison
// orders them.  Ranks by counting: every workgroup loads the whole sample into LDS and each of
// its waves ranks four elements, the lanes striding over the sample.
constexpr int kSampleThreads = 1024;
constexpr int kOversample = 4;
constexpr int kSampleMax = 2048;
constexpr int kSamplePerWave = 1;
constexpr int kSamplePer = kSamplePerWave * kSampleThreads / kLanes;    // elements ranked by one workgroup
__global__ __launch_bounds__(kSampleThreads) void sample_splitters_kernel(const double *fit_row, const double *slot_score,
                                                                         const uint32_t *row_of, uint32_t P,
                                                                         uint32_t sample, uint32_t nb,
                                                                         uint64_t *split, uint32_t *count) {
  __shared__ uint64_t sk[kSampleMax];
  static_assert(kSampleMax <= 4096, "the position in the sample takes the low 12 bits of a score");
  const uint32_t per = sample / nb;                   // sample points per bucket: kOversample, or fewer with kMaxBuckets buckets
  const uint32_t t = threadIdx.x;
  const uint32_t sample_log2 = 31 - __clz(static_cast<int>(sample));
  if (blockIdx.x == 0)
    for (uint32_t c = t; c < static_cast<uint32_t>(kBucketCounters); c += kSampleThreads) count[c] = 0;
  uint64_t mine_of[kSampleMax / kSampleThreads];
#pragma unroll
  for (int u = 0; u < kSampleMax / kSampleThreads; ++u) {          // all loads first, then the stores
    const uint32_t e = t + u * kSampleThreads;
    // slot floor(e P / sample); sample is a power of two
    const uint32_t p = static_cast<uint32_t>((static_cast<uint64_t>(e) * P) >> sample_log2);
    mine_of[u] = e < sample ? static_cast<uint64_t>(__double_as_longlong(slot_score ? slot_score[p] : fit_row[row_of[p]])) : 0ull;
  }
#pragma unroll
  for (int u = 0; u < kSampleMax / kSampleThreads; ++u) {
    const uint32_t e = t + u * kSampleThreads;
    sk[e] = e < sample ? (mine_of[u] & ~0xFFFull) | e : ~0ull;     // the padding is never below an element
  }
  __syncthreads();
  const uint32_t lane = t % kLanes;
  const uint32_t first = blockIdx.x * kSamplePer + (t / kLanes) * kSamplePerWave;   // sample = kSamplePer * the workgroups
  uint64_t key[kSamplePerWave];
  uint32_t below[kSamplePerWave];
#pragma unroll
  for (int m = 0; m < kSamplePerWave; ++m) { key[m] = sk[first + m]; below[m] = 0; }
  for (uint32_t q = lane; q < sample; q += 2 * kLanes) {           // sample is a multiple of 128
    const uint64_t a = sk[q], b = sk[q + kLanes];
#pragma unroll
    for (int m = 0; m < kSamplePerWave; ++m) below[m] += (a < key[m] ? 1u : 0u) + (b < key[m] ? 1u : 0u);
  }
#pragma unroll
  for (int m = 0; m < kSamplePerWave; ++m) {
    const uint32_t r = wave_sum_u32(below[m]);
    // rank per * (c + 1) - 1 makes splitter c; the last bucket has none
    if (lane == 0 && r % per == per - 1 && r / per + 1 < nb) split[r / per] = key[m];
  }
  // the splitters beyond are +inf: nothing lands in those buckets
  if (blockIdx.x == 0)
    for (uint32_t c = nb - 1 + t; c < static_cast<uint32_t>(kMaxBuckets); c += kSampleThreads) split[c] = ~0ull;
}

// Bucket of a score = number of splitters <= it (equal scores share a bucket).  A workgroup
// first counts its candidates per bucket in LDS and reserves their places with one global
// atomic per bucket, instead of one per candidate.
constexpr int kDropThreads = 1024;
__global__ __launch_bounds__(kDropThreads) void drop_all_kernel(const double *fit_row, const double *slot_score,
                                                               const uint32_t *row_of, uint32_t P, BucketArgs bk) {
  __shared__ uint64_t split[kMaxBuckets];
  __shared__ uint32_t here[kMaxBuckets], base[kMaxBuckets];
  const uint32_t t = threadIdx.x, nb = bk.nb;
  for (uint32_t c = t; c < nb; c += kDropThreads) { split[c] = bk.split[c]; here[c] = 0; }
  __syncthreads();
  const uint32_t p = blockIdx.x * kDropThreads + t;
  uint64_t key = 0;
  uint32_t b = 0, r = 0;
  if (p < P) {
    key = static_cast<uint64_t>(__double_as_longlong(slot_score ? slot_score[p] : fit_row[row_of[p]]));
    uint32_t lo = 0, hi = nb - 1;                    // splitters 0 .. nb-2
    while (lo < hi) {
      const uint32_t mid = (lo + hi) >> 1;
      if (split[mid] <= key) lo = mid + 1; else hi = mid;
    }
    b = lo;
    r = atomicAdd(&here[b], 1u);
  }
  __syncthreads();
  for (uint32_t c = t; c < nb; c += kDropThreads) base[c] = here[c] ? atomicAdd(&bk.count[c], here[c]) : 0u;
  __syncthreads();
  if (p < P) {
    const uint32_t slot = base[b] + r;
    if (slot < bk.seg) {
      const size_t at = static_cast<size_t>(b) * bk.seg + slot;
      bk.keys[at] = key;
      bk.idx[at] = p;
    } else {                                         // bucket full: shared spill list (holds a whole pool)
      const uint32_t at = atomicAdd(&bk.count[kSpillCounter], 1u);
      bk.spill_keys[at] = key;
      bk.spill_idx[at] = p;
      bk.spill_bucket[at] = b;
    }
  }
}

__global__ void zero_words_kernel(uint32_t *words, uint32_t n) {
  const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) words[i] = 0;
}

// Splitters after a selection by the general path.
__global__ void splitters_kernel(const double *fit_row, const uint32_t *row_of, const int32_t *sel, uint32_t K,
                                 uint32_t nb, uint64_t *split, uint64_t *thresh, uint32_t *count0,
                                 uint32_t *count1) {
  const uint32_t c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c < static_cast<uint32_t>(kBucketCounters)) { count0[c] = 0; count1[c] = 0; }
  if (c < static_cast<uint32_t>(kMaxBuckets))
    split[c] = (c + 1 < nb) ? static_cast<uint64_t>(__double_as_longlong(fit_row[row_of[sel[bucket_bound(c + 1, K, nb)]]]))
                            : 0x7FF0000000000000ull;          // +infinity pads the table
  if (c == 0) *thresh = static_cast<uint64_t>(__double_as_longlong(fit_row[row_of[sel[K - 1]]]));
}

// What the kernels need of one job slot, derived from the validated raw table.
struct SlotValues { uint32_t cstart, cmax, info; double abl, cc, d, Y; };

__device__ __forceinline__ SlotValues derive_slot(const RawJobs &raw, uint32_t j) {
  const uint32_t w = raw.rawinfo[j];
  const int lo = w & 31, hi = (w >> 5) & 31, mu = (w >> 10) & 31;
  if (!((w >> 15) & 1u)) return SlotValues{0u, 0u, 0u, 0.0, 0.0, 0.0, 0.0};
  const int bl = min(mu, hi);                       // log2 of the local batch of a running job
  const int gstart = max(lo, bl);                   // batch a waiting job resumes with
  SlotValues v;
  v.cstart = 1u << max(0, gstart - mu);
  v.cmax = 1u << max(0, hi - mu);
  v.info = static_cast<uint32_t>(lo) | (static_cast<uint32_t>(hi - lo + 2) << 5) | (static_cast<uint32_t>(mu) << 11) |
           (static_cast<uint32_t>(bl) << 16) | (1u << 21) | (((w >> 16) & 1u) << 22);
  v.abl = raw.a[j] * static_cast<double>(1u << bl);
  v.cc = raw.c[j];
  v.d = raw.d[j];
  v.Y = raw.Y[j];
  return v;
}

// A new job table in one launch.  The first table_blocks workgroups derive the per-slot values
// and the term table (thread q: entry q of the term table; the thread of a slot's code 0 also
// writes the slot's values); the workgroups behind them set the n_changed slots that changed
// hands to "waiting" in every genome row (one thread per (row, changed slot), the slots of a
// row next to each other).
constexpr int kTableThreads = 256;
__global__ __launch_bounds__(kTableThreads) void table_change_kernel(RawJobs raw, JobTable tab, uint32_t Jp,
                                                                     uint32_t table_blocks, int32_t *genes,
                                                                     const uint32_t *slots, uint32_t n_changed,
                                                                     uint32_t rows) {
  if (blockIdx.x < table_blocks) {
    const uint32_t q = blockIdx.x * kTableThreads + threadIdx.x;
    const uint32_t E = tab.term_E;
    if (q >= Jp * E) return;
    const uint32_t lane = q % kLanes, e = (q / kLanes) % E, row = q / (kLanes * E);
    const uint32_t j = row * kLanes + lane;
    const SlotValues v = derive_slot(raw, j);
    tab.terms[q] = term_of(v.abl, v.cc, v.d, v.Y, info_blexp(v.info), e);
    if (e == 0) {
      tab.cstart[j] = v.cstart; tab.cmax[j] = v.cmax; tab.info[j] = v.info;
      tab.abl[j] = v.abl; tab.cc[j] = v.cc; tab.d[j] = v.d; tab.Y[j] = v.Y;
    }
    return;
  }
  const uint32_t n = rows * n_changed;               // at most 1.25 * 2^20 * 2048 < 2^32
  const uint32_t reset_blocks = gridDim.x - table_blocks;
  for (uint32_t e = (blockIdx.x - table_blocks) * kTableThreads + threadIdx.x; e < n; e += reset_blocks * kTableThreads) {
    const uint32_t row = e / n_changed, k = e - row * n_changed;
    genes[static_cast<size_t>(row) * Jp + slots[k]] = 0;
  }
}

// Term table: the score formula evaluated once per (slot, GPU-count code), same operations in
// the same order as the per-gene evaluation, so both give the same bits.
__global__ void build_terms_kernel(JobTable tab, uint32_t Jp) {
  const uint32_t q = blockIdx.x * blockDim.x + threadIdx.x;
  const uint32_t E = tab.term_E;
  if (q >= Jp * E) return;
  const uint32_t lane = q % kLanes, e = (q / kLanes) % E, row = q / (kLanes * E);
  const uint32_t j = row * kLanes + lane;
  tab.terms[q] = term_of(tab.abl[j], tab.cc[j], tab.d[j], tab.Y[j], info_blexp(tab.info[j]), e);
}

__global__ void best_kernel(const int32_t *genes, const double *fit_row, const uint32_t *row_of, const int32_t *sel,
                            const uint32_t *info, uint32_t Jn, uint32_t Jp, int32_t *batch_out, int32_t *gpus_out,
                            double *fit_out, const uint32_t *err_in, uint32_t *err_out) {
  const uint32_t best = row_of[sel[0]];
  const int32_t *row = genes + static_cast<size_t>(best) * Jp;
  for (uint32_t j = threadIdx.x; j < Jn; j += blockDim.x) {
    const uint32_t B = static_cast<uint32_t>(row[j]);
    batch_out[j] = static_cast<int32_t>(B);
    gpus_out[j] = static_cast<int32_t>(B ? max(1u, B >> info_mu(info[j])) : 0u);
  }
  if (threadIdx.x == 0) {
    *fit_out = fit_row[best];
    err_out[0] = err_in[0];                          // the two error words travel to the host with the winner
    err_out[1] = err_in[1];
  }
}

// The winner unrolled over the GPUs (Eq. 1, reorder): every workgroup scans the jobs' GPU
// counts in LDS (at most 2048 slots), then each thread finds the job of one GPU by binary
// search over the prefix sums.
constexpr int kPlaceThreads = 1024;
__global__ __launch_bounds__(kPlaceThreads) void placement_kernel(const int32_t *genes, const uint32_t *row_of,
                                                                 const int32_t *sel, const uint32_t *info, uint32_t Jn,
                                                                 uint32_t Jp, uint32_t G, int32_t *slot_of_gpu,
                                                                 int32_t *batch_of_gpu) {
  __shared__ uint32_t first[2 * kPlaceThreads + 1];    // first GPU of every slot, then the GPUs in use
  __shared__ uint32_t per_gpu[2 * kPlaceThreads];      // local batch of every slot's workers
  __shared__ uint32_t wave_total[kPlaceThreads / kLanes];
  const int32_t *row = genes + static_cast<size_t>(row_of[sel[0]]) * Jp;
  const uint32_t t = threadIdx.x;
  // thread t owns slots 2t and 2t + 1
  uint32_t c[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const uint32_t j = 2 * t + u;
    const uint32_t B = j < Jn ? static_cast<uint32_t>(row[j]) : 0u;
    c[u] = B ? max(1u, B >> info_mu(info[j < Jn ? j : 0])) : 0u;
    per_gpu[j] = B ? B / c[u] : 0u;
  }
  const uint32_t mine = c[0] + c[1];
  uint32_t incl = mine;
#pragma unroll
  for (int d = 1; d < kLanes; d <<= 1) {
    const uint32_t up = __shfl_up(incl, d, kLanes);
    if ((t & (kLanes - 1)) >= static_cast<uint32_t>(d)) incl += up;
  }
  if ((t & (kLanes - 1)) == kLanes - 1) wave_total[t / kLanes] = incl;
  __syncthreads();
  uint32_t before = 0;
  for (uint32_t w = 0; w < t / kLanes; ++w) before += wave_total[w];
  const uint32_t excl = before + incl - mine;
  first[2 * t] = excl;
  first[2 * t + 1] = excl + c[0];
  if (t == kPlaceThreads - 1) first[2 * kPlaceThreads] = excl + mine;
  __syncthreads();
  const uint32_t used = first[2 * kPlaceThreads];
  for (uint32_t i = blockIdx.x * kPlaceThreads + t; i < G; i += gridDim.x * kPlaceThreads) {
    int32_t slot = -1, batch = 0;
    if (i < used) {
      uint32_t lo = 0, hi = 2 * kPlaceThreads;       // last slot with first[slot] <= i
      while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (first[mid] <= i) lo = mid; else hi = mid;
      }
      slot = static_cast<int32_t>(lo);
      batch = static_cast<int32_t>(per_gpu[lo]);
    }
    if (slot_of_gpu) slot_of_gpu[i] = slot;
    if (batch_of_gpu) batch_of_gpu[i] = batch;
  }
}

}  // namespace

hipError_t launch_build_terms(const JobTable &tab, uint32_t Jp, hipStream_t s) {
  const uint32_t n = Jp * tab.term_E;
  hipLaunchKernelGGL(build_terms_kernel, dim3((n + 255) / 256), dim3(256), 0, s, tab, Jp);
  return hipGetLastError();
}

hipError_t launch_table_change(const RawJobs &raw, const JobTable &tab, uint32_t Jp, int32_t *genes, const uint32_t *slots,
                               uint32_t n_changed, uint32_t rows, hipStream_t s) {
  const uint32_t table_blocks = (Jp * tab.term_E + kTableThreads - 1) / kTableThreads;
  const uint64_t n = static_cast<uint64_t>(rows) * n_changed;
  if (n > 0xFFFFFFFFull) return hipErrorInvalidValue;
  const uint32_t reset_blocks = static_cast<uint32_t>(std::min<uint64_t>((n + kTableThreads - 1) / kTableThreads, 16384));
  hipLaunchKernelGGL(table_change_kernel, dim3(table_blocks + reset_blocks), dim3(kTableThreads), 0, s, raw, tab, Jp,
                     table_blocks, genes, slots, n_changed, rows);
  return hipGetLastError();
}

hipError_t launch_zero_words(uint32_t *words, uint32_t n, hipStream_t s) {
  hipLaunchKernelGGL(zero_words_kernel, dim3((n + 255) / 256), dim3(256), 0, s, words, n);
  return hipGetLastError();
}

hipError_t launch_select(const double *fit, const double *slot_score, const RowPlan &rp, uint32_t P, uint32_t K,
                         const BucketArgs &store, int32_t *sel, hipStream_t s) {
  if (P <= kRankPoolMax) {
    const uint32_t rank_blocks = (P + kRankPoolPer - 1) / kRankPoolPer;
    constexpr uint32_t kStep = 8 * (kSortThreads / kRankPoolPer);
    const size_t lds = static_cast<size_t>((P + kStep - 1) / kStep * kStep) * 8 + kRankPoolPer * 4;
    hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void *>(rank_pool_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (rc != hipSuccess) return rc;
    hipLaunchKernelGGL(rank_pool_kernel, dim3(rank_blocks), dim3(kSortThreads), lds, s, fit, slot_score, rp, P, K, sel);
    return hipGetLastError();
  }
  // 64 to 127 candidates per bucket (more in pools beyond 2^17), kOversample sample points per
  // bucket while the sample stays within kSampleMax
  BucketArgs bk = store;
  uint32_t nb = 32;
  while (nb < static_cast<uint32_t>(kMaxBuckets) && nb * 128 <= P) nb <<= 1;
  const uint32_t sample = std::min<uint32_t>(kOversample * nb, kSampleMax);   // a power of two, 256 .. kSampleMax
  bk.seg = static_cast<uint32_t>(static_cast<size_t>(store.nb) * store.seg / nb);   // the same storage, re-divided
  bk.nb = nb;
  hipLaunchKernelGGL(sample_splitters_kernel, dim3(sample / kSamplePer), dim3(kSampleThreads), 0, s, fit, slot_score,
                     rp.row_of_cur, P, sample, nb, const_cast<uint64_t *>(bk.split), bk.count);
  hipError_t rc = hipGetLastError();
  if (rc != hipSuccess) return rc;
  hipLaunchKernelGGL(drop_all_kernel, dim3((P + kDropThreads - 1) / kDropThreads), dim3(kDropThreads), 0, s, fit,
                     slot_score, rp.row_of_cur, P, bk);
  rc = hipGetLastError();
  if (rc != hipSuccess) return rc;
  hipLaunchKernelGGL((bucket_select_kernel<false, kBucketCount>), dim3(nb), dim3(kBucketCount), 0, s, nullptr, nullptr,
                     bk, rp, K, nullptr, sel);
  return hipGetLastError();
}

hipError_t launch_bucket_select(const double *fit_row, const uint32_t *parent_row, const BucketArgs &bk,
                                const RowPlan &rp, uint32_t K, uint32_t *count_next, int32_t *sel, hipStream_t s) {
  hipLaunchKernelGGL((bucket_select_kernel<true, kBucketThreads>), dim3(bk.nb), dim3(kBucketThreads), 0, s, fit_row,
                     parent_row, bk, rp, K, count_next, sel);
  return hipGetLastError();
}

hipError_t launch_splitters(const double *fit_row, const uint32_t *row_of, const int32_t *sel, uint32_t K,
                            uint32_t nb, uint64_t *split, uint64_t *thresh, uint32_t *count0, uint32_t *count1,
                            hipStream_t s) {
  hipLaunchKernelGGL(splitters_kernel, dim3((kBucketCounters + 255) / 256), dim3(256), 0, s, fit_row, row_of, sel, K,
                     nb, split, thresh, count0, count1);
  return hipGetLastError();
}

hipError_t launch_placement(const int32_t *genes, const uint32_t *row_of, const int32_t *sel, const uint32_t *info,
                            uint32_t Jn, uint32_t Jp, uint32_t G, int32_t *slot_of_gpu, int32_t *batch_of_gpu,
                            hipStream_t s) {
  const uint32_t blocks = std::max<uint32_t>(1u, std::min<uint32_t>((G + kPlaceThreads - 1) / kPlaceThreads, 1024u));
  hipLaunchKernelGGL(placement_kernel, dim3(blocks), dim3(kPlaceThreads), 0, s, genes, row_of, sel, info, Jn, Jp, G,
                     slot_of_gpu, batch_of_gpu);
  return hipGetLastError();
}

hipError_t launch_best(const int32_t *genes, const double *fit_row, const uint32_t *row_of, const int32_t *sel,
                       const uint32_t *info, uint32_t Jn, uint32_t Jp, int32_t *batch_out, int32_t *gpus_out,
                       double *fit_out, const uint32_t *err_in, uint32_t *err_out, hipStream_t s) {
  hipLaunchKernelGGL(best_kernel, dim3(1), dim3(256), 0, s, genes, fit_row, row_of, sel, info, Jn, Jp, batch_out,
                     gpus_out, fit_out, err_in, err_out);
  return hipGetLastError();
}

}  // namespace ones
