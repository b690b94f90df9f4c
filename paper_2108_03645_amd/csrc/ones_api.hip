// Host side of libones: argument validation, workspace layout, launch sequencing.
// The boundary is declared and documented in include/ones.h.
#include "ones.h"
#include "ones_device.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <vector>

// Scratch of ones_generation_static: one copy per GPU, held by every device that runs the
// library until the process ends.  Host code must not use this name as an address: the
// per-device address comes from hipGetSymbolAddress (static_scratch_of below).
static __device__ __align__(256) unsigned char scratch[ONES_STATIC_SCRATCH_BYTES];

namespace {

using namespace ones;

thread_local char g_hip_msg[256] = "HIP call failed";

int hip_fail(hipError_t e, const char *what) {
  snprintf(g_hip_msg, sizeof(g_hip_msg), "HIP call failed: %s: %s", what, hipGetErrorString(e));
  return ONES_E_HIP;
}
#define HIP_TRY(expr)                                         \
  do {                                                        \
    hipError_t e__ = (expr);                                  \
    if (e__ != hipSuccess) return hip_fail(e__, #expr);       \
  } while (0)

template <typename F>
int guarded(F &&body) noexcept {
  try {
    return body();
  } catch (const std::bad_alloc &) {
    snprintf(g_hip_msg, sizeof(g_hip_msg), "out of host memory");
  } catch (...) {
    snprintf(g_hip_msg, sizeof(g_hip_msg), "unexpected C++ exception");
  }
  return ONES_E_HIP;
}

size_t align_up(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }

// Device address of the static scratch array on the current device, resolved once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
char *g_scratch_ptr[kMaxDevices];

int static_scratch_of(int device, char **out) {
  if (device < 0 || device >= kMaxDevices) {
    snprintf(g_hip_msg, sizeof(g_hip_msg), "device ordinal %d outside 0..%d", device, kMaxDevices - 1);
    return ONES_E_HIP;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void *ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));   // for the device that is current
    g_scratch_ptr[device] = static_cast<char *>(ptr);
  }
  *out = g_scratch_ptr[device];
  return ONES_OK;
}

// Scratch of the selection: nothing in it outlives the generations of one ones_generation call
// except the splitters, the threshold and the cleared counter sets, which the next call may use
// (ctx->splitters_valid).  Offsets from the block's base, which lies in the caller's workspace
// or, for ones_generation_static, in the library's static array.
struct ScratchLayout {
  size_t split, thresh, bcount[2], bkeys, bidx, skeys, sidx, sbucket, pkeys, pidx, total;
};

struct Layout {
  size_t genes, fit_row, slot_score, row_of[2], parent_row[2], occupied[2], sel, fsync, xkeys, scratch, cstart, cmax, info, abl, cc, d, Y[kDrawRing], terms[kDrawRing];
  size_t rawinfo, changed, ra, rc, rd, rY, alpha, beta, processed, time_rank, best_batch, best_gpus, best_fit, best_err, place_slot, place_batch, total;
  ScratchLayout S;
};

// Buckets of the selection: about 16 survivors each, at most kMaxBuckets.  A bucket stores eight
// times its fair share of the 3P/4 children and mutants (at least 256, a power of two); the
// surplus goes to a spill list that can hold a whole pool (the general selection drops every
// candidate, and equal scores all land in one bucket), and buckets too large for LDS are sorted
// in a scratch pool (each takes a power-of-two slice below twice its size).  The general
// selection re-divides the same bucket space among its own number of buckets.
struct BucketPlan { uint32_t nb, seg, spill, pool; };
constexpr uint32_t kMinBucketPool = 256;
uint32_t pow2_at_least(uint32_t v) { uint32_t n = 1; while (n < v) n <<= 1; return n; }
BucketPlan bucket_plan(uint32_t P) {
  if (P < kMinBucketPool) return BucketPlan{0, 0, 0, 0};      // tiny pools: one short sort is as fast
  const uint32_t K = P / 4;
  BucketPlan bp;
  bp.nb = std::min<uint32_t>(kMaxBuckets, std::max<uint32_t>(1, K / 16));
  bp.spill = P;                                            // the general selection may spill a whole pool
  bp.pool = 2 * pow2_at_least(P);                          // every slice is a power of two below twice its bucket
  bp.seg = std::min(pow2_at_least(std::max<uint32_t>(256, 8 * ((3 * K + bp.nb - 1) / bp.nb))), bp.pool / 4);
  return bp;
}

// Pools whose generations run in one launch per ones_generation call (ones_fused.hip).  The
// launch is a cooperative one, which costs about 20 us where an ordinary launch costs 2.5, so
// calls of one or two generations are cheaper as two ordinary launches per generation.
constexpr int32_t kFusedMinGenerations = 3;
bool fused_pool(uint32_t P, uint32_t Jp) { return Jp == static_cast<uint32_t>(kLanes) && P <= kFusedMaxPool; }

ScratchLayout make_scratch_layout(uint32_t P) {
  ScratchLayout S;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t at = off; off = align_up(off + bytes); return at; };
  const BucketPlan bp = bucket_plan(P);
  S.split = take(kMaxBuckets * 8); S.thresh = take(8);
  S.bcount[0] = take(kBucketCounters * 4); S.bcount[1] = take(kBucketCounters * 4);
  S.bkeys = take(static_cast<size_t>(bp.nb) * bp.seg * 8);
  S.bidx = take(static_cast<size_t>(bp.nb) * bp.seg * 4);
  S.skeys = take(static_cast<size_t>(bp.spill) * 8);
  S.sidx = take(static_cast<size_t>(bp.spill) * 4);
  S.sbucket = take(static_cast<size_t>(bp.spill) * 4);
  S.pkeys = take(static_cast<size_t>(bp.pool) * 8);
  S.pidx = take(static_cast<size_t>(bp.pool) * 4);
  S.total = off;
  return S;
}

Layout make_layout(uint32_t P, uint32_t Jp, uint32_t G) {
  Layout L;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t at = off; off = align_up(off + bytes); return at; };
  const size_t rows = static_cast<size_t>(P) + P / 4;      // a pool of P slots lives in P + K physical rows
  L.genes = take(rows * Jp * 4);
  L.fit_row = take(rows * 8);
  L.slot_score = take(static_cast<size_t>(P) * 8);
  L.row_of[0] = take(static_cast<size_t>(P) * 4);
  L.row_of[1] = take(static_cast<size_t>(P) * 4);
  L.parent_row[0] = take(static_cast<size_t>(P / 4) * 4);
  L.parent_row[1] = take(static_cast<size_t>(P / 4) * 4);
  L.occupied[0] = take((rows + 31) / 32 * 4);     // bitmaps of the rows the survivors keep
  L.occupied[1] = take((rows + 31) / 32 * 4);
  L.sel = take(static_cast<size_t>(P / 4) * 4);
  // single-launch generations of small pools: arrival counter + error word, scores exchanged by slot
  L.fsync = take(256);
  L.xkeys = take(fused_pool(P, Jp) ? fused_exchange_bytes(P) : 0);
  // the selection's scratch: splitters, counters, bucket storage, spill list, scratch pool
  L.S = make_scratch_layout(P);
  L.scratch = take(L.S.total);
  L.cstart = take(Jp * 4); L.cmax = take(Jp * 4); L.info = take(Jp * 4);
  L.abl = take(Jp * 8); L.cc = take(Jp * 8); L.d = take(Jp * 8);
  // remaining work and the term table built from it, a ring of kDrawRing pairs at equal distances:
  // under probability sampling the draws of that many generations are made in one launch, and
  // generation g is scored with pair g mod kDrawRing
  for (int k = 0; k < kDrawRing; ++k) { L.Y[k] = take(Jp * 8); L.terms[k] = take(static_cast<size_t>(Jp) * kMaxTermEntries * 8); }
  L.rawinfo = take(Jp * 4); L.changed = take(Jp * 4);
  L.ra = take(Jp * 8); L.rc = take(Jp * 8); L.rd = take(Jp * 8); L.rY = take(Jp * 8);
  L.alpha = take(Jp * 8); L.beta = take(Jp * 8); L.processed = take(Jp * 8);
  L.time_rank = take(Jp * 4);
  L.best_batch = take(Jp * 4); L.best_gpus = take(Jp * 4); L.best_fit = take(8); L.best_err = take(8);
  L.place_slot = take(static_cast<size_t>(G) * 4); L.place_batch = take(static_cast<size_t>(G) * 4);
  L.total = off;
  return L;
}

// Host transfers go through one pinned staging buffer, a single copy per call: the arrays that
// travel together lie next to each other in the workspace (every size below is a multiple of the
// 256-byte alignment except the last of a group).
size_t stage_bytes(const Layout &L, uint32_t Jp, uint32_t G) {
  const size_t table = L.rY + static_cast<size_t>(Jp) * 8 - L.rawinfo;        // rawinfo, changed, a, c, d, Y
  const size_t progress = L.processed + static_cast<size_t>(Jp) * 8 - L.alpha; // alpha, beta, processed
  const size_t best = L.best_err + 8 - L.best_batch;                           // batch, gpus, fitness, error words
  const size_t place = L.place_batch + static_cast<size_t>(G) * 4 - L.place_slot;
  return std::max({table, progress, best, place, static_cast<size_t>(Jp) * 4});
}

int check_config(const ones_config *cfg) {
  if (!cfg) return ONES_E_INVALID_ARG;
  if (cfg->n_gpus < 0 || cfg->n_gpus > ONES_MAX_GPUS) return ONES_E_INVALID_ARG;
  if (cfg->n_slots < 0 || cfg->n_slots > ONES_MAX_SLOTS) return ONES_E_INVALID_ARG;
  if (cfg->population <= 0 || cfg->population % 4 != 0 || cfg->population > ONES_MAX_POPULATION)
    return ONES_E_INVALID_ARG;
  if (!(cfg->mutation_rate >= 0.0 && cfg->mutation_rate <= 1.0)) return ONES_E_INVALID_ARG;
  if (!(cfg->crossover_rate >= 0.0 && cfg->crossover_rate <= 1.0)) return ONES_E_INVALID_ARG;
  return ONES_OK;
}

// A rate becomes a threshold on a uniform 32-bit word: min(2^32 - 1, floor(rate * 2^32)).
uint32_t rate_threshold(double rate) {
  const double v = std::floor(rate * 4294967296.0);
  return v >= 4294967295.0 ? 0xFFFFFFFFu : static_cast<uint32_t>(v);
}

int log2_pow2(int32_t v) {           // -1 unless v is a power of two
  if (v <= 0 || (v & (v - 1)) != 0) return -1;
  return 31 - __builtin_clz(static_cast<uint32_t>(v));
}

int check_param(double v) {
  if (!std::isfinite(v)) return ONES_E_NONFINITE;
  if (v < 0.0) return ONES_E_INVALID_ARG;
  if (v > ONES_MAX_PARAM) return ONES_E_BOUNDS;
  return ONES_OK;
}

struct HostJobs {                     // validated, padded staging copy of a job table
  std::vector<uint32_t> rawinfo;
  std::vector<double> a, c, d, Y;
  std::vector<int64_t> id;
  uint32_t term_E = 2;                // waiting + GPU-count codes up to the largest bmax / gpu_max_batch
};

int stage_jobs(int Jn, int Jp, const ones_jobs *jobs, HostJobs &h) {
  h.rawinfo.assign(Jp, 0u);
  h.a.assign(Jp, 0.0); h.c.assign(Jp, 0.0); h.d.assign(Jp, 0.0); h.Y.assign(Jp, 0.0);
  h.id.assign(Jp, 0);
  h.term_E = 2;
  if (Jn > 0 && (!jobs || !jobs->job_id || !jobs->active || !jobs->bmin || !jobs->bmax ||
                 !jobs->gpu_max_batch || !jobs->a || !jobs->c || !jobs->d || !jobs->remaining))
    return ONES_E_INVALID_ARG;
  for (int j = 0; j < Jn; ++j) {
    h.id[j] = jobs->job_id[j];
    if (!jobs->active[j]) continue;
    const int lo = log2_pow2(jobs->bmin[j]), hi = log2_pow2(jobs->bmax[j]);
    const int mu = log2_pow2(jobs->gpu_max_batch[j]);
    if (lo < 0 || hi < 0 || mu < 0) return ONES_E_NOT_POW2;
    if (lo > hi || hi > 30 || hi - mu > 20) return ONES_E_BOUNDS;
    int rc;
    if ((rc = check_param(jobs->a[j])) || (rc = check_param(jobs->c[j])) ||
        (rc = check_param(jobs->d[j])) || (rc = check_param(jobs->remaining[j])))
      return rc;
    h.rawinfo[j] = static_cast<uint32_t>(lo) | (static_cast<uint32_t>(hi) << 5) |
                   (static_cast<uint32_t>(mu) << 10) | (1u << 15);
    h.a[j] = jobs->a[j]; h.c[j] = jobs->c[j]; h.d[j] = jobs->d[j]; h.Y[j] = jobs->remaining[j];
    h.term_E = std::max<uint32_t>(h.term_E, static_cast<uint32_t>(std::max(0, hi - mu)) + 2);
  }
  return ONES_OK;
}

struct EventPair { hipEvent_t start, stop; };

}  // namespace

struct ones_ctx {
  ones_config cfg;
  uint32_t P, K, Jn, Jp, R, G;
  uint32_t T_mut, T_x;
  hipStream_t stream;
  char *ws;
  char *stage;                // pinned host staging buffer (stage_bytes), free between calls
  char *stage_dev;            // the same buffer as the device addresses it (ones_best's kernel writes the winner there)
  Layout L;
  int cur;                    // which row_of array describes the current generation
  bool table_changed;         // job table replaced since the current generation was computed
  bool no_schedule;           // ... by ones_set_jobs: the winner is not a schedule under the new table
  bool new_jobs_first;        // option: the generation after ones_set_jobs serves the arrived jobs first
  bool sampling;              // remaining work drawn per generation (Alg. 1) instead of the table's
  int y_cur;                  // which remaining-work array and term table the last generation was scored with
  int64_t drawn_from, drawn_to;  // the ring holds the draws of generations [drawn_from, drawn_to) (equal: none)
  bool per_gpu;               // uniform crossover over the GPUs instead of the jobs (ones_set_crossover)
  bool has_times;             // executed times known (ones_set_processed_time): their ranks are on the device
  BucketPlan bp;              // nb == 0: pool small enough for the single-chunk sort
  int bucket_phase;           // which counter set the next bucketed generation fills
  bool splitters_valid;       // the workspace's selection scratch holds the splitters of the current survivors
                              // and cleared counter sets: a bucketed generation may follow
  bool poisoned;              // a launch failed in the middle of a generation: the state is inconsistent
  bool fused;                 // small pool: all generations of a call in one cooperative launch
  uint32_t fused_generations; // generations those launches have run so far
  uint32_t fused_changes;     // ... of them generations that also exchanged the survivors' scores
  uint32_t fused_draws;       // ... of them generations with a drawn remaining work
  uint32_t spin_limit;        // polls before a device-wide wait gives up
  int device;                 // the device the context was created on
  char *static_scratch;       // this device's copy of the library's static scratch array
  int n_cus;
  uint32_t term_E;            // entries per job of the term table
  int64_t t;                  // generation counter
  std::vector<int64_t> ids;   // job identity per slot, to detect slots that change hands
  // measurement
  bool profiling;
  int profile_every;          // bracket the kernels of every profile_every-th generation
  int64_t profile_tick;
  std::vector<EventPair> evolve_ev, select_ev;
  size_t evolve_used, select_used;

  template <typename T> T *at(size_t off) const { return reinterpret_cast<T *>(ws + off); }
  JobTable table(int which) const {     // with the remaining work and term table number `which`
    return JobTable{at<uint32_t>(L.cstart), at<uint32_t>(L.cmax), at<uint32_t>(L.info),
                    at<double>(L.abl), at<double>(L.cc), at<double>(L.d), at<double>(L.Y[which]),
                    at<double>(L.terms[which]), term_E};
  }
  JobTable table() const { return table(y_cur); }
};

namespace {

int upload_table(ones_ctx *c, const HostJobs &h, const std::vector<uint32_t> *changed) {
  const size_t n4 = static_cast<size_t>(c->Jp) * 4, n8 = static_cast<size_t>(c->Jp) * 8;
  const Layout &L = c->L;
  auto staged = [&](size_t off) { return c->stage + (off - L.rawinfo); };   // laid out as in the workspace
  memcpy(staged(L.rawinfo), h.rawinfo.data(), n4);
  const size_t n_changed = changed ? changed->size() : 0;          // the slots that changed hands, as a list
  if (n_changed) memcpy(staged(L.changed), changed->data(), n_changed * 4);
  memset(staged(L.changed) + n_changed * 4, 0, n4 - n_changed * 4);
  memcpy(staged(L.ra), h.a.data(), n8);
  memcpy(staged(L.rc), h.c.data(), n8);
  memcpy(staged(L.rd), h.d.data(), n8);
  memcpy(staged(L.rY), h.Y.data(), n8);
  HIP_TRY(hipMemcpyAsync(c->ws + L.rawinfo, c->stage, L.rY + n8 - L.rawinfo, hipMemcpyHostToDevice, c->stream));
  RawJobs raw{c->at<uint32_t>(c->L.rawinfo), c->at<double>(c->L.ra), c->at<double>(c->L.rc),
              c->at<double>(c->L.rd), c->at<double>(c->L.rY)};
  c->term_E = h.term_E;
  // every physical row, whether a candidate lives in it or not
  HIP_TRY(launch_table_change(raw, c->table(), c->Jp, c->at<int32_t>(c->L.genes), c->at<uint32_t>(c->L.changed),
                              static_cast<uint32_t>(n_changed), c->P + c->K, c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));     // the staging buffer is free again
  return ONES_OK;
}

int timed(ones_ctx *c, std::vector<EventPair> &pool, size_t &used, bool begin) {
  if (!c->profiling || c->profile_tick % c->profile_every != 0) return ONES_OK;
  if (begin) {
    if (used == pool.size()) {
      EventPair e;
      HIP_TRY(hipEventCreate(&e.start));
      HIP_TRY(hipEventCreate(&e.stop));
      pool.push_back(e);
    }
    HIP_TRY(hipEventRecord(pool[used].start, c->stream));
  } else {
    HIP_TRY(hipEventRecord(pool[used].stop, c->stream));
    ++used;
  }
  return ONES_OK;
}

// scratch: base of the selection's scratch block (the workspace's, or the static array);
// splitters_valid: that block holds the current survivors' splitters and cleared counters.
int run_generation(ones_ctx *c, uint32_t t, char *scratch, bool &splitters_valid, bool events) {
  EvolveArgs a;
  const ScratchLayout &S = c->L.S;
  auto sc = [&](size_t off) { return scratch + off; };
  // generation 0 fills row_of[cur]; later generations complete the array whose first K entries
  // the last selection wrote
  const int next = t == 0 ? c->cur : c->cur ^ 1;
  a.genes = c->at<int32_t>(c->L.genes);
  a.fit_row = c->at<double>(c->L.fit_row);
  a.parent_row = c->at<uint32_t>(c->L.parent_row[next]);
  a.row_of = c->at<uint32_t>(c->L.row_of[next]);
  a.occupied = c->at<uint32_t>(c->L.occupied[c->cur]);          // set by the last selection
  a.occupied_other = c->at<uint32_t>(c->L.occupied[c->cur ^ 1]);
  // Under probability sampling this generation is scored with its own place of the ring of
  // remaining-work arrays and term tables: a launch of an earlier generation has filled it
  // already, or the draws of this and the next generations are made now.
  const bool sampled = t != 0 && c->sampling;
  const int y_this = sampled ? static_cast<int>(t % kDrawRing) : c->y_cur;
  a.tab = c->table(y_this);
  a.G = c->G; a.P = c->P; a.K = c->K; a.Jp = c->Jp;
  a.key0 = static_cast<uint32_t>(c->cfg.seed);
  a.key1 = static_cast<uint32_t>(c->cfg.seed >> 32);
  a.t = t; a.T_mut = c->T_mut; a.T_x = c->T_x;
  // same table: the survivors are fixed points of the repair.  Under probability sampling their
  // scores still change with every draw of the remaining work, so they are scored again.
  const bool same_table = t != 0 && !c->table_changed;
  a.rescore = same_table && sampled ? 1u : 0u;
  a.new_first = c->new_jobs_first && c->no_schedule ? 1u : 0u;   // the table's "arrived" marks are fresh
  a.per_gpu = c->per_gpu ? 1u : 0u;
  a.stash_stride = 0;                                            // the launcher sets it
  a.fault = c->at<uint32_t>(c->L.fsync) + 2;
  a.slot_score = c->at<double>(c->L.slot_score);
  a.time_rank = c->has_times ? c->at<uint32_t>(c->L.time_rank) : nullptr;
  // quantile buckets: only when the survivors reappear with the scores they had
  const bool buckets = same_table && !sampled && c->bp.nb != 0 && splitters_valid;
  a.bk.nb = buckets ? c->bp.nb : 0;
  a.bk.seg = c->bp.seg;
  a.bk.split = a.bk.split_next = reinterpret_cast<uint64_t *>(sc(S.split));
  a.bk.thresh = a.bk.thresh_next = reinterpret_cast<uint64_t *>(sc(S.thresh));
  a.bk.count = reinterpret_cast<uint32_t *>(sc(S.bcount[c->bucket_phase]));
  a.bk.keys = reinterpret_cast<uint64_t *>(sc(S.bkeys));
  a.bk.idx = reinterpret_cast<uint32_t *>(sc(S.bidx));
  a.bk.spill_keys = reinterpret_cast<uint64_t *>(sc(S.skeys));
  a.bk.spill_idx = reinterpret_cast<uint32_t *>(sc(S.sidx));
  a.bk.spill_bucket = reinterpret_cast<uint32_t *>(sc(S.sbucket));
  a.bk.pool_keys = reinterpret_cast<uint64_t *>(sc(S.pkeys));
  a.bk.pool_idx = reinterpret_cast<uint32_t *>(sc(S.pidx));
  // the selection notes the rows the survivors keep: parents and first K slots of the next pool
  RowPlan rp;
  rp.row_of_cur = a.row_of;
  rp.parent_next = c->at<uint32_t>(c->L.parent_row[next ^ 1]);
  rp.row_of_next = c->at<uint32_t>(c->L.row_of[next ^ 1]);
  rp.occupied = c->at<uint32_t>(c->L.occupied[next]);
  int rc;
  const Progress pr{c->at<double>(c->L.alpha), c->at<double>(c->L.beta), c->at<double>(c->L.processed)};
  if (sampled && !(c->drawn_from <= static_cast<int64_t>(t) && static_cast<int64_t>(t) < c->drawn_to)) {
    const uint32_t count = static_cast<uint32_t>(std::min<int64_t>(kDrawRing, 0x100000000ll - static_cast<int64_t>(t)));
    // places lie at equal distances (make_layout); counted in doubles
    const uint32_t ring_stride = static_cast<uint32_t>((c->L.Y[1] - c->L.Y[0]) / 8);
    HIP_TRY(launch_sample_remaining(pr, c->table(0), ring_stride, c->Jn, c->Jp, a.key0, a.key1, t, count, c->stream));
    c->drawn_from = t;
    c->drawn_to = static_cast<int64_t>(t) + count;
  }
  if (events && (rc = timed(c, c->evolve_ev, c->evolve_used, true))) return rc;
  HIP_TRY(launch_evolve(a, static_cast<int>(c->R), same_table, c->n_cus, c->stream));
  if (events && (rc = timed(c, c->evolve_ev, c->evolve_used, false))) return rc;
  if (events && (rc = timed(c, c->select_ev, c->select_used, true))) return rc;
  if (buckets) {
    HIP_TRY(launch_bucket_select(a.fit_row, a.parent_row, a.bk, rp, c->K,
                                 reinterpret_cast<uint32_t *>(sc(S.bcount[c->bucket_phase ^ 1])),
                                 c->at<int32_t>(c->L.sel), c->stream));
    c->bucket_phase ^= 1;
  } else {
    BucketArgs store = a.bk;                       // same storage; always the first counter set
    store.nb = c->bp.nb;
    store.count = reinterpret_cast<uint32_t *>(sc(S.bcount[0]));
    // the launch scored the whole pool (initial population, refresh under a new table, survivors
    // scored again under a new draw): its scores by slot are complete
    const bool all_scored = t == 0 || !same_table || a.rescore != 0;
    HIP_TRY(launch_select(a.fit_row, all_scored ? a.slot_score : nullptr, rp, c->P, c->K, store,
                          c->at<int32_t>(c->L.sel), c->stream));
    splitters_valid = false;
    if (c->bp.nb != 0 && !sampled && same_table) {
      // Splitters for the bucketed generations that follow; clears both counter sets.  Under sampling
      // no bucketed generation can follow.  Nor after an initial population or a refresh under a new
      // table: the scores of such survivors say little about where their children will fall (nearly
      // all children of a random population beat its best members and would crowd into the first
      // bucket, more than a workgroup sorts in LDS), so the generation after it is ranked in full
      // once more and the buckets start from survivors that the search itself produced.
      HIP_TRY(launch_splitters(a.fit_row, a.row_of, c->at<int32_t>(c->L.sel), c->K, c->bp.nb,
                               reinterpret_cast<uint64_t *>(sc(S.split)), reinterpret_cast<uint64_t *>(sc(S.thresh)),
                               reinterpret_cast<uint32_t *>(sc(S.bcount[0])),
                               reinterpret_cast<uint32_t *>(sc(S.bcount[1])), c->stream));
      splitters_valid = true;
    }
  }
  if (events && (rc = timed(c, c->select_ev, c->select_used, false))) return rc;
  c->cur = next;
  c->y_cur = y_this;
  c->table_changed = false;
  c->no_schedule = false;
  c->profile_tick += 1;
  return ONES_OK;
}

}  // namespace

extern "C" {

int32_t ones_padded_jobs(int32_t n_slots) {
  const int32_t n = n_slots < 1 ? 1 : n_slots;
  return kLanes * ((n + kLanes - 1) / kLanes);
}

size_t ones_workspace_bytes(const ones_config *cfg) {
  if (check_config(cfg) != ONES_OK) return 0;
  return make_layout(static_cast<uint32_t>(cfg->population), static_cast<uint32_t>(ones_padded_jobs(cfg->n_slots)),
                     static_cast<uint32_t>(cfg->n_gpus)).total;
}

static int init_impl(ones_ctx **out, const ones_config *cfg, const ones_jobs *jobs, void *d_workspace,
                     size_t workspace_bytes, void *hip_stream) {
  if (!out) return ONES_E_INVALID_ARG;
  int rc = check_config(cfg);
  if (rc) return rc;
  const int Jp = ones_padded_jobs(cfg->n_slots);
  HostJobs h;
  if ((rc = stage_jobs(cfg->n_slots, Jp, jobs, h))) return rc;
  const Layout L = make_layout(static_cast<uint32_t>(cfg->population), static_cast<uint32_t>(Jp),
                               static_cast<uint32_t>(cfg->n_gpus));
  if (!d_workspace) return ONES_E_INVALID_ARG;
  if (workspace_bytes < L.total || (reinterpret_cast<uintptr_t>(d_workspace) & 255u) != 0)
    return ONES_E_WORKSPACE_TOO_SMALL;
  std::unique_ptr<ones_ctx, void (*)(ones_ctx *)> owner(new ones_ctx(), ones_destroy);   // freed on every way out but the last
  ones_ctx *c = owner.get();
  c->cfg = *cfg;
  c->P = static_cast<uint32_t>(cfg->population); c->K = c->P / 4;
  c->Jn = static_cast<uint32_t>(cfg->n_slots); c->Jp = static_cast<uint32_t>(Jp); c->R = c->Jp / kLanes;
  c->G = static_cast<uint32_t>(cfg->n_gpus);
  c->T_mut = rate_threshold(cfg->mutation_rate);
  c->T_x = rate_threshold(cfg->crossover_rate);
  c->stream = static_cast<hipStream_t>(hip_stream);
  c->ws = static_cast<char *>(d_workspace);
  c->L = L;
  c->stage = nullptr;
  c->stage_dev = nullptr;
  {
    void *pinned = nullptr;
    HIP_TRY(hipHostMalloc(&pinned, stage_bytes(L, static_cast<uint32_t>(Jp), static_cast<uint32_t>(cfg->n_gpus)),
                          hipHostMallocDefault));
    c->stage = static_cast<char *>(pinned);
    void *mapped = nullptr;
    HIP_TRY(hipHostGetDevicePointer(&mapped, pinned, 0));
    c->stage_dev = static_cast<char *>(mapped);
  }
  c->cur = 0; c->t = 0;
  c->table_changed = false;
  c->no_schedule = false;
  c->new_jobs_first = false;
  c->sampling = false;
  c->y_cur = 0;
  c->drawn_from = c->drawn_to = 0;
  c->has_times = false;
  c->per_gpu = false;
  c->bp = bucket_plan(c->P);
  c->bucket_phase = 0;
  c->splitters_valid = false;
  c->poisoned = false;
  c->fused = false;
  c->fused_generations = 0;
  c->fused_changes = 0;
  c->fused_draws = 0;
  c->spin_limit = 1u << 22;   // a few seconds of polling
  c->ids = h.id;
  {
    int dev = 0;
    hipDeviceProp_t prop;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDeviceProperties");
    c->n_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    c->device = dev;
    c->static_scratch = nullptr;
    if ((rc = static_scratch_of(dev, &c->static_scratch))) return rc;
    // the single-launch path needs a launch whose workgroups are all resident at once
    c->fused = fused_pool(c->P, c->Jp) && prop.cooperativeLaunch != 0 &&
               fused_grid_limit(c->P) <= static_cast<uint32_t>(c->n_cus);
  }
  c->profiling = false; c->profile_every = 1; c->profile_tick = 0; c->evolve_used = c->select_used = 0;
  {
    const uint32_t words = (c->P + c->K + 31) / 32;
    hipError_t e = launch_zero_words(c->at<uint32_t>(c->L.occupied[0]), words, c->stream);
    if (e == hipSuccess) e = launch_zero_words(c->at<uint32_t>(c->L.occupied[1]), words, c->stream);
    if (e == hipSuccess) e = launch_zero_words(c->at<uint32_t>(c->L.fsync), 64, c->stream);
    if (e == hipSuccess && fused_pool(c->P, c->Jp))   // the exchange buffers of the single-launch path: every tag starts at 0
      e = launch_zero_words(c->at<uint32_t>(c->L.xkeys), static_cast<uint32_t>(fused_exchange_bytes(c->P) / 4), c->stream);
    if (e != hipSuccess) return hip_fail(e, "launch_zero_words");
  }
  if ((rc = upload_table(c, h, nullptr)) ||
      (rc = run_generation(c, 0, c->ws + c->L.scratch, c->splitters_valid, false)))
    return rc;
  hipError_t e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
  *out = owner.release();
  return ONES_OK;
}

static int set_jobs_impl(ones_ctx *c, const ones_jobs *jobs) {
  if (!c) return ONES_E_INVALID_ARG;
  HostJobs h;
  int rc = stage_jobs(static_cast<int>(c->Jn), static_cast<int>(c->Jp), jobs, h);
  if (rc) return rc;
  std::vector<uint32_t> changed;                                  // the slots that changed hands
  for (uint32_t j = 0; j < c->Jn; ++j)
    if (h.id[j] != c->ids[j]) {
      changed.push_back(j);
      if ((h.rawinfo[j] >> 15) & 1u) h.rawinfo[j] |= 1u << 16;   // an active job arrived in this slot
    }
  if ((rc = upload_table(c, h, changed.empty() ? nullptr : &changed))) return rc;
  c->ids = h.id;
  c->table_changed = true;
  c->no_schedule = true;
  c->drawn_from = c->drawn_to = 0;   // the draws made ahead built their term tables from the old job table
  return ONES_OK;
}

static int set_progress_impl(ones_ctx *c, const double *alpha, const double *beta, const double *processed) {
  if (!c) return ONES_E_INVALID_ARG;
  if (!alpha && !beta && !processed) {
    if (c->sampling) {
      // back to the table's remaining work (still staged on the device); every score is stale
      HIP_TRY(hipMemcpyAsync(c->ws + c->L.Y[c->y_cur], c->ws + c->L.rY, static_cast<size_t>(c->Jp) * 8,
                             hipMemcpyDeviceToDevice, c->stream));
      HIP_TRY(launch_build_terms(c->table(), c->Jp, c->stream));
      HIP_TRY(hipStreamSynchronize(c->stream));
      c->sampling = false;
      c->drawn_from = c->drawn_to = 0;
      c->table_changed = true;
    }
    return ONES_OK;
  }
  if (!alpha || !beta || !processed) return ONES_E_INVALID_ARG;
  for (uint32_t j = 0; j < c->Jn; ++j) {
    if (!std::isfinite(alpha[j]) || !std::isfinite(beta[j]) || !std::isfinite(processed[j])) return ONES_E_NONFINITE;
    if (alpha[j] < 1.0 || beta[j] < 1.0 || processed[j] < 0.0) return ONES_E_INVALID_ARG;
    if (alpha[j] > ONES_MAX_PARAM || beta[j] > ONES_MAX_PARAM || processed[j] > ONES_MAX_PARAM) return ONES_E_BOUNDS;
  }
  const Layout &L = c->L;
  auto staged = [&](size_t off) { return reinterpret_cast<double *>(c->stage + (off - L.alpha)); };
  double *ha = staged(L.alpha), *hb = staged(L.beta), *hp = staged(L.processed);   // laid out as in the workspace
  for (uint32_t j = 0; j < c->Jp; ++j) {
    const bool real = j < c->Jn;
    ha[j] = real ? alpha[j] : 1.0; hb[j] = real ? beta[j] : 1.0; hp[j] = real ? processed[j] : 0.0;
  }
  HIP_TRY(hipMemcpyAsync(c->ws + L.alpha, c->stage, L.processed + static_cast<size_t>(c->Jp) * 8 - L.alpha,
                         hipMemcpyHostToDevice, c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));     // the staging buffer is free again
  c->sampling = true;
  c->drawn_from = c->drawn_to = 0;   // the draws made ahead used the old parameters
  return ONES_OK;
}

static int set_new_jobs_first_impl(ones_ctx *c, int32_t on) {
  if (!c) return ONES_E_INVALID_ARG;
  c->new_jobs_first = on != 0;
  return ONES_OK;
}

static int set_crossover_impl(ones_ctx *c, int32_t mode) {
  if (!c || (mode != ONES_CROSSOVER_JOBS && mode != ONES_CROSSOVER_GPUS)) return ONES_E_INVALID_ARG;
  if (mode == ONES_CROSSOVER_GPUS && c->G > static_cast<uint32_t>(kMaxCoinGpus)) return ONES_E_BOUNDS;
  c->per_gpu = mode == ONES_CROSSOVER_GPUS;
  return ONES_OK;
}

static int set_processed_time_impl(ones_ctx *c, const double *t_processed) {
  if (!c) return ONES_E_INVALID_ARG;
  if (!t_processed) { c->has_times = false; return ONES_OK; }
  for (uint32_t j = 0; j < c->Jn; ++j) {
    int rc = check_param(t_processed[j]);
    if (rc) return rc;
  }
  // position of every slot in ascending (time, slot) order; the padding slots count as time 0
  std::vector<uint32_t> order(c->Jp);
  uint32_t *rank = reinterpret_cast<uint32_t *>(c->stage);
  for (uint32_t j = 0; j < c->Jp; ++j) order[j] = j;
  auto time_of = [&](uint32_t j) { return j < c->Jn ? t_processed[j] : 0.0; };
  std::stable_sort(order.begin(), order.end(), [&](uint32_t x, uint32_t y) { return time_of(x) < time_of(y); });
  for (uint32_t pos = 0; pos < c->Jp; ++pos) rank[order[pos]] = pos;
  HIP_TRY(hipMemcpyAsync(c->ws + c->L.time_rank, rank, static_cast<size_t>(c->Jp) * 4, hipMemcpyHostToDevice,
                         c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));     // the staging buffer is free again
  c->has_times = true;
  return ONES_OK;
}

static int export_remaining_impl(ones_ctx *c, double *remaining_out) {
  if (!c || !remaining_out) return ONES_E_INVALID_ARG;
  HIP_TRY(hipStreamSynchronize(c->stream));
  if (c->Jn) HIP_TRY(hipMemcpy(remaining_out, c->ws + c->L.Y[c->y_cur], static_cast<size_t>(c->Jn) * 8, hipMemcpyDeviceToHost));
  return ONES_OK;
}

// All n generations in one cooperative launch (small pools).
static int run_fused(ones_ctx *c, uint32_t n, bool events) {
  FusedArgs fa;
  EvolveArgs &a = fa.ev;
  a.genes = c->at<int32_t>(c->L.genes);
  a.fit_row = c->at<double>(c->L.fit_row);
  a.parent_row = nullptr; a.row_of = nullptr; a.occupied = nullptr; a.occupied_other = nullptr;
  a.slot_score = nullptr;                              // no selection kernel follows
  a.tab = c->table();
  a.G = c->G; a.P = c->P; a.K = c->K; a.Jp = c->Jp;
  a.key0 = static_cast<uint32_t>(c->cfg.seed);
  a.key1 = static_cast<uint32_t>(c->cfg.seed >> 32);
  a.t = static_cast<uint32_t>(c->t);
  a.T_mut = c->T_mut; a.T_x = c->T_x;
  a.new_first = c->new_jobs_first && c->no_schedule ? 1u : 0u;
  a.time_rank = c->has_times ? c->at<uint32_t>(c->L.time_rank) : nullptr;
  a.rescore = 0;
  a.per_gpu = c->per_gpu ? 1u : 0u;
  a.stash_stride = 0; a.term_lds = 0;
  a.fault = c->at<uint32_t>(c->L.fsync) + 2;
  a.bk = BucketArgs{};
  const int next = c->cur ^ 1;
  fa.parent_rows = c->at<uint32_t>(c->L.parent_row[next]);
  fa.row_of_next = c->at<uint32_t>(c->L.row_of[next]);
  fa.row_of_cur = c->at<uint32_t>(c->L.row_of[c->cur]);
  fa.occupied = c->at<uint32_t>(c->L.occupied[c->cur]);
  fa.sel = c->at<int32_t>(c->L.sel);
  fa.xkeys = c->at<uint64_t>(c->L.xkeys);
  fa.xsurv = fa.xkeys + static_cast<size_t>(2) * c->P;
  fa.xrank = fa.xsurv + static_cast<size_t>(2) * c->K;
  fa.xdraw = fa.xrank + c->P;
  fa.draws_before = c->fused_draws;
  fa.sampled = c->sampling ? 1u : 0u;
  fa.pr = Progress{c->at<double>(c->L.alpha), c->at<double>(c->L.beta), c->at<double>(c->L.processed)};
  fa.n_slots = c->Jn;
  fa.y_out = c->at<double>(c->L.Y[c->y_cur]);      // what ones_export_remaining reads
  fa.sync = c->at<uint32_t>(c->L.fsync);
  fa.generations_before = c->fused_generations;
  fa.changes_before = c->fused_changes;
  fa.n_generations = n;
  fa.first_changed = c->table_changed ? 1u : 0u;
  fa.spin_limit = c->spin_limit;
  int rc;
  if (events && (rc = timed(c, c->evolve_ev, c->evolve_used, true))) return rc;
  HIP_TRY(launch_fused(fa, c->stream));
  if (events && (rc = timed(c, c->evolve_ev, c->evolve_used, false))) return rc;
  c->fused_generations += n;
  c->fused_changes += c->sampling ? n : fa.first_changed;
  if (c->sampling) {
    c->fused_draws += n;
    c->drawn_from = c->drawn_to = 0;   // the ring may hold tables this launch wrote over (y_out); the two-launch path draws again
  }
  c->table_changed = false;
  c->no_schedule = false;
  c->splitters_valid = false;       // the two-launch path ranks the pool in full before it uses buckets again
  c->profile_tick += 1;
  return ONES_OK;
}

static int poisoned_error() {
  snprintf(g_hip_msg, sizeof(g_hip_msg), "an earlier launch failed in the middle of a generation; destroy the context");
  return ONES_E_HIP;
}

static int generation_impl(ones_ctx *c, int32_t n_generations, bool in_static_scratch) {
  if (!c || n_generations < 0) return ONES_E_INVALID_ARG;
  if (c->t + n_generations > 0xFFFFFFFFll) return ONES_E_INVALID_ARG;
  if (c->poisoned) return poisoned_error();
  char *block = c->ws + c->L.scratch;
  bool static_valid = false;      // the static array holds whatever the last call on this GPU left
  if (in_static_scratch) {
    if (c->L.S.total > ONES_STATIC_SCRATCH_BYTES) return ONES_E_STATIC_LIMIT;
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev != c->device) return ONES_E_INVALID_ARG;
    block = c->static_scratch;
    if (n_generations > 0) c->splitters_valid = false;   // the workspace's splitters fall behind
  }
  if (c->fused && n_generations >= kFusedMinGenerations) {
    // uses no scratch at all: every workgroup ranks the pool in its LDS
    int rc = run_fused(c, static_cast<uint32_t>(n_generations), !in_static_scratch);
    if (rc) { c->poisoned = true; return rc; }
    c->t += n_generations;
    return ONES_OK;
  }
  for (int32_t i = 0; i < n_generations; ++i) {
    int rc = run_generation(c, static_cast<uint32_t>(c->t + 1), block,
                            in_static_scratch ? static_valid : c->splitters_valid, !in_static_scratch);
    if (rc) { c->poisoned = true; return rc; }
    c->t += 1;
  }
  return ONES_OK;
}

// A device-wide wait of a single-launch generation gave up (it never does on a healthy device):
// the population is inconsistent from then on.
static int wait_gave_up(ones_ctx *c) {
  c->poisoned = true;
  snprintf(g_hip_msg, sizeof(g_hip_msg), "a device-wide wait inside the generation kernel gave up; destroy the context");
  return ONES_E_HIP;
}

// A kernel had to pull a row index back into the genome array: the row bookkeeping is wrong
// (a defect of the library, never of the caller's input).
static int row_fault(ones_ctx *c) {
  c->poisoned = true;
  snprintf(g_hip_msg, sizeof(g_hip_msg), "internal error: a genome row index was out of range; destroy the context");
  return ONES_E_HIP;
}

// For the calls that synchronise without reading the winner: fetches the error words the
// kernels leave (a wait of a single-launch generation gave up; a row index was out of range).
// The stream must be idle.
static int check_waits(ones_ctx *c) {
  if (c->poisoned) return poisoned_error();
  uint32_t words[2] = {0, 0};
  HIP_TRY(hipMemcpy(words, c->ws + c->L.fsync + 4, 8, hipMemcpyDeviceToHost));
  if (words[0]) return wait_gave_up(c);
  return words[1] ? row_fault(c) : ONES_OK;
}

static int best_impl(ones_ctx *c, int32_t *batch_out, int32_t *gpus_out, double *fitness_out) {
  if (!c) return ONES_E_INVALID_ARG;
  if (c->poisoned) return poisoned_error();
  // The kernel writes the winner and the two error words straight into the pinned host buffer
  // (a few hundred bytes to a few kilobytes), laid out as the best_* block of the workspace:
  // one launch and one wait, no copy.
  const Layout &L = c->L;
  auto mapped = [&](size_t off) { return c->stage_dev + (off - L.best_batch); };
  HIP_TRY(launch_best(c->at<int32_t>(c->L.genes), c->at<double>(c->L.fit_row), c->at<uint32_t>(c->L.row_of[c->cur]),
                      c->at<int32_t>(c->L.sel), c->at<uint32_t>(c->L.info), c->Jn, c->Jp,
                      reinterpret_cast<int32_t *>(mapped(L.best_batch)), reinterpret_cast<int32_t *>(mapped(L.best_gpus)),
                      reinterpret_cast<double *>(mapped(L.best_fit)), c->at<uint32_t>(c->L.fsync) + 1,
                      reinterpret_cast<uint32_t *>(mapped(L.best_err)), c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));
  auto staged = [&](size_t off) { return c->stage + (off - L.best_batch); };   // laid out as in the workspace
  uint32_t words[2] = {0, 0};
  memcpy(words, staged(L.best_err), 8);
  if (words[0]) return wait_gave_up(c);
  if (words[1]) return row_fault(c);
  if (batch_out && c->Jn) memcpy(batch_out, staged(L.best_batch), c->Jn * 4);
  if (gpus_out && c->Jn) memcpy(gpus_out, staged(L.best_gpus), c->Jn * 4);
  if (fitness_out) memcpy(fitness_out, staged(L.best_fit), 8);
  return ONES_OK;
}

static int placement_impl(ones_ctx *c, int32_t *slot_of_gpu, int32_t *batch_of_gpu) {
  if (!c || c->no_schedule) return ONES_E_INVALID_ARG;
  if (c->poisoned) return poisoned_error();
  const size_t n4 = static_cast<size_t>(c->G) * 4;
  HIP_TRY(launch_placement(c->at<int32_t>(c->L.genes), c->at<uint32_t>(c->L.row_of[c->cur]), c->at<int32_t>(c->L.sel),
                           c->at<uint32_t>(c->L.info), c->Jn, c->Jp, c->G, c->at<int32_t>(c->L.place_slot),
                           c->at<int32_t>(c->L.place_batch), c->stream));
  const Layout &L = c->L;
  if (c->G)
    HIP_TRY(hipMemcpyAsync(c->stage, c->ws + L.place_slot, L.place_batch + n4 - L.place_slot, hipMemcpyDeviceToHost,
                           c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));
  if (int rc = check_waits(c)) return rc;
  auto staged = [&](size_t off) { return c->stage + (off - L.place_slot); };   // laid out as in the workspace
  if (slot_of_gpu && c->G) memcpy(slot_of_gpu, staged(L.place_slot), n4);
  if (batch_of_gpu && c->G) memcpy(batch_of_gpu, staged(L.place_batch), n4);
  return ONES_OK;
}

static int export_impl(ones_ctx *c, int32_t *genes, double *fit, int32_t *sel, int64_t *generation) {
  if (!c) return ONES_E_INVALID_ARG;
  HIP_TRY(hipStreamSynchronize(c->stream));
  if (int rc = check_waits(c)) return rc;
  // candidates live in physical rows: fetch the rows and put them in slot order on the host
  const size_t rows = static_cast<size_t>(c->P) + c->K, Jp = c->Jp;
  std::vector<uint32_t> row_of(c->P);
  std::vector<int32_t> g;
  std::vector<double> f;
  HIP_TRY(hipMemcpy(row_of.data(), c->ws + c->L.row_of[c->cur], static_cast<size_t>(c->P) * 4, hipMemcpyDeviceToHost));
  if (genes) {
    g.resize(rows * Jp);
    HIP_TRY(hipMemcpy(g.data(), c->ws + c->L.genes, rows * Jp * 4, hipMemcpyDeviceToHost));
  }
  if (fit) {
    f.resize(rows);
    HIP_TRY(hipMemcpy(f.data(), c->ws + c->L.fit_row, rows * 8, hipMemcpyDeviceToHost));
  }
  if (sel) HIP_TRY(hipMemcpy(sel, c->ws + c->L.sel, static_cast<size_t>(c->K) * 4, hipMemcpyDeviceToHost));
  for (uint32_t p = 0; p < c->P; ++p) {
    if (genes) memcpy(genes + static_cast<size_t>(p) * Jp, g.data() + static_cast<size_t>(row_of[p]) * Jp, Jp * 4);
    if (fit) fit[p] = f[row_of[p]];
  }
  if (generation) *generation = c->t;
  return ONES_OK;
}

static int profile_enable_impl(ones_ctx *c, int32_t on) {
  if (!c) return ONES_E_INVALID_ARG;
  HIP_TRY(hipStreamSynchronize(c->stream));
  c->profiling = on > 0;
  c->profile_every = on > 0 ? on : 1;
  c->profile_tick = 0;
  c->evolve_used = c->select_used = 0;
  return ONES_OK;
}

static int profile_read_impl(ones_ctx *c, double *evolve_ms, int64_t *evolve_launches, double *select_ms,
                      int64_t *select_launches) {
  if (!c) return ONES_E_INVALID_ARG;
  HIP_TRY(hipStreamSynchronize(c->stream));
  double em = 0.0, sm = 0.0;
  for (size_t i = 0; i < c->evolve_used; ++i) {
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, c->evolve_ev[i].start, c->evolve_ev[i].stop));
    em += ms;
  }
  for (size_t i = 0; i < c->select_used; ++i) {
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, c->select_ev[i].start, c->select_ev[i].stop));
    sm += ms;
  }
  if (evolve_ms) *evolve_ms = em;
  if (evolve_launches) *evolve_launches = static_cast<int64_t>(c->evolve_used);
  if (select_ms) *select_ms = sm;
  if (select_launches) *select_launches = static_cast<int64_t>(c->select_used);
  return ONES_OK;
}

static int update_limits_impl(int32_t n_slots, const ones_limit_inputs *in, double sigma, int32_t *limit) {
  if (n_slots < 0 || n_slots > ONES_MAX_SLOTS) return ONES_E_INVALID_ARG;
  if (n_slots > 0 && (!in || !limit || !in->state || !in->bmin || !in->bcap || !in->gpu_max_batch ||
                      !in->last_batch || !in->finished_epoch || !in->elapsed))
    return ONES_E_INVALID_ARG;
  if (!std::isfinite(sigma)) return ONES_E_NONFINITE;
  if (sigma < 0.0) return ONES_E_INVALID_ARG;
  std::vector<int32_t> next(static_cast<size_t>(n_slots), 0);
  for (int32_t j = 0; j < n_slots; ++j) {
    const uint8_t state = in->state[j];
    if (state > 3) return ONES_E_INVALID_ARG;
    if (state == 0) continue;
    if (log2_pow2(in->bmin[j]) < 0 || log2_pow2(in->bcap[j]) < 0 || log2_pow2(in->gpu_max_batch[j]) < 0)
      return ONES_E_NOT_POW2;
    if (in->bmin[j] > in->bcap[j] || in->bcap[j] > (1 << 30)) return ONES_E_BOUNDS;
    int64_t r = limit[j];
    if (state == 1) {                              // Start
      r = in->gpu_max_batch[j];
    } else {
      if (r < 1) return ONES_E_INVALID_ARG;
      if (state == 2) {                            // Resume
        if (in->last_batch[j] < 0) return ONES_E_INVALID_ARG;
        r = in->last_batch[j] > 0 ? std::min<int64_t>(r, in->last_batch[j]) : r / 2;
      } else {                                     // Scale-up with the Scale-down penalty
        const double T = in->elapsed[j];
        if (!std::isfinite(T)) return ONES_E_NONFINITE;
        if (T < 0.0) return ONES_E_INVALID_ARG;
        if (sigma * T > 1e15) return ONES_E_BOUNDS;
        if (in->finished_epoch[j]) {
          const int64_t penalty = static_cast<int64_t>(std::ceil(sigma * T + 1.0));
          r = (2 * r + penalty - 1) / penalty;
        }
      }
    }
    r = std::min<int64_t>(std::max<int64_t>(r, in->bmin[j]), in->bcap[j]);
    next[j] = 1 << (63 - __builtin_clzll(static_cast<unsigned long long>(r)));   // largest power of two <= r
  }
  if (n_slots) memcpy(limit, next.data(), static_cast<size_t>(n_slots) * 4);
  return ONES_OK;
}

// The entry points proper: nothing is thrown across the C boundary (the staging vectors may run out of host
// memory).

int ones_init(ones_ctx **out, const ones_config *cfg, const ones_jobs *jobs, void *d_workspace, size_t workspace_bytes, void *hip_stream) {
  return guarded([&] { return init_impl(out, cfg, jobs, d_workspace, workspace_bytes, hip_stream); });
}

int ones_set_jobs(ones_ctx *c, const ones_jobs *jobs) {
  return guarded([&] { return set_jobs_impl(c, jobs); });
}

int ones_set_crossover(ones_ctx *c, int32_t mode) {
  return guarded([&] { return set_crossover_impl(c, mode); });
}

int ones_set_processed_time(ones_ctx *c, const double *t_processed) {
  return guarded([&] { return set_processed_time_impl(c, t_processed); });
}

int ones_set_progress(ones_ctx *c, const double *alpha, const double *beta, const double *processed) {
  return guarded([&] { return set_progress_impl(c, alpha, beta, processed); });
}

int ones_set_new_jobs_first(ones_ctx *c, int32_t on) {
  return guarded([&] { return set_new_jobs_first_impl(c, on); });
}

int ones_export_remaining(ones_ctx *c, double *remaining_out) {
  return guarded([&] { return export_remaining_impl(c, remaining_out); });
}

int ones_generation(ones_ctx *c, int32_t n_generations) {
  return guarded([&] { return generation_impl(c, n_generations, false); });
}

int ones_set_wait_limit(ones_ctx *c, uint32_t polls) {
  if (!c) return ONES_E_INVALID_ARG;
  c->spin_limit = polls;
  return ONES_OK;
}

int ones_generation_static(ones_ctx *c, int32_t n_generations) {
  return guarded([&] { return generation_impl(c, n_generations, true); });
}

int ones_best(ones_ctx *c, int32_t *batch_out, int32_t *gpus_out, double *fitness_out) {
  return guarded([&] { return best_impl(c, batch_out, gpus_out, fitness_out); });
}

int ones_placement(ones_ctx *c, int32_t *slot_of_gpu, int32_t *batch_of_gpu) {
  return guarded([&] { return placement_impl(c, slot_of_gpu, batch_of_gpu); });
}

int ones_export(ones_ctx *c, int32_t *genes, double *fit, int32_t *sel, int64_t *generation) {
  return guarded([&] { return export_impl(c, genes, fit, sel, generation); });
}

int ones_profile_enable(ones_ctx *c, int32_t on) {
  return guarded([&] { return profile_enable_impl(c, on); });
}

int ones_profile_read(ones_ctx *c, double *evolve_ms, int64_t *evolve_launches, double *select_ms, int64_t *select_launches) {
  return guarded([&] { return profile_read_impl(c, evolve_ms, evolve_launches, select_ms, select_launches); });
}

int ones_update_limits(int32_t n_slots, const ones_limit_inputs *in, double sigma, int32_t *limit) {
  return guarded([&] { return update_limits_impl(n_slots, in, sigma, limit); });
}

void ones_destroy(ones_ctx *c) {
  if (!c) return;
  for (auto &e : c->evolve_ev) { (void)hipEventDestroy(e.start); (void)hipEventDestroy(e.stop); }
  for (auto &e : c->select_ev) { (void)hipEventDestroy(e.start); (void)hipEventDestroy(e.stop); }
  if (c->stage) (void)hipHostFree(c->stage);
  delete c;
}

const char *ones_strerror(int code) {
  switch (code) {
    case ONES_OK: return "ok";
    case ONES_E_INVALID_ARG: return "invalid argument";
    case ONES_E_NOT_POW2: return "bmin, bmax and gpu_max_batch of an active slot must be powers of two";
    case ONES_E_BOUNDS: return "batch window or model parameter out of bounds";
    case ONES_E_NONFINITE: return "NaN or infinity in a job parameter";
    case ONES_E_WORKSPACE_TOO_SMALL: return "workspace too small or not 256-byte aligned";
    case ONES_E_HIP: return g_hip_msg;
    case ONES_E_STATIC_LIMIT: return "population too large for the static scratch of ones_generation_static";
    default: return "unknown error code";
  }
}

}  // extern "C"

