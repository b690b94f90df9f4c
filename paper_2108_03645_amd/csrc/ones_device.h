// Internal interface between the host side of libones (ones_api.hip) and its kernels
// (ones_evolve.hip, ones_select.hip, ones_sample.hip).  Not installed; the public boundary is include/ones.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ones {

constexpr int kLanes = 64;          // one candidate schedule per wave64, job columns across lanes
constexpr int kMaxRows = 32;        // 2048 job slots / 64 columns
constexpr int kMaxTermEntries = 22; // waiting + GPU counts 2^0 .. 2^20
constexpr int kMaxCoinGpus = 8192;  // crossover over the GPUs: one Philox block of 128 coins per lane
#ifndef ONES_SORT_CHUNK
#define ONES_SORT_CHUNK 4096
#endif
constexpr int kSortChunk = ONES_SORT_CHUNK;   // largest pool that one workgroup sorts in LDS

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11).
struct Words { uint32_t w[4]; };

__device__ __forceinline__ Words philox4x32_10(uint32_t x0, uint32_t x1, uint32_t x2, uint32_t x3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint64_t pa = static_cast<uint64_t>(x0) * 0xD2511F53ull;
    const uint64_t pb = static_cast<uint64_t>(x2) * 0xCD9E8D57ull;
    // three-input xor in one instruction (truth table 0x96)
    const uint32_t n0 = __builtin_amdgcn_bitop3_b32(static_cast<uint32_t>(pb >> 32), x1, k0, 0x96);
    const uint32_t n2 = __builtin_amdgcn_bitop3_b32(static_cast<uint32_t>(pa >> 32), x3, k1, 0x96);
    x1 = static_cast<uint32_t>(pb);
    x3 = static_cast<uint32_t>(pa);
    x0 = n0;
    x2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Words{{x0, x1, x2, x3}};
}

// Per-slot constants derived from the job table, structure of arrays over the padded
// slots (column = slot mod 64, row = slot div 64).  A gene is handled on the device as
// the job's GPU count c (0 = waiting): after the free lift to the per-GPU max batch the
// global batch is B = c << bl_exp, so c in {0} U {cstart, 2 cstart, .., cmax} says it all.
struct JobTable {
  uint32_t *cstart;   // GPU count a waiting job resumes with; 0 for an empty slot
  uint32_t *cmax;     // GPU count at the batch-size limit R_j;  0 for an empty slot
  uint32_t *info;     // bits 0-4 lo, 5-10 (hi-lo+2), 11-15 mu, 16-20 bl_exp, 21 active, 22 arrived with this table
  double   *abl;      // a * 2^bl_exp: compute time of one iteration at the local batch
  double   *cc;       // synchronisation cost per doubling of the GPU count
  double   *d;        // fixed cost per iteration
  double   *Y;        // remaining samples
  // term table: T_j c_j of slot (row, lane) running on 2^(e-1) GPUs at [(row*term_E + e)*64 + lane],
  // e = 0 (waiting, +0.0) .. term_E-1; the value the score formula gives, precomputed per table
  double   *terms;
  uint32_t  term_E;
};

__host__ __device__ inline uint32_t info_lo(uint32_t w)     { return w & 31u; }
__host__ __device__ inline uint32_t info_n(uint32_t w)      { return (w >> 5) & 63u; }
__host__ __device__ inline uint32_t info_mu(uint32_t w)     { return (w >> 11) & 31u; }
__host__ __device__ inline uint32_t info_blexp(uint32_t w)  { return (w >> 16) & 31u; }
__host__ __device__ inline uint32_t info_active(uint32_t w) { return (w >> 21) & 1u; }
__host__ __device__ inline uint32_t info_new(uint32_t w)    { return (w >> 22) & 1u; }

// Quantile buckets of the selection (valid while the job table stays the same): children and
// mutants that beat the K-th survivor are dropped into the bucket of the survivors they fall
// between.  nb == 0 switches the mechanism off.  A bucket stores up to seg offspring; the rare
// surplus goes to one shared spill list, and a bucket too large for LDS is sorted in a slice of
// a shared scratch pool.
constexpr int kMaxBuckets = 1024;
constexpr int kSpillCounter = kMaxBuckets;       // count[kSpillCounter]: records in the spill list
constexpr int kPoolCounter = kMaxBuckets + 1;    // count[kPoolCounter]: scratch pool entries handed out
constexpr int kBucketCounters = kMaxBuckets + 2;
constexpr int kRowGroupWords = 64;               // bitmap words per entry of the free-row index (one per lane)
struct BucketArgs {
  const uint64_t *split;      // [kMaxBuckets] score bits of survivor ranks c*K/nb, c = 1..nb-1, then +inf
  const uint64_t *thresh;     // [1] score bits of the K-th survivor
  uint32_t       *count;      // [kBucketCounters] offspring per bucket (spilled ones included), this generation
  uint64_t       *keys;       // [nb][seg] score bits of the bucket's offspring
  uint32_t       *idx;        // [nb][seg] their pool slots
  uint64_t       *spill_keys; // [P] surplus candidates: score bits, slot, bucket
  uint32_t       *spill_idx;
  uint32_t       *spill_bucket;
  uint64_t       *pool_keys;  // [pool] scratch for buckets that do not fit LDS
  uint32_t       *pool_idx;
  uint64_t       *split_next; // splitters and threshold for the next generation (same arrays)
  uint64_t       *thresh_next;
  uint32_t        nb, seg;
};

// Remaining work of slot j under probability sampling (Alg. 1, Eq. 7) for generation t:
// tab.Y[j] = processed[j] * (1/rho - 1), rho ~ Be(alpha[j], beta[j]), for j < Jn; then the
// slot's entries of the term table.
struct Progress {
  const double *alpha, *beta, *processed;   // [Jp]
};
// The draws depend on nothing but (seed, slot, generation), so they are made ahead, kDrawRing
// generations in one launch: generation g's remaining work and term table sit at place
// g mod kDrawRing of a ring of (Y, terms) pairs.
constexpr int kDrawRing = 8;

// Genomes live in physical rows; a candidate keeps its row for as long as it survives, so a
// survivor is never copied.  The pool of P slots uses P + K rows, K of them held by the
// survivors (the selection marks them in a bitmap).  Of the P free rows in ascending order,
// slot K + q of the new pool takes the q-th; a survivor that must be refreshed after a table
// change (rank p) takes the (3K + p)-th.  The evolve kernel looks its rows up in the bitmap.
struct EvolveArgs {
  int32_t        *genes;      // [P + K][Jp] genome rows (global batch sizes)
  double         *fit_row;    // [P + K] score of the genome in each row
  const uint32_t *parent_row; // [K] rows of the survivors, best first
  uint32_t       *row_of;     // [P] row of every slot of the new pool: entries [0,K) prefilled
                              //     (survivors keep their rows), the others written here
  const uint32_t *occupied;   // bitmap over the P + K rows: the survivors' rows
  uint32_t       *occupied_other;  // the other bitmap, cleared here for the coming selection
  JobTable       tab;
  uint32_t       G, P, K, Jp;
  uint32_t       key0, key1;  // seed
  uint32_t       t;           // generation counter (0 = initial population)
  uint32_t       T_mut, T_x;  // rate thresholds on a 32-bit word
  uint32_t       new_first;   // after a table change: the jobs that arrived with it are served first
  const uint32_t *time_rank;  // [Jp] with new_first: position of every slot in ascending order of executed
                              //      time, the order the other jobs are admitted in; null = visiting order
  uint32_t       rescore;     // the survivors' scores are stale (remaining work redrawn): score them again
  uint32_t       per_gpu;     // the uniform crossover scans the GPUs (Eq. 1) instead of the jobs; needs G <= kMaxCoinGpus
  uint32_t       stash_stride; // set by the launcher: bytes of LDS scratch per wave
  uint32_t       term_lds;    // set by the launcher: entries per job of the term table in LDS, 0 = none
  uint32_t       *fault;      // [1] raised when a row index had to be pulled back into the genome array
  double         *slot_score; // [P] the score of every candidate this launch scores, by pool slot (written when
                              //     the buckets are off): what the general selection reads when the launch scored
                              //     the whole pool, in place of slot -> row -> score
  BucketArgs     bk;
};

// All generations of one ones_generation call in a single launch, for pools that are small
// enough to be ranked inside every workgroup's LDS (one row of 64 job columns, at most
// kFusedMaxPool candidates).  ev describes the problem as for the evolve kernel; of its row
// bookkeeping only genes, fit_row and tab are used, and ev.t is the generation counter BEFORE
// the call (the launch runs generations ev.t + 1 .. ev.t + n_generations).
constexpr uint32_t kFusedMaxPool = 2048;
struct FusedArgs {
  EvolveArgs ev;
  uint32_t *parent_rows;    // [K] in: rows of the survivors, best first; out: of the new survivors
  uint32_t *row_of_next;    // [P] out, entries [0,K): the same rows (the next pool's first K slots)
  uint32_t *row_of_cur;     // [P] out: row of every slot of the last generation's pool
  uint32_t *occupied;       // bitmap over the P + K rows, in: the survivors' rows; out likewise
  int32_t  *sel;            // [K] out: survivor slots of the last generation's pool, best first
  // exchange between the workgroups, zeroed when the context is created, then only written by these launches:
  uint64_t *xkeys;          // [2][P] tagged score bits of the children by pool slot, a buffer per generation parity
  uint64_t *xsurv;          // [2][K] the same for survivors refreshed after a table change
  uint64_t *xrank;          // [P] ranks from a ranking by counting, stamped with the generation
  uint64_t *xdraw;          // [4][64] tagged draws of the remaining work (probability sampling), four generations rotating
  uint32_t *sync;           // [1] set when a poll ran out
  uint32_t generations_before;  // generations these launches have run for the context so far
  uint32_t changes_before;      // ... of them generations that also exchanged the survivors' scores
  uint32_t draws_before;        // ... of them generations with a drawn remaining work
  uint32_t sampled;             // probability sampling (Alg. 1): every generation draws the remaining work anew
  Progress pr;                  // its inputs
  uint32_t n_slots;             // Jn: slots at or beyond it have no remaining work
  double  *y_out;               // [64] out: the remaining work the last generation was scored with
  uint32_t n_generations;   // > 0
  uint32_t first_changed;   // the job table changed since the survivors were scored: the first generation refreshes them
  uint32_t spin_limit;      // polls before a wait gives up (0: gives up at once; for tests of that path)
  uint32_t table_lds;       // set by the launcher: bytes of LDS the staged job table takes
  uint32_t work_groups;     // set by the launcher: workgroups that compute candidates (the grid's first ones)
};
// Workgroups to launch for a pool of P (the launch must be co-resident: cooperative).
uint32_t fused_workgroups(uint32_t P, bool sampled);
uint32_t fused_grid_limit(uint32_t P);      // the largest grid a launch for a pool of P uses
size_t fused_exchange_bytes(uint32_t P);    // xkeys, xsurv and xrank, consecutive
hipError_t launch_fused(const FusedArgs &fa, hipStream_t s);

// What a selection records besides the survivor list: the survivors keep their rows.
struct RowPlan {
  const uint32_t *row_of_cur;   // [P] row of every slot of the pool being ranked
  uint32_t       *parent_next;  // [K] rows of the new survivors, best first
  uint32_t       *row_of_next;  // [P] rows of the next pool; entries [0,K) are written here
  uint32_t       *occupied;     // bitmap over the P + K rows, zero on entry; survivors' rows get set
};

// T_j c_j of a job at GPU-count code e (0 = waiting, e = 1 + log2 of the GPU count): Eq. 3
// with T = Y / X (Eq. 5) and the iteration time a*b + c*log2(g) + d at the job's local batch
// b = 2^blexp; abl = a * b.  Same operations in the same order wherever a term is computed.
__device__ __forceinline__ double term_of(double abl, double cc, double d, double Y, uint32_t blexp, uint32_t e) {
  if (e == 0) return 0.0;
  const double lg = static_cast<double>(e - 1);
  const double inv_bl = __hiloint2double(static_cast<int>((1023u - blexp) << 20), 0);
  const double t = (abl + cc * lg) + d;
  return (Y * t) * inv_bl;
}

struct RawJobs {              // uploaded by the host after validation, [Jp] each
  const uint32_t *rawinfo;    // bits 0-4 lo, 5-9 hi, 10-14 mu, 15 active, 16 arrived with this table
  const double   *a, *c, *d, *Y;
};

// launchers (each returns the hipGetLastError of its launch)
// The per-slot values and the term table from the raw table, and the n_changed slots (may be 0)
// that changed hands set to "waiting" in every one of the genome rows; one launch.
hipError_t launch_table_change(const RawJobs &raw, const JobTable &tab, uint32_t Jp, int32_t *genes, const uint32_t *slots,
                               uint32_t n_changed, uint32_t rows, hipStream_t s);
hipError_t launch_build_terms(const JobTable &tab, uint32_t Jp, hipStream_t s);
// ring: the job table with Y and terms pointing at place 0 of the ring, whose places lie
// ring_stride doubles apart; draws generations t .. t + count - 1 (count <= kDrawRing).
hipError_t launch_sample_remaining(const Progress &pr, const JobTable &ring, uint32_t ring_stride, uint32_t Jn,
                                   uint32_t Jp, uint32_t key0, uint32_t key1, uint32_t t, uint32_t count,
                                   hipStream_t s);
// same_table: the job table is the one the previous generation was repaired and scored with
hipError_t launch_evolve_group0(const EvolveArgs &a, int rows, bool same_table, int n_cus, hipStream_t s);
hipError_t launch_evolve_group1(const EvolveArgs &a, int rows, bool same_table, int n_cus, hipStream_t s);
hipError_t launch_evolve_group2(const EvolveArgs &a, int rows, bool same_table, int n_cus, hipStream_t s);
hipError_t launch_evolve_group3(const EvolveArgs &a, int rows, bool same_table, int n_cus, hipStream_t s);
inline hipError_t launch_evolve(const EvolveArgs &a, int rows, bool same_table, int n_cus, hipStream_t s) {
  switch ((rows - 1) / 8) {
    case 0: return launch_evolve_group0(a, rows, same_table, n_cus, s);
    case 1: return launch_evolve_group1(a, rows, same_table, n_cus, s);
    case 2: return launch_evolve_group2(a, rows, same_table, n_cus, s);
    case 3: return launch_evolve_group3(a, rows, same_table, n_cus, s);
    default: return hipErrorInvalidValue;
  }
}
// General selection (any scores).  store: the bucket storage (count, keys, idx, spill and pool
// arrays, split as scratch for the splitters, nb * seg entries of bucket space); used by pools
// too large for the single launch that ranks a whole pool.  slot_score: the pool's scores by slot
// when the evolve launch wrote them all, else null (they are then looked up through the rows).
hipError_t launch_select(const double *fit_row, const double *slot_score, const RowPlan &rp, uint32_t P, uint32_t K,
                         const BucketArgs &store, int32_t *sel, hipStream_t s);
hipError_t launch_zero_words(uint32_t *words, uint32_t n, hipStream_t s);
hipError_t launch_bucket_select(const double *fit_row, const uint32_t *parent_row, const BucketArgs &bk,
                                const RowPlan &rp, uint32_t K, uint32_t *count_next, int32_t *sel, hipStream_t s);
hipError_t launch_splitters(const double *fit_row, const uint32_t *row_of, const int32_t *sel, uint32_t K,
                            uint32_t nb, uint64_t *split, uint64_t *thresh, uint32_t *count0, uint32_t *count1,
                            hipStream_t s);
// Eq. 1 for the winner: GPU i runs slot slot_of_gpu[i] (-1 = idle) with batch_of_gpu[i] samples;
// jobs in slot order on consecutive GPUs.  G entries each.
hipError_t launch_placement(const int32_t *genes, const uint32_t *row_of, const int32_t *sel, const uint32_t *info,
                            uint32_t Jn, uint32_t Jp, uint32_t G, int32_t *slot_of_gpu, int32_t *batch_of_gpu,
                            hipStream_t s);
hipError_t launch_best(const int32_t *genes, const double *fit_row, const uint32_t *row_of, const int32_t *sel,
                       const uint32_t *info,
                       uint32_t Jn, uint32_t Jp, int32_t *batch_out, int32_t *gpus_out, double *fit_out,
                       const uint32_t *err_in, uint32_t *err_out, hipStream_t s);

}  // namespace ones
