// Internal interface between the host side of libones (ones_api.hip) and its kernels
// (ones_evolve.hip, ones_select.hip).  Not installed; the public boundary is include/ones.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ones {

constexpr int kLanes = 64;          // one candidate schedule per wave64, job columns across lanes
constexpr int kMaxRows = 32;        // 2048 job slots / 64 columns
constexpr int kSortChunk = 4096;    // keys sorted per workgroup in LDS

// Per-slot constants derived from the job table, structure of arrays over the padded
// slots (column = slot mod 64, row = slot div 64).  A gene is handled on the device as
// the job's GPU count c (0 = waiting): after the free lift to the per-GPU max batch the
// global batch is B = c << bl_exp, so c in {0} U {cstart, 2 cstart, .., cmax} says it all.
struct JobTable {
  uint32_t *cstart;   // GPU count a waiting job resumes with; 0 for an empty slot
  uint32_t *cmax;     // GPU count at the batch-size limit R_j;  0 for an empty slot
  uint32_t *info;     // bits 0-4 lo, 5-10 (hi-lo+2), 11-15 mu, 16-20 bl_exp, 21 active
  double   *abl;      // a * 2^bl_exp: compute time of one iteration at the local batch
  double   *cc;       // synchronisation cost per doubling of the GPU count
  double   *d;        // fixed cost per iteration
  double   *Y;        // remaining samples
};

__host__ __device__ inline uint32_t info_lo(uint32_t w)     { return w & 31u; }
__host__ __device__ inline uint32_t info_n(uint32_t w)      { return (w >> 5) & 63u; }
__host__ __device__ inline uint32_t info_mu(uint32_t w)     { return (w >> 11) & 31u; }
__host__ __device__ inline uint32_t info_blexp(uint32_t w)  { return (w >> 16) & 31u; }
__host__ __device__ inline uint32_t info_active(uint32_t w) { return (w >> 21) & 1u; }

struct EvolveArgs {
  const int32_t *genes_old;   // [P][Jp] previous generation (unused by the initial population)
  int32_t       *genes_new;   // [P][Jp]
  const int32_t *sel;         // [K] survivors of the previous generation, best first
  double        *fit;         // [P] scores of the new generation
  const double  *fit_old;     // [P] scores of the previous generation
  JobTable       tab;
  uint32_t       G, P, K, Jp;
  uint32_t       key0, key1;  // seed
  uint32_t       t;           // generation counter (0 = initial population)
  uint32_t       T_mut, T_x;  // rate thresholds on a 32-bit word
};

struct RawJobs {              // uploaded by the host after validation, [Jp] each
  const uint32_t *rawinfo;    // bits 0-4 lo, 5-9 hi, 10-14 mu, 15 active
  const double   *a, *c, *d, *Y;
};

// launchers (each returns the hipGetLastError of its launch)
hipError_t launch_prepare_table(const RawJobs &raw, const JobTable &tab, uint32_t Jp, hipStream_t s);
hipError_t launch_reset_slots(int32_t *genes, const uint32_t *changed, uint32_t P, uint32_t Jp, hipStream_t s);
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
hipError_t launch_select(const double *fit, uint32_t P, uint32_t K, uint64_t *keys, uint32_t *idx,
                         int32_t *sel, hipStream_t s);
hipError_t launch_best(const int32_t *genes, const double *fit, const int32_t *sel, const uint32_t *info,
                       uint32_t Jn, uint32_t Jp, int32_t *batch_out, int32_t *gpus_out, double *fit_out,
                       hipStream_t s);

}  // namespace ones
