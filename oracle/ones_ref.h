/*
 * CPU oracle for one generation of the ONES evolutionary search (arXiv 2108.03645,
 * Section 3.2).  TEST INFRASTRUCTURE ONLY: plain, slow, scalar C; it exists to check
 * the GPU library and to be timed as a CPU baseline.  It shares no code, header,
 * table or constant with the GPU library and must never be called from it.
 *
 * Parity status of each function (what pins it, other than itself):
 *   ones_ref_philox4x32_10 : published known-answer vectors + a big-integer Python
 *                            transcription of the SC'11 definition.
 *   ones_ref_repair_genome : hand-worked example, Eq. 4 capacity, maximality,
 *                            idempotence, closed-form special cases, brute force.
 *   ones_ref_score_genome  : hand values, exact rational recomputation of
 *                            Eq. 3 / Eq. 5, monotonicity.
 *   ones_ref_select        : numpy lexsort on (fitness, index).
 *   compose (crossover, mutation, init): complementarity of children, coin
 *                            frequencies, chi-square on redraws and parent ranks,
 *                            theta = chi = 0 and chi = 1 special cases.
 *   ones_ref_log           : the C library's log within 2 ulp over the whole range.
 *   ones_ref_gamma_draw    : mean = variance = shape, Kolmogorov-Smirnov against the
 *                            gamma distribution function, shape 1 = exponential.
 *   ones_ref_sampled_remaining : Beta mean alpha/(alpha+beta) and variance
 *                            alpha*beta/((alpha+beta)^2 (alpha+beta+1)), KS against the
 *                            Beta distribution function, Be(1,1) uniform,
 *                            E[1/rho - 1] = beta/(alpha-1), a Python transcription.
 *   ones_ref_placement     : Eq. 2 (B_j and c_j recovered from the per-GPU batches), one job
 *                            per GPU, packing in slot order, a hand-worked example.
 *   ones_ref_update_limits : the four policies worked by hand (doubling at T = 0, the
 *                            printed penalty formula at several sigma*T, halving on rejection,
 *                            the cap at the batch before pre-emption), monotonicity in T.
 *   new jobs first         : a hand-worked two-GPU example, every new job running in every
 *                            candidate when the capacity allows, Eq. 4, no effect when off or
 *                            when no job is new.
 *   ones_ref_repair_arrivals / ones_ref_set_processed_time : a sequential Python
 *                            transcription on random cases, a hand-worked example (the job
 *                            with the largest T_processed gives up its GPUs), equal times =
 *                            slot order, the admitted jobs form a prefix of the time order.
 *   ones_ref_gpu_crossover / ones_ref_set_crossover(1) : every GPU's job goes to exactly one
 *                            child (n1 + n2 = the parents' counts inside the cluster), equal
 *                            parents give equal children, coin frequencies, a Python
 *                            transcription with the coins recomputed from Philox, a hand-worked
 *                            example; in the search: Eq. 4, children between their parents.
 *   scheduling quality against the paper's JCT numbers: parity unpinned (the paper's
 *                            trace, jobs and comparison schedulers do not exist here).
 */
#ifndef ONES_REF_H
#define ONES_REF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ones_ref_ctx ones_ref_ctx;

typedef struct {
  int32_t  n_gpus;         /* |C| of Table 1 */
  int32_t  n_slots;        /* job slots Jn */
  int32_t  population;     /* pool size P = 4K (K elites + 2K children + K mutants) */
  uint64_t seed;
  double   mutation_rate;  /* theta, Section 3.2.2 "Uniform mutation" */
  double   crossover_rate; /* per-gene swap probability of the uniform crossover */
} ones_ref_config;

typedef struct {           /* arrays of length n_slots, host memory */
  const int64_t *job_id;
  const uint8_t *active;
  const int32_t *bmin, *bmax, *gpu_max_batch;
  const double  *a, *c, *d;
  const double  *remaining;
} ones_ref_jobs;

enum {
  ONES_REF_OK = 0,
  ONES_REF_E_INVALID_ARG = -1,
  ONES_REF_E_NOT_POW2 = -2,
  ONES_REF_E_BOUNDS = -3,
  ONES_REF_E_NONFINITE = -4
};

/* whole-search entry points, same call sequence as the GPU library */
int  ones_ref_init(ones_ref_ctx **out, const ones_ref_config *cfg, const ones_ref_jobs *jobs);
int  ones_ref_set_jobs(ones_ref_ctx *ctx, const ones_ref_jobs *jobs);
int  ones_ref_generation(ones_ref_ctx *ctx, int32_t n_generations);
int  ones_ref_best(ones_ref_ctx *ctx, int32_t *batch_out, int32_t *gpus_out, double *fitness_out);
int  ones_ref_export(ones_ref_ctx *ctx, int32_t *genes, double *fit, int32_t *sel, int64_t *generation);
void ones_ref_destroy(ones_ref_ctx *ctx);
int  ones_ref_padded_jobs(int32_t n_slots);     /* Jp = 64*ceil(max(n,1)/64) */
void ones_ref_set_threads(int n);               /* candidates split over n OpenMP threads */
int  ones_ref_get_threads(void);

/* Probability sampling (Alg. 1, Eq. 7).  HOST arrays of n_slots entries: alpha_j, beta_j
 * (each in [1, 1e100]: the thresholded parameters of the progress distribution Be_j) and
 * the samples job j has processed (in [0, 1e100]).  From the next generation on, every
 * generation first draws rho_j ~ Be(alpha_j, beta_j) for every slot and scores the whole
 * pool with Y_j = processed_j * (1/rho_j - 1).  Three NULL pointers switch back to the
 * job table's fixed remaining work. */
int  ones_ref_set_progress(ones_ref_ctx *ctx, const double *alpha, const double *beta,
                           const double *processed);
/* Option (off at first): the first generation after ones_ref_set_jobs serves the jobs that
 * arrived with that table first (refresh (3) of Section 3.2.2): in every candidate, in visiting
 * order, each new job starts with the batch a waiting job resumes with while the capacity
 * lasts; the other jobs are admitted to what is left, then the fill runs as always. */
int  ones_ref_set_new_jobs_first(ones_ref_ctx *ctx, int32_t on);
/* Which positions the uniform crossover scans (Section 3.2.2): 0 (at first) the jobs, a coin
 * per job with the configured rate; 1 the GPUs of the paper's encoding (Eq. 1), a fair coin per
 * GPU, the parents laid out as the reorder operator leaves them (ones_ref_gpu_crossover); a
 * child then runs each job on the largest power-of-two number of GPUs it inherited for it.
 * Mode 1 needs n_gpus <= 8192 (ONES_REF_E_BOUNDS). */
int  ones_ref_set_crossover(ones_ref_ctx *ctx, int32_t mode);
/* The time every slot's job has executed (T_processed; n_slots finite entries >= 0), or NULL to
 * forget it.  While set, the generation that serves new jobs first admits the other jobs in
 * ascending order of that time (equal times: lower slot first) instead of the rotated order:
 * when the new jobs leave too little room, the GPUs are taken from the jobs with the largest
 * T_processed (same passage).  The fill rounds keep the rotated order. */
int  ones_ref_set_processed_time(ones_ref_ctx *ctx, const double *t_processed);

/* the remaining work Y_j (n_slots entries) the last generation was scored with */
int  ones_ref_export_remaining(ones_ref_ctx *ctx, double *remaining_out);

/* The winner as the paper's mapping from (job, GPU) to a local batch (Eq. 1), packed the way
 * the reorder operator leaves it (Section 3.2.2): the jobs in slot order, each on c_j
 * consecutive GPUs with B_j / c_j samples per GPU.  n_gpus entries each: the slot whose worker
 * GPU i runs (-1 = idle) and that worker's batch (0 = idle); either may be NULL.  Fails with
 * ONES_REF_E_INVALID_ARG between ones_ref_set_jobs and the next generation, when no schedule
 * exists under the current job table. */
int  ones_ref_placement(ones_ref_ctx *ctx, int32_t *slot_of_gpu, int32_t *batch_of_gpu);

/* The batch-size limit policies of Section 3.3.2, the producer of bmax_j between scheduling
 * epochs.  state_j: 0 empty slot (limit 0), 1 Start (the job arrived or is still warming up:
 * limit = one GPU's batch), 2 Resume (the job is waiting: the first update after it was
 * pre-empted, marked by last_batch_j > 0, caps the limit at that batch; every further one
 * halves it), 3 running (when it finished an epoch: R' = ceil(2R / ceil(sigma*T + 1)), the
 * doubling of Scale-up with the penalty of Scale-down; otherwise unchanged).  Results are
 * rounded down to a power of two and kept inside [bmin_j, bcap_j].  limit: in/out. */
typedef struct {
  const uint8_t *state;
  const int32_t *bmin, *bcap, *gpu_max_batch;   /* powers of two, bmin <= bcap */
  const int32_t *last_batch;                    /* waiting jobs: batch before pre-emption, or 0 */
  const uint8_t *finished_epoch;                /* running jobs */
  const double  *elapsed;                       /* running jobs: T_processed in seconds */
} ones_ref_limit_inputs;
int  ones_ref_update_limits(int32_t n_slots, const ones_ref_limit_inputs *in, double sigma,
                            int32_t *limit);

/* single steps, exposed so that tests can pin them one at a time */
double ones_ref_log(double x);                  /* natural logarithm of a positive normal number */
/* Gamma(shape, 1) draw number `which` (1 or 2) of slot j in generation t, shape >= 1;
 * attempts_out (may be NULL) receives the number of candidate draws used */
double ones_ref_gamma_draw(uint64_t seed, uint32_t j, uint32_t t, uint32_t which, double shape,
                           int *attempts_out);
/* Eq. 7 with rho ~ Be(alpha, beta); rho_out may be NULL */
double ones_ref_sampled_remaining(uint64_t seed, uint32_t j, uint32_t t, double alpha, double beta,
                                  double processed, double *rho_out);
void ones_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
/* GPUs per job each child of a pair inherits under the crossover over the GPUs (mode 1 of
 * ones_ref_set_crossover): cA, cB, n1, n2 have n entries (GPU counts per job) */
void ones_ref_gpu_crossover(uint64_t seed, uint32_t p0, uint32_t t, int32_t n_gpus, int32_t n,
                            const int32_t *cA, const int32_t *cB, int32_t *n1, int32_t *n2);
/* genes: n_slots int32 batch sizes (0 or a power of two), repaired in place with
 * rotation r in [0,Jp); fill_rounds_out (may be NULL) receives the number of fill rounds */
int  ones_ref_repair_genome(const ones_ref_config *cfg, const ones_ref_jobs *jobs,
                            int32_t *genes, uint32_t r, int32_t *fill_rounds_out);
/* The same with the refresh (3) of Section 3.2.2: arrived (n_slots bytes) marks the slots whose
 * jobs arrived (their genes start from waiting and they are served first); t_processed
 * (n_slots entries or NULL) is the executed time that orders the admission of the others. */
int  ones_ref_repair_arrivals(const ones_ref_config *cfg, const ones_ref_jobs *jobs, int32_t *genes, uint32_t r,
                              const uint8_t *arrived, const double *t_processed, int32_t *fill_rounds_out);
int  ones_ref_score_genome(const ones_ref_config *cfg, const ones_ref_jobs *jobs,
                           const int32_t *genes, double *fitness_out);
void ones_ref_select(const double *fit, int32_t population, int32_t *sel /* population/4 */);
/* the genome slot p of generation t+1 would hold BEFORE repair, and its rotation */
int  ones_ref_compose_slot(ones_ref_ctx *ctx, int32_t p, int32_t *genes_out, uint32_t *r_out,
                           int32_t *parent_a_out, int32_t *parent_b_out);

/* the random genome slot p of the initial population holds BEFORE repair (n_slots genes) */
int  ones_ref_initial_genome(const ones_ref_config *cfg, const ones_ref_jobs *jobs, int32_t p,
                             int32_t *genes_out, uint32_t *r_out);

#ifdef __cplusplus
}
#endif
#endif
