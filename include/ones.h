/*
 * libones - one generation of the ONES evolutionary search on an AMD MI355X (gfx950).
 *
 * ONES (arXiv 2108.03645) schedules the batch size of every deep-learning job in a
 * shared GPU cluster by evolving a population of candidate schedules (Section 3.2).
 * This library runs that search on one GPU: the initial population, and per generation
 * the refresh / uniform crossover / uniform mutation operators (Section 3.2.2), the
 * repair of every candidate to the cluster's capacity (Eq. 4), the scoring with the
 * "smallest remaining utilisation" objective sum_j T_j * c_j (Eq. 3 with T = Y/X,
 * Eq. 5 / Eq. 8) and the selection of the best K candidates; optionally with the remaining
 * work Y_j drawn per generation from the jobs' progress distributions (Alg. 1, Eq. 7), and
 * with the winner unrolled into the paper's map from GPUs to jobs (Eq. 1).
 *
 * Encoding.  A schedule is one gene per job slot: the job's global batch size B_j,
 * either 0 (the job waits, "B_j = c_j = 0" of Section 3) or a power of two inside
 * [bmin_j, bmax_j]; bmax_j is the batch-size limit R_j of Section 3.2.2.  The job then
 * runs on c_j = ceil(B_j / gpu_max_batch_j) GPUs with equal local batches.  The pool
 * holds P = 4K candidates: slots [0,K) the refreshed survivors in rank order, [K,3K)
 * the children of K parent pairs, [3K,4K) K mutants.
 *
 * Conventions.  Every function returns ONES_OK (0) or a negative ONES_E_* code; nothing
 * aborts or throws across this boundary and outputs are untouched on error.  All job
 * arrays are HOST pointers owned by the caller and copied during the call.  The device
 * workspace and the HIP stream are owned by the caller and must outlive the context;
 * the library allocates no device memory.  A context must be used by one thread at a
 * time.  Calls on the same context execute in order on the context's stream.
 */
#ifndef ONES_H
#define ONES_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ONES_MAX_SLOTS      2048      /* job slots per cluster                         */
#define ONES_MAX_GPUS       1048576   /* cluster size |C|                              */
#define ONES_MAX_POPULATION 1048576   /* pool size P                                   */
#define ONES_MAX_PARAM      1e100     /* upper bound of a, c, d, remaining             */
#define ONES_STATIC_SCRATCH_BYTES (16u << 20)  /* scratch of ones_generation_static, per GPU */

enum {
  ONES_OK = 0,
  ONES_E_INVALID_ARG = -1,         /* null pointer, negative or out-of-range scalar      */
  ONES_E_NOT_POW2 = -2,            /* bmin / bmax / gpu_max_batch of an active slot      */
  ONES_E_BOUNDS = -3,              /* bmin > bmax, bmax > 2^30, bmax/gpu_max_batch > 2^20,
                                      or a model parameter above ONES_MAX_PARAM          */
  ONES_E_NONFINITE = -4,           /* NaN or infinity in a, c, d or remaining            */
  ONES_E_WORKSPACE_TOO_SMALL = -5, /* workspace_bytes < ones_workspace_bytes(cfg), or
                                      the workspace pointer is not 256-byte aligned      */
  ONES_E_HIP = -6,                 /* a HIP call failed, or host memory ran out;
                                      ones_strerror says which (per thread).  After a launch
                                      that failed in the middle of a generation the context is
                                      inconsistent: ones_generation and ones_generation_static
                                      keep returning this code until ones_destroy            */
  ONES_E_STATIC_LIMIT = -7         /* ones_generation_static: the population needs more
                                      scratch than ONES_STATIC_SCRATCH_BYTES                 */
};

typedef struct ones_ctx ones_ctx;  /* opaque, host side; owns no device memory */

/* The search problem (Table 1: the GPU set C, the population; Section 3.2.2: theta). */
typedef struct {
  int32_t  n_gpus;         /* |C|, 0..ONES_MAX_GPUS                                      */
  int32_t  n_slots;        /* job slots, 0..ONES_MAX_SLOTS; fixed for the context        */
  int32_t  population;     /* pool size P > 0, multiple of 4; K = P/4 survive            */
  uint64_t seed;           /* key of the counter-based generator                         */
  double   mutation_rate;  /* theta in [0,1]: each job of a mutant is redrawn with it    */
  double   crossover_rate; /* in [0,1]: per-gene probability that the children swap      */
} ones_config;

/* The job set J, one entry per slot (structure of arrays, each of length n_slots).
 * Values of an inactive slot other than job_id are ignored. */
typedef struct {
  const int64_t *job_id;        /* identity; a change resets the slot's genes to "waiting" */
  const uint8_t *active;        /* 0 = empty slot                                          */
  const int32_t *bmin;          /* smallest allowed global batch, power of two             */
  const int32_t *bmax;          /* limit R_j, power of two, bmin <= bmax <= 2^30           */
  const int32_t *gpu_max_batch; /* per-GPU max batch, power of two, bmax/it <= 2^20        */
  const double  *a, *c, *d;     /* iteration time t(B,g) = a*B/g + c*log2(g) + d seconds,
                                   each finite, in [0, ONES_MAX_PARAM]                     */
  const double  *remaining;     /* Y_j, remaining samples (Eq. 5), same range              */
} ones_jobs;

/* Bytes of device memory ones_init needs for cfg; 0 if cfg is invalid. */
size_t ones_workspace_bytes(const ones_config *cfg);

/* Creates a context and the initial population G_0 (Section 3.2.2 "Initialization"):
 * P random genomes, each gene uniform over {waiting, bmin..bmax}, repaired, scored and
 * ranked.  d_workspace: DEVICE pointer, 256-byte aligned, workspace_bytes long.
 * hip_stream: a hipStream_t (NULL = the default stream).  Synchronises the stream
 * before returning.  *out is written only on success.  Besides the context the library
 * allocates one pinned host buffer (a few bytes per slot and per GPU) through which every
 * later host transfer goes in a single copy; ones_destroy frees both.  A context is used by
 * one thread at a time. */
int ones_init(ones_ctx **out, const ones_config *cfg, const ones_jobs *jobs,
              void *d_workspace, size_t workspace_bytes, void *hip_stream);

/* Replaces the job table between scheduling epochs (the "real-time job status" the
 * refresh operator reads, Section 3.2.2).  Slots whose job_id changed are set to
 * "waiting" in every candidate; nothing else happens until the next generation, whose
 * repair projects every candidate, survivors included, onto the new table.  The
 * generation counter keeps running.  Synchronises the stream. */
int ones_set_jobs(ones_ctx *ctx, const ones_jobs *jobs);

/* Probability sampling (Alg. 1, Eq. 7): instead of a fixed remaining work, every generation
 * from the next one on first draws the progress rho_j ~ Be(alpha_j, beta_j) of every slot
 * and scores the whole pool, survivors included, with Y_j = processed_j * (1/rho_j - 1),
 * capped at ONES_MAX_PARAM.  alpha, beta, processed: HOST arrays of n_slots entries, copied
 * during the call; alpha_j, beta_j in [1, ONES_MAX_PARAM] (the thresholded parameters of
 * Section 3.2.1), processed_j (samples job j has processed) in [0, ONES_MAX_PARAM]; entries
 * of empty slots are checked too.  The draw of slot j in generation t is a function of
 * (seed, j, t) only: rho = Ga / (Ga + Gb) with Marsaglia-Tsang gamma deviates fed by
 * Philox4x32-10 counters (n, j, t, 1) and (n, j, t, 2), n = 0, 1, ... the candidate number.
 * The values persist across ones_set_jobs.  Three NULL pointers switch back to the job
 * table's remaining work.  Errors: ONES_E_INVALID_ARG (only some pointers NULL, alpha or
 * beta below 1, processed negative), ONES_E_NONFINITE, ONES_E_BOUNDS.  Synchronises. */
int ones_set_progress(ones_ctx *ctx, const double *alpha, const double *beta,
                      const double *processed);

/* Option, off at first.  When on, the first generation after ones_set_jobs serves the jobs that
 * arrived with that table (active slots whose job_id changed) first, in every candidate
 * (refresh (3) of Section 3.2.2: new jobs are allocated before the others so that they do
 * not starve): in the candidate's visiting order each new job starts with the batch a waiting
 * job resumes with while the cluster's capacity lasts; the other jobs are admitted to what is
 * left; then the fill runs as always.  Later generations treat those jobs like any other. */
int ones_set_new_jobs_first(ones_ctx *ctx, int32_t on);

/* Which positions the uniform crossover scans (Section 3.2.2).
 *   ONES_CROSSOVER_JOBS (at first): the jobs; per job the two children swap their parents' batch
 *     sizes with the configured crossover_rate.
 *   ONES_CROSSOVER_GPUS: the GPUs of the paper's encoding (Eq. 1, a schedule maps every GPU to
 *     the job whose worker it hosts).  Both parents are laid out as the reorder operator leaves
 *     them (jobs in slot order on consecutive GPUs); every GPU has a fair coin (crossover_rate is
 *     not used): heads, the first parent's job on that GPU goes to the first child and the
 *     second parent's to the second child; tails, the other way round.  A child runs each job on
 *     the largest power-of-two number of GPUs it inherited for it, at the job's local batch,
 *     pulled inside the job's window; then the repair runs as always.  Coin of GPU i of the pair
 *     whose first child is pool slot p0 in generation t: bit i mod 32 of word (i mod 128) div 32
 *     of the Philox4x32-10 block with counter (i div 128, p0, t, 3).  Needs n_gpus <= 8192.
 * Takes effect with the next generation.  Errors: ONES_E_INVALID_ARG (unknown mode),
 * ONES_E_BOUNDS (ONES_CROSSOVER_GPUS on a larger cluster). */
#define ONES_CROSSOVER_JOBS 0
#define ONES_CROSSOVER_GPUS 1
int ones_set_crossover(ones_ctx *ctx, int32_t mode);

/* The time the job of every slot has executed (T_processed; HOST array of n_slots finite
 * entries in [0, 1e100], copied; empty slots' entries are ignored), or NULL to forget the
 * times.  While they are known, the generation that serves new jobs first admits the other
 * jobs in ascending order of executed time (equal times: lower slot first) instead of the
 * candidate's visiting order, so that the GPUs the new jobs need are taken from the jobs with
 * the largest T_processed (same passage).  The fill keeps the visiting order.  The times
 * persist across ones_set_jobs; a scheduler sets them anew with every table.  Errors:
 * ONES_E_NONFINITE, ONES_E_INVALID_ARG (negative), ONES_E_BOUNDS.  Synchronises. */
int ones_set_processed_time(ones_ctx *ctx, const double *t_processed);

/* The remaining work Y_j the last generation was scored with (HOST array of n_slots
 * entries): the job table's, or the last draw under ones_set_progress.  Synchronises. */
int ones_export_remaining(ones_ctx *ctx, double *remaining_out);

/* Runs n_generations >= 0 generations (compose, repair, score, select), asynchronously
 * on the stream. */
int ones_generation(ones_ctx *ctx, int32_t n_generations);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): ones_generation with the selection's scratch (splitters, counters,
 * bucket storage, spill list, sort pool) in a static device array of ONES_STATIC_SCRATCH_BYTES
 * that the library's code object holds on every GPU it runs on until the process ends, instead of
 * the caller's workspace.  The population, scores and survivor list stay in the workspace as
 * always, and the results are those of ones_generation bit for bit; the two calls may be mixed
 * freely on one context.  Calls no hipMalloc, hipFree, hipHostMalloc, event or other allocating
 * routine and takes no HIP events (the measurement hook does not see these generations).
 * Every context on a GPU shares that GPU's array, which keeps the last call's contents: each call
 * sets up by itself what it reads (its first generation ranks the pool without relying on
 * anything left there), so calls may follow each other in any order, but two calls that overlap
 * in time on one GPU (different streams or threads) race.  Must be called with the context's
 * device current.  Errors: ONES_E_STATIC_LIMIT when the population's scratch exceeds the array
 * (populations up to 65536 fit; nothing is launched), ONES_E_INVALID_ARG (null context, negative
 * count, another device current), ONES_E_HIP. */
int ones_generation_static(ones_ctx *ctx, int32_t n_generations);

/* Pools of at most 64 job slots and 2048 candidates with a fixed remaining work run all
 * generations of a ones_generation call of three or more generations in ONE launch whose
 * workgroups exchange results while it runs; a workgroup polls for the others' results at most
 * `polls` times (at first 2^22, a few seconds) and then gives up: the launch ends, the next call
 * that synchronises (ones_best, ones_export, ones_placement) returns ONES_E_HIP, and the context
 * only accepts ones_destroy from then on.  This never happens on a healthy device; polls = 0
 * makes every wait give up at once, which is how the error path is tested. */
int ones_set_wait_limit(ones_ctx *ctx, uint32_t polls);

/* The winner S* (Alg. 1: smallest score): global batch and GPU count per slot (HOST
 * arrays of n_slots entries, either may be NULL) and its score.  Between ones_set_jobs and the
 * next generation no schedule exists under the new table: the call then returns the last
 * winner as it is stored (slots that changed hands already set to waiting) with the score it had
 * under the old table; run a generation first.  Synchronises. */
int ones_best(ones_ctx *ctx, int32_t *batch_out, int32_t *gpus_out, double *fitness_out);

/* The winner as the paper's mapping from (job, GPU) to a local batch (Eq. 1), packed the way
 * the reorder operator leaves it (Section 3.2.2): the jobs in slot order, each on c_j
 * consecutive GPUs with B_j / c_j samples per GPU, idle GPUs last.  HOST arrays of n_gpus
 * entries, either may be NULL: the slot whose worker GPU i runs (-1 = idle) and that worker's
 * batch (0 = idle).  Eq. 2 recovers ones_best's outputs from them.  ONES_E_INVALID_ARG between
 * ones_set_jobs and the next generation (no schedule exists under the current job table).
 * Synchronises. */
int ones_placement(ones_ctx *ctx, int32_t *slot_of_gpu, int32_t *batch_of_gpu);

/* Copies the whole state to HOST arrays (any may be NULL): genes[P][Jp] batch sizes with
 * Jp = ones_padded_jobs(n_slots), fit[P], sel[K] (survivor slots by ascending
 * (fitness, slot)), generation counter.  For parity checks and checkpoints.  Synchronises.
 * Also reports, as ONES_E_HIP, a defect of the library's own row bookkeeping that its kernels
 * detected (a genome row index outside the array, which they pull back inside before use). */
int ones_export(ones_ctx *ctx, int32_t *genes, double *fit, int32_t *sel, int64_t *generation);

/* Job slots padded to whole rows of 64 columns: 64 * ceil(max(n_slots,1) / 64). */
int32_t ones_padded_jobs(int32_t n_slots);

/* Measurement hook.  With every = n > 0 the evolve and the select kernels of every n-th
 * generation are bracketed by HIP events on the context's stream (n = 1: every generation;
 * an event costs a few microseconds of stream time); every <= 0 switches it off.
 * A small pool (at most 64 job slots and 2048 candidates, fixed remaining work) runs all
 * generations of a ones_generation call of three or more generations in one launch: that
 * launch counts as one evolve launch (every n-th call is bracketed) and there is no select
 * launch.
 * ones_profile_read synchronises and returns the accumulated kernel time in milliseconds
 * and the number of bracketed launches since the last ones_profile_enable call (any output
 * may be NULL). */
int ones_profile_enable(ones_ctx *ctx, int32_t every);
int ones_profile_read(ones_ctx *ctx, double *evolve_ms, int64_t *evolve_launches,
                      double *select_ms, int64_t *select_launches);

/* The batch-size limit policies of Section 3.3.2: produces the limits R_j (the bmax of the
 * next ones_set_jobs) from the cluster's state between two scheduling epochs.  Host code, no
 * context, no device work.  One entry per slot, all HOST arrays:
 *   state 0  empty slot: limit 0.
 *   state 1  Start: the job arrived, or is still in its warm-up steps: limit = gpu_max_batch
 *            (it must fit one GPU).
 *   state 2  Resume: the job waits.  The first update after it was pre-empted (marked by
 *            last_batch > 0, its global batch before pre-emption) caps the limit at that
 *            batch; every further update finds it rejected again and halves the limit.
 *   state 3  running: when finished_epoch is set, R' = ceil(2R / ceil(sigma * elapsed + 1)):
 *            the doubling of Scale-up (elapsed = 0) with the penalty of Scale-down for long
 *            executed time; otherwise unchanged.  sigma: the paper suggests the job arrival
 *            rate.
 * Every result is rounded down to a power of two and kept inside [bmin, bcap] (bcap: the
 * job's own largest batch).  limit is read (states 2, 3) and written.  Nothing is written
 * on error: ONES_E_INVALID_ARG (null pointer, state above 3, n_slots outside
 * 0..ONES_MAX_SLOTS, negative sigma / elapsed / last_batch, limit below 1 for a waiting or
 * running job), ONES_E_NOT_POW2, ONES_E_BOUNDS (bmin > bcap, bcap > 2^30, sigma * elapsed >
 * 1e15), ONES_E_NONFINITE. */
typedef struct {
  const uint8_t *state;
  const int32_t *bmin, *bcap, *gpu_max_batch;
  const int32_t *last_batch;
  const uint8_t *finished_epoch;
  const double  *elapsed;
} ones_limit_inputs;
int ones_update_limits(int32_t n_slots, const ones_limit_inputs *in, double sigma, int32_t *limit);

void ones_destroy(ones_ctx *ctx);           /* NULL is allowed */
const char *ones_strerror(int code);        /* static or thread-local storage */

#ifdef __cplusplus
}
#endif
#endif
