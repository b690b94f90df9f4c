/*
 * CPU oracle for one generation of the ONES evolutionary search (arXiv 2108.03645,
 * Section 3.2: population of candidate schedules, refresh / uniform crossover /
 * uniform mutation, scoring with the "smallest remaining utilisation" objective
 * Eq. 3 with T = Y/X of Eq. 5, selection of the best K).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain scalar loops in the order the method states them;
 * no blocking, fusion or reordering.  Build: gcc -O2 -ffp-contract=off -fopenmp.
 *
 * Encoding.  The paper's schedule maps (job, GPU) to a local batch (Eq. 1); the
 * objective only needs the global batch B_j and GPU count c_j (Eq. 2, Eq. 3), so a
 * genome here is one gene per job: B_j = 0 (the job waits, Section 3 "B_j = c_j = 0")
 * or a power of two inside the job's window [bmin_j, bmax_j] (bmax_j is the limit R_j
 * of Section 3.2.2).  GPU count c = ceil(B / per-GPU max batch); local batches equal.
 * Inside this file a gene is its exponent g = log2 B, or WAIT.
 */
#include "ones_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define WAIT (-1)
#define LANES 64
#define MAX_SLOTS 2048
#define MAX_POPULATION (1 << 20)
#define MAX_GPUS (1 << 20)
#define MAX_PARAM 1e100

typedef struct {
  int     active;
  int     lo, hi, mu;      /* log2 of bmin, bmax, per-GPU max batch */
  double  a, cc, d, Y;
  int64_t id;
} slot_t;

struct ones_ref_ctx {
  int      G, Jn, Jp, R, P, K;
  uint32_t key[2];
  uint32_t T_mut, T_x;
  slot_t  *tab;            /* Jp entries */
  int32_t *genes[2];       /* [P][Jp] batch sizes, ping-pong */
  double  *fit;            /* [P] */
  int32_t *sel;            /* [K] */
  int      cur;
  int64_t  t;              /* generation counter; 0 = initial population */
  int      stale;          /* job table replaced since the last generation */
  int      new_jobs_first; /* option: the first generation after a table change serves new jobs first */
  int      serve_new;      /* ... and this is that generation */
  uint8_t *is_new;         /* Jp entries: slot changed hands in the last ones_ref_set_jobs */
  double  *t_processed;    /* Jp entries: executed time per slot, or NULL (ones_ref_set_processed_time) */
  int     *by_time;        /* Jp entries: the slots in ascending (t_processed, slot) order */
  int      per_gpu;        /* uniform crossover scans the GPUs (the paper's encoding) instead of the jobs */
  int      sampling;       /* Alg. 1: remaining work drawn per generation */
  double  *alpha, *beta, *processed, *Y_fixed;   /* Jn entries each */
};

static int g_threads = 1;
void ones_ref_set_threads(int n) { g_threads = n < 1 ? 1 : n; }
int  ones_ref_get_threads(void) { return g_threads; }

int ones_ref_padded_jobs(int32_t n_slots) {
  int n = n_slots < 1 ? 1 : n_slots;
  return LANES * ((n + LANES - 1) / LANES);
}

/* ------------------------------------------------------------------ RNG ---------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds; each round multiplies
 * counter words 0 and 2 by two fixed constants, the high halves are xored with words
 * 1 and 3 and the round key, the low halves move to words 1 and 3; the key is bumped
 * by two Weyl constants between rounds. */
void ones_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t x0 = ctr[0], x1 = ctr[1], x2 = ctr[2], x3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t p0 = (uint64_t)0xD2511F53u * x0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * x2;
    uint32_t y0 = (uint32_t)(p1 >> 32) ^ x1 ^ k0;
    uint32_t y1 = (uint32_t)p1;
    uint32_t y2 = (uint32_t)(p0 >> 32) ^ x3 ^ k1;
    uint32_t y3 = (uint32_t)p0;
    x0 = y0; x1 = y1; x2 = y2; x3 = y3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = x0; out[1] = x1; out[2] = x2; out[3] = x3;
}

static uint32_t bounded(uint32_t w, uint32_t n) { return (uint32_t)(((uint64_t)w * n) >> 32); }

/* per-candidate draw: ranks of the two parents among the survivors, repair rotation */
static void candidate_draw(const ones_ref_ctx *c, uint32_t p, uint32_t t,
                           uint32_t *ra, uint32_t *rb, uint32_t *r) {
  uint32_t ctr[4] = {0xFFFFFFFFu, p, t, 0u}, w[4];
  ones_ref_philox4x32_10(ctr, c->key, w);
  *ra = bounded(w[0], (uint32_t)c->K);
  *rb = bounded(w[1], (uint32_t)c->K);
  *r  = bounded(w[2], (uint32_t)c->Jp);
}

/* one 32-bit word per (candidate, generation, job): job j lives in column j mod 64,
 * row j div 64; four consecutive rows of a column share one Philox block */
static uint32_t gene_word(const ones_ref_ctx *c, uint32_t p, uint32_t t, int j) {
  int l = j % LANES, i = j / LANES;
  uint32_t ctr[4] = {(uint32_t)((i / 4) * LANES + l), p, t, 0u}, w[4];
  ones_ref_philox4x32_10(ctr, c->key, w);
  return w[i % 4];
}

/* ------------------------------------------------------------- job table --------- */
static int ilog2_exact(int32_t v) {           /* -1 unless v is a power of two */
  if (v <= 0 || (v & (v - 1)) != 0) return -1;
  int e = 0;
  while ((1 << e) != v) ++e;
  return e;
}

static int check_config(const ones_ref_config *cfg) {
  if (!cfg) return ONES_REF_E_INVALID_ARG;
  if (cfg->n_gpus < 0 || cfg->n_gpus > MAX_GPUS) return ONES_REF_E_INVALID_ARG;
  if (cfg->n_slots < 0 || cfg->n_slots > MAX_SLOTS) return ONES_REF_E_INVALID_ARG;
  if (cfg->population <= 0 || cfg->population % 4 != 0 || cfg->population > MAX_POPULATION)
    return ONES_REF_E_INVALID_ARG;
  if (!(cfg->mutation_rate >= 0.0 && cfg->mutation_rate <= 1.0)) return ONES_REF_E_INVALID_ARG;
  if (!(cfg->crossover_rate >= 0.0 && cfg->crossover_rate <= 1.0)) return ONES_REF_E_INVALID_ARG;
  return ONES_REF_OK;
}

static int check_param(double v) {
  if (!isfinite(v)) return ONES_REF_E_NONFINITE;
  if (v < 0.0) return ONES_REF_E_INVALID_ARG;
  if (v > MAX_PARAM) return ONES_REF_E_BOUNDS;
  return ONES_REF_OK;
}

/* fills tab[0..Jp); slots that are empty or beyond n_slots become inactive */
static int build_table(int Jn, int Jp, const ones_ref_jobs *jobs, slot_t *tab) {
  memset(tab, 0, sizeof(slot_t) * (size_t)Jp);
  if (Jn > 0) {
    if (!jobs || !jobs->job_id || !jobs->active || !jobs->bmin || !jobs->bmax ||
        !jobs->gpu_max_batch || !jobs->a || !jobs->c || !jobs->d || !jobs->remaining)
      return ONES_REF_E_INVALID_ARG;
  }
  for (int j = 0; j < Jn; ++j) {
    slot_t *s = &tab[j];
    s->id = jobs->job_id[j];
    if (!jobs->active[j]) continue;
    int lo = ilog2_exact(jobs->bmin[j]), hi = ilog2_exact(jobs->bmax[j]);
    int mu = ilog2_exact(jobs->gpu_max_batch[j]);
    if (lo < 0 || hi < 0 || mu < 0) return ONES_REF_E_NOT_POW2;
    if (lo > hi || hi > 30 || hi - mu > 20) return ONES_REF_E_BOUNDS;
    int rc;
    if ((rc = check_param(jobs->a[j])) || (rc = check_param(jobs->c[j])) ||
        (rc = check_param(jobs->d[j])) || (rc = check_param(jobs->remaining[j])))
      return rc;
    s->active = 1; s->lo = lo; s->hi = hi; s->mu = mu;
    s->a = jobs->a[j]; s->cc = jobs->c[j]; s->d = jobs->d[j]; s->Y = jobs->remaining[j];
  }
  return ONES_REF_OK;
}

static uint32_t rate_threshold(double rate) {   /* min(2^32-1, floor(rate * 2^32)) */
  double v = floor(rate * 4294967296.0);
  return v >= 4294967295.0 ? 0xFFFFFFFFu : (uint32_t)v;
}

/* --------------------------------------------------------- gene helpers ---------- */
static int64_t gpus_of(int g, int mu) {           /* c(g): ceil(2^g / 2^mu), 0 if waiting */
  if (g == WAIT) return 0;
  return (int64_t)1 << (g > mu ? g - mu : 0);
}
static int32_t batch_of(int g) { return g == WAIT ? 0 : (int32_t)1 << g; }
static int exponent_of(int32_t batch) { return batch == 0 ? WAIT : ilog2_exact(batch); }
static int imin(int x, int y) { return x < y ? x : y; }
static int imax(int x, int y) { return x > y ? x : y; }

/* uniform draw over {WAIT, lo..hi} from k in [0, hi-lo+2) */
static int gene_from_draw(const slot_t *s, uint32_t k) {
  if (!s->active || k == 0) return WAIT;
  return s->lo + (int)k - 1;
}

/* ------------------------------------------------------------- repair ------------ */
/* The paper's refresh (Section 3.2.2): (1) drop finished jobs, (2) scale down to the
 * limit R_j, (3) make room when capacity is exceeded (Eq. 4: a GPU hosts one worker),
 * then fill idle GPUs by resuming waiting jobs or scaling up running ones until no
 * single step fits.  Jobs are visited in a fixed order rotated by r. */
/* is_new (may be NULL): slots of jobs that arrived with the last job table.  They are
 * served first ("allocates N new jobs with N available GPUs ... avoid starvation of new jobs
 * by the preferential allocation", Section 3.2.2 refresh (3)): in visiting order each starts
 * with the batch a waiting job resumes with while the capacity lasts, and only what they leave
 * is shared out among the others.
 * by_time (may be NULL; only looked at together with is_new): the slots in ascending order of
 * the time their jobs have executed.  The others are then admitted in that order instead of
 * the rotated one, so that the room for the new jobs is taken from the jobs with the largest
 * T_processed (same passage). */
static int repair(const slot_t *tab, int Jp, int R, int64_t G, int *g, uint32_t r, const uint8_t *is_new,
                  const int *by_time) {
  int order[MAX_SLOTS];
  for (int j = 0; j < Jp; ++j) {
    int sigma = (j % LANES) * R + (j / LANES);
    int pi = (sigma + Jp - (int)r) % Jp;
    order[pi] = j;
  }
  /* 1. clamp: empty slot waits; a running job is pulled inside its window */
  for (int j = 0; j < Jp; ++j) {
    if (!tab[j].active) g[j] = WAIT;
    else if (g[j] != WAIT) g[j] = imin(imax(g[j], tab[j].lo), tab[j].hi);
  }
  /* 2. lift: a larger batch that needs no extra GPU */
  for (int j = 0; j < Jp; ++j)
    if (g[j] != WAIT) g[j] = imax(g[j], imin(tab[j].mu, tab[j].hi));
  /* 2b. new jobs first */
  int64_t Q = 0, taken = 0;
  if (is_new) {
    for (int pos = 0; pos < Jp; ++pos) {
      int j = order[pos];
      if (!is_new[j] || !tab[j].active) continue;
      int start = imax(tab[j].lo, imin(tab[j].mu, tab[j].hi));
      Q += gpus_of(start, tab[j].mu);
      if (Q <= G) { g[j] = start; taken = Q; } else g[j] = WAIT;
    }
  }
  /* 3. admit: prefix sum of GPU counts in visiting order; beyond capacity -> wait */
  Q = 0;
  for (int pos = 0; pos < Jp; ++pos) {
    int j = (is_new && by_time) ? by_time[pos] : order[pos];
    if (g[j] == WAIT || (is_new && is_new[j])) continue;
    Q += gpus_of(g[j], tab[j].mu);
    if (Q > G - taken) g[j] = WAIT;
  }
  /* 4. fill */
  int rounds = 0;
  for (;;) {
    int64_t used = 0;
    for (int j = 0; j < Jp; ++j) used += gpus_of(g[j], tab[j].mu);
    int64_t idle = G - used;
    int     target[MAX_SLOTS];
    int64_t cost[MAX_SLOTS];
    int any = 0;
    for (int j = 0; j < Jp; ++j) {
      const slot_t *s = &tab[j];
      target[j] = WAIT; cost[j] = -1;              /* no proposal */
      if (!s->active) continue;
      if (g[j] == WAIT) {
        target[j] = imax(s->lo, imin(s->mu, s->hi));
        cost[j] = gpus_of(target[j], s->mu);
      } else if (g[j] < s->hi) {
        target[j] = g[j] + 1;
        cost[j] = gpus_of(target[j], s->mu) - gpus_of(g[j], s->mu);
      }
      if (cost[j] >= 0 && cost[j] > idle) { target[j] = WAIT; cost[j] = -1; } /* not participating */
      if (cost[j] >= 0) any = 1;
    }
    if (!any) break;
    ++rounds;
    Q = 0;
    for (int pos = 0; pos < Jp; ++pos) {
      int j = order[pos];
      if (cost[j] < 0) continue;
      Q += cost[j];
      if (Q <= idle) g[j] = target[j];
    }
  }
  return rounds;
}

/* -------------------------------------------------------------- score ------------ */
/* Eq. 3 with Eq. 5: sum over running jobs of T_j * c_j, T_j = Y_j / X_j, throughput
 * X_j = B_j / t_j, iteration time t(b,g) = a*b/g + c*log2(g) + d with b/g the local
 * batch.  T_j*c_j = Y_j * t_j / (B_j/c_j).  Fixed summation order: column sums over the
 * rows top to bottom, then a xor-butterfly over the 64 columns. */
static double score(const slot_t *tab, int R, const int *g) {
  double part[LANES], next[LANES];
  for (int l = 0; l < LANES; ++l) {
    double acc = 0.0;
    for (int i = 0; i < R; ++i) {
      int j = l + LANES * i;
      double term = 0.0;
      if (g[j] != WAIT) {
        const slot_t *s = &tab[j];
        double bf = (double)((int64_t)1 << imin(g[j], s->mu));   /* local batch */
        double lg = (double)imax(0, g[j] - s->mu);               /* log2(GPU count) */
        double prod_a = s->a * bf;
        double prod_c = s->cc * lg;
        double t = (prod_a + prod_c) + s->d;
        double yt = s->Y * t;
        term = yt / bf;
      }
      acc = acc + term;
    }
    part[l] = acc;
  }
  for (int s = 32; s >= 1; s >>= 1) {
    for (int l = 0; l < LANES; ++l) next[l] = part[l] + part[l ^ s];
    memcpy(part, next, sizeof(part));
  }
  return part[0];
}

/* ------------------------------------------------------------- select ------------ */
typedef struct { double f; int32_t idx; } keyed_t;
static int keyed_cmp(const void *x, const void *y) {
  const keyed_t *u = (const keyed_t *)x, *v = (const keyed_t *)y;
  if (u->f < v->f) return -1;
  if (u->f > v->f) return 1;
  return (u->idx > v->idx) - (u->idx < v->idx);
}
/* the K = P/4 slots with the smallest (fitness, slot index), in that order */
void ones_ref_select(const double *fit, int32_t population, int32_t *sel) {
  keyed_t *k = (keyed_t *)malloc(sizeof(keyed_t) * (size_t)population);
  for (int32_t p = 0; p < population; ++p) { k[p].f = fit[p]; k[p].idx = p; }
  qsort(k, (size_t)population, sizeof(keyed_t), keyed_cmp);
  for (int32_t i = 0; i < population / 4; ++i) sel[i] = k[i].idx;
  free(k);
}

/* ------------------------------------------- crossover over the GPUs ------------- */
/* Uniform crossover as the paper states it (Section 3.2.2), on the encoding of Eq. 1: a
 * schedule maps every GPU to the job whose worker it hosts.  The parents are laid out the way
 * the reorder operator leaves them (jobs in slot order on consecutive GPUs, cA[j] resp. cB[j]
 * GPUs each, GPUs beyond the cluster do not exist), every GPU is scanned on its own, and
 * with a fair coin the job of the first parent goes to the first child and the job of the
 * second parent to the second child, or the other way round.  n1[j], n2[j]: the number of GPUs
 * on which each child inherited job j.
 * Coin of GPU i for the pair whose first child is pool slot p0, generation t: bit i mod 32 of
 * word (i mod 128) div 32 of the Philox block with counter (i div 128, p0, t, 3). */
void ones_ref_gpu_crossover(uint64_t seed, uint32_t p0, uint32_t t, int32_t n_gpus, int32_t n,
                            const int32_t *cA, const int32_t *cB, int32_t *n1, int32_t *n2) {
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  int32_t *gpuA = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_gpus > 0 ? n_gpus : 1));
  int32_t *gpuB = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_gpus > 0 ? n_gpus : 1));
  for (int which = 0; which < 2; ++which) {
    const int32_t *c = which ? cB : cA;
    int32_t *gpu = which ? gpuB : gpuA;
    int32_t pos = 0;
    for (int32_t j = 0; j < n; ++j)
      for (int32_t k = 0; k < c[j] && pos < n_gpus; ++k) gpu[pos++] = j;
    while (pos < n_gpus) gpu[pos++] = -1;              /* idle */
  }
  for (int32_t j = 0; j < n; ++j) n1[j] = n2[j] = 0;
  for (int32_t i = 0; i < n_gpus; ++i) {
    uint32_t ctr[4] = {(uint32_t)(i / 128), p0, t, 3u}, w[4];
    ones_ref_philox4x32_10(ctr, key, w);
    int coin = (int)((w[(i % 128) / 32] >> (i % 32)) & 1u);
    int32_t to_first = coin ? gpuA[i] : gpuB[i];
    int32_t to_second = coin ? gpuB[i] : gpuA[i];
    if (to_first >= 0) n1[to_first] += 1;
    if (to_second >= 0) n2[to_second] += 1;
  }
  free(gpuA); free(gpuB);
}

/* GPUs a parent's gene stands for under the current job table (what clamp and lift of the
 * repair make of it); an empty slot or a waiting job holds none */
static int32_t parent_gpus(const slot_t *s, int32_t batch) {
  int g = exponent_of(batch);
  if (!s->active || g == WAIT) return 0;
  g = imin(imax(g, s->lo), s->hi);
  g = imax(g, imin(s->mu, s->hi));
  return (int32_t)gpus_of(g, s->mu);
}

/* ------------------------------------------------------------ compose ------------ */
/* Genome of pool slot p of generation t, before repair, read from the previous
 * generation through its survivor list.  Pool = K refreshed survivors, K parent pairs
 * giving 2K crossover children, K mutants (Section 3.2.2). */
static void compose(const ones_ref_ctx *c, const int32_t *prev, uint32_t t, int p, int *g,
                    uint32_t *r_out, int *pa_out, int *pb_out) {
  const int K = c->K, Jp = c->Jp;
  uint32_t ra, rb, r;
  candidate_draw(c, (uint32_t)p, t, &ra, &rb, &r);     /* rotation: always the slot's own */
  *r_out = r;
  *pa_out = *pb_out = -1;
  if (p < K) {                                          /* refreshed survivor */
    const int32_t *src = prev + (size_t)c->sel[p] * Jp;
    for (int j = 0; j < Jp; ++j) g[j] = exponent_of(src[j]);
    *pa_out = c->sel[p];
  } else if (p < 3 * K) {                               /* uniform crossover */
    int q = (p - K) / 2, side = (p - K) % 2, p0 = K + 2 * q;
    uint32_t unused;
    candidate_draw(c, (uint32_t)p0, t, &ra, &rb, &unused);   /* both children share parents */
    const int32_t *A = prev + (size_t)c->sel[ra] * Jp;
    const int32_t *B = prev + (size_t)c->sel[rb] * Jp;
    if (c->per_gpu) {
      /* a child runs job j with the largest power-of-two GPU count among the GPUs it
       * inherited for it, at the job's local batch; the repair does the rest */
      int32_t cA[MAX_SLOTS], cB[MAX_SLOTS], n1[MAX_SLOTS], n2[MAX_SLOTS];
      for (int j = 0; j < Jp; ++j) { cA[j] = parent_gpus(&c->tab[j], A[j]); cB[j] = parent_gpus(&c->tab[j], B[j]); }
      uint64_t seed = ((uint64_t)c->key[1] << 32) | c->key[0];
      ones_ref_gpu_crossover(seed, (uint32_t)p0, t, c->G, Jp, cA, cB, n1, n2);
      for (int j = 0; j < Jp; ++j) {
        int32_t n = side == 0 ? n1[j] : n2[j];
        if (n == 0) { g[j] = WAIT; continue; }
        int lg = 0;
        while ((n >> (lg + 1)) != 0) ++lg;
        g[j] = imin(c->tab[j].mu, c->tab[j].hi) + lg;
      }
    } else
    for (int j = 0; j < Jp; ++j) {
      int swap = gene_word(c, (uint32_t)p0, t, j) < c->T_x;
      int from_b = side == 0 ? swap : !swap;            /* the children are complementary */
      g[j] = exponent_of(from_b ? B[j] : A[j]);
    }
    *pa_out = c->sel[ra]; *pb_out = c->sel[rb];
  } else {                                              /* uniform mutation */
    const int32_t *A = prev + (size_t)c->sel[ra] * Jp;
    for (int j = 0; j < Jp; ++j) {
      uint32_t w = gene_word(c, (uint32_t)p, t, j);
      const slot_t *s = &c->tab[j];
      if (w < c->T_mut) {
        uint32_t n = (uint32_t)(s->hi - s->lo + 2);
        uint32_t k = ((w & 0xFFFFu) * n) >> 16;         /* k = 0: the job is pre-empted */
        g[j] = gene_from_draw(s, k);
      } else {
        g[j] = exponent_of(A[j]);
      }
    }
    *pa_out = c->sel[ra];
  }
}

static void initial_genome(const ones_ref_ctx *c, int p, int *g, uint32_t *r_out) {
  uint32_t ra, rb;
  candidate_draw(c, (uint32_t)p, 0u, &ra, &rb, r_out);
  for (int j = 0; j < c->Jp; ++j) {
    const slot_t *s = &c->tab[j];
    uint32_t n = (uint32_t)(s->hi - s->lo + 2);
    g[j] = gene_from_draw(s, bounded(gene_word(c, (uint32_t)p, 0u, j), n));
  }
}

static void finish_slot(ones_ref_ctx *c, int32_t *dst, int p, int *g, uint32_t r) {
  repair(c->tab, c->Jp, c->R, c->G, g, r, c->serve_new ? c->is_new : NULL, c->t_processed ? c->by_time : NULL);
  c->fit[p] = score(c->tab, c->R, g);
  int32_t *row = dst + (size_t)p * c->Jp;
  for (int j = 0; j < c->Jp; ++j) row[j] = batch_of(g[j]);
}

/* ------------------------------------------------- probability sampling ---------- */
/* Natural logarithm of a positive normal double, by the textbook route: x = m * 2^e with m
 * in [sqrt(1/2), sqrt(2)), ln m = 2 artanh(s) with s = (m-1)/(m+1) = f/(2+f), f = m-1, and the
 * artanh series s + s^3/3 + s^5/5 + ... cut after s^23/23 (|s| < 0.1716, so the next term is
 * below 2e-20 of the first).  Every operation is a plain IEEE double operation in the order
 * written, so that any other implementation of these lines gives the same bits.  ln 2 is
 * split into a 32-bit head (e * head is exact) and a tail. */
double ones_ref_log(double x) {
  uint64_t bits;
  memcpy(&bits, &x, sizeof bits);
  int e = (int)((bits >> 52) & 0x7FF) - 1023;
  bits = (bits & 0x000FFFFFFFFFFFFFull) | 0x3FF0000000000000ull;
  double m;
  memcpy(&m, &bits, sizeof m);
  if (m > 1.4142135623730951) { m = m * 0.5; e = e + 1; }
  double f = m - 1.0;
  double s = f / (2.0 + f);
  double z = s * s;
  double p = 1.0 / 23.0;
  for (int k = 21; k >= 3; k -= 2) p = p * z + 1.0 / (double)k;
  double s2 = 2.0 * s;
  double lm = s2 + s2 * (z * p);
  double ef = (double)e;
  return ef * 0.6931471803691238 + (ef * 1.9082149292705877e-10 + lm);
}

/* Gamma(shape, 1), shape >= 1, by Marsaglia and Tsang's method (ACM TOMS 26, 2000): with
 * d = shape - 1/3 and c = 1/sqrt(9 d), draw x ~ N(0,1), v = (1 + c x)^3, and accept d*v when
 * v > 0 and ln u < x^2/2 + d - d v + d ln v for a uniform u.  The normal deviate comes from
 * the polar method (a point uniform in the unit disc, rejected outside).  Candidate draw
 * n = 0, 1, ... takes its four random words from Philox with counter (n, j, t, which):
 * words 0, 1 the point, words 2, 3 a 52-bit uniform.  After 64 rejected candidates the
 * draw gives up and returns d (probability below 1e-30). */
#define GAMMA_ATTEMPTS 64
double ones_ref_gamma_draw(uint64_t seed, uint32_t j, uint32_t t, uint32_t which, double shape,
                           int *attempts_out) {
  const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
  const double d = shape - 1.0 / 3.0;
  const double c = 1.0 / sqrt(9.0 * d);
  for (uint32_t n = 0; n < GAMMA_ATTEMPTS; ++n) {
    if (attempts_out) *attempts_out = (int)n + 1;
    const uint32_t ctr[4] = {n, j, t, which};
    uint32_t w[4];
    ones_ref_philox4x32_10(ctr, key, w);
    const double u1 = ((double)w[0] + 0.5) * (1.0 / 2147483648.0) - 1.0;    /* in (-1, 1) */
    const double u2 = ((double)w[1] + 0.5) * (1.0 / 2147483648.0) - 1.0;
    const double s = u1 * u1 + u2 * u2;
    if (s >= 1.0) continue;
    const double x = u1 * sqrt((-2.0 * ones_ref_log(s)) / s);
    const double t1 = 1.0 + c * x;
    if (t1 <= 0.0) continue;
    const double v = (t1 * t1) * t1;
    const uint64_t k = ((uint64_t)w[2] << 20) | (uint64_t)(w[3] >> 12);
    const double u = ((double)k + 0.5) * (1.0 / 4503599627370496.0);        /* in (0, 1) */
    const double bound = ((0.5 * (x * x) + d) - d * v) + d * ones_ref_log(v);
    if (ones_ref_log(u) < bound) return d * v;
  }
  return d;
}

/* rho ~ Be(alpha, beta) as Ga/(Ga + Gb) with independent Ga ~ Gamma(alpha), Gb ~ Gamma(beta);
 * then Eq. 7.  The ratio 1/rho - 1 and the product are capped at the largest parameter. */
double ones_ref_sampled_remaining(uint64_t seed, uint32_t j, uint32_t t, double alpha, double beta,
                                  double processed, double *rho_out) {
  const double ga = ones_ref_gamma_draw(seed, j, t, 1u, alpha, NULL);
  const double gb = ones_ref_gamma_draw(seed, j, t, 2u, beta, NULL);
  const double rho = ga / (ga + gb);
  if (rho_out) *rho_out = rho;
  double ratio = 1.0 / rho - 1.0;
  if (ratio > MAX_PARAM) ratio = MAX_PARAM;
  double y = processed * ratio;
  if (y > MAX_PARAM) y = MAX_PARAM;
  return y;
}

int ones_ref_set_progress(ones_ref_ctx *c, const double *alpha, const double *beta, const double *processed) {
  if (!c) return ONES_REF_E_INVALID_ARG;
  if (!alpha && !beta && !processed) {
    if (c->sampling) for (int j = 0; j < c->Jn; ++j) c->tab[j].Y = c->Y_fixed[j];
    c->sampling = 0;
    return ONES_REF_OK;
  }
  if (!alpha || !beta || !processed) return ONES_REF_E_INVALID_ARG;
  for (int j = 0; j < c->Jn; ++j) {
    if (!isfinite(alpha[j]) || !isfinite(beta[j]) || !isfinite(processed[j])) return ONES_REF_E_NONFINITE;
    if (alpha[j] < 1.0 || beta[j] < 1.0 || processed[j] < 0.0) return ONES_REF_E_INVALID_ARG;
    if (alpha[j] > MAX_PARAM || beta[j] > MAX_PARAM || processed[j] > MAX_PARAM) return ONES_REF_E_BOUNDS;
  }
  for (int j = 0; j < c->Jn; ++j) {
    c->alpha[j] = alpha[j]; c->beta[j] = beta[j]; c->processed[j] = processed[j];
  }
  c->sampling = 1;
  return ONES_REF_OK;
}

int ones_ref_set_crossover(ones_ref_ctx *c, int32_t mode) {
  if (!c || (mode != 0 && mode != 1)) return ONES_REF_E_INVALID_ARG;
  if (mode == 1 && c->G > 8192) return ONES_REF_E_BOUNDS;
  c->per_gpu = mode;
  return ONES_REF_OK;
}

int ones_ref_set_new_jobs_first(ones_ref_ctx *c, int32_t on) {
  if (!c) return ONES_REF_E_INVALID_ARG;
  c->new_jobs_first = on != 0;
  return ONES_REF_OK;
}

/* slots in ascending (time, slot) order: insertion into a sorted list, stable by construction */
static void order_by_time(const double *time, int Jp, int *out) {
  for (int j = 0; j < Jp; ++j) {
    int pos = j;
    while (pos > 0 && time[out[pos - 1]] > time[j]) { out[pos] = out[pos - 1]; --pos; }
    out[pos] = j;
  }
}

static int check_times(const double *t, int n) {
  for (int j = 0; j < n; ++j) {
    if (!isfinite(t[j])) return ONES_REF_E_NONFINITE;
    if (t[j] < 0.0) return ONES_REF_E_INVALID_ARG;
    if (t[j] > MAX_PARAM) return ONES_REF_E_BOUNDS;
  }
  return ONES_REF_OK;
}

int ones_ref_set_processed_time(ones_ref_ctx *c, const double *t_processed) {
  if (!c) return ONES_REF_E_INVALID_ARG;
  if (!t_processed) {
    free(c->t_processed); free(c->by_time);
    c->t_processed = NULL; c->by_time = NULL;
    return ONES_REF_OK;
  }
  int rc = check_times(t_processed, c->Jn);
  if (rc) return rc;
  if (!c->t_processed) {
    c->t_processed = (double *)calloc((size_t)c->Jp, sizeof(double));
    c->by_time = (int *)calloc((size_t)c->Jp, sizeof(int));
  }
  for (int j = 0; j < c->Jp; ++j) c->t_processed[j] = j < c->Jn ? t_processed[j] : 0.0;
  order_by_time(c->t_processed, c->Jp, c->by_time);
  return ONES_REF_OK;
}

int ones_ref_export_remaining(ones_ref_ctx *c, double *remaining_out) {
  if (!c || !remaining_out) return ONES_REF_E_INVALID_ARG;
  for (int j = 0; j < c->Jn; ++j) remaining_out[j] = c->tab[j].Y;
  return ONES_REF_OK;
}

/* ------------------------------------------------------------- public ------------ */
int ones_ref_init(ones_ref_ctx **out, const ones_ref_config *cfg, const ones_ref_jobs *jobs) {
  if (!out) return ONES_REF_E_INVALID_ARG;
  int rc = check_config(cfg);
  if (rc) return rc;
  ones_ref_ctx *c = (ones_ref_ctx *)calloc(1, sizeof(*c));
  c->G = cfg->n_gpus; c->Jn = cfg->n_slots; c->Jp = ones_ref_padded_jobs(cfg->n_slots);
  c->R = c->Jp / LANES; c->P = cfg->population; c->K = c->P / 4;
  c->key[0] = (uint32_t)cfg->seed; c->key[1] = (uint32_t)(cfg->seed >> 32);
  c->T_mut = rate_threshold(cfg->mutation_rate);
  c->T_x = rate_threshold(cfg->crossover_rate);
  c->tab = (slot_t *)malloc(sizeof(slot_t) * (size_t)c->Jp);
  rc = build_table(c->Jn, c->Jp, jobs, c->tab);
  if (rc) { free(c->tab); free(c); return rc; }
  size_t n = (size_t)c->P * c->Jp;
  c->genes[0] = (int32_t *)calloc(n, sizeof(int32_t));
  c->genes[1] = (int32_t *)calloc(n, sizeof(int32_t));
  c->fit = (double *)calloc((size_t)c->P, sizeof(double));
  c->sel = (int32_t *)calloc((size_t)c->K, sizeof(int32_t));
  size_t jn = (size_t)(c->Jn > 0 ? c->Jn : 1);
  c->alpha = (double *)calloc(jn, sizeof(double));
  c->beta = (double *)calloc(jn, sizeof(double));
  c->processed = (double *)calloc(jn, sizeof(double));
  c->Y_fixed = (double *)calloc(jn, sizeof(double));
  c->is_new = (uint8_t *)calloc((size_t)c->Jp, 1);
  for (int j = 0; j < c->Jn; ++j) c->Y_fixed[j] = c->tab[j].Y;
  c->cur = 0; c->t = 0;
  /* initial population: random genomes, repaired, scored, ranked */
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int p = 0; p < c->P; ++p) {
    int g[MAX_SLOTS]; uint32_t r;
    initial_genome(c, p, g, &r);
    finish_slot(c, c->genes[0], p, g, r);
  }
  ones_ref_select(c->fit, c->P, c->sel);
  *out = c;
  return ONES_REF_OK;
}

int ones_ref_set_jobs(ones_ref_ctx *c, const ones_ref_jobs *jobs) {
  if (!c) return ONES_REF_E_INVALID_ARG;
  slot_t *tab = (slot_t *)malloc(sizeof(slot_t) * (size_t)c->Jp);
  int rc = build_table(c->Jn, c->Jp, jobs, tab);
  if (rc) { free(tab); return rc; }
  /* a slot that changed hands starts from "waiting" in every candidate */
  memset(c->is_new, 0, (size_t)c->Jp);
  for (int j = 0; j < c->Jn; ++j) {
    if (tab[j].id == c->tab[j].id) continue;
    c->is_new[j] = 1;
    for (int p = 0; p < c->P; ++p) c->genes[c->cur][(size_t)p * c->Jp + j] = 0;
  }
  free(c->tab);
  c->tab = tab;
  c->stale = 1;
  for (int j = 0; j < c->Jn; ++j) c->Y_fixed[j] = tab[j].Y;
  return ONES_REF_OK;
}

int ones_ref_generation(ones_ref_ctx *c, int32_t n_generations) {
  if (!c || n_generations < 0) return ONES_REF_E_INVALID_ARG;
  if (c->t + n_generations > 0xFFFFFFFFll) return ONES_REF_E_INVALID_ARG;
  for (int32_t it = 0; it < n_generations; ++it) {
    const int32_t *prev = c->genes[c->cur];
    int32_t *next = c->genes[c->cur ^ 1];
    uint32_t t = (uint32_t)(c->t + 1);
    c->serve_new = c->new_jobs_first && c->stale;
    if (c->sampling) {               /* Alg. 1: one draw of every job's progress per selection */
      uint64_t seed = ((uint64_t)c->key[1] << 32) | c->key[0];
      for (int j = 0; j < c->Jn; ++j)
        c->tab[j].Y = ones_ref_sampled_remaining(seed, (uint32_t)j, t, c->alpha[j], c->beta[j],
                                                 c->processed[j], NULL);
    }
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int p = 0; p < c->P; ++p) {
      int g[MAX_SLOTS], pa, pb; uint32_t r;
      compose(c, prev, t, p, g, &r, &pa, &pb);
      finish_slot(c, next, p, g, r);
    }
    ones_ref_select(c->fit, c->P, c->sel);
    c->cur ^= 1;
    c->t += 1;
    c->stale = 0;
  }
  return ONES_REF_OK;
}

int ones_ref_best(ones_ref_ctx *c, int32_t *batch_out, int32_t *gpus_out, double *fitness_out) {
  if (!c) return ONES_REF_E_INVALID_ARG;
  int best = c->sel[0];                                 /* smallest score wins (Alg. 1) */
  const int32_t *row = c->genes[c->cur] + (size_t)best * c->Jp;
  for (int j = 0; j < c->Jn; ++j) {
    if (batch_out) batch_out[j] = row[j];
    if (gpus_out) gpus_out[j] = (int32_t)gpus_of(exponent_of(row[j]), c->tab[j].mu);
  }
  if (fitness_out) *fitness_out = c->fit[best];
  return ONES_REF_OK;
}

/* Eq. 1 for the winner after the reorder operator: walk the slots in order and hand each
 * running job its c_j GPUs, B_j / c_j samples each; what is left is idle. */
int ones_ref_placement(ones_ref_ctx *c, int32_t *slot_of_gpu, int32_t *batch_of_gpu) {
  if (!c || c->stale) return ONES_REF_E_INVALID_ARG;
  const int32_t *row = c->genes[c->cur] + (size_t)c->sel[0] * c->Jp;
  int gpu = 0;
  for (int j = 0; j < c->Jn; ++j) {
    int64_t gpus = gpus_of(exponent_of(row[j]), c->tab[j].mu);
    for (int64_t k = 0; k < gpus && gpu < c->G; ++k, ++gpu) {
      if (slot_of_gpu) slot_of_gpu[gpu] = j;
      if (batch_of_gpu) batch_of_gpu[gpu] = (int32_t)(row[j] / gpus);
    }
  }
  for (; gpu < c->G; ++gpu) {
    if (slot_of_gpu) slot_of_gpu[gpu] = -1;
    if (batch_of_gpu) batch_of_gpu[gpu] = 0;
  }
  return ONES_REF_OK;
}

/* ------------------------------------------------ batch-size limit policies ------ */
static int32_t floor_pow2(int64_t v) {
  int32_t p = 1;
  while ((int64_t)p * 2 <= v) p *= 2;
  return p;
}

int ones_ref_update_limits(int32_t n_slots, const ones_ref_limit_inputs *in, double sigma, int32_t *limit) {
  if (n_slots < 0 || n_slots > MAX_SLOTS) return ONES_REF_E_INVALID_ARG;
  if (n_slots > 0 && (!in || !limit || !in->state || !in->bmin || !in->bcap || !in->gpu_max_batch ||
                      !in->last_batch || !in->finished_epoch || !in->elapsed))
    return ONES_REF_E_INVALID_ARG;
  if (!isfinite(sigma)) return ONES_REF_E_NONFINITE;
  if (sigma < 0.0) return ONES_REF_E_INVALID_ARG;
  for (int j = 0; j < n_slots; ++j) {            /* check everything before changing anything */
    if (in->state[j] > 3) return ONES_REF_E_INVALID_ARG;
    if (in->state[j] == 0) continue;
    if (ilog2_exact(in->bmin[j]) < 0 || ilog2_exact(in->bcap[j]) < 0 || ilog2_exact(in->gpu_max_batch[j]) < 0)
      return ONES_REF_E_NOT_POW2;
    if (in->bmin[j] > in->bcap[j] || in->bcap[j] > (1 << 30)) return ONES_REF_E_BOUNDS;
    if (in->state[j] >= 2 && limit[j] < 1) return ONES_REF_E_INVALID_ARG;
    if (in->state[j] == 2 && in->last_batch[j] < 0) return ONES_REF_E_INVALID_ARG;
    if (in->state[j] == 3) {
      if (!isfinite(in->elapsed[j])) return ONES_REF_E_NONFINITE;
      if (in->elapsed[j] < 0.0) return ONES_REF_E_INVALID_ARG;
      if (sigma * in->elapsed[j] > 1e15) return ONES_REF_E_BOUNDS;
    }
  }
  for (int j = 0; j < n_slots; ++j) {
    int64_t r = limit[j];
    switch (in->state[j]) {
      case 0: limit[j] = 0; continue;
      case 1: r = in->gpu_max_batch[j]; break;                       /* Start: one GPU */
      case 2:                                                         /* Resume */
        if (in->last_batch[j] > 0) { if (r > in->last_batch[j]) r = in->last_batch[j]; }
        else r = r / 2;
        break;
      default:                                                        /* Scale-up and Scale-down */
        if (in->finished_epoch[j]) {
          int64_t den = (int64_t)ceil(sigma * in->elapsed[j] + 1.0);
          r = (2 * r + den - 1) / den;
        }
        break;
    }
    if (r < in->bmin[j]) r = in->bmin[j];
    if (r > in->bcap[j]) r = in->bcap[j];
    limit[j] = floor_pow2(r);
  }
  return ONES_REF_OK;
}

int ones_ref_export(ones_ref_ctx *c, int32_t *genes, double *fit, int32_t *sel, int64_t *generation) {
  if (!c) return ONES_REF_E_INVALID_ARG;
  if (genes) memcpy(genes, c->genes[c->cur], sizeof(int32_t) * (size_t)c->P * c->Jp);
  if (fit) memcpy(fit, c->fit, sizeof(double) * (size_t)c->P);
  if (sel) memcpy(sel, c->sel, sizeof(int32_t) * (size_t)c->K);
  if (generation) *generation = c->t;
  return ONES_REF_OK;
}

void ones_ref_destroy(ones_ref_ctx *c) {
  if (!c) return;
  free(c->tab); free(c->genes[0]); free(c->genes[1]); free(c->fit); free(c->sel);
  free(c->alpha); free(c->beta); free(c->processed); free(c->Y_fixed); free(c->is_new);
  free(c->t_processed); free(c->by_time); free(c);
}

int ones_ref_compose_slot(ones_ref_ctx *c, int32_t p, int32_t *genes_out, uint32_t *r_out,
                          int32_t *parent_a_out, int32_t *parent_b_out) {
  if (!c || p < 0 || p >= c->P || !genes_out) return ONES_REF_E_INVALID_ARG;
  int g[MAX_SLOTS], pa, pb; uint32_t r;
  compose(c, c->genes[c->cur], (uint32_t)(c->t + 1), p, g, &r, &pa, &pb);
  for (int j = 0; j < c->Jp; ++j) genes_out[j] = batch_of(g[j]);
  if (r_out) *r_out = r;
  if (parent_a_out) *parent_a_out = pa;
  if (parent_b_out) *parent_b_out = pb;
  return ONES_REF_OK;
}

/* single-genome entry points for the pins */
int ones_ref_initial_genome(const ones_ref_config *cfg, const ones_ref_jobs *jobs, int32_t p,
                            int32_t *genes_out, uint32_t *r_out) {
  int rc = check_config(cfg);
  if (rc) return rc;
  if (p < 0 || p >= cfg->population || !genes_out) return ONES_REF_E_INVALID_ARG;
  ones_ref_ctx c;
  memset(&c, 0, sizeof(c));
  c.Jn = cfg->n_slots; c.Jp = ones_ref_padded_jobs(cfg->n_slots); c.R = c.Jp / LANES;
  c.P = cfg->population; c.K = c.P / 4;
  c.key[0] = (uint32_t)cfg->seed; c.key[1] = (uint32_t)(cfg->seed >> 32);
  slot_t tab[MAX_SLOTS]; int g[MAX_SLOTS]; uint32_t r;
  if ((rc = build_table(c.Jn, c.Jp, jobs, tab))) return rc;
  c.tab = tab;
  initial_genome(&c, p, g, &r);
  for (int j = 0; j < c.Jn; ++j) genes_out[j] = batch_of(g[j]);
  if (r_out) *r_out = r;
  return ONES_REF_OK;
}

static int load_genome(const slot_t *tab, int Jn, int Jp, const int32_t *genes, int *g) {
  (void)tab;
  for (int j = 0; j < Jp; ++j) {
    int32_t b = j < Jn ? genes[j] : 0;
    if (b < 0) return ONES_REF_E_INVALID_ARG;
    int e = exponent_of(b);
    if (b != 0 && e < 0) return ONES_REF_E_NOT_POW2;
    g[j] = e;
  }
  return ONES_REF_OK;
}

int ones_ref_repair_genome(const ones_ref_config *cfg, const ones_ref_jobs *jobs,
                           int32_t *genes, uint32_t r, int32_t *fill_rounds_out) {
  int rc = check_config(cfg);
  if (rc) return rc;
  int Jn = cfg->n_slots, Jp = ones_ref_padded_jobs(Jn);
  if ((int64_t)r >= Jp || !genes) return ONES_REF_E_INVALID_ARG;
  slot_t tab[MAX_SLOTS]; int g[MAX_SLOTS];
  if ((rc = build_table(Jn, Jp, jobs, tab))) return rc;
  if ((rc = load_genome(tab, Jn, Jp, genes, g))) return rc;
  int rounds = repair(tab, Jp, Jp / LANES, cfg->n_gpus, g, r, NULL, NULL);
  for (int j = 0; j < Jn; ++j) genes[j] = batch_of(g[j]);
  if (fill_rounds_out) *fill_rounds_out = rounds;
  return ONES_REF_OK;
}

int ones_ref_repair_arrivals(const ones_ref_config *cfg, const ones_ref_jobs *jobs, int32_t *genes, uint32_t r,
                             const uint8_t *arrived, const double *t_processed, int32_t *fill_rounds_out) {
  int rc = check_config(cfg);
  if (rc) return rc;
  int Jn = cfg->n_slots, Jp = ones_ref_padded_jobs(Jn);
  if ((int64_t)r >= Jp || !genes || !arrived) return ONES_REF_E_INVALID_ARG;
  if (t_processed && (rc = check_times(t_processed, Jn))) return rc;
  slot_t tab[MAX_SLOTS]; int g[MAX_SLOTS];
  if ((rc = build_table(Jn, Jp, jobs, tab))) return rc;
  if ((rc = load_genome(tab, Jn, Jp, genes, g))) return rc;
  uint8_t is_new[MAX_SLOTS];
  double time[MAX_SLOTS];
  int by_time[MAX_SLOTS];
  for (int j = 0; j < Jp; ++j) {
    is_new[j] = j < Jn && arrived[j] != 0;
    time[j] = (t_processed && j < Jn) ? t_processed[j] : 0.0;
    if (is_new[j]) g[j] = WAIT;                 /* the slot changed hands: it starts from waiting */
  }
  order_by_time(time, Jp, by_time);
  int rounds = repair(tab, Jp, Jp / LANES, cfg->n_gpus, g, r, is_new, t_processed ? by_time : NULL);
  for (int j = 0; j < Jn; ++j) genes[j] = batch_of(g[j]);
  if (fill_rounds_out) *fill_rounds_out = rounds;
  return ONES_REF_OK;
}

int ones_ref_score_genome(const ones_ref_config *cfg, const ones_ref_jobs *jobs,
                          const int32_t *genes, double *fitness_out) {
  int rc = check_config(cfg);
  if (rc) return rc;
  int Jn = cfg->n_slots, Jp = ones_ref_padded_jobs(Jn);
  if (!genes || !fitness_out) return ONES_REF_E_INVALID_ARG;
  slot_t tab[MAX_SLOTS]; int g[MAX_SLOTS];
  if ((rc = build_table(Jn, Jp, jobs, tab))) return rc;
  if ((rc = load_genome(tab, Jn, Jp, genes, g))) return rc;
  for (int j = 0; j < Jp; ++j) if (!tab[j].active) g[j] = WAIT;
  *fitness_out = score(tab, Jp / LANES, g);
  return ONES_REF_OK;
}
