/*
 * CPU oracle for ExDyna's per-iteration gradient-selection path.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, single-threaded
 * transcription of the paper's definitions (Alg. 1-5, Eq. 1, 5, 6) used to
 * check the GPU library and as the timed CPU baseline.  Nothing in the
 * product path may include, link or call it, and it shares no code with the
 * HIP kernels.
 *
 * Precision: the gradient data and the residual are fp32 (the tensors the
 * paper's implementation operates on); one accumulate is one fp32 add.  All
 * control arithmetic (partial-k vector, det/det2, k_move, exam) is fp64.
 * The threshold is an fp32 scalar scaled by an fp32 factor.
 *
 * Pins: every function below is pinned by tests that do not call it to
 * produce their expectation (hand-evaluated cases stored as text fixtures,
 * numpy sort / nonzero brute force, invariants).  The output-capacity rule
 * and the default hyper-parameters are this build's reading, not the
 * paper's: "parity unpinned" for those two (see exo_step).  The n-worker
 * form (exo_workers_*) is pinned by the same definitions written in numpy,
 * by its reduction to the one-device form for n = 1 and for identical
 * gradients, and by Alg. 3 (cyclic allocation) for the re-indexing ahead of the sweep; the
 * order of the AllReduce sum (rank order) is this build's reading.
 */
#ifndef EXDYNA_ORACLE_H
#define EXDYNA_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Alg. 2 (block size): block size from a block count: floor(n_g / n_b) rounded
 * down to a multiple of 32. */
uint64_t exo_block_size(uint64_t n_g, uint64_t n_b);

/* Alg. 2 (topology): initial topology.  blk_part[i] = quotient (+1 for the
 * first `remainder` partitions); blk_pos = exclusive prefix sum. */
void exo_partition(uint64_t n_b, uint32_t n, int64_t *blk_part, int64_t *blk_pos);

/* Alg. 3 (the sweep over adjacent pairs): one sweep over adjacent partition pairs.  kvec (fp64,
 * length n) is the partial-k vector in partition order and is updated in
 * place, as are blk_part / blk_pos.  A sum of zero (nothing selected) leaves
 * everything unchanged.  Returns the number of boundary moves made. */
int exo_allocate(double *kvec, int64_t *blk_part, int64_t *blk_pos, uint32_t n,
                 uint64_t n_g, uint64_t sz_blk, int64_t blk_move, int64_t min_blk,
                 double alpha);

/* Alg. 3 (cyclic allocation): the partition that worker `rank` owns at iteration t. */
uint32_t exo_owner(uint64_t t, uint32_t rank, uint32_t n);

/* Alg. 4: ascending indices i in [st, end) with |acc[i]| >= delta
 * (cmp_mode 0, the paper's comparator) or > delta (cmp_mode 1).  Writes at
 * most `cap` indices to out_idx (may be NULL when cap == 0) and returns the
 * full count. */
uint64_t exo_select(const float *acc, uint64_t st, uint64_t end, float delta,
                    int cmp_mode, uint32_t *out_idx, uint64_t cap);

/* Alg. 5: scaling factor chosen from exam = k'/k against beta and 1/beta,
 * returned as fp32; the caller multiplies the fp32 threshold by it. */
float exo_scale_factor(double k, double k_actual, double beta, double gamma);
float exo_estimate(double k, double k_actual, float delta, double beta, double gamma);

/* ---- whole-step state machine (Alg. 1 (initialisation and iteration body)) ------------- */

typedef struct exo_state exo_state;

/* Returns NULL on invalid arguments or allocation failure.  cap = 0 selects
 * the default capacity max(ceil(4k), 1024) clamped to n_g. */
exo_state *exo_create(uint64_t n_g, uint32_t block_size, uint32_t n_parts,
                      double density, float threshold0, double alpha, double beta,
                      double gamma, uint32_t blk_move, uint32_t min_blk,
                      uint32_t cmp_mode, uint64_t cap);
void exo_destroy(exo_state *s);

/* One iteration on gradient g (n_g fp32, already scaled by the learning
 * rate).  Order follows Alg. 1: accumulate, Allocate, Sparsify every
 * partition in ascending partition order, count, Estimate, zero selected,
 * carry the residual. */
void exo_step(exo_state *s, const float *g);

/* The same iteration with Alg. 1 (accumulate) as printed, acc = e + eta * G, for
 * gradients stored as fp32 (dtype 0), bf16 (1) or fp16 (2): fl(e + fl(eta * g)). */
void exo_step_scaled(exo_state *s, const void *g, int dtype, float eta);

/* Accessors: pointers stay valid until the next exo_step / exo_destroy. */
uint64_t        exo_n_blocks(const exo_state *s);
uint64_t        exo_capacity(const exo_state *s);
uint64_t        exo_iteration(const exo_state *s);      /* t of the NEXT step */
float           exo_threshold(const exo_state *s);      /* delta for the next step */
float           exo_threshold_used(const exo_state *s); /* delta the last step compared with */
float          *exo_residual(exo_state *s);             /* n_g */
const uint32_t *exo_out_idx(const exo_state *s);        /* k_emitted */
const float    *exo_out_val(const exo_state *s);        /* k_emitted */
const uint64_t *exo_part_off(const exo_state *s);       /* P+1, clamped to capacity */
const uint64_t *exo_part_count(const exo_state *s);     /* P, untruncated */
const uint32_t *exo_block_count(const exo_state *s);    /* n_b, untruncated */
uint64_t        exo_k_actual(const exo_state *s);
uint64_t        exo_k_emitted(const exo_state *s);
/* which = 0: topology the last step selected with; 1: current (next step's
 * input to Allocate). */
const int64_t  *exo_blk_part(const exo_state *s, int which);
const int64_t  *exo_blk_pos(const exo_state *s, int which);
double          exo_err_norm(const exo_state *s);  /* Eq. 1, one worker: ||e_{t+1}||_2 */
double          exo_density_error(const exo_state *s); /* Eq. 6 */
double          exo_traffic_ratio(const exo_state *s); /* Eq. 5; 0 when k' = 0 */

/* ---- Alg. 1 with n workers (each its own gradient and residual) ------- */

/* Alg. 3 (re-indexing of the partial-k vector): partial-k vector from rank order (as all-gathered after
 * iteration t-1) to partition order, k_part[((t-1) mod n + i) mod n] = k_rank[i]. */
void exo_reindex(const double *k_rank, uint32_t n, uint64_t t, double *k_part);

typedef struct exo_workers exo_workers;

/* Same arguments and checks as exo_create; n workers = n partitions.  The
 * capacity is per worker (each worker's own index list). */
exo_workers *exo_workers_create(uint64_t n_g, uint32_t block_size, uint32_t n,
                                double density, float threshold0, double alpha, double beta,
                                double gamma, uint32_t blk_move, uint32_t min_blk,
                                uint32_t cmp_mode, uint64_t cap);
void exo_workers_destroy(exo_workers *s);

/* One iteration of Alg. 1 (the iteration body) for all workers; g[i] = worker i's
 * gradient (n_g fp32, learning rate applied).  AllGather concatenates the
 * workers' lists in rank order; AllReduce sums in rank order in fp32. */
void exo_workers_step(exo_workers *s, const float *const *g);

uint64_t        exo_workers_capacity(const exo_workers *s);
uint64_t        exo_workers_n_blocks(const exo_workers *s);
uint64_t        exo_workers_iteration(const exo_workers *s);
float           exo_workers_threshold(const exo_workers *s);
float           exo_workers_threshold_used(const exo_workers *s);
float          *exo_workers_residual(exo_workers *s, uint32_t i);      /* e_i, n_g */
const uint64_t *exo_workers_k_rank(const exo_workers *s);              /* k_{i,t}, n, untruncated */
const uint64_t *exo_workers_rank_off(const exo_workers *s);            /* n+1 offsets into idx_t */
const uint32_t *exo_workers_idx(const exo_workers *s);                 /* idx_t */
const float    *exo_workers_values(const exo_workers *s, uint32_t i);  /* g_i = acc_i[idx_t] */
const float    *exo_workers_sum(const exo_workers *s);                 /* g_t */
uint64_t        exo_workers_k_actual(const exo_workers *s);            /* k' */
const int64_t  *exo_workers_blk_part(const exo_workers *s, int which);
const int64_t  *exo_workers_blk_pos(const exo_workers *s, int which);
double          exo_workers_err_norm(const exo_workers *s, uint32_t i); /* Eq. 1; i == n: the mean */
double          exo_workers_traffic_ratio(const exo_workers *s);        /* Eq. 5 */

/* Eq. 2-4: the padding an AllGather of equal-sized lists adds, C_t = n * sum_i
 * (max_j k_j - k_i), from the n selection counts of one iteration. */
uint64_t exo_padding_overhead(const uint64_t *k, uint32_t n);

/* Alg. 1 (model update) restricted to the sent entries: x[idx_t[j]] -= scale * g_t[j]
 * (scale = 1/n; fp32 product, then fp32 difference). */
void exo_apply_update(float *x, const uint32_t *idx_t, const float *g_t, uint64_t len, float scale);

#ifdef __cplusplus
}
#endif
#endif
