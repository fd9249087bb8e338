/*
 * CPU oracle for ExDyna's per-iteration gradient-selection path.
 * TEST INFRASTRUCTURE ONLY -- see exdyna_oracle.h.
 *
 * Written from the paper's definitions, one plain loop per statement, in
 * the paper's order.  No blocking, fusion or threading.
 * Build: gcc -O2 -std=c99 -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include "exdyna_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Alg. 2 (block size)                                                   */
uint64_t exo_block_size(uint64_t n_g, uint64_t n_b)
{
    if (n_b == 0) return 0;
    uint64_t temp = n_g / n_b;
    return temp - temp % 32;
}

/* Alg. 2 (topology), Sec. 4.1: the n_b blocks are dealt to the n partitions as evenly as whole
 * blocks allow -- every partition holds floor(n_b / n) blocks and the first n_b mod n of them
 * hold one more -- and a partition starts where the one before it ends.                     */
void exo_partition(uint64_t n_b, uint32_t n, int64_t *blk_part, int64_t *blk_pos)
{
    const int64_t share = (int64_t)(n_b / n);
    const int64_t extra = (int64_t)(n_b % n);
    int64_t first = 0;
    for (uint32_t p = 0; p < n; ++p) {
        blk_part[p] = share + ((int64_t)p < extra ? 1 : 0);
        blk_pos[p]  = first;
        first += blk_part[p];
    }
}

/* Alg. 3 (the sweep over adjacent pairs), Sec. 4.2.  A partition's load is its count of the
 * last iteration over the fair share k'/n.  Walking the shared boundaries left to right, a
 * boundary moves by blk_move blocks toward the overloaded side's interior when one side's load
 * is above alpha and the other's below 1/alpha, unless the side that gives blocks away would
 * be left with fewer than min_blk.  The counts are then corrected by what the moved blocks are
 * expected to hold at the last iteration's overall density, so the next pair sees the
 * corrected count of the partition the two pairs share.  kvec is indexed by partition: the
 * re-indexing from rank order that precedes the sweep is the caller's.  alpha >= 1 makes the
 * two cases exclude each other.  Returns the number of boundaries moved.                    */
int exo_allocate(double *kvec, int64_t *blk_part, int64_t *blk_pos, uint32_t n,
                 uint64_t n_g, uint64_t sz_blk, int64_t blk_move, int64_t min_blk,
                 double alpha)
{
    double selected = 0.0;
    for (uint32_t p = 0; p < n; ++p) selected += kvec[p];
    /* Nothing selected: every load would be 0/0.  No boundary moves. */
    if (!(selected > 0.0)) return 0;

    const double fair_share = selected / (double)n;
    const double density    = selected / (double)n_g;
    const double carried    = (double)blk_move * (double)sz_blk * density; /* count that moves along */
    const double low        = 1.0 / alpha;
    int moved = 0;

    for (uint32_t left = 0; left + 1 < n; ++left) {
        const uint32_t right = left + 1;
        const double load_left  = kvec[left] / fair_share;
        const double load_right = kvec[right] / fair_share;
        if (load_left > alpha && load_right < low) {
            /* the left partition hands its last blocks to the right one */
            if (blk_part[left] - blk_move < min_blk) continue;
            blk_part[left]  -= blk_move;
            blk_part[right] += blk_move;
            blk_pos[right]  -= blk_move;
            kvec[left]      -= carried;
            kvec[right]     += carried;
            ++moved;
        } else if (load_left < low && load_right > alpha) {
            /* the right partition hands its first blocks to the left one */
            if (blk_part[right] - blk_move < min_blk) continue;
            blk_part[left]  += blk_move;
            blk_part[right] -= blk_move;
            blk_pos[right]  += blk_move;
            kvec[left]      += carried;
            kvec[right]     -= carried;
            ++moved;
        }
    }
    return moved;
}

/* Alg. 3 (cyclic allocation)                                                     */
uint32_t exo_owner(uint64_t t, uint32_t rank, uint32_t n)
{
    return (uint32_t)((t % n + rank) % n);
}

/* Alg. 4: where(|g[st:end]| >= delta) + st                            */
uint64_t exo_select(const float *acc, uint64_t st, uint64_t end, float delta,
                    int cmp_mode, uint32_t *out_idx, uint64_t cap)
{
    uint64_t count = 0;
    for (uint64_t i = st; i < end; ++i) {
        float a = fabsf(acc[i]);
        int sel = cmp_mode ? (a > delta) : (a >= delta);
        if (sel) {
            if (count < cap) out_idx[count] = (uint32_t)i;
            ++count;
        }
    }
    return count;
}

/* Alg. 5 (choice of the scaling factor)                                                   */
float exo_scale_factor(double k, double k_actual, double beta, double gamma)
{
    double exam = k_actual / k;
    double sf;
    if (exam > beta)
        sf = 1.0 + gamma;
    else if (exam > 1.0 / beta)
        sf = 1.0 + 0.25 * gamma;
    else
        sf = 1.0 - gamma;
    return (float)sf;
}

/* Alg. 5 (threshold scaling)                                                      */
float exo_estimate(double k, double k_actual, float delta, double beta, double gamma)
{
    float sf = exo_scale_factor(k, k_actual, beta, gamma);
    return delta * sf;
}

/* ------------------------------------------------------------------ */
struct exo_state {
    uint64_t n_g, n_b, cap, t;
    uint32_t b, n, blk_move, min_blk, cmp_mode;
    double   k, alpha, beta, gamma;
    float    delta, delta_used;
    float   *e;                  /* residual; holds acc during a step */
    double  *kvec;               /* partial-k vector, partition order */
    int64_t *blk_part, *blk_pos; /* current topology */
    int64_t *used_part, *used_pos; /* topology the last step selected with */
    uint32_t *out_idx;
    float    *out_val;
    uint64_t *part_off, *part_cnt;
    uint32_t *blk_cnt;
    uint64_t k_actual, k_emitted;
};

exo_state *exo_create(uint64_t n_g, uint32_t block_size, uint32_t n_parts,
                      double density, float threshold0, double alpha, double beta,
                      double gamma, uint32_t blk_move, uint32_t min_blk,
                      uint32_t cmp_mode, uint64_t cap)
{
    if (n_g == 0 || n_g > 0xFFFFFFFFull) return NULL;
    if (block_size == 0 || block_size % 32 != 0) return NULL;
    uint64_t n_b = (n_g + block_size - 1) / block_size;
    if (n_parts == 0 || n_parts > n_b) return NULL;
    if (!(density > 0.0 && density <= 1.0)) return NULL;
    if (!(threshold0 > 0.0f) || isinf(threshold0)) return NULL;
    if (!(alpha >= 1.0) || !(beta > 1.0) || !(gamma >= 0.0 && gamma < 1.0)) return NULL;
    if (min_blk == 0 || cmp_mode > 1) return NULL;

    exo_state *s = (exo_state *)calloc(1, sizeof *s);
    if (!s) return NULL;
    s->n_g = n_g; s->b = block_size; s->n = n_parts; s->n_b = n_b;
    s->k = density * (double)n_g;
    s->alpha = alpha; s->beta = beta; s->gamma = gamma;
    s->blk_move = blk_move; s->min_blk = min_blk; s->cmp_mode = cmp_mode;
    if (cap == 0) {
        double c = ceil(4.0 * s->k);
        cap = c < 1024.0 ? 1024 : (uint64_t)c;
    }
    if (cap > n_g) cap = n_g;
    s->cap = cap;
    s->delta = threshold0;          /* Alg. 1 (threshold initialisation) */
    s->delta_used = threshold0;
    s->t = 0;

    s->e         = (float *)calloc(n_g, sizeof(float));        /* Alg. 1 (local-error initialisation) */
    s->kvec      = (double *)malloc(n_parts * sizeof(double));
    s->blk_part  = (int64_t *)malloc(n_parts * sizeof(int64_t));
    s->blk_pos   = (int64_t *)malloc(n_parts * sizeof(int64_t));
    s->used_part = (int64_t *)malloc(n_parts * sizeof(int64_t));
    s->used_pos  = (int64_t *)malloc(n_parts * sizeof(int64_t));
    s->out_idx   = (uint32_t *)malloc(cap * sizeof(uint32_t));
    s->out_val   = (float *)malloc(cap * sizeof(float));
    s->part_off  = (uint64_t *)calloc(n_parts + 1, sizeof(uint64_t));
    s->part_cnt  = (uint64_t *)calloc(n_parts, sizeof(uint64_t));
    s->blk_cnt   = (uint32_t *)calloc(n_b, sizeof(uint32_t));
    if (!s->e || !s->kvec || !s->blk_part || !s->blk_pos || !s->used_part ||
        !s->used_pos || !s->out_idx || !s->out_val || !s->part_off ||
        !s->part_cnt || !s->blk_cnt) {
        exo_destroy(s);
        return NULL;
    }
    for (uint32_t i = 0; i < n_parts; ++i)                      /* Alg. 1 (partial-k initialisation) */
        s->kvec[i] = s->k / (double)n_parts;
    exo_partition(n_b, n_parts, s->blk_part, s->blk_pos);       /* Alg. 1 (partition initialisation) */
    memcpy(s->used_part, s->blk_part, n_parts * sizeof(int64_t));
    memcpy(s->used_pos, s->blk_pos, n_parts * sizeof(int64_t));
    return s;
}

void exo_destroy(exo_state *s)
{
    if (!s) return;
    free(s->e); free(s->kvec); free(s->blk_part); free(s->blk_pos);
    free(s->used_part); free(s->used_pos); free(s->out_idx); free(s->out_val);
    free(s->part_off); free(s->part_cnt); free(s->blk_cnt);
    free(s);
}

static void step_after_accumulate(exo_state *s);

void exo_step(exo_state *s, const float *g)
{
    const uint64_t n_g = s->n_g;
    float *acc = s->e;

    /* Alg. 1 (accumulate): acc = e + g (g carries the learning rate already). */
    for (uint64_t i = 0; i < n_g; ++i) {
        float a = acc[i] + g[i];
        acc[i] = a;
    }
    step_after_accumulate(s);
}

/* bf16 is the upper half of an fp32. */
static float bf16_to_float(uint16_t h)
{
    uint32_t bits = (uint32_t)h << 16;
    float v;
    memcpy(&v, &bits, sizeof v);
    return v;
}

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
static float half_to_float(uint16_t h)
{
    uint32_t sign = (h >> 15) & 1u, ex = (h >> 10) & 31u, man = h & 1023u;
    float v;
    if (ex == 0)
        v = ldexpf((float)man, -24);                       /* subnormal or zero */
    else if (ex == 31)
        v = man ? NAN : INFINITY;
    else
        v = ldexpf((float)(man | 1024u), (int)ex - 25);    /* 1.f x 2^(ex-15) */
    return sign ? -v : v;
}

/* Alg. 1 (accumulate) as printed: acc = e + eta * G, with G in fp32 (dtype 0), bf16
 * (1) or fp16 (2).  The gradient is widened exactly, the product is rounded
 * to fp32, then the sum is rounded to fp32 (no fused multiply-add: the file
 * is built with -ffp-contract=off). */
void exo_step_scaled(exo_state *s, const void *g, int dtype, float eta)
{
    const uint64_t n_g = s->n_g;
    float *acc = s->e;
    for (uint64_t i = 0; i < n_g; ++i) {
        float gi;
        if (dtype == 0)
            gi = ((const float *)g)[i];
        else if (dtype == 1)
            gi = bf16_to_float(((const uint16_t *)g)[i]);
        else
            gi = half_to_float(((const uint16_t *)g)[i]);
        float p = eta * gi;
        float a = acc[i] + p;
        acc[i] = a;
    }
    step_after_accumulate(s);
}

static void step_after_accumulate(exo_state *s)
{
    const uint64_t n_g = s->n_g;
    const uint32_t n = s->n;
    float *acc = s->e;

    /* Alg. 1 (Allocate): Allocate adjusts the topology from last iteration's
     * per-partition counts; selection below uses the adjusted topology. */
    exo_allocate(s->kvec, s->blk_part, s->blk_pos, n, n_g, s->b,
                 (int64_t)s->blk_move, (int64_t)s->min_blk, s->alpha);
    memcpy(s->used_part, s->blk_part, n * sizeof(int64_t));
    memcpy(s->used_pos, s->blk_pos, n * sizeof(int64_t));

    /* Alg. 1 (Sparsify, AllGather, value gather): every partition is selected by exactly one worker
     * (Alg. 3 (cyclic allocation) is a bijection rank -> partition at fixed t), so on
     * one device the gathered index list is the partitions' lists; they are
     * laid out here in ascending partition order. */
    const float delta = s->delta;
    s->delta_used = delta;
    memset(s->blk_cnt, 0, s->n_b * sizeof(uint32_t));
    uint64_t emitted = 0, total = 0;
    for (uint32_t p = 0; p < n; ++p) {
        /* Alg. 3 (partition range), with the last block allowed to be short. */
        uint64_t st  = (uint64_t)s->used_pos[p] * s->b;
        uint64_t end = (uint64_t)(s->used_pos[p] + s->used_part[p]) * s->b;
        if (end > n_g) end = n_g;
        if (st > n_g) st = n_g;
        s->part_off[p] = emitted;
        uint64_t room = s->cap - emitted;
        /* Alg. 4 */
        uint64_t cnt = exo_select(acc, st, end, delta, (int)s->cmp_mode,
                                  s->out_idx + emitted, room);
        uint64_t take = cnt < room ? cnt : room;
        /* per-block counts (scaffold for the device compaction; untruncated) */
        for (uint64_t i = st; i < end; ++i) {
            float a = fabsf(acc[i]);
            int sel = s->cmp_mode ? (a > delta) : (a >= delta);
            if (sel) s->blk_cnt[i / s->b] += 1;
        }
        /* Alg. 1 (value gather): values at the selected indices. */
        for (uint64_t j = 0; j < take; ++j)
            s->out_val[emitted + j] = acc[s->out_idx[emitted + j]];
        s->part_cnt[p] = cnt;
        emitted += take;
        total += cnt;
    }
    s->part_off[n] = emitted;
    s->k_actual = total;        /* Alg. 1 (k' sum) */
    s->k_emitted = emitted;

    /* Alg. 1 (Estimate): Estimate. */
    s->delta = exo_estimate(s->k, (double)total, delta, s->beta, s->gamma);

    /* Alg. 1 (AllGather counts, partial-k carry): the partial-k vector for the next Allocate. */
    for (uint32_t p = 0; p < n; ++p) s->kvec[p] = (double)s->part_cnt[p];

    /* Alg. 1 (zeroing of the sent entries): zero what was sent (only what fitted the output). */
    for (uint64_t j = 0; j < emitted; ++j) acc[s->out_idx[j]] = 0.0f;

    /* Alg. 1 (residual carry): e_{t+1} = acc (same buffer). */
    s->t += 1;
}

uint64_t        exo_n_blocks(const exo_state *s)       { return s->n_b; }
uint64_t        exo_capacity(const exo_state *s)       { return s->cap; }
uint64_t        exo_iteration(const exo_state *s)      { return s->t; }
float           exo_threshold(const exo_state *s)      { return s->delta; }
float           exo_threshold_used(const exo_state *s) { return s->delta_used; }
float          *exo_residual(exo_state *s)             { return s->e; }
const uint32_t *exo_out_idx(const exo_state *s)        { return s->out_idx; }
const float    *exo_out_val(const exo_state *s)        { return s->out_val; }
const uint64_t *exo_part_off(const exo_state *s)       { return s->part_off; }
const uint64_t *exo_part_count(const exo_state *s)     { return s->part_cnt; }
const uint32_t *exo_block_count(const exo_state *s)    { return s->blk_cnt; }
uint64_t        exo_k_actual(const exo_state *s)       { return s->k_actual; }
uint64_t        exo_k_emitted(const exo_state *s)      { return s->k_emitted; }
const int64_t  *exo_blk_part(const exo_state *s, int which) { return which ? s->blk_part : s->used_part; }
const int64_t  *exo_blk_pos(const exo_state *s, int which)  { return which ? s->blk_pos : s->used_pos; }

/* Eq. 1 with one worker: the L2 norm of the residual, summed in fp64. */
double exo_err_norm(const exo_state *s)
{
    double acc = 0.0;
    for (uint64_t i = 0; i < s->n_g; ++i) {
        double v = (double)s->e[i];
        acc += v * v;
    }
    return sqrt(acc);
}

/* Eq. 6: |k - k'| / n_g */
double exo_density_error(const exo_state *s)
{
    return fabs(s->k - (double)s->k_actual) / (double)s->n_g;
}

/* Eq. 5: n * max_i k_i / k' */
double exo_traffic_ratio(const exo_state *s)
{
    if (s->k_actual == 0) return 0.0;
    uint64_t m = 0;
    for (uint32_t p = 0; p < s->n; ++p)
        if (s->part_cnt[p] > m) m = s->part_cnt[p];
    return (double)s->n * (double)m / (double)s->k_actual;
}

/* ================================================================== */
/* Alg. 1 with n workers, each with its own gradient and residual.     */
/* One statement of the algorithm = one loop below, workers in rank    */
/* order; the two collectives are plain loops over the workers.        */

/* Alg. 3 (re-indexing of the partial-k vector): the all-gathered partial-k vector is indexed by rank;
 * rank i selected partition ((t-1) mod n + i) mod n at iteration t-1, so
 * temp[that partition] = k_t[i].  The modulo is the mathematical one
 * ((-1) mod n = n-1), which only matters at t = 0. */
void exo_reindex(const double *k_rank, uint32_t n, uint64_t t, double *k_part)
{
    uint64_t shift = (t == 0) ? (uint64_t)(n - 1) : (t - 1) % n;
    for (uint32_t i = 0; i < n; ++i) {
        uint32_t j = (uint32_t)((shift + i) % n);
        k_part[j] = k_rank[i];
    }
}

struct exo_workers {
    uint64_t n_g, n_b, cap, t;
    uint32_t b, n, blk_move, min_blk, cmp_mode;
    double   k, alpha, beta, gamma;
    float    delta, delta_used;
    float  **e;                    /* e[i]: worker i's residual; holds acc_i during a step */
    double  *k_t;                  /* partial-k vector in RANK order, as all-gathered */
    double  *temp;                 /* the same in partition order */
    int64_t *blk_part, *blk_pos, *used_part, *used_pos;
    uint32_t **idx;                /* idx[i]: worker i's own index list */
    uint64_t *k_rank;              /* k_{i,t}, untruncated */
    uint64_t *rank_off;            /* n+1 offsets of the workers' lists inside idx_t */
    uint32_t *idx_t;               /* gathered list, rank order */
    float  **g;                    /* g[i] = acc_i[idx_t] */
    float   *g_t;                  /* sum over workers */
    uint64_t k_actual;
};

void exo_workers_destroy(exo_workers *s)
{
    if (!s) return;
    for (uint32_t i = 0; i < s->n; ++i) {
        if (s->e) free(s->e[i]);
        if (s->idx) free(s->idx[i]);
        if (s->g) free(s->g[i]);
    }
    free(s->e); free(s->idx); free(s->g);
    free(s->k_t); free(s->temp); free(s->blk_part); free(s->blk_pos);
    free(s->used_part); free(s->used_pos); free(s->k_rank); free(s->rank_off);
    free(s->idx_t); free(s->g_t);
    free(s);
}

exo_workers *exo_workers_create(uint64_t n_g, uint32_t block_size, uint32_t n,
                                double density, float threshold0, double alpha, double beta,
                                double gamma, uint32_t blk_move, uint32_t min_blk,
                                uint32_t cmp_mode, uint64_t cap)
{
    if (n_g == 0 || n_g > 0xFFFFFFFFull) return NULL;
    if (block_size == 0 || block_size % 32 != 0) return NULL;
    uint64_t n_b = (n_g + block_size - 1) / block_size;
    if (n == 0 || n > n_b) return NULL;
    if (!(density > 0.0 && density <= 1.0)) return NULL;
    if (!(threshold0 > 0.0f) || isinf(threshold0)) return NULL;
    if (!(alpha >= 1.0) || !(beta > 1.0) || !(gamma >= 0.0 && gamma < 1.0)) return NULL;
    if (min_blk == 0 || cmp_mode > 1) return NULL;

    exo_workers *s = (exo_workers *)calloc(1, sizeof *s);
    if (!s) return NULL;
    s->n_g = n_g; s->b = block_size; s->n = n; s->n_b = n_b;
    s->k = density * (double)n_g;
    s->alpha = alpha; s->beta = beta; s->gamma = gamma;
    s->blk_move = blk_move; s->min_blk = min_blk; s->cmp_mode = cmp_mode;
    if (cap == 0) {
        double c = ceil(4.0 * s->k);
        cap = c < 1024.0 ? 1024 : (uint64_t)c;
    }
    if (cap > n_g) cap = n_g;
    s->cap = cap;
    s->delta = threshold0;
    s->delta_used = threshold0;

    s->e   = (float **)calloc(n, sizeof(float *));
    s->idx = (uint32_t **)calloc(n, sizeof(uint32_t *));
    s->g   = (float **)calloc(n, sizeof(float *));
    s->k_t = (double *)malloc(n * sizeof(double));
    s->temp = (double *)malloc(n * sizeof(double));
    s->blk_part = (int64_t *)malloc(n * sizeof(int64_t));
    s->blk_pos = (int64_t *)malloc(n * sizeof(int64_t));
    s->used_part = (int64_t *)malloc(n * sizeof(int64_t));
    s->used_pos = (int64_t *)malloc(n * sizeof(int64_t));
    s->k_rank = (uint64_t *)calloc(n, sizeof(uint64_t));
    s->rank_off = (uint64_t *)calloc(n + 1, sizeof(uint64_t));
    s->idx_t = (uint32_t *)malloc(n * cap * sizeof(uint32_t));
    s->g_t = (float *)malloc(n * cap * sizeof(float));
    int ok = s->e && s->idx && s->g && s->k_t && s->temp && s->blk_part && s->blk_pos &&
             s->used_part && s->used_pos && s->k_rank && s->rank_off && s->idx_t && s->g_t;
    for (uint32_t i = 0; ok && i < n; ++i) {
        s->e[i]   = (float *)calloc(n_g, sizeof(float));            /* Alg. 1 (local-error initialisation) */
        s->idx[i] = (uint32_t *)malloc(cap * sizeof(uint32_t));
        s->g[i]   = (float *)malloc(n * cap * sizeof(float));
        ok = s->e[i] && s->idx[i] && s->g[i];
    }
    if (!ok) {
        exo_workers_destroy(s);
        return NULL;
    }
    for (uint32_t i = 0; i < n; ++i) s->k_t[i] = s->k / (double)n;  /* Alg. 1 (partial-k initialisation) */
    exo_partition(n_b, n, s->blk_part, s->blk_pos);                  /* Alg. 1 (partition initialisation) */
    memcpy(s->used_part, s->blk_part, n * sizeof(int64_t));
    memcpy(s->used_pos, s->blk_pos, n * sizeof(int64_t));
    return s;
}

/* One iteration of Alg. 1 for all n workers.  g[i] is worker i's gradient,
 * already scaled by the learning rate (n_g fp32 each). */
void exo_workers_step(exo_workers *s, const float *const *g)
{
    const uint64_t n_g = s->n_g;
    const uint32_t n = s->n;
    const float delta = s->delta;
    s->delta_used = delta;

    /* accumulate: acc_i = e_i + g_i */
    for (uint32_t i = 0; i < n; ++i) {
        float *acc = s->e[i];
        for (uint64_t j = 0; j < n_g; ++j) {
            float a = acc[j] + g[i][j];
            acc[j] = a;
        }
    }

    /* Allocate.  Every worker computes the same thing from the same
     * gathered vector, so it is computed once. */
    exo_reindex(s->k_t, n, s->t, s->temp);
    exo_allocate(s->temp, s->blk_part, s->blk_pos, n, n_g, s->b,
                 (int64_t)s->blk_move, (int64_t)s->min_blk, s->alpha);
    memcpy(s->used_part, s->blk_part, n * sizeof(int64_t));
    memcpy(s->used_pos, s->blk_pos, n * sizeof(int64_t));

    /* Sparsify: every worker sparsifies its own partition of its own acc */
    for (uint32_t i = 0; i < n; ++i) {
        uint32_t alloc = exo_owner(s->t, i, n);                      /* Alg. 3 (cyclic allocation) */
        uint64_t st  = (uint64_t)s->used_pos[alloc] * s->b;          /* Alg. 3 (partition range) */
        uint64_t end = (uint64_t)(s->used_pos[alloc] + s->used_part[alloc]) * s->b;
        if (end > n_g) end = n_g;
        if (st > n_g) st = n_g;
        s->k_rank[i] = exo_select(s->e[i], st, end, delta, (int)s->cmp_mode, s->idx[i], s->cap);
    }

    /* AllGather of the index lists (rank order) and of the counts */
    uint64_t total = 0, len = 0;
    for (uint32_t i = 0; i < n; ++i) {
        uint64_t sent = s->k_rank[i] < s->cap ? s->k_rank[i] : s->cap;
        s->rank_off[i] = len;
        for (uint64_t j = 0; j < sent; ++j) s->idx_t[len + j] = s->idx[i][j];
        len += sent;
        total += s->k_rank[i];
        s->k_t[i] = (double)s->k_rank[i];                            /* also the partial-k carry */
    }
    s->rank_off[n] = len;

    /* value gather: g_i = acc_i[idx_t] */
    for (uint32_t i = 0; i < n; ++i)
        for (uint64_t j = 0; j < len; ++j) s->g[i][j] = s->e[i][s->idx_t[j]];

    /* AllReduce(SUM); the order of the sum is rank order here */
    for (uint64_t j = 0; j < len; ++j) {
        float sum = s->g[0][j];
        for (uint32_t i = 1; i < n; ++i) sum = sum + s->g[i][j];
        s->g_t[j] = sum;
    }

    /* k' sum and Estimate */
    s->k_actual = total;
    s->delta = exo_estimate(s->k, (double)total, delta, s->beta, s->gamma);

    /* zeroing: every worker zeroes its acc at the gathered indices */
    for (uint32_t i = 0; i < n; ++i)
        for (uint64_t j = 0; j < len; ++j) s->e[i][s->idx_t[j]] = 0.0f;

    /* residual carry: e_{i,t+1} = acc_i (same buffer) */
    s->t += 1;
}

uint64_t        exo_workers_capacity(const exo_workers *s)        { return s->cap; }
uint64_t        exo_workers_n_blocks(const exo_workers *s)        { return s->n_b; }
uint64_t        exo_workers_iteration(const exo_workers *s)       { return s->t; }
float           exo_workers_threshold(const exo_workers *s)       { return s->delta; }
float           exo_workers_threshold_used(const exo_workers *s)  { return s->delta_used; }
float          *exo_workers_residual(exo_workers *s, uint32_t i)  { return s->e[i]; }
const uint64_t *exo_workers_k_rank(const exo_workers *s)          { return s->k_rank; }
const uint64_t *exo_workers_rank_off(const exo_workers *s)        { return s->rank_off; }
const uint32_t *exo_workers_idx(const exo_workers *s)             { return s->idx_t; }
const float    *exo_workers_values(const exo_workers *s, uint32_t i) { return s->g[i]; }
const float    *exo_workers_sum(const exo_workers *s)             { return s->g_t; }
uint64_t        exo_workers_k_actual(const exo_workers *s)        { return s->k_actual; }
const int64_t  *exo_workers_blk_part(const exo_workers *s, int which) { return which ? s->blk_part : s->used_part; }
const int64_t  *exo_workers_blk_pos(const exo_workers *s, int which)  { return which ? s->blk_pos : s->used_pos; }

/* Eq. 1: the mean over the workers of ||e_{i,t+1}||_2, each summed in fp64;
 * one worker's term when `i` < n, the mean when i == n. */
double exo_workers_err_norm(const exo_workers *s, uint32_t i)
{
    double mean = 0.0;
    for (uint32_t w = 0; w < s->n; ++w) {
        double acc = 0.0;
        for (uint64_t j = 0; j < s->n_g; ++j) {
            double v = (double)s->e[w][j];
            acc += v * v;
        }
        if (w == i) return sqrt(acc);
        mean += sqrt(acc);
    }
    return mean / (double)s->n;
}

/* Eq. 5: n * max_i k_{i,t} / k' (0 when nothing was selected) */
double exo_workers_traffic_ratio(const exo_workers *s)
{
    if (s->k_actual == 0) return 0.0;
    uint64_t m = 0;
    for (uint32_t i = 0; i < s->n; ++i)
        if (s->k_rank[i] > m) m = s->k_rank[i];
    return (double)s->n * (double)m / (double)s->k_actual;
}

/* Alg. 1 (model update) on the entries that were sent: x[idx_t] <- x[idx_t] - (1/n) g_t.
 * `scale` is the 1/n of the paper as an fp32 number; the product is rounded
 * to fp32, then the difference is. */
void exo_apply_update(float *x, const uint32_t *idx_t, const float *g_t, uint64_t len, float scale)
{
    for (uint64_t j = 0; j < len; ++j) {
        float p = scale * g_t[j];
        float v = x[idx_t[j]] - p;
        x[idx_t[j]] = v;
    }
}

/* Eq. 2-4: m_t = max_i k_{i,t}; c_i = m_t - k_{i,t} elements padded by worker i;
 * C_t = n * sum_i c_i. */
uint64_t exo_padding_overhead(const uint64_t *k, uint32_t n)
{
    uint64_t m_t = 0;
    for (uint32_t i = 0; i < n; ++i)
        if (k[i] > m_t) m_t = k[i];
    uint64_t sum = 0;
    for (uint32_t i = 0; i < n; ++i) {
        uint64_t c_i = m_t - k[i];
        sum += c_i;
    }
    return (uint64_t)n * sum;
}
