/*
 * exdyna.h -- C ABI of the MI355X (gfx950) ExDyna gradient-selection library.
 *
 * One `exdyna_step` is one iteration of the sparsifier inside the paper's
 * distributed SGD (the body of Alg. 1's loop) on ONE device that plays all P workers:
 *   acc = residual + grad                          (Alg. 1, accumulate; Sec. 2)
 *   select |acc| >= delta inside every partition   (Alg. 4, Sec. 4.3)
 *   emit (index, value) pairs, ascending           (Alg. 1, Sparsify and value gather)
 *   residual = acc with the emitted entries zeroed (Alg. 1, zeroing and residual carry)
 *   delta   <- online threshold scaling            (Alg. 5, Sec. 4.4)
 *   topology <- adjacent-partition rebalancing     (Alg. 3, the sweep; Sec. 4.2)
 * The two collectives of Alg. 1 (AllGather, AllReduce) are not part of this
 * library; the model update is available for the selected entries as
 * exdyna_apply_update.  The "worker view" calls further down split the
 * iteration at those collectives for callers that have one context per worker.
 *
 * Conventions
 *  - Pointers named d_* are DEVICE pointers, h_* are HOST pointers.
 *  - The caller owns d_grad, d_residual, d_workspace and the HIP stream; the
 *    library owns only the host-side context.  The library never allocates
 *    device memory.
 *  - Every call returns EXDYNA_OK (0) or a negative error; nothing throws or
 *    aborts.  Arguments are validated on the host before anything is launched.
 *  - exdyna_step only enqueues work on `hip_stream` and never synchronises.
 *    The getters that fill host memory synchronise that stream.
 *  - One context must not be used from two host threads at once, and steps of
 *    one context must all be enqueued on streams that are ordered with respect
 *    to each other.
 */
#ifndef EXDYNA_H
#define EXDYNA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    EXDYNA_OK      = 0,
    EXDYNA_EINVAL  = -1, /* a configuration value is out of range            */
    EXDYNA_ENULL   = -2, /* a required pointer is NULL                       */
    EXDYNA_EALIGN  = -3, /* a device pointer is not aligned as required      */
    EXDYNA_ESTATE  = -4, /* context is not initialised / already destroyed / no step run yet */
    EXDYNA_ENOMEM  = -5, /* workspace too small, or host allocation failed   */
    EXDYNA_EHIP    = -6  /* a HIP runtime call failed (see exdyna_last_hip_error) */
};

/* gradient element types of exdyna_step_scaled */
enum { EXDYNA_F32 = 0, EXDYNA_BF16 = 1, EXDYNA_F16 = 2 };

typedef struct exdyna_ctx exdyna_ctx; /* opaque, host memory, library-owned */

/* Problem statement of Alg. 1 / Alg. 3 / Alg. 5.  The paper names alpha, beta,
 * gamma, blk_move and min_blk but gives them no values; exdyna_default_config
 * fills this build's defaults. */
typedef struct {
    uint64_t n_g;          /* number of gradients, 1 <= n_g < 2^32 (indices are u32)        */
    uint32_t block_size;   /* b: gradients per block, > 0 and a multiple of 32 (Sec. 4.1,
                              Alg. 2's rounding).  Any such size runs at about the same
                              speed; multiples of 4096 (one streaming workgroup) need no
                              per-block counters at all                                    */
    uint32_t n_parts;      /* P = number of workers n, 1 <= P <= min(n_b, 1024)             */
    double   density;      /* d in (0, 1]; k = d * n_g is kept in fp64 (Sec. 1)             */
    float    threshold0;   /* delta_0 > 0, finite (Alg. 1, threshold initialisation)        */
    uint32_t cmp_mode;     /* 0: |acc| >= delta (Alg. 4's comparison); 1: |acc| > delta     */
    double   alpha;        /* >= 1, imbalance band of Alg. 3's two overload tests           */
    double   beta;         /* > 1, density band of Alg. 5's two tests on exam               */
    double   gamma;        /* in [0, 1), threshold step of Alg. 5's scaling factors; 0 keeps
                              delta fixed (the hard-threshold sparsifier of Sec. 3)         */
    uint32_t blk_move;     /* blocks moved per adjustment (Alg. 3's k_move); 0 = static
                              partitions (the coarse-grained partitioning of Sec. 4.1)      */
    uint32_t min_blk;      /* >= 1, smallest partition in blocks (Alg. 3's min_blk guards)  */
    uint64_t max_selected; /* output capacity in pairs; 0 = max(ceil(4k), 1024), <= n_g     */
    uint32_t want_err_norm;/* != 0: also compute ||residual||_2 (Eq. 1, one worker)         */
    uint32_t reserved;     /* must be 0                                                     */
} exdyna_config;

/* Per-step scalars, all produced on the device by the finishing kernel. */
typedef struct {
    uint64_t t;             /* iterations completed                                         */
    uint64_t k_actual;      /* k' = number of gradients that passed the comparison          */
    uint64_t k_emitted;     /* min(k', capacity): pairs actually written and zeroed         */
    uint64_t k_max_part;    /* m_t = max_p k_{p,t} (Eq. 2)                                  */
    double   density_error; /* eps_t = |k - k'| / n_g (Eq. 6)                               */
    double   traffic_ratio; /* f(t) = P * m_t / k' (Eq. 5); 0 when k' = 0                   */
    double   err_norm;      /* ||e_{t+1}||_2 (Eq. 1 with one worker); -1 when not requested */
    float    delta_used;    /* delta_t the step compared with                               */
    float    delta_next;    /* delta_{t+1} (Alg. 5, threshold scaling)                      */
    uint32_t overflow;      /* 1 when k' > capacity (worker view: some worker's k_i > capacity) */
    uint32_t moves;         /* boundary moves Alg. 3 made for the next iteration            */
    uint32_t bad_index;     /* worker view: gathered indices >= n_g, skipped by the exchange */
    uint32_t reserved;
    uint64_t padding_overhead; /* C_t = P * sum_p (m_t - k_{p,t}) (Eq. 3-4): what an AllGather of
                                  equal-sized lists pads, summed over the receivers        */
} exdyna_stats;

/* Fill *cfg with defaults: alpha 1.0, beta 1.1, gamma 0.01, blk_move 1,
 * min_blk 1, cmp_mode 0, max_selected 0, want_err_norm 0.  n_g, block_size,
 * n_parts, density and threshold0 are left 0 for the caller to set. */
int exdyna_default_config(exdyna_config *cfg);

/* Alg. 2 (block size), for callers that think in a block count n_b: floor(n_g /
 * n_b) rounded down to the granularity `multiple` (the paper uses 32, which
 * this library accepts; 256 selects its leaner kernel variant).  Writes 0 when fewer than `multiple` gradients
 * would fall in a block.  Host only. */
int exdyna_block_size_from_nb(uint64_t n_g, uint64_t n_b, uint32_t multiple, uint32_t *h_block_size);

/* Bytes of device workspace exdyna_init needs for this configuration
 * (state, per-block / per-segment / per-tile counters, the staging slots the
 * streaming pass writes selected pairs into, and the output pairs).  Host only, launches nothing. */
int exdyna_workspace_bytes(const exdyna_config *cfg, size_t *h_bytes);

/* Alg. 1 (initialisation): residual <- 0, partial-k vector <- k/P, delta <- delta_0,
 * topology <- Alg. 2.  d_residual: n_g floats, 16-byte aligned, zeroed here
 * and updated in place by every step.  d_workspace: 256-byte aligned,
 * ws_bytes >= exdyna_workspace_bytes().  Both must stay valid until
 * exdyna_destroy.  Work is enqueued on hip_stream (a hipStream_t; NULL = the
 * default stream).  *out receives the context. */
int exdyna_init(exdyna_ctx **out, const exdyna_config *cfg, float *d_residual,
                void *d_workspace, size_t ws_bytes, void *hip_stream);

/* exdyna_init for callers that cannot allocate device memory -- code running under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc: the state, counters,
 * tables and staging slots that exdyna_init lays into a caller-provided workspace live in a
 * device array built into the library instead (EXDYNA_STATIC_SCRATCH_BYTES per device, held
 * from the first call on that device until the process ends).  The caller still passes the
 * residual and the two output arrays: d_out_idx and d_out_val, cfg->max_selected entries
 * each (max_selected must be set, not 0), 4-byte aligned; exdyna_get_selected returns these
 * same pointers.  The context itself is built-in storage too, so neither this call nor any
 * later call on the context (steps, getters, exdyna_destroy) allocates or frees device
 * memory, and this call allocates no host memory either.  Everything else -- exdyna_step
 * and the other entry points, results, error codes -- is exactly as for a context made by
 * exdyna_init.
 *  - EXDYNA_ENOMEM: the configuration needs more scratch than the built-in array holds
 *    (25 million gradients at density 0.01 or 138 million at 0.001, with four times
 *    the target count as capacity, still fit; the exact need is exdyna_workspace_bytes
 *    minus 8 bytes per output pair).
 *  - EXDYNA_ESTATE: the current device's built-in context is still live.  There is ONE per
 *    device because all of them would share that device's array: destroy it before making
 *    the next (whose set-up clears what must start at zero; the rest of the array keeps the
 *    last context's contents and is overwritten before it is read).  Work of a destroyed
 *    built-in context that is still running on the device when the next one is created
 *    races with it: drain the stream first, as before freeing a workspace.
 *  - EXDYNA_EINVAL also for max_selected = 0 and for a device ordinal above 15.
 * The device that is current at the call is the one whose array is used. */
#define EXDYNA_STATIC_SCRATCH_BYTES (64u << 20)
int exdyna_init_static(exdyna_ctx **out, const exdyna_config *cfg, float *d_residual,
                       uint32_t *d_out_idx, float *d_out_val, void *hip_stream);

/* One iteration (see the top of this file).  d_grad: n_g floats, 16-byte
 * aligned, read only, already scaled by the learning rate (the accumulate is a
 * single fp32 add).  Asynchronous: returns after enqueueing two kernels.
 *
 * HIP graphs: the two launches are plain kernel nodes (no memset, no event
 * unless profiling is on), all state they read or write is in the workspace,
 * and consecutive iterations alternate between two sets of counters.  A
 * stream capture of an EVEN number of consecutive exdyna_step calls (with
 * profiling off and fixed d_grad addresses) can therefore be replayed any
 * number of times; each replay advances the device state by that many
 * iterations and the getters keep reporting the last iteration (every getter
 * that synchronises also takes the iteration count from the device, so the
 * host side follows the replays).
 *
 * Errors: every argument check happens before the first launch, so a negative
 * return other than EXDYNA_EHIP means nothing was enqueued.  EXDYNA_EHIP means
 * the HIP runtime refused a launch or an event record; the iteration counter
 * has not advanced, but the first kernel may have run and left this
 * iteration's counters and the residual half-updated: the context must not be
 * stepped again -- restore the residual and call exdyna_set_state, or destroy
 * the context. */
int exdyna_step(exdyna_ctx *ctx, const float *d_grad, void *hip_stream);

/* The same iteration with the learning rate fused in and a choice of gradient
 * element type (Alg. 1's accumulate as printed: acc = e + eta * G).  d_grad: n_g
 * elements of grad_dtype (EXDYNA_F32 / EXDYNA_BF16 / EXDYNA_F16), 16-byte
 * aligned.  Each gradient is widened to fp32 exactly, multiplied by eta in fp32
 * (rounded), then added to the residual in fp32 (rounded): fl(e + fl(eta * g)),
 * never a fused multiply-add.  With 16-bit gradients the streaming pass moves
 * 10 instead of 12 bytes per gradient.  eta must be finite.  Steps of both
 * kinds can be mixed freely on one context. */
int exdyna_step_scaled(exdyna_ctx *ctx, const void *d_grad, int grad_dtype, float eta,
                       void *hip_stream);

/* ---- worker view --------------------------------------------------------
 * For callers that run Alg. 1 as printed, one context per worker, each with its
 * own gradient and residual, and do the two collectives (AllGather and
 * AllReduce) themselves.  An iteration is exdyna_worker_select, the caller's
 * AllGather, exdyna_worker_exchange, the caller's AllReduce.  All contexts of
 * a job are created with the same configuration (n_parts = number of workers)
 * and stay replicas of each other in threshold and topology, because Alg. 5
 * and Alg. 3 see the same gathered counts everywhere.
 *
 * exdyna_worker_select (Alg. 1's accumulate, Allocate and Sparsify for worker
 * `rank`): acc = e + eta * g over all n_g gradients as in exdyna_step_scaled (same d_grad, grad_dtype,
 * eta rules; eta = 1 with EXDYNA_F32 is bit-identical to the single add of
 * exdyna_step), but the comparison runs only inside the partition that worker
 * `rank` < n_parts owns at this iteration, (t mod P + rank) mod P of the
 * current topology (Alg. 3, cyclic allocation and partition range).
 * Afterwards exdyna_get_selected gives this worker's list idx_{i,t} (ascending, cut at the capacity; the values are
 * acc at them; k_actual is the uncut count k_{i,t}), and those entries of the
 * residual are already zero.  Threshold, topology and t do not change yet.
 * Returns EXDYNA_ESTATE if a selection is already waiting for its exchange;
 * exdyna_step / exdyna_step_scaled return it too while one is.
 *
 * exdyna_worker_exchange (Alg. 1's value gather, k' sum, Estimate, partial-k
 * carry and zeroing, and the next iteration's Allocate):
 *  d_idx_all        the gathered lists, P rows of `stride` indices; row r holds
 *                   worker r's list in its first min(k_r, capacity, stride)
 *                   entries, the rest of the row is ignored.  Row `rank` must
 *                   be this context's own list.
 *  d_counts_by_rank P uint64, k_{r,t} of worker r (not cut), 8-byte aligned.
 *  d_val_all        P rows of `stride` floats, written here: this worker's acc
 *                   at every gathered index (g_{i,t}, the value gather), 0 in the
 *                   unused part of each row, so that a SUM AllReduce over the
 *                   whole buffer gives g_t.
 * Every gathered entry of the residual is then cleared (the zeroing step); an index
 * >= n_g is skipped and counted in exdyna_stats.bad_index.  The counts are
 * moved from rank order to partition order (Alg. 3's re-indexing of the
 * partial-k vector) and drive Alg. 5 and Alg. 3 exactly as in exdyna_step; t advances.  stride may be 0 when
 * nothing was selected anywhere (the pointers may then be NULL).  Two kernels
 * in `select`, one in `exchange`; nothing synchronises.  The partition a worker
 * owns and the re-indexing offset are computed inside the kernels from the
 * iteration counter in device memory, so a worker-view iteration that follows
 * a replayed HIP graph of steps selects the right partition, and an even number
 * of select/exchange pairs can itself be captured under the rules given for
 * exdyna_step. */
int exdyna_worker_select(exdyna_ctx *ctx, const void *d_grad, int grad_dtype, float eta,
                         uint32_t rank, void *hip_stream);
int exdyna_worker_exchange(exdyna_ctx *ctx, const uint32_t *d_idx_all,
                           const uint64_t *d_counts_by_rank, uint64_t stride, float *d_val_all,
                           void *hip_stream);

/* Alg. 1 (model update) restricted to the selected entries: for every listed index i,
 * d_model[i] <- fl(d_model[i] - fl(scale * value)), scale = 1/n in the paper
 * (two fp32 roundings, no fused multiply-add).  d_idx / d_val: n_rows rows of
 * `stride` entries each (indices and the values to apply, e.g. the gathered
 * list and the all-reduced buffer of the worker view, or, with n_rows = 1 and
 * stride = capacity, the whole step's own output); row r uses its first
 * min(d_counts[r], capacity, stride) entries.  d_counts: n_rows uint64 in device
 * memory (exdyna_get_count_pointers gives one for the context's own list).
 * d_model: n_g floats.  Indices must not repeat (they do not in the library's
 * own lists: partitions are disjoint); an index >= n_g is skipped and counted
 * in exdyna_stats.bad_index.  One kernel, asynchronous.  1 <= n_rows <= 1024. */
int exdyna_apply_update(exdyna_ctx *ctx, float *d_model, const uint32_t *d_idx, const float *d_val,
                        const uint64_t *d_counts, uint32_t n_rows, uint64_t stride, float scale,
                        void *hip_stream);

/* Results of the last step.  *d_idx / *d_val: device arrays of k_emitted
 * ascending gradient indices and the accumulated values at them (Alg. 1,
 * Sparsify and value gather); *d_part_off: device array of P+1 offsets, partition p's pairs are
 * [part_off[p], part_off[p+1]).  They point into the workspace and are
 * overwritten by the next step.  Any of the three may be NULL.  If h_k_actual
 * or h_k_emitted is non-NULL the stream is synchronised and the counts are
 * copied to the host. */
int exdyna_get_selected(exdyna_ctx *ctx, const uint32_t **d_idx, const float **d_val,
                        const uint64_t **d_part_off, uint64_t *h_k_actual, uint64_t *h_k_emitted);

/* Device addresses of the two counts exdyna_get_selected copies to the host
 * (k_actual: gradients that passed the comparison in the last selection pass,
 * k_emitted: pairs written), for callers that feed them to a collective or a
 * kernel without a host round trip -- in the worker view k_actual is the
 * k_{i,t} that Alg. 1's AllGather carries.  The pointers stay valid for
 * the life of the context; the values are rewritten by every selection pass.
 * Host only, does not synchronise. */
int exdyna_get_count_pointers(exdyna_ctx *ctx, const uint64_t **d_k_actual,
                              const uint64_t **d_k_emitted);

/* Topology (Alg. 2 / Alg. 3): which = 0 is what the last step selected with,
 * which = 1 what the next step will select with.  Host arrays of P entries
 * each; any may be NULL.  h_elem_end is clamped to n_g (the last block may be
 * short).  h_owner_rank[p] is the worker that owns partition p at that
 * iteration under Alg. 3's cyclic allocation.  Synchronises. */
int exdyna_get_partitions(exdyna_ctx *ctx, int which, uint32_t *h_blk_pos, uint32_t *h_blk_part,
                          uint64_t *h_elem_start, uint64_t *h_elem_end, uint32_t *h_owner_rank);

/* Untruncated per-block counts of the last step (n_b entries) and
 * per-partition counts k_{p,t} (P entries).  Synchronise. */
int exdyna_get_block_counts(exdyna_ctx *ctx, uint32_t *h_counts);
int exdyna_get_part_counts(exdyna_ctx *ctx, uint64_t *h_counts);

/* Scalars of the last step.  Synchronises. */
int exdyna_get_stats(exdyna_ctx *ctx, exdyna_stats *h_out);

/* Capacity and block count the context was created with.  Host only. */
int exdyna_get_dims(const exdyna_ctx *ctx, uint64_t *h_n_blocks, uint64_t *h_capacity);

/* Checkpoint / resume.  Besides the residual (caller-owned device memory: save
 * and restore those n_g floats yourself) the loop of Alg. 1 carries the iteration
 * number t, the threshold delta_t and the partition topology; the partial-k
 * vector needs no saving because Alg. 3 has already been applied for the next
 * iteration.  exdyna_state_bytes gives the size of that state for this context,
 * exdyna_get_state synchronises and writes it to host memory, exdyna_set_state
 * loads it into a context created with the same n_g, block_size and n_parts
 * (EXDYNA_EINVAL otherwise, or if the topology does not tile the blocks) and
 * synchronises hip_stream.  After set_state plus restoring the residual, further
 * steps give bit-identical results to the run that was saved.  Profiling, if on,
 * is turned off by set_state. */
int exdyna_state_bytes(const exdyna_ctx *ctx, size_t *h_bytes);
int exdyna_get_state(exdyna_ctx *ctx, void *h_state, size_t bytes);
int exdyna_set_state(exdyna_ctx *ctx, const void *h_state, size_t bytes, void *hip_stream);

/* Per-kernel timing for benchmarks.  exdyna_set_profiling(ctx, n_slots, every)
 * with n_slots > 0 makes later steps record HIP events around their two
 * kernels on the step's stream: the iteration it is called before and every
 * `every`-th (>= 1) after it, into a ring of n_slots (<= 65536) event sets;
 * n_slots = 0 turns it off.  Recording costs a few microseconds per step (the
 * event markers keep consecutive launches from overlapping), which is why a
 * benchmark samples.  exdyna_get_kernel_ms waits for iteration `iteration`
 * (0-based, a recorded one among the last n_slots recorded) and returns its
 * durations in milliseconds: [0] the streaming pass, [1] the finishing kernel
 * (control + compaction). */
int exdyna_set_profiling(exdyna_ctx *ctx, uint32_t n_slots, uint32_t every);
int exdyna_get_kernel_ms(exdyna_ctx *ctx, uint64_t iteration, float *h_ms2);

const char *exdyna_strerror(int code);
/* Text of the last HIP error seen by this context's calls ("" if none). */
const char *exdyna_last_hip_error(const exdyna_ctx *ctx);

/* Frees the host context.  Does not touch device memory; the caller must make
 * sure the stream has drained before freeing d_residual / d_workspace.  The
 * library keeps a table of its live contexts and looks every handle up there
 * before reading it: destroying a context twice, using it after exdyna_destroy,
 * or passing memory that never was a context returns EXDYNA_ESTATE without
 * touching that memory.  At most 1024 contexts can be live in one process
 * (exdyna_init returns EXDYNA_ENOMEM beyond that). */
int exdyna_destroy(exdyna_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif
