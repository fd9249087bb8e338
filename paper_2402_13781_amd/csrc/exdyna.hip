// ExDyna gradient-selection hot path for MI355X (gfx950, wave64).
//
// Two kernels per iteration, both enqueued by exdyna_step with no host round
// trip (threshold, topology and counters live in device memory):
//
//   k_stream   acc = e + g (Alg. 1, accumulate), |acc| cmp delta (Alg. 4).
//              Each wavefront owns 1024 contiguous gradients (a "wave tile").
//              It ranks its selected gradients with ballots, writes their
//              (index, value) pairs in index order into the tile's staging
//              slots, writes the residual -- with those entries already zeroed
//              (Alg. 1, zeroing and residual carry) when the tile's output rank
//              of the iteration before says they will fit the output -- stores
//              the tile's count word, and adds the count to its segment's
//              counter: a segment is the four tiles of one workgroup (longer
//              vectors: 16 to 64 tiles), because adds to one address serialise
//              and a wavefront does not retire before its add has returned.
//              Blocks that are not whole segments are counted as well; the
//              counts of those that are follow from the segment counters in
//              k_finish.  A tile whose rank lay far beyond the output
//              capacity, or with more selected gradients than slots, is only
//              counted and flagged.  Pure streaming: 8 B read + 4 B written per
//              gradient, no workgroup barrier, no fence.
//   k_finish   workgroup 0 = control: per-partition counts k_{p,t} and k'
//              (Alg. 1, the gathered counts and their sum), output segment
//              offsets, threshold scaling (Alg. 5), adjacent-partition
//              rebalancing (Alg. 3's sweep), Eq. 2/5/6 statistics.
//              The other workgroups place the pairs.  Each builds the same small
//              offset table from the segment counters in LDS.  Some then work by
//              tile (ranks of the tiles -> the next iteration's staging slots
//              and zeroing rights); the rest work by OUTPUT RANK: a window of
//              consecutive output positions per workgroup, whose tiles' running
//              counts are spread out in LDS so that every thread finds its
//              ranks' pairs with a short search and copies them (Alg. 1,
//              Sparsify and value gather).  Work is therefore proportional to
//              min(k', capacity) however the selected gradients are spread over
//              the vector, also while the threshold is still catching up and
//              k' is far above the capacity.
//              Control and placement read the same finished counters and do
//              not depend on each other, so they overlap inside one launch.
//
// Variants of the same two kernels: gradients stored as fp32, bf16 or fp16 with
// the learning rate applied inside the accumulate (Alg. 1 as printed);
// block sizes that are multiples of 32 but not of 256 (per-lane masks and
// counters instead of per-granule ones); and the "worker view", in which one
// context is one worker of Alg. 1: k_stream compares only inside the partition
// that worker owns at this iteration (Alg. 3, cyclic allocation), k_finish stops
// at the offsets of the worker's own list, and after the caller's AllGather a
// third kernel finishes the iteration:
//
//   k_exchange rows r < P: read this worker's acc at rank r's gathered indices
//              into the value buffer the AllReduce will sum, and clear them
//              (Alg. 1, value gather and zeroing).  Row P: the control workgroup
//              on the gathered counts, moved from rank to partition order (Alg. 3
//              re-indexing) -- the same Alg. 5 / Alg. 3 code as in k_finish.
//
// Partitions are contiguous and ascending (Sec. 4.1), so the concatenation of
// the per-partition index lists in partition order is the global ascending
// list: a pair's output position is the number of selected gradients in front
// of it, and partition p's segment starts at the sum of the counts of the
// partitions before it.
//
// What the measurements on this part ruled out: a device-scope fence or a
// "last workgroup done" ticket per workgroup (about 150 ns each, serialised),
// counters shared by many workgroups (16 tiles per counter cost the streaming
// pass 4 % when every tile adds, 64 tiles 15 %; 4 tiles under 1 %), summing a
// workgroup's counts in LDS first (the barrier costs more than the adds),
// a workgroup barrier in the streaming pass (6 % slower), gathering the
// selected values from the residual afterwards (random 4-byte reads over
// gigabytes), and dealing the placement out by tile (a threshold transient
// packs the whole output into a few per cent of the tiles: a few wavefronts
// then copy thousands of pairs each while the rest idle).  In the finishing
// kernel every first touch of memory costs 1.5-2 us and every shuffle through
// the LDS crossbar about 60 ns, so loads are issued before anything waits and
// wavefront scans use the vector ALU's lane-shift path.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "exdyna.h"

#include "device_common.h"
#include "k_stream.h"
#include "k_finish.h"
#include "k_exchange.h"
#include "k_setup.h"

namespace {

struct Layout {
    size_t state, parts, part_cnt, part_off, blk_cnt, blk_out, seg_cnt, tile_cnt, err_slots, stage,
        out_idx, out_val, total;
    size_t n_tiles, n_segs, n_groups, pool_pairs;
    size_t blk_stride, seg_stride, out_stride;  // entries between the two parities' arrays (padded to 64)
    size_t tile_pad;                // entries of tile_cnt (n_tiles rounded up to 1024, the rest stays 0)
    uint32_t segs_per_blk; // blocks are this many whole segments (0: they are not; the streaming pass counts blocks too)
    uint32_t rep_shift;    // ... then with 2^rep_shift counters to a block, one per streaming workgroup in turn
    size_t slot_tab;
    uint32_t pool_extra; // staging pairs handed out in proportion to the last counts
    uint32_t slots;      // staging slots every wave tile always has
    uint32_t seg_shift;  // log2(wave tiles per segment counter)
    uint32_t grp_shift;  // log2(segment counters per entry of the placement's offset table)
    uint32_t tile_wgs, rank_wgs;  // placement workgroups per launch: by tile, by output rank
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

// ---------------------------------------------------------------------------
// host side

struct exdyna_ctx {
    uint64_t      magic;
    exdyna_config cfg;
    CtrlParams    prm;
    Layout        lay;
    uint64_t      n_b, cap;
    uint64_t      t;  // iterations completed (enqueued)
    uint32_t      phase;     // worker view: 1 between exdyna_worker_select and exdyna_worker_exchange
    uint32_t      rank;      // worker view: the rank of the pending selection
    uint32_t      sel_rank;  // worker whose partition the current selection pass compares, or kAllParts
    float        *d_residual;
    char         *ws;
    uint32_t     *d_out_idx;   // output pairs: inside the workspace, or the caller's arrays
    float        *d_out_val;
    int           static_dev;  // >= 0: this is the built-in context of that device (its scratch is the static array)
    hipStream_t   stream;  // stream of the most recent call
    uint32_t      prof_slots;  // 0 = profiling off
    uint64_t      prof_since;  // first iteration recorded with the current events
    uint32_t      prof_every;  // every how many iterations events are recorded
    hipEvent_t   *ev;          // prof_slots x 3 events, slot = iteration % prof_slots
    char          hip_err[256];
};

namespace {

int validate_config(const exdyna_config *c, uint64_t *n_b_out, uint64_t *cap_out)
{
    if (c->n_g == 0 || c->n_g > 0xFFFFFFFFull) return EXDYNA_EINVAL;
    if (c->block_size == 0 || c->block_size % 32 != 0) return EXDYNA_EINVAL;
    const uint64_t n_b = (c->n_g + c->block_size - 1) / c->block_size;
    if (c->n_parts == 0 || c->n_parts > n_b || c->n_parts > kMaxParts) return EXDYNA_EINVAL;
    if (!(c->density > 0.0 && c->density <= 1.0)) return EXDYNA_EINVAL;
    if (!(c->threshold0 > 0.0f) || std::isinf(c->threshold0)) return EXDYNA_EINVAL;
    if (c->cmp_mode > 1) return EXDYNA_EINVAL;
    if (!(c->alpha >= 1.0) || std::isinf(c->alpha)) return EXDYNA_EINVAL;
    if (!(c->beta > 1.0) || std::isinf(c->beta)) return EXDYNA_EINVAL;
    if (!(c->gamma >= 0.0 && c->gamma < 1.0)) return EXDYNA_EINVAL;  // 0: fixed threshold
    if (c->min_blk == 0) return EXDYNA_EINVAL;
    if (c->reserved != 0) return EXDYNA_EINVAL;
    if (c->max_selected > c->n_g) return EXDYNA_EINVAL;
    uint64_t cap = c->max_selected;
    if (cap == 0) {
        const double want = std::ceil(4.0 * c->density * (double)c->n_g);
        cap = want < 1024.0 ? 1024 : (uint64_t)want;
        if (cap > c->n_g) cap = c->n_g;
    }
    *n_b_out = n_b;
    *cap_out = cap;
    return EXDYNA_OK;
}

// Staging slots every wave tile has: room for four times the expected number of
// selected gradients in 1024 (density d), 32 or 64 (16 pairs = one 128-byte line).
// Not fewer than 32: a tile beyond its fixed slots depends on the slots the finishing
// kernel gave it from its last count, four per pair, and with 16 fixed slots the tiles
// that had 3 to 7 pairs and now have 17 or more (a few per thousand while the threshold is
// still catching up) would be left without room and have to be read again.
uint32_t staging_slots(double density)
{
    const double want = 4.0 * density * (double)kTile + 4.0;
    uint32_t s = 32;
    while (s < 64 && (double)s < want) s <<= 1;
    return s;
}

// Wave tiles per segment counter.  Every tile with a selected gradient adds to
// its segment's counter, and same-address atomics from many workgroups
// serialise; the segment is sized so that about ten tiles per segment are
// expected to add anything (a tile does with probability 1 - exp(-1024 d)).
uint32_t segment_shift(double density)
{
    const double p_hit = 1.0 - std::exp(-(double)kTile * density);
    uint32_t sh = kSegShift;
    while (sh > 2 && (double)(1u << sh) * p_hit > 12.0) --sh;
    return sh;
}

// the placement keeps one prefix entry per group of 1, 4 or 16 segments in LDS
bool groups_fit(size_t n_tiles, uint32_t sh)
{
    const size_t n_segs = (n_tiles + (1u << sh) - 1) >> sh;
    return (n_segs + 15) / 16 <= kMaxGroups;
}

Layout make_layout(const exdyna_config *c, uint64_t n_b, uint64_t cap, bool with_outputs = true)
{
    Layout L{};
    const size_t P = c->n_parts;
    L.n_tiles  = (c->n_g + kTile - 1) / kTile;
    L.slots    = staging_slots(c->density);
    // One counter per workgroup of the streaming pass (four tiles) while the finishing kernel
    // can still read them all (every placement workgroup does); coarser ones for longer vectors.
    if ((L.n_tiles + 3) / 4 <= kMaxFineSegs) {
        L.seg_shift = 2;
    } else {
        L.seg_shift = segment_shift(c->density);
        while (!groups_fit(L.n_tiles, L.seg_shift)) ++L.seg_shift;  // 64 tiles per segment always fit
    }
    // Blocks that are whole segments are not counted by the streaming pass: the control
    // workgroup adds their segments up.
    {
        const uint64_t seg_elems = (uint64_t)kTile << L.seg_shift;
        L.segs_per_blk = c->block_size % seg_elems == 0 ? (uint32_t)(c->block_size / seg_elems) : 0u;
        // Other blocks are counted by the streaming pass itself.  Large ones get several
        // counters, used by consecutive workgroups in turn, so that about four tiles add to one.
        L.rep_shift = 0;
        if (!L.segs_per_blk)
            while (L.rep_shift < 4 && ((uint64_t)4 * kTile << L.rep_shift) < c->block_size) ++L.rep_shift;
    }
    L.n_segs   = (L.n_tiles + (1u << L.seg_shift) - 1) >> L.seg_shift;
    // few entries make the table quick to build; every level below it costs one more lookup
    L.grp_shift = L.n_segs > 4096 ? 4 : L.n_segs > 1024 ? 2 : 0;
    L.n_groups = (L.n_segs + (1u << L.grp_shift) - 1) >> L.grp_shift;
    // the placement reads counters 16 and 64 at a time: arrays are padded with zeros that nothing writes
    L.blk_stride = align_up(n_b << L.rep_shift, 64);
    L.out_stride = align_up(n_b, 64);
    L.seg_stride = align_up(std::max<size_t>(L.n_segs, (size_t)n_b * L.segs_per_blk), 64);  // whole blocks' worth
    L.tile_pad   = align_up(L.n_tiles, 1024);  // whole groups of segments (at most 16 x 64 tiles)
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    L.state     = take(sizeof(DevState));
    L.parts     = take(4 * P * sizeof(int32_t));             // slot0 part,pos ; slot1 part,pos
    L.part_cnt  = take(P * sizeof(uint64_t));
    L.part_off  = take((P + 1) * sizeof(uint64_t));
    L.blk_cnt   = take(2 * L.blk_stride * sizeof(uint32_t));  // two alternating counter arrays
    L.blk_out   = take(2 * L.out_stride * sizeof(uint32_t));  // the per-block counts as the getters see them
    L.seg_cnt   = take(2 * L.seg_stride * sizeof(uint32_t));  // likewise
    L.tile_cnt  = take(L.tile_pad * sizeof(uint32_t));
    L.err_slots = take(2 * 2 * kErrSlots * sizeof(double));   // per parity: unselected, then left-behind selected
    // staging pool: slots for every tile plus up to four per pair for one and a half output capacities
    {
        uint64_t extra = (6 * cap + 15) & ~15ull;
        const uint64_t fixed = (uint64_t)L.n_tiles * L.slots;
        if (fixed + extra > 0xFFFF0000ull) extra = (0xFFFF0000ull - fixed) & ~15ull;  // slot offsets are u32
        L.pool_extra = (uint32_t)extra;
        L.pool_pairs = fixed + extra;
    }
    L.slot_tab  = take(2 * L.n_tiles * sizeof(uint2));        // {first slot, slots} per tile, two parities
    L.stage     = take(L.pool_pairs * sizeof(uint2));
    if (with_outputs) {
        L.out_idx = take(cap * sizeof(uint32_t));
        L.out_val = take(cap * sizeof(float));
    }
    L.total     = off;
    // placement workgroups: one per 4096 tiles and one per window of 1024 output ranks, but no
    // more than the chip holds at once; they stride over the rest
    {
        const uint64_t rounds  = (L.n_tiles + kFinishWG * kTilesPerThr - 1) / (kFinishWG * kTilesPerThr);
        const uint64_t windows = (cap + kFinishWG - 1) / kFinishWG;
        L.tile_wgs = (uint32_t)(rounds < kMaxTileWG ? rounds : kMaxTileWG);
        if (L.tile_wgs == 0) L.tile_wgs = 1;
        L.rank_wgs = (uint32_t)(windows < kMaxPlaceWG - L.tile_wgs ? windows : kMaxPlaceWG - L.tile_wgs);
        if (L.tile_wgs == 0) L.tile_wgs = 1;
        if (L.rank_wgs == 0) L.rank_wgs = 1;
    }
    return L;
}

// Live contexts.  A handle is looked up here before it is dereferenced, so a
// destroyed context, or memory that never was one, is turned away without being
// read.  Fixed size: registering a context allocates nothing.
constexpr uint32_t kMaxLive = 1024;
std::mutex         g_live_mu;
const exdyna_ctx  *g_live[kMaxLive];
uint32_t           g_live_hi = 0;  // slots [0, g_live_hi) may be in use

bool ctx_ok(const exdyna_ctx *c)
{
    if (!c) return false;
    std::lock_guard<std::mutex> lock(g_live_mu);
    for (uint32_t i = 0; i < g_live_hi; ++i)
        if (g_live[i] == c) return c->magic == kMagic;
    return false;
}

bool ctx_register(const exdyna_ctx *c)
{
    std::lock_guard<std::mutex> lock(g_live_mu);
    for (uint32_t i = 0; i < kMaxLive; ++i)
        if (!g_live[i]) {
            g_live[i] = c;
            if (i >= g_live_hi) g_live_hi = i + 1;
            return true;
        }
    return false;
}

bool ctx_unregister(const exdyna_ctx *c)
{
    std::lock_guard<std::mutex> lock(g_live_mu);
    for (uint32_t i = 0; i < g_live_hi; ++i)
        if (g_live[i] == c) {
            g_live[i] = nullptr;
            while (g_live_hi && !g_live[g_live_hi - 1]) --g_live_hi;
            return true;
        }
    return false;
}

int hip_fail(exdyna_ctx *c, hipError_t e, const char *what)
{
    if (c) snprintf(c->hip_err, sizeof c->hip_err, "%s: %s", what, hipGetErrorString(e));
    return EXDYNA_EHIP;
}

#define HIP_TRY(ctx, call)                                       \
    do {                                                         \
        hipError_t e__ = (call);                                 \
        if (e__ != hipSuccess) return hip_fail(ctx, e__, #call); \
    } while (0)

template <typename T> T *at(exdyna_ctx *c, size_t off) { return reinterpret_cast<T *>(c->ws + off); }

int32_t *slot_part(exdyna_ctx *c, uint64_t slot) { return at<int32_t>(c, c->lay.parts) + (slot & 1) * 2 * c->cfg.n_parts; }
int32_t *slot_pos(exdyna_ctx *c, uint64_t slot) { return slot_part(c, slot) + c->cfg.n_parts; }
uint32_t *blk_cnt_of(exdyna_ctx *c, uint64_t t) { return at<uint32_t>(c, c->lay.blk_cnt) + (t & 1) * c->lay.blk_stride; }
uint32_t *seg_cnt_of(exdyna_ctx *c, uint64_t t);
// Where iteration t's per-block counts are: the counters themselves when a block has exactly one
// (its own, or its one segment's), else the sums the control workgroup stores.
uint32_t *blk_out_of(exdyna_ctx *c, uint64_t t)
{
    if (c->lay.segs_per_blk == 1) return seg_cnt_of(c, t);
    if (c->lay.segs_per_blk == 0 && c->lay.rep_shift == 0) return blk_cnt_of(c, t);
    return at<uint32_t>(c, c->lay.blk_out) + (t & 1) * c->lay.out_stride;
}
double *err_slots_of(exdyna_ctx *c, uint64_t t) { return at<double>(c, c->lay.err_slots) + (t & 1) * 2 * kErrSlots; }

uint2 *slot_tab_of(exdyna_ctx *c, uint64_t t) { return at<uint2>(c, c->lay.slot_tab) + (t & 1) * c->lay.n_tiles; }
uint32_t *seg_cnt_of(exdyna_ctx *c, uint64_t t) { return at<uint32_t>(c, c->lay.seg_cnt) + (t & 1) * c->lay.seg_stride; }

template <int CMP, bool NORM, int GT, bool SCALE, bool GEN>
void launch_stream(exdyna_ctx *c, const void *g, float eta, hipStream_t s)
{
    StreamArgs A;
    A.g = g;
    A.eta = eta;
    A.e = c->d_residual;
    A.st = at<DevState>(c, c->lay.state);
    A.stage = at<uint2>(c, c->lay.stage);
    A.stage_extra = A.stage + c->lay.n_tiles * c->lay.slots;
    A.slots_min = c->lay.slots;
    A.pack_off = c->lay.pool_extra <= kMaxPackedExtra;
    A.slot_tab = slot_tab_of(c, c->t);
    A.tile_cnt = at<uint32_t>(c, c->lay.tile_cnt);
    A.blk_cnt = blk_cnt_of(c, c->t);
    A.seg_cnt = seg_cnt_of(c, c->t);
    A.seg_shift = c->lay.seg_shift;
    A.seg_only = c->lay.segs_per_blk != 0;
    A.rep_shift = c->lay.rep_shift;
    A.err_slots = err_slots_of(c, c->t);
    A.n_g = (uint32_t)c->cfg.n_g;
    A.n_tiles = (uint32_t)c->lay.n_tiles;
    A.gran_per_blk = c->cfg.block_size / kGran;
    A.gpb_shift = 32;
    for (uint32_t sh = 0; sh < 32; ++sh)
        if ((1u << sh) == A.gran_per_blk) A.gpb_shift = sh;
    A.parity = (uint32_t)(c->t & 1);
    A.sel_rank = c->sel_rank;
    A.n_parts = c->cfg.n_parts;
    A.cur_part = slot_part(c, c->t);
    A.cur_pos = slot_pos(c, c->t);
    A.block_size = c->cfg.block_size;
    const uint32_t grid = (uint32_t)((c->lay.n_tiles + kWavesPerWG - 1) / kWavesPerWG);
    hipLaunchKernelGGL((k_stream<CMP, NORM, GT, SCALE, GEN>), dim3(grid), dim3(kStreamWG), 0, s, A);
}

FinishArgs finish_args(exdyna_ctx *c, uint32_t mode)
{
    const uint64_t t = c->t;
    FinishArgs A;
    A.st = at<DevState>(c, c->lay.state);
    A.e = c->d_residual;
    A.stage = at<uint2>(c, c->lay.stage);
    A.stage_extra = A.stage + c->lay.n_tiles * c->lay.slots;
    A.slot_tab = slot_tab_of(c, t);
    A.slot_tab_next = slot_tab_of(c, t + 1);
    A.n_tile_wgs = c->lay.tile_wgs;
    A.grp_shift = c->lay.grp_shift;
    A.pack_off = c->lay.pool_extra <= kMaxPackedExtra;
    A.slots_min = c->lay.slots;
    A.tile_cnt = at<uint32_t>(c, c->lay.tile_cnt);
    A.seg_cnt = seg_cnt_of(c, t);
    A.seg_cnt_next = seg_cnt_of(c, t + 1);
    if (c->lay.segs_per_blk) {  // a block's count: the sum of its segments' counters
        A.blk_src = A.seg_cnt;
        A.blk_clear = nullptr;  // the placement clears the segment counters
        A.per_blk = c->lay.segs_per_blk;
    } else {                    // ... or of its own counters
        A.blk_src = blk_cnt_of(c, t);
        A.blk_clear = blk_cnt_of(c, t + 1);
        A.per_blk = 1u << c->lay.rep_shift;
    }
    A.blk_out = blk_out_of(c, t);
    A.cur_part = slot_part(c, t);
    A.cur_pos = slot_pos(c, t);
    A.nxt_part = slot_part(c, t + 1);
    A.nxt_pos = slot_pos(c, t + 1);
    A.part_cnt = at<uint64_t>(c, c->lay.part_cnt);
    A.part_off = at<uint64_t>(c, c->lay.part_off);
    A.out_idx = c->d_out_idx;
    A.out_val = c->d_out_val;
    A.err_slots = err_slots_of(c, t);
    A.err_slots_next = err_slots_of(c, t + 1);
    A.n_tiles = (uint32_t)c->lay.n_tiles;
    A.n_segs = (uint32_t)c->lay.n_segs;
    A.n_groups = (uint32_t)c->lay.n_groups;
    A.search_step = 0;  // largest power of two <= n_groups - 1: the first stride of the offset search
    for (uint32_t p2 = 1; p2 < A.n_groups; p2 <<= 1) A.search_step = p2;
    A.seg_shift = c->lay.seg_shift;
    A.pool_extra = c->lay.pool_extra;
    A.parity = (uint32_t)(t & 1);
    A.mode = mode;
    A.sel_rank = c->sel_rank;
    A.block_size = c->cfg.block_size;
    A.n_parts = c->cfg.n_parts;
    return A;
}

template <bool NORM, int CMP>
void launch_finish(exdyna_ctx *c, uint32_t mode, hipStream_t s)
{
    const FinishArgs A = finish_args(c, mode);
    const uint32_t grid = 1u + c->lay.tile_wgs + c->lay.rank_wgs;
    hipLaunchKernelGGL((k_finish<NORM, CMP>), dim3(grid), dim3(kFinishWG), 0, s, A, c->prm);
}

template <int GT, bool SCALE, bool GEN>
void dispatch_stream2(exdyna_ctx *c, const void *g, float eta, hipStream_t s)
{
    const bool norm = c->cfg.want_err_norm != 0;
    if (c->cfg.cmp_mode == 0) {
        if (norm) launch_stream<0, true, GT, SCALE, GEN>(c, g, eta, s); else launch_stream<0, false, GT, SCALE, GEN>(c, g, eta, s);
    } else {
        if (norm) launch_stream<1, true, GT, SCALE, GEN>(c, g, eta, s); else launch_stream<1, false, GT, SCALE, GEN>(c, g, eta, s);
    }
}

template <int GT, bool SCALE>
void dispatch_stream(exdyna_ctx *c, const void *g, float eta, hipStream_t s)
{
    if (c->cfg.block_size % kGran != 0)
        dispatch_stream2<GT, SCALE, true>(c, g, eta, s);   // blocks are not whole granules
    else
        dispatch_stream2<GT, SCALE, false>(c, g, eta, s);
}

// grad_dtype < 0: the unscaled fp32 path of exdyna_step (one add per gradient).
// worker_rank < 0: one device plays every worker; otherwise only that worker's
// partition is compared and the control stops at the own list's offsets.
int step_impl(exdyna_ctx *c, const void *d_grad, int grad_dtype, float eta, int64_t worker_rank,
              void *hip_stream)
{
    if (!ctx_ok(c)) return c ? EXDYNA_ESTATE : EXDYNA_ENULL;
    if (!d_grad) return EXDYNA_ENULL;
    if (grad_dtype > EXDYNA_F16) return EXDYNA_EINVAL;
    if (grad_dtype >= 0 && !std::isfinite(eta)) return EXDYNA_EINVAL;
    if (worker_rank >= (int64_t)c->cfg.n_parts) return EXDYNA_EINVAL;
    if ((uintptr_t)d_grad % 16 != 0) return EXDYNA_EALIGN;
    if (c->phase != 0) return EXDYNA_ESTATE;  // a worker's selection is waiting for its exchange
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    c->stream = s;
    const bool norm = c->cfg.want_err_norm != 0;
    const bool prof = c->prof_slots != 0 && (c->t - c->prof_since) % c->prof_every == 0;
    hipEvent_t *ev = prof ? c->ev + 3 * (((c->t - c->prof_since) / c->prof_every) % c->prof_slots) : nullptr;
    // the kernels work out which partition that worker owns from the device's iteration counter
    c->sel_rank = worker_rank < 0 ? kAllParts : (uint32_t)worker_rank;
    const uint32_t mode = worker_rank < 0 ? kCtrlFull : kCtrlSelect;

    if (prof) HIP_TRY(c, hipEventRecord(ev[0], s));
    switch (grad_dtype) {
    case EXDYNA_F32: dispatch_stream<EXDYNA_F32, true>(c, d_grad, eta, s); break;
    case EXDYNA_BF16: dispatch_stream<EXDYNA_BF16, true>(c, d_grad, eta, s); break;
    case EXDYNA_F16: dispatch_stream<EXDYNA_F16, true>(c, d_grad, eta, s); break;
    default: dispatch_stream<EXDYNA_F32, false>(c, d_grad, 1.0f, s); break;
    }
    if (prof) HIP_TRY(c, hipEventRecord(ev[1], s));

    if (c->cfg.cmp_mode == 0) {
        if (norm) launch_finish<true, 0>(c, mode, s); else launch_finish<false, 0>(c, mode, s);
    } else {
        if (norm) launch_finish<true, 1>(c, mode, s); else launch_finish<false, 1>(c, mode, s);
    }
    if (prof) HIP_TRY(c, hipEventRecord(ev[2], s));
    HIP_TRY(c, hipGetLastError());
    if (worker_rank < 0) {
        c->t += 1;
    } else {
        c->rank = (uint32_t)worker_rank;
        c->phase = 1;  // the iteration ends with exdyna_worker_exchange
    }
    return EXDYNA_OK;
}

// The device counts its iterations itself (a replayed HIP graph advances it without the
// host's knowledge), so whenever a getter has synchronised and read the device state the host
// counter is set from it.
void adopt_device_iteration(exdyna_ctx *c, const DevState &st) { c->t = st.t; }

// Iteration whose selection the getters describe: the last finished one, or the
// one whose worker-view selection is waiting for its exchange.
bool have_iteration(const exdyna_ctx *c) { return c->t + c->phase > 0; }
uint64_t last_iteration(const exdyna_ctx *c) { return c->t + c->phase - 1; }


// ---- the entry point for callers that cannot allocate -------------------------------
// Everything exdyna_init lays into the caller's workspace except the output pairs lives in
// this file-scope device array instead.  Each device the library runs on holds its own
// copy; host code uses the address hipGetSymbolAddress returns for the current device,
// never the array's name.
constexpr size_t kStaticScratchBytes = (size_t)EXDYNA_STATIC_SCRATCH_BYTES;
constexpr int    kMaxStaticDevices   = 16;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

struct StaticContext {
    char      *scratch_ptr;  // device address of `scratch` on this device, once asked for
    bool       live;
    exdyna_ctx ctx;          // the built-in context itself: no host allocation either
};
StaticContext g_static[kMaxStaticDevices];
std::mutex    g_static_mu;

// Fills *c and enqueues the set-up kernels (Alg. 1 (initialisation), Alg. 2): the part
// exdyna_init and exdyna_init_static share.  Counters, tables and state are cleared here,
// so whatever an earlier context left in the scratch memory does not matter; the staging
// pool and the outputs are written before they are read in every iteration.
int init_context(exdyna_ctx *c, const exdyna_config *cfg, const Layout &L, uint64_t n_b, uint64_t cap,
                 float *d_residual, char *ws, uint32_t *d_out_idx, float *d_out_val, int static_dev,
                 void *hip_stream)
{
    c->cfg = *cfg;
    c->lay = L;
    c->n_b = n_b;
    c->cap = cap;
    c->t = 0;
    c->phase = 0;
    c->rank = 0;
    c->sel_rank = kAllParts;
    c->d_residual = d_residual;
    c->ws = ws;
    c->d_out_idx = d_out_idx;
    c->d_out_val = d_out_val;
    c->static_dev = static_dev;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->prof_slots = 0;
    c->prof_every = 1;
    c->ev = nullptr;
    c->hip_err[0] = 0;

    CtrlParams &p = c->prm;
    p.n_g = cfg->n_g;
    p.cap = cap;
    p.k = cfg->density * (double)cfg->n_g;
    p.alpha = cfg->alpha;
    p.inv_alpha = 1.0 / cfg->alpha;
    p.beta = cfg->beta;
    p.inv_beta = 1.0 / cfg->beta;
    p.sf_hi = (float)(1.0 + cfg->gamma);           // Alg. 5 (factor above beta)
    p.sf_mid = (float)(1.0 + 0.25 * cfg->gamma);   // Alg. 5 (factor inside the band)
    p.sf_lo = (float)(1.0 - cfg->gamma);           // Alg. 5 (factor below 1/beta)
    p.n_b = (uint32_t)n_b;
    p.n_parts = cfg->n_parts;
    p.block_size = cfg->block_size;
    p.blk_move = cfg->blk_move;
    p.min_blk = cfg->min_blk;

    hipStream_t s = c->stream;
    const uint32_t P = cfg->n_parts;
    // residual <- 0 (Alg. 1 (local-error initialisation)); counters start clean
    hipLaunchKernelGGL(k_fill_u32, dim3(2048), dim3(256), 0, s,
                       reinterpret_cast<uint32_t *>(d_residual), 0u, (size_t)cfg->n_g);
    hipLaunchKernelGGL(k_fill_u32, dim3(256), dim3(256), 0, s, at<uint32_t>(c, L.blk_cnt), 0u,
                       (size_t)(2 * L.blk_stride));
    hipLaunchKernelGGL(k_fill_u32, dim3(64), dim3(256), 0, s, at<uint32_t>(c, L.seg_cnt), 0u,
                       (size_t)(2 * L.seg_stride));
    hipLaunchKernelGGL(k_fill_u32, dim3(256), dim3(256), 0, s, at<uint32_t>(c, L.tile_cnt), 0u,
                       L.tile_pad);
    hipLaunchKernelGGL(k_init_slot_tab, dim3(256), dim3(256), 0, s, slot_tab_of(c, 0), slot_tab_of(c, 1),
                       (uint32_t)L.n_tiles);
    const uint32_t init_threads = (P + 1 > 4 * kErrSlots ? P + 1 : 4 * kErrSlots);
    hipLaunchKernelGGL(k_init_state, dim3((init_threads + 255) / 256), dim3(256), 0, s,
                       at<DevState>(c, L.state), slot_part(c, 0), slot_pos(c, 0), slot_part(c, 1),
                       slot_pos(c, 1), at<uint64_t>(c, L.part_cnt), at<uint64_t>(c, L.part_off),
                       at<double>(c, L.err_slots), cfg->threshold0, (uint32_t)n_b, P);
    if (hipGetLastError() != hipSuccess) return EXDYNA_EHIP;
    c->magic = kMagic;
    return EXDYNA_OK;
}
}  // namespace

extern "C" {

int exdyna_default_config(exdyna_config *cfg)
{
    if (!cfg) return EXDYNA_ENULL;
    memset(cfg, 0, sizeof *cfg);
    cfg->alpha = 1.0;
    cfg->beta = 1.1;
    cfg->gamma = 0.01;
    cfg->blk_move = 1;
    cfg->min_blk = 1;
    return EXDYNA_OK;
}

int exdyna_block_size_from_nb(uint64_t n_g, uint64_t n_b, uint32_t multiple, uint32_t *h_block_size)
{
    if (!h_block_size) return EXDYNA_ENULL;
    if (n_b == 0 || multiple == 0) return EXDYNA_EINVAL;
    const uint64_t temp = n_g / n_b;
    const uint64_t sz = temp - temp % multiple;
    if (sz > 0xFFFFFFFFull) return EXDYNA_EINVAL;
    *h_block_size = (uint32_t)sz;
    return EXDYNA_OK;
}

int exdyna_workspace_bytes(const exdyna_config *cfg, size_t *h_bytes)
{
    if (!cfg || !h_bytes) return EXDYNA_ENULL;
    uint64_t n_b, cap;
    int rc = validate_config(cfg, &n_b, &cap);
    if (rc) return rc;
    *h_bytes = make_layout(cfg, n_b, cap).total;
    return EXDYNA_OK;
}

int exdyna_init(exdyna_ctx **out, const exdyna_config *cfg, float *d_residual, void *d_workspace,
                size_t ws_bytes, void *hip_stream)
{
    if (!out) return EXDYNA_ENULL;
    *out = nullptr;
    if (!cfg || !d_residual || !d_workspace) return EXDYNA_ENULL;
    uint64_t n_b, cap;
    int rc = validate_config(cfg, &n_b, &cap);
    if (rc) return rc;
    if ((uintptr_t)d_residual % 16 != 0 || (uintptr_t)d_workspace % 256 != 0) return EXDYNA_EALIGN;
    const Layout L = make_layout(cfg, n_b, cap);
    if (ws_bytes < L.total) return EXDYNA_ENOMEM;

    exdyna_ctx *c = new (std::nothrow) exdyna_ctx();
    if (!c) return EXDYNA_ENOMEM;
    char *ws = static_cast<char *>(d_workspace);
    rc = init_context(c, cfg, L, n_b, cap, d_residual, ws, reinterpret_cast<uint32_t *>(ws + L.out_idx),
                      reinterpret_cast<float *>(ws + L.out_val), -1, hip_stream);
    if (rc == EXDYNA_OK && !ctx_register(c)) rc = EXDYNA_ENOMEM;  // more live contexts than the table holds
    if (rc != EXDYNA_OK) {
        delete c;
        return rc;
    }
    *out = c;
    return EXDYNA_OK;
}

int exdyna_init_static(exdyna_ctx **out, const exdyna_config *cfg, float *d_residual,
                       uint32_t *d_out_idx, float *d_out_val, void *hip_stream)
{
    if (!out) return EXDYNA_ENULL;
    *out = nullptr;
    if (!cfg || !d_residual || !d_out_idx || !d_out_val) return EXDYNA_ENULL;
    uint64_t n_b, cap;
    int rc = validate_config(cfg, &n_b, &cap);
    if (rc) return rc;
    if (cfg->max_selected == 0) return EXDYNA_EINVAL;  // the caller sized its output arrays: it must say how
    if ((uintptr_t)d_residual % 16 != 0 || (uintptr_t)d_out_idx % 4 != 0 || (uintptr_t)d_out_val % 4 != 0)
        return EXDYNA_EALIGN;
    const Layout L = make_layout(cfg, n_b, cap, false);
    if (L.total > kStaticScratchBytes) return EXDYNA_ENOMEM;  // beyond what the static array holds

    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return EXDYNA_EHIP;
    if (dev < 0 || dev >= kMaxStaticDevices) return EXDYNA_EINVAL;
    std::lock_guard<std::mutex> lock(g_static_mu);
    StaticContext &sc = g_static[dev];
    if (sc.live) return EXDYNA_ESTATE;  // one built-in context per device: its scratch is shared
    if (!sc.scratch_ptr) {
        // the array's name is a host-side stand-in; its address on this device is asked for once
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return EXDYNA_EHIP;
        sc.scratch_ptr = static_cast<char *>(ptr);
    }
    exdyna_ctx *c = &sc.ctx;
    *c = exdyna_ctx();
    rc = init_context(c, cfg, L, n_b, cap, d_residual, sc.scratch_ptr, d_out_idx, d_out_val, dev, hip_stream);
    if (rc == EXDYNA_OK && !ctx_register(c)) rc = EXDYNA_ENOMEM;
    if (rc != EXDYNA_OK) {
        c->magic = 0;
        return rc;
    }
    sc.live = true;
    *out = c;
    return EXDYNA_OK;
}

int exdyna_step(exdyna_ctx *c, const float *d_grad, void *hip_stream)
{
    return step_impl(c, d_grad, -1, 1.0f, -1, hip_stream);
}

int exdyna_step_scaled(exdyna_ctx *c, const void *d_grad, int grad_dtype, float eta, void *hip_stream)
{
    if (grad_dtype < EXDYNA_F32) return c ? EXDYNA_EINVAL : EXDYNA_ENULL;
    return step_impl(c, d_grad, grad_dtype, eta, -1, hip_stream);
}

int exdyna_worker_select(exdyna_ctx *c, const void *d_grad, int grad_dtype, float eta, uint32_t rank,
                         void *hip_stream)
{
    if (grad_dtype < EXDYNA_F32) return c ? EXDYNA_EINVAL : EXDYNA_ENULL;
    return step_impl(c, d_grad, grad_dtype, eta, (int64_t)rank, hip_stream);
}

int exdyna_worker_exchange(exdyna_ctx *c, const uint32_t *d_idx_all, const uint64_t *d_counts_by_rank,
                           uint64_t stride, float *d_val_all, void *hip_stream)
{
    if (!ctx_ok(c)) return c ? EXDYNA_ESTATE : EXDYNA_ENULL;
    if (!d_counts_by_rank) return EXDYNA_ENULL;
    if (stride > 0 && (!d_idx_all || !d_val_all)) return EXDYNA_ENULL;
    if (stride > c->cfg.n_g) return EXDYNA_EINVAL;
    if ((uintptr_t)d_counts_by_rank % 8 != 0 || (uintptr_t)d_idx_all % 4 != 0 ||
        (uintptr_t)d_val_all % 4 != 0)
        return EXDYNA_EALIGN;
    if (c->phase != 1) return EXDYNA_ESTATE;  // no selection is waiting
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    c->stream = s;
    const uint32_t P = c->cfg.n_parts;
    const FinishArgs A = finish_args(c, kCtrlUpdate);
    ExchangeArgs X;
    X.idx_all = d_idx_all;
    X.counts = d_counts_by_rank;
    X.val_all = d_val_all;
    X.own_val = c->d_out_val;
    X.stride = stride;
    X.rank = c->rank;
    const uint64_t gx = (stride + kFinishWG - 1) / kFinishWG;
    const dim3 grid((uint32_t)(gx ? gx : 1), P + 1);
    if (c->cfg.want_err_norm)
        hipLaunchKernelGGL((k_exchange<true>), grid, dim3(kFinishWG), 0, s, A, c->prm, X);
    else
        hipLaunchKernelGGL((k_exchange<false>), grid, dim3(kFinishWG), 0, s, A, c->prm, X);
    HIP_TRY(c, hipGetLastError());
    c->t += 1;
    c->phase = 0;
    c->sel_rank = kAllParts;
    return EXDYNA_OK;
}

int exdyna_apply_update(exdyna_ctx *c, float *d_model, const uint32_t *d_idx, const float *d_val,
                        const uint64_t *d_counts, uint32_t n_rows, uint64_t stride, float scale,
                        void *hip_stream)
{
    if (!ctx_ok(c)) return c ? EXDYNA_ESTATE : EXDYNA_ENULL;
    if (!d_model || !d_counts) return EXDYNA_ENULL;
    if (stride > 0 && (!d_idx || !d_val)) return EXDYNA_ENULL;
    if (n_rows == 0 || n_rows > kMaxParts || stride > c->cfg.n_g || !std::isfinite(scale)) return EXDYNA_EINVAL;
    if ((uintptr_t)d_model % 4 != 0 || (uintptr_t)d_idx % 4 != 0 || (uintptr_t)d_val % 4 != 0 ||
        (uintptr_t)d_counts % 8 != 0)
        return EXDYNA_EALIGN;
    if (stride == 0) return EXDYNA_OK;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    c->stream = s;
    const dim3 grid((uint32_t)((stride + 255) / 256), n_rows);
    hipLaunchKernelGGL(k_apply, grid, dim3(256), 0, s, d_model, d_idx, d_val, d_counts, stride,
                       (uint64_t)c->cap, (uint32_t)c->cfg.n_g, scale, at<DevState>(c, c->lay.state));
    HIP_TRY(c, hipGetLastError());
    return EXDYNA_OK;
}

int exdyna_get_selected(exdyna_ctx *c, const uint32_t **d_idx, const float **d_val,
                        const uint64_t **d_part_off, uint64_t *h_k_actual, uint64_t *h_k_emitted)
{
    if (!ctx_ok(c)) return c ? EXDYNA_ESTATE : EXDYNA_ENULL;
    if (d_idx) *d_idx = c->d_out_idx;
    if (d_val) *d_val = c->d_out_val;
    if (d_part_off) *d_part_off = at<uint64_t>(c, c->lay.part_off);
    if (h_k_actual || h_k_emitted) {
        DevState st;
        HIP_TRY(c, hipMemcpyAsync(&st, at<DevState>(c, c->lay.state), sizeof st,
                                  hipMemcpyDeviceToHost, c->stream));
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        adopt_device_iteration(c, st);
        if (h_k_actual) *h_k_actual = st.own_actual;
        if (h_k_emitted) *h_k_emitted = st.own_emitted;
    }
    return EXDYNA_OK;
}

int exdyna_get_count_pointers(exdyna_ctx *c, const uint64_t **d_k_actual, const uint64_t **d_k_emitted)
{
    if (!ctx_ok(c)) return c ? EXDYNA_ESTATE : EXDYNA_ENULL;
    DevState *st = at<DevState>(c, c->lay.state);
    if (d_k_actual) *d_k_actual = &st->own_actual;
    if (d_k_emitted) *d_k_emitted = &st->own_emitted;
    return EXDYNA_OK;
}

int exdyna_get_partitions(exdyna_ctx *c, int which, uint32_t *h_blk_pos, uint32_t *h_blk_part,
                          uint64_t *h_elem_start, uint64_t *h_elem_end, uint32_t *h_owner_rank)
{
    if (!ctx_ok(c)) return c ? EXDYNA_ESTATE : EXDYNA_ENULL;
    if (which != 0 && which != 1) return EXDYNA_EINVAL;
    {
        DevState st;
        HIP_TRY(c, hipMemcpyAsync(&st, at<DevState>(c, c->lay.state), sizeof st, hipMemcpyDeviceToHost,
                                  c->stream));
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        adopt_device_iteration(c, st);
    }
    if (which == 0 && !have_iteration(c)) return EXDYNA_ESTATE;  // no step has selected yet
    if (which == 1 && c->phase) return EXDYNA_ESTATE;  // the pending exchange computes it
    const uint32_t P = c->cfg.n_parts;
    // iteration whose topology is asked for
    const uint64_t it = which == 0 ? last_iteration(c) : c->t;
    int32_t *tmp = static_cast<int32_t *>(malloc(2 * (size_t)P * sizeof(int32_t)));
    if (!tmp) return EXDYNA_ENOMEM;
    hipError_t e = hipMemcpyAsync(tmp, slot_part(c, it), 2 * (size_t)P * sizeof(int32_t),
                                  hipMemcpyDeviceToHost, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) {
        free(tmp);
        return hip_fail(c, e, "copy topology");
    }
    const int32_t *part = tmp, *pos = tmp + P;
    for (uint32_t p = 0; p < P; ++p) {
        if (h_blk_part) h_blk_part[p] = (uint32_t)part[p];
        if (h_blk_pos) h_blk_pos[p] = (uint32_t)pos[p];
        // Alg. 3 (partition range), the last block may be short
        uint64_t st = (uint64_t)pos[p] * c->cfg.block_size;
        uint64_t en = (uint64_t)(pos[p] + part[p]) * c->cfg.block_size;
        if (st > c->cfg.n_g) st = c->cfg.n_g;
        if (en > c->cfg.n_g) en = c->cfg.n_g;
        if (h_elem_start) h_elem_start[p] = st;
        if (h_elem_end) h_elem_end[p] = en;
        // Alg. 3 (cyclic allocation): alloc = (t mod P + rank) mod P  <=>  rank = (alloc - t) mod P
        if (h_owner_rank) h_owner_rank[p] = (uint32_t)((p + P - (uint32_t)(it % P)) % P);
    }
    free(tmp);
    return EXDYNA_OK;
}

int exdyna_get_block_counts(exdyna_ctx *c, uint32_t *h_counts)
{
    if (!ctx_ok(c)) return c ? EXDYNA_ESTATE : EXDYNA_ENULL;
    if (!h_counts) return EXDYNA_ENULL;
    if (!have_iteration(c)) return EXDYNA_ESTATE;
    HIP_TRY(c, hipMemcpyAsync(h_counts, blk_out_of(c, last_iteration(c)), c->n_b * sizeof(uint32_t),
                              hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return EXDYNA_OK;
}

int exdyna_get_part_counts(exdyna_ctx *c, uint64_t *h_counts)
{
    if (!ctx_ok(c)) return c ? EXDYNA_ESTATE : EXDYNA_ENULL;
    if (!h_counts) return EXDYNA_ENULL;
    if (!have_iteration(c)) return EXDYNA_ESTATE;
    HIP_TRY(c, hipMemcpyAsync(h_counts, at<uint64_t>(c, c->lay.part_cnt),
                              c->cfg.n_parts * sizeof(uint64_t), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return EXDYNA_OK;
}

int exdyna_get_stats(exdyna_ctx *c, exdyna_stats *h_out)
{
    if (!ctx_ok(c)) return c ? EXDYNA_ESTATE : EXDYNA_ENULL;
    if (!h_out) return EXDYNA_ENULL;
    if (c->cfg.want_err_norm && have_iteration(c))
        hipLaunchKernelGGL(k_norm_finalize, dim3(1), dim3(kErrSlots), 0, c->stream,
                           at<DevState>(c, c->lay.state), err_slots_of(c, last_iteration(c)),
                           (uint32_t)(last_iteration(c) & 1));
    DevState st;
    HIP_TRY(c, hipMemcpyAsync(&st, at<DevState>(c, c->lay.state), sizeof st, hipMemcpyDeviceToHost,
                              c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    adopt_device_iteration(c, st);
    h_out->t = st.t;
    h_out->k_actual = st.k_actual;
    h_out->k_emitted = st.k_emitted;
    h_out->k_max_part = st.k_max_part;
    h_out->density_error = st.density_error;
    h_out->traffic_ratio = st.traffic_ratio;
    h_out->err_norm = (c->cfg.want_err_norm && have_iteration(c)) ? st.err_norm : -1.0;
    h_out->delta_used = st.delta_used;
    h_out->delta_next = st.delta_next;
    h_out->overflow = st.overflow;
    h_out->moves = st.moves;
    h_out->bad_index = st.bad_index;
    h_out->reserved = 0;
    h_out->padding_overhead = st.padding;
    return EXDYNA_OK;
}

int exdyna_get_dims(const exdyna_ctx *c, uint64_t *h_n_blocks, uint64_t *h_capacity)
{
    if (!ctx_ok(c)) return c ? EXDYNA_ESTATE : EXDYNA_ENULL;
    if (h_n_blocks) *h_n_blocks = c->n_b;
    if (h_capacity) *h_capacity = c->cap;
    return EXDYNA_OK;
}

namespace {
void drop_events(exdyna_ctx *c)
{
    if (c->ev) {
        for (uint32_t i = 0; i < 3 * c->prof_slots; ++i) (void)hipEventDestroy(c->ev[i]);
        free(c->ev);
    }
    c->ev = nullptr;
    c->prof_slots = 0;
}

// Saved state (Alg. 1's loop-carried variables other than the residual, which the
// caller owns): a small header, then blk_part[P] and blk_pos[P] of the topology
// the next iteration will select with.
struct StateHeader {
    uint64_t magic, n_g, t;
    uint32_t block_size, n_parts;
    float    delta;
    uint32_t pad;
};
constexpr uint64_t kStateMagic = 0x4578447953743031ull;
}  // namespace

int exdyna_state_bytes(const exdyna_ctx *c, size_t *h_bytes)
{
    if (!ctx_ok(c)) return c ? EXDYNA_ESTATE : EXDYNA_ENULL;
    if (!h_bytes) return EXDYNA_ENULL;
    *h_bytes = sizeof(StateHeader) + 2 * (size_t)c->cfg.n_parts * sizeof(int32_t);
    return EXDYNA_OK;
}

int exdyna_get_state(exdyna_ctx *c, void *h_state, size_t bytes)
{
    if (!ctx_ok(c)) return c ? EXDYNA_ESTATE : EXDYNA_ENULL;
    if (!h_state) return EXDYNA_ENULL;
    if (c->phase) return EXDYNA_ESTATE;  // in the middle of a worker-view iteration
    const size_t P = c->cfg.n_parts;
    if (bytes < sizeof(StateHeader) + 2 * P * sizeof(int32_t)) return EXDYNA_ENOMEM;
    DevState st;
    char *out = static_cast<char *>(h_state);
    HIP_TRY(c, hipMemcpyAsync(&st, at<DevState>(c, c->lay.state), sizeof st, hipMemcpyDeviceToHost,
                              c->stream));
    HIP_TRY(c, hipMemcpyAsync(out + sizeof(StateHeader), slot_part(c, c->t),
                              2 * P * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    adopt_device_iteration(c, st);
    StateHeader h{};
    h.magic = kStateMagic;
    h.n_g = c->cfg.n_g;
    h.t = st.t;
    h.block_size = c->cfg.block_size;
    h.n_parts = c->cfg.n_parts;
    h.delta = st.delta_next;
    memcpy(out, &h, sizeof h);
    return EXDYNA_OK;
}

int exdyna_set_state(exdyna_ctx *c, const void *h_state, size_t bytes, void *hip_stream)
{
    if (!ctx_ok(c)) return c ? EXDYNA_ESTATE : EXDYNA_ENULL;
    if (!h_state) return EXDYNA_ENULL;
    const size_t P = c->cfg.n_parts;
    if (bytes < sizeof(StateHeader) + 2 * P * sizeof(int32_t)) return EXDYNA_EINVAL;
    StateHeader h;
    memcpy(&h, h_state, sizeof h);
    if (h.magic != kStateMagic || h.n_g != c->cfg.n_g || h.block_size != c->cfg.block_size ||
        h.n_parts != c->cfg.n_parts || !(h.delta > 0.0f) || std::isinf(h.delta))
        return EXDYNA_EINVAL;
    // the topology must tile the blocks: positive sizes, contiguous, covering n_b
    const int32_t *part = reinterpret_cast<const int32_t *>(static_cast<const char *>(h_state) + sizeof h);
    const int32_t *pos = part + P;
    int64_t next = 0;
    for (size_t p = 0; p < P; ++p) {
        if (part[p] < 1 || pos[p] != next) return EXDYNA_EINVAL;
        next += part[p];
    }
    if ((uint64_t)next != c->n_b) return EXDYNA_EINVAL;

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    c->stream = s;
    if (c->prof_slots) {
        HIP_TRY(c, hipStreamSynchronize(s));
        drop_events(c);
    }
    c->t = h.t;
    c->phase = 0;  // a selection waiting for its exchange is dropped
    c->sel_rank = kAllParts;
    const Layout &L = c->lay;
    HIP_TRY(c, hipMemcpyAsync(slot_part(c, c->t), part, 2 * P * sizeof(int32_t),
                              hipMemcpyHostToDevice, s));
    HIP_TRY(c, hipMemcpyAsync(slot_part(c, c->t + 1), part, 2 * P * sizeof(int32_t),
                              hipMemcpyHostToDevice, s));
    hipLaunchKernelGGL(k_restore_state, dim3(1), dim3(1), 0, s, at<DevState>(c, L.state), h.t, h.delta);
    hipLaunchKernelGGL(k_fill_u32, dim3(256), dim3(256), 0, s, at<uint32_t>(c, L.blk_cnt), 0u,
                       (size_t)(2 * L.blk_stride));
    hipLaunchKernelGGL(k_fill_u32, dim3(64), dim3(256), 0, s, at<uint32_t>(c, L.seg_cnt), 0u,
                       (size_t)(2 * L.seg_stride));
    hipLaunchKernelGGL(k_fill_u32, dim3(64), dim3(256), 0, s, at<uint32_t>(c, L.err_slots), 0u,
                       (size_t)(4 * kErrSlots * 2));
    hipLaunchKernelGGL(k_init_slot_tab, dim3(256), dim3(256), 0, s, slot_tab_of(c, 0), slot_tab_of(c, 1),
                       (uint32_t)L.n_tiles);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(s));  // h_state may be freed by the caller on return
    return EXDYNA_OK;
}

int exdyna_set_profiling(exdyna_ctx *c, uint32_t n_slots, uint32_t every)
{
    if (!ctx_ok(c)) return c ? EXDYNA_ESTATE : EXDYNA_ENULL;
    if (n_slots > 65536 || (n_slots && every == 0)) return EXDYNA_EINVAL;
    if (c->prof_slots) {
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        drop_events(c);
    }
    if (n_slots == 0) return EXDYNA_OK;
    c->ev = static_cast<hipEvent_t *>(calloc(3 * (size_t)n_slots, sizeof(hipEvent_t)));
    if (!c->ev) return EXDYNA_ENOMEM;
    for (uint32_t i = 0; i < 3 * n_slots; ++i) {
        hipError_t e = hipEventCreate(&c->ev[i]);
        if (e != hipSuccess) {
            for (uint32_t j = 0; j < i; ++j) (void)hipEventDestroy(c->ev[j]);
            free(c->ev);
            c->ev = nullptr;
            return hip_fail(c, e, "hipEventCreate");
        }
    }
    c->prof_slots = n_slots;
    c->prof_every = every;
    c->prof_since = c->t;
    return EXDYNA_OK;
}

int exdyna_get_kernel_ms(exdyna_ctx *c, uint64_t iteration, float *h_ms2)
{
    if (!ctx_ok(c)) return c ? EXDYNA_ESTATE : EXDYNA_ENULL;
    if (!h_ms2) return EXDYNA_ENULL;
    if (!c->prof_slots) return EXDYNA_ESTATE;
    // only recorded iterations, enqueued while profiling was on and not yet overwritten
    if (iteration >= c->t || iteration < c->prof_since) return EXDYNA_EINVAL;
    if ((iteration - c->prof_since) % c->prof_every != 0) return EXDYNA_EINVAL;
    const uint64_t sample = (iteration - c->prof_since) / c->prof_every;
    const uint64_t latest = (c->t - 1 - c->prof_since) / c->prof_every;
    if (latest - sample >= c->prof_slots) return EXDYNA_EINVAL;
    hipEvent_t *ev = c->ev + 3 * (sample % c->prof_slots);
    HIP_TRY(c, hipEventSynchronize(ev[2]));
    for (int i = 0; i < 2; ++i) HIP_TRY(c, hipEventElapsedTime(&h_ms2[i], ev[i], ev[i + 1]));
    return EXDYNA_OK;
}

const char *exdyna_strerror(int code)
{
    switch (code) {
    case EXDYNA_OK: return "ok";
    case EXDYNA_EINVAL: return "configuration value out of range";
    case EXDYNA_ENULL: return "required pointer is NULL";
    case EXDYNA_EALIGN: return "device pointer not aligned as required";
    case EXDYNA_ESTATE: return "context not initialised, destroyed, or no step run yet";
    case EXDYNA_ENOMEM: return "workspace too small or host allocation failed";
    case EXDYNA_EHIP: return "HIP runtime call failed";
    default: return "unknown error code";
    }
}

const char *exdyna_last_hip_error(const exdyna_ctx *c) { return ctx_ok(c) ? c->hip_err : ""; }

int exdyna_destroy(exdyna_ctx *c)
{
    if (!c) return EXDYNA_ENULL;
    if (!ctx_unregister(c)) return EXDYNA_ESTATE;  // never a context, or destroyed already: not touched
    drop_events(c);
    c->magic = 0;
    if (c->static_dev >= 0) {
        // a built-in context is not heap memory: its device's scratch becomes free for the next one
        std::lock_guard<std::mutex> lock(g_static_mu);
        g_static[c->static_dev].live = false;
    } else {
        delete c;
    }
    return EXDYNA_OK;
}

}  // extern "C"
