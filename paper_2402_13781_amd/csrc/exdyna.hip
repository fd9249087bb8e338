// ExDyna gradient-selection hot path for MI355X (gfx950, wave64).
//
// Two kernels per iteration, both enqueued by exdyna_step with no host round
// trip (threshold, topology and counters live in device memory):
//
//   k_stream   acc = e + g (Alg. 1, accumulate), |acc| cmp delta (Alg. 4).
//              Each wavefront owns 1024 contiguous gradients (a "wave tile").
//              It ranks its selected gradients with ballots, writes their
//              (index, value) pairs in index order into the tile's staging
//              slots, writes the residual with those entries already zeroed
//              (Alg. 1, zeroing and residual carry), stores the tile's count, and
//              adds the count to a per-block and a per-segment counter.  A tile with
//              more selected gradients than it has slots is only counted and
//              flagged; its residual is written unzeroed.
//              Pure streaming: 8 B read + 4 B written per gradient, no
//              workgroup barrier, no fence.
//   k_finish   workgroup 0 = control: per-partition counts k_{p,t} and k'
//              (Alg. 1, the gathered counts and their sum), output segment
//              offsets, threshold scaling (Alg. 5), adjacent-partition
//              rebalancing (Alg. 3's sweep), Eq. 2/5/6 statistics.
//              other workgroups = compaction, one wavefront per chunk of up to
//              64 wave tiles: prefix of the segment counters in front (summed
//              by the whole workgroup), a wave scan of the tile counts, then
//              all lanes copy the chunk's staged pairs to their final
//              positions (Alg. 1, Sparsify and value gather).  Flagged tiles are
//              re-read from the residual and compacted by the whole wave.  Pairs beyond the
//              output capacity are put back into the residual.  The same
//              prefix lays out the next iteration's staging slots: a tile gets
//              slots in proportion to what it selected this time, so dense
//              regions and threshold transients stay on the staged path.
//              Control and compaction read the same finished counters and do
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
// hot counters shared by many workgroups (same cost per same-address atomic),
// a workgroup barrier in the streaming pass (6 % slower), and gathering the
// selected values from the residual afterwards (random 4-byte reads over
// gigabytes cost more than the whole compaction does now).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "exdyna.h"

namespace {

constexpr uint32_t kGran        = 256;   // gradients per wave load: 64 lanes x float4
constexpr uint32_t kTileGran    = 4;     // granules per wave tile
constexpr uint32_t kTile        = kGran * kTileGran;  // 1024 gradients per wavefront
constexpr uint32_t kStreamWG    = 256;   // k_stream: 4 wavefronts = 4096 contiguous gradients
constexpr uint32_t kWavesPerWG  = kStreamWG / 64;
constexpr uint32_t kChunkShift  = 6;     // at most 64 wave tiles (65536 gradients) per compaction wavefront
constexpr uint32_t kMaxParts    = 1024;
constexpr uint32_t kFinishWG    = 1024;  // k_finish: 16 waves = control, or 16 chunks
constexpr uint32_t kErrSlots    = 256;
constexpr uint32_t kFlag        = 0x80000000u;  // tile count flag: pairs not staged
constexpr uint32_t kAllParts    = 0xFFFFFFFFu;  // selection over every partition (one device plays all workers)
constexpr uint64_t kMagic       = 0x45784479'6e61'0002ull;

// Device-resident scalar state.  One instance at the start of the workspace.
struct DevState {
    float    delta[2];    // delta[t & 1] is what iteration t compares with
    float    delta_used;  // threshold the last iteration compared with
    float    delta_next;  // threshold the next iteration will compare with
    uint32_t overflow;
    uint32_t moves;
    uint64_t t;
    uint64_t k_actual;
    uint64_t k_emitted;
    uint64_t k_max_part;
    double   density_error;
    double   traffic_ratio;
    double   err_norm;
    uint64_t own_actual;   // what the output lists hold: selected / emitted by the last selection pass
    uint64_t own_emitted;  // (one worker's share in the worker view, everything otherwise)
    uint32_t bad_index;    // worker view: gathered indices >= n_g that were skipped
    uint32_t pad;
};

struct CtrlParams {
    uint64_t n_g;
    uint64_t cap;
    double   k;          // d * n_g
    double   alpha, inv_alpha, beta, inv_beta;
    float    sf_hi, sf_mid, sf_lo;
    uint32_t n_b, n_parts, block_size, blk_move, min_blk;
};

struct Layout {
    size_t state, parts, part_cnt, part_off, blk_cnt, seg_cnt, tile_cnt, err_slots, stage,
        out_idx, out_val, total;
    size_t n_tiles, n_chunks, n_segs, pool_pairs;
    uint32_t chunk_shift; // log2(wave tiles per compaction wavefront)
    uint32_t one_counter; // blocks coincide with segments: one counter array serves both
    size_t slot_tab;
    uint32_t pool_extra; // staging pairs handed out in proportion to the last counts
    uint32_t slots;      // staging slots every wave tile always has
    uint32_t seg_shift;  // log2(wave tiles per segment counter)
};

typedef float f32x4 __attribute__((ext_vector_type(4)));

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---------------------------------------------------------------------------
// device helpers

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, uint32_t lane)
{
#pragma unroll
    for (uint32_t d = 1; d < 64; d <<= 1) {
        uint32_t t = __shfl_up(v, d, 64);
        if (lane >= d) v += t;
    }
    return v;
}

template <int CMP>
__device__ __forceinline__ uint32_t sel(float a, float delta)
{
    // |NaN| never compares true, +-Inf always does.
    return CMP ? (__builtin_fabsf(a) > delta) : (__builtin_fabsf(a) >= delta);
}

// number of set bits of `m` in lanes below this one
__device__ __forceinline__ uint32_t lanes_below(uint64_t m)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// Flags of one granule (nib: bit q <-> gradient 4*lane + q) -> how many are
// set in the whole granule, and how many precede this lane's, in index order.
__device__ __forceinline__ void granule_ranks(uint32_t nib, uint32_t &count, uint32_t &below)
{
    const uint64_t b0 = __ballot(nib & 1u), b1 = __ballot(nib & 2u), b2 = __ballot(nib & 4u),
                   b3 = __ballot(nib & 8u);
    count = (uint32_t)(__popcll(b0) + __popcll(b1) + __popcll(b2) + __popcll(b3));
    below = lanes_below(b0) + lanes_below(b1) + lanes_below(b2) + lanes_below(b3);
}

// Gradient element types of exdyna_step_scaled.  16-bit inputs are widened to
// fp32 exactly (bf16: the bits are the upper half of an fp32; fp16: hardware
// conversion), then the accumulate is fl(e + fl(eta * g)): one fp32 multiply,
// one fp32 add, never contracted into an FMA (the file is built with
// -ffp-contract=off and the pragma below repeats it).
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

template <int GT>
__device__ __forceinline__ f32x4 load_grad4(const void *g, size_t elem)
{
    if (GT == EXDYNA_F32) {
        return __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(static_cast<const float *>(g) + elem));
    } else if (GT == EXDYNA_BF16) {
        const u16x4 r = __builtin_nontemporal_load(
            reinterpret_cast<const u16x4 *>(static_cast<const unsigned short *>(g) + elem));
        f32x4 v;
        v.x = __uint_as_float((uint32_t)r.x << 16);
        v.y = __uint_as_float((uint32_t)r.y << 16);
        v.z = __uint_as_float((uint32_t)r.z << 16);
        v.w = __uint_as_float((uint32_t)r.w << 16);
        return v;
    } else {
        const f16x4 r = __builtin_nontemporal_load(
            reinterpret_cast<const f16x4 *>(static_cast<const _Float16 *>(g) + elem));
        return __builtin_convertvector(r, f32x4);
    }
}

template <int GT>
__device__ __forceinline__ float load_grad1(const void *g, uint64_t elem)
{
    if (GT == EXDYNA_F32) return static_cast<const float *>(g)[elem];
    if (GT == EXDYNA_BF16)
        return __uint_as_float((uint32_t) static_cast<const unsigned short *>(g)[elem] << 16);
    return (float)static_cast<const _Float16 *>(g)[elem];
}

template <bool SCALE>
__device__ __forceinline__ float accumulate(float e, float g, float eta)
{
#pragma clang fp contract(off)
    if (SCALE) {
        const float p = eta * g;  // rounded to fp32 before the add
        return e + p;
    }
    return e + g;
}

// ---------------------------------------------------------------------------
// k_stream: error-feedback accumulate + compare + rank + stage + zeroed
// write-back.  Workgroup w streams gradients [4096 w, 4096 (w+1)); its wave v
// owns wave tile 4w + v = four consecutive granules.
struct StreamArgs {
    const void     *g;          // n_g gradients of the kernel's element type
    float           eta;        // learning rate (used by the scaled variants only)
    float          *e;
    const DevState *st;
    uint2          *stage;      // staging pool of (index, value bits) pairs
    const uint2    *slot_tab;   // per tile: {first slot, number of slots} for this iteration
    uint32_t       *tile_cnt;   // n_tiles: selected in the tile, kFlag if not staged
    uint32_t       *blk_cnt;    // this iteration's per-block counters (zero on entry)
    uint32_t       *seg_cnt;    // this iteration's per-segment counters (zero on entry)
    double         *err_slots;
    uint32_t        n_g, n_tiles, gran_per_blk, parity;
    uint32_t        gpb_shift;  // log2(gran_per_blk) when it is a power of two, else 32
    uint32_t        seg_shift;  // log2(wave tiles per segment counter), 2..6
    uint32_t        one_counter;  // a block is exactly one segment: blk_cnt doubles as seg_cnt
    // worker view (Alg. 1 (Sparsify)): compare only inside partition own_part of this
    // iteration's topology; kAllParts = everywhere
    uint32_t        own_part;
    const int32_t  *cur_part;
    const int32_t  *cur_pos;
    uint32_t        block_size;  // b (the generic variant counts and masks by element index)
};

// Gradient range [lo, hi) of partition p, cut at n_g (Alg. 3 (partition range)).
__device__ __forceinline__ void partition_elems(const int32_t *part, const int32_t *pos, uint32_t p,
                                                uint32_t block_size, uint32_t n_g, uint32_t &lo, uint32_t &hi)
{
    const uint64_t a = (uint64_t)(uint32_t)pos[p] * block_size;
    const uint64_t b = (uint64_t)((uint32_t)pos[p] + (uint32_t)part[p]) * block_size;
    lo = (uint32_t)(a < n_g ? a : n_g);
    hi = (uint32_t)(b < n_g ? b : n_g);
}

// Granule range [lo, hi) of partition p: blocks are whole granules (b % 256 == 0).
__device__ __forceinline__ void partition_granules(const int32_t *part, const int32_t *pos, uint32_t p,
                                                   uint32_t gran_per_blk, uint32_t &lo, uint32_t &hi)
{
    const uint32_t ps = (uint32_t)pos[p], pn = (uint32_t)part[p];
    lo = ps * gran_per_blk;
    hi = (ps + pn) * gran_per_blk;
}

// GEN: block sizes that are multiples of 32 but not of 256.  Block and partition
// boundaries then fall inside granules (always between lanes: a lane's four
// gradients share a 32-aligned group), so the comparison is masked per lane
// and every lane adds its own selected gradients to its block's counter.
template <int CMP, bool NORM, int GT, bool SCALE, bool GEN>
__global__ void __launch_bounds__(kStreamWG)
k_stream(StreamArgs A)
{
    const float    delta  = A.st->delta[A.parity];
    const uint32_t lane   = threadIdx.x & 63u;
    const uint32_t wave   = threadIdx.x >> 6;
    // the tile index is the same in all lanes: keep it in a scalar register
    const uint32_t tile   = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerWG + wave);
    const uint32_t gran0  = tile * kTileGran;
    const uint32_t n_full = A.n_g >> 8;  // complete granules
    const bool     live   = tile < A.n_tiles;            // wave-uniform
    const bool     fast   = gran0 + kTileGran <= n_full;  // wave-uniform: no ragged end inside
    float nrm = 0.f;
    uint32_t g_lo = 0u, g_hi = 0xFFFFFFFFu;  // granules that are compared at all
    uint32_t e_lo = 0u, e_hi = 0xFFFFFFFFu;  // GEN: the same as a gradient range
    if (A.own_part != kAllParts) {
        if (GEN)
            partition_elems(A.cur_part, A.cur_pos, A.own_part, A.block_size, A.n_g, e_lo, e_hi);
        else
            partition_granules(A.cur_part, A.cur_pos, A.own_part, A.gran_per_blk, g_lo, g_hi);
    }

    if (live && fast) {
        f32x4    a[kTileGran];
        uint32_t nib[kTileGran];
        const uint2 tab = A.slot_tab[tile];  // requested with the data, used only if something is selected
        {
            f32x4 gv[kTileGran], ev[kTileGran];
#pragma unroll
            for (uint32_t u = 0; u < kTileGran; ++u) {
                const size_t off = ((size_t)(gran0 + u) << 8) + lane * 4u;
                gv[u] = load_grad4<GT>(A.g, off);
                ev[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(A.e + off));
            }
#pragma unroll
            for (uint32_t u = 0; u < kTileGran; ++u) {
                a[u].x = accumulate<SCALE>(ev[u].x, gv[u].x, A.eta);
                a[u].y = accumulate<SCALE>(ev[u].y, gv[u].y, A.eta);
                a[u].z = accumulate<SCALE>(ev[u].z, gv[u].z, A.eta);
                a[u].w = accumulate<SCALE>(ev[u].w, gv[u].w, A.eta);
                nib[u] = sel<CMP>(a[u].x, delta) | (sel<CMP>(a[u].y, delta) << 1) |
                         (sel<CMP>(a[u].z, delta) << 2) | (sel<CMP>(a[u].w, delta) << 3);
                if (GEN) {
                    const uint32_t i0 = ((gran0 + u) << 8) + lane * 4u;
                    if (i0 < e_lo || i0 >= e_hi) nib[u] = 0u;
                } else if (gran0 + u < g_lo || gran0 + u >= g_hi) {
                    nib[u] = 0u;  // wave-uniform: another worker's partition
                }
            }
        }

        if (NORM) {
#pragma unroll
            for (uint32_t u = 0; u < kTileGran; ++u) {
                nrm += (nib[u] & 1u) ? 0.f : a[u].x * a[u].x;
                nrm += (nib[u] & 2u) ? 0.f : a[u].y * a[u].y;
                nrm += (nib[u] & 4u) ? 0.f : a[u].z * a[u].z;
                nrm += (nib[u] & 8u) ? 0.f : a[u].w * a[u].w;
            }
        }

        uint32_t total = 0, word = 0;
        if (__ballot((nib[0] | nib[1] | nib[2] | nib[3]) != 0)) {  // wave-uniform
            uint32_t cu[kTileGran], below[kTileGran];
#pragma unroll
            for (uint32_t u = 0; u < kTileGran; ++u) {
                cu[u] = 0;
                below[u] = 0;
                if (__ballot(nib[u] != 0)) granule_ranks(nib[u], cu[u], below[u]);  // wave-uniform
                total += cu[u];
            }
            word = total;
            if (total <= tab.y) {
                // staged: pairs in index order, residual zeroed where sent (+0)
                uint2   *slot = A.stage + tab.x;
                uint32_t pre  = 0;
#pragma unroll
                for (uint32_t u = 0; u < kTileGran; ++u) {
                    if (nib[u]) {
                        uint32_t       r  = pre + below[u];
                        const uint32_t i0 = ((gran0 + u) << 8) + lane * 4u;
                        if (nib[u] & 1u) { slot[r++] = make_uint2(i0, __float_as_uint(a[u].x)); a[u].x = 0.f; }
                        if (nib[u] & 2u) { slot[r++] = make_uint2(i0 + 1u, __float_as_uint(a[u].y)); a[u].y = 0.f; }
                        if (nib[u] & 4u) { slot[r++] = make_uint2(i0 + 2u, __float_as_uint(a[u].z)); a[u].z = 0.f; }
                        if (nib[u] & 8u) { slot[r++] = make_uint2(i0 + 3u, __float_as_uint(a[u].w)); a[u].w = 0.f; }
                    }
                    pre += cu[u];
                }
            } else {
                word = total | kFlag;  // too many for the slots: compaction re-reads this tile
            }
            if (GEN) {
#pragma unroll
                for (uint32_t u = 0; u < kTileGran; ++u)
                    if (nib[u])
                        atomicAdd(&A.blk_cnt[(((gran0 + u) << 8) + lane * 4u) / A.block_size],
                                  (uint32_t)__popc(nib[u]));
                if (lane == 0) atomicAdd(&A.seg_cnt[tile >> A.seg_shift], total);
            } else if (lane == 0) {
                // One counter per block / segment keeps same-address atomics rare (they
                // serialise at roughly 150 ns each across the dies).
                if (A.one_counter) {
                    // a block is exactly one segment: the same counter serves both
                    atomicAdd(&A.blk_cnt[tile >> A.seg_shift], total);
                } else {
                    // per-block counters; consecutive granules of one block are added together
                    uint32_t blk = A.gpb_shift < 32u ? gran0 >> A.gpb_shift : gran0 / A.gran_per_blk;
                    uint32_t in_blk = gran0 - blk * A.gran_per_blk;  // granule's position inside its block
                    uint32_t run = cu[0];
#pragma unroll
                    for (uint32_t u = 1; u < kTileGran; ++u) {
                        if (++in_blk == A.gran_per_blk) {  // granule gran0 + u starts the next block
                            if (run) atomicAdd(&A.blk_cnt[blk], run);
                            ++blk;
                            in_blk = 0;
                            run = 0;
                        }
                        run += cu[u];
                    }
                    if (run) atomicAdd(&A.blk_cnt[blk], run);
                    atomicAdd(&A.seg_cnt[tile >> A.seg_shift], total);
                }
            }
        }

#pragma unroll
        for (uint32_t u = 0; u < kTileGran; ++u) {
            const size_t off = ((size_t)(gran0 + u) << 8) + lane * 4u;
            __builtin_nontemporal_store(a[u], reinterpret_cast<f32x4 *>(A.e + off));
        }
        if (lane == 0) A.tile_cnt[tile] = word;
    } else if (live) {
        // The ragged end of the vector (at most the last workgroup): guarded
        // scalar accesses, one granule at a time.  The tile is only counted and
        // flagged; compaction ranks and zeroes it from the residual.
        uint32_t total = 0;
#pragma unroll 1
        for (uint32_t u = 0; u < kTileGran; ++u) {
            const uint64_t base = ((uint64_t)(gran0 + u) << 8) + lane * 4u;
            uint32_t f = 0;
            const bool mine = GEN ? (base >= e_lo && base < e_hi)
                                  : (gran0 + u >= g_lo && gran0 + u < g_hi);  // wave-uniform unless GEN
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q) {
                if (base + q < A.n_g) {
                    const float v = accumulate<SCALE>(A.e[base + q], load_grad1<GT>(A.g, base + q), A.eta);
                    A.e[base + q] = v;
                    const uint32_t hit = mine ? sel<CMP>(v, delta) : 0u;
                    f |= hit << q;
                    if (NORM) nrm += hit ? 0.f : v * v;
                }
            }
            uint32_t cu, below;
            granule_ranks(f, cu, below);
            if (GEN) {
                if (f) atomicAdd(&A.blk_cnt[(uint32_t)base / A.block_size], (uint32_t)__popc(f));
            } else if (cu && lane == 0) {
                atomicAdd(&A.blk_cnt[(gran0 + u) / A.gran_per_blk], cu);  // = its segment if one_counter
            }
            total += cu;
        }
        if (lane == 0) {
            if (total && !A.one_counter) atomicAdd(&A.seg_cnt[tile >> A.seg_shift], total);
            A.tile_cnt[tile] = total ? (total | kFlag) : 0u;
        }
    }

    if (NORM) {
        __shared__ double wsum[kWavesPerWG];
        double s = (double)nrm;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d, 64);
        if (lane == 0) wsum[wave] = s;
        __syncthreads();
        if (threadIdx.x == 0) {
            double tot = wsum[0] + wsum[1] + wsum[2] + wsum[3];
            atomicAdd(&A.err_slots[blockIdx.x % kErrSlots], tot);
        }
    }
}

// ---------------------------------------------------------------------------
struct FinishArgs {
    DevState       *st;
    float          *e;
    const uint2    *stage;
    const uint2    *slot_tab;        // this iteration's {first slot, slots} per tile
    uint2          *slot_tab_next;   // the next iteration's, written here
    const uint32_t *tile_cnt;
    const uint32_t *blk_cnt;         // this iteration's per-block counters (complete)
    const uint32_t *seg_cnt;         // this iteration's per-segment counters (complete)
    uint32_t       *blk_cnt_next;    // the other parity's counters, cleared here
    uint32_t       *seg_cnt_next;
    const int32_t  *cur_part;        // topology this iteration selected with
    const int32_t  *cur_pos;
    int32_t        *nxt_part;        // receives Alg. 3's adjusted topology
    int32_t        *nxt_pos;
    uint64_t       *part_cnt;
    uint64_t       *part_off;
    uint32_t       *out_idx;
    float          *out_val;
    double         *err_slots;       // this iteration's norm partials
    double         *err_slots_next;  // cleared here
    uint32_t        n_tiles, n_chunks, n_segs, seg_shift, chunk_shift, slots_min, pool_extra, parity;
    uint32_t        mode;            // kCtrlFull or kCtrlSelect
    uint32_t        own_part;        // worker view: the partition that was compared; else kAllParts
    uint32_t        block_size;
};

// ---- control: workgroup 0 of k_finish (1024 threads) ----
//
// Alg. 3's sweep looks sequential (pair i sees what pair i-1 did), but pair
// i-1 can leave pair i in only three states: untouched, or k[i] and
// blk_part[i] raised, or lowered, by one move.  So every pair's decision is
// tabulated for the three states side by side, and the chain of tables is
// resolved with a prefix scan of table compositions.  A table is three 2-bit
// actions (0 none, 1 blocks go right: the first move, 2 blocks go left: the
// second), and the action a pair takes is the state it hands to the next pair.
__device__ __forceinline__ uint32_t compose(uint32_t later, uint32_t earlier)
{
    // (later o earlier)[s] = later[earlier[s]]
    return ((later >> (2u * (earlier & 3u))) & 3u) |
           (((later >> (2u * ((earlier >> 2) & 3u))) & 3u) << 2) |
           (((later >> (2u * ((earlier >> 4) & 3u))) & 3u) << 4);
}

// Shared-memory scratch of the control workgroup.
struct CtrlShared {
    uint32_t cnt[kMaxParts];    // selected per partition
    int32_t  lpos[kMaxParts];   // topology the iteration selected with
    int32_t  lpart[kMaxParts];
    uint8_t  flags[kMaxParts];
    uint32_t wsum[kFinishWG / 64];
    uint32_t wmax[kFinishWG / 64];
    uint32_t wfun[kFinishWG / 64];
    uint32_t wcarry[kFinishWG / 64];
    uint32_t n_moves;
    uint64_t k_total;
};

// What the control workgroup does with the per-partition counts.
enum : uint32_t {
    kCtrlFull   = 0,  // one device plays every worker: offsets, Alg. 5, Alg. 3, statistics
    kCtrlSelect = 1,  // worker view, after the selection pass: output offsets of the own list only
    kCtrlUpdate = 2   // worker view, after the exchange: Alg. 5, Alg. 3, statistics from the gathered counts
};

// k_{p,t} from the per-block counters (Sec. 4.2: the workload of a partition).
// Each wave takes a contiguous run of the counters, 64 at a time; its first
// slices are requested before anything waits on memory.  Also clears the other
// parity's block counters and norm partials for the next iteration.
__device__ void control_counts(const FinishArgs &A, const CtrlParams &prm, CtrlShared &S)
{
    constexpr uint32_t kWaves = kFinishWG / 64;
    const uint32_t tid  = threadIdx.x;
    const uint32_t lane = tid & 63u;
    const uint32_t wave = tid >> 6;
    const uint32_t P    = prm.n_parts;
    const uint32_t n_b  = prm.n_b;

    const uint32_t per_wave = (n_b + kWaves - 1) / kWaves;
    const uint32_t beg      = wave * per_wave < n_b ? wave * per_wave : n_b;
    const uint32_t end      = beg + per_wave < n_b ? beg + per_wave : n_b;
    constexpr uint32_t kAhead = 4;
    uint32_t cbuf[kAhead];
#pragma unroll
    for (uint32_t q = 0; q < kAhead; ++q) {
        const uint32_t i = beg + q * 64u + lane;
        cbuf[q] = i < end ? A.blk_cnt[i] : 0u;
    }
    if (tid < P) {
        S.cnt[tid]   = 0u;
        S.lpos[tid]  = A.cur_pos[tid];
        S.lpart[tid] = A.cur_part[tid];
    }
    if (tid < kErrSlots) A.err_slots_next[tid] = 0.0;
    __syncthreads();

    if (beg < end) {  // wave-uniform
        // partition of the run's first block: the largest p with blk_pos[p] <= beg
        uint32_t plo = 0, phi = P - 1;
        while (plo < phi) {
            const uint32_t mid = (plo + phi + 1) >> 1;
            if ((uint32_t)S.lpos[mid] <= beg) plo = mid; else phi = mid - 1;
        }
        uint32_t pcur       = plo;
        uint32_t next_start = pcur + 1 < P ? (uint32_t)S.lpos[pcur + 1] : 0xFFFFFFFFu;
        uint32_t acc        = 0;  // this lane's share of partition pcur so far
        for (uint32_t i0 = beg; i0 < end; i0 += kAhead * 64u) {
            if (i0 != beg) {
#pragma unroll
                for (uint32_t q = 0; q < kAhead; ++q) {
                    const uint32_t i = i0 + q * 64u + lane;
                    cbuf[q] = i < end ? A.blk_cnt[i] : 0u;
                }
            }
#pragma unroll
            for (uint32_t q = 0; q < kAhead; ++q) {
                const uint32_t s0 = i0 + q * 64u;  // first block of this slice
                const uint32_t i  = s0 + lane;
                if (i < end) A.blk_cnt_next[i] = 0u;  // clean block counters for the next iteration
                uint32_t c = cbuf[q];
                while (next_start < s0 + 64u && next_start < end) {  // the slice reaches the next partition
                    acc += i < next_start ? c : 0u;
                    c = i < next_start ? 0u : c;
#pragma unroll
                    for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
                    if (lane == 0 && acc) atomicAdd(&S.cnt[pcur], acc);
                    acc = 0;
                    ++pcur;
                    next_start = pcur + 1 < P ? (uint32_t)S.lpos[pcur + 1] : 0xFFFFFFFFu;
                }
                acc += c;
            }
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
        if (lane == 0 && acc) atomicAdd(&S.cnt[pcur], acc);
    }
    __syncthreads();
}

// Everything that follows from the per-partition counts in S.cnt (S.lpos /
// S.lpart hold the topology they were counted with).
__device__ void control_decide(const FinishArgs &A, const CtrlParams &prm, CtrlShared &S, uint32_t mode)
{
    constexpr uint32_t kWaves = kFinishWG / 64;
    constexpr uint32_t kIdent = 0u | (1u << 2) | (2u << 4);  // s -> s
    const uint32_t tid  = threadIdx.x;
    const uint32_t lane = tid & 63u;
    const uint32_t wave = tid >> 6;
    const uint32_t P    = prm.n_parts;

    float    delta  = 0.f;
    uint64_t t_done = 0;
    if (tid == 0) {
        delta  = A.st->delta[A.parity];
        t_done = A.st->t;
        S.n_moves = 0u;
    }
    const int32_t part = tid < P ? S.lpart[tid] : 0;
    const int32_t pos  = tid < P ? S.lpos[tid] : 0;

    // exclusive scan and maximum of the P counts (P <= 1024 = one value per thread)
    const uint32_t c    = tid < P ? S.cnt[tid] : 0u;
    const uint32_t incl = wave_incl_scan(c, lane);
    uint32_t mx = c;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t o = __shfl_xor(mx, d, 64);
        mx = o > mx ? o : mx;
    }
    if (lane == 63) S.wsum[wave] = incl;
    if (lane == 0) S.wmax[wave] = mx;
    __syncthreads();
    if (wave == 0) {
        const uint32_t v  = lane < kWaves ? S.wsum[lane] : 0u;
        const uint32_t vi = wave_incl_scan(v, lane);
        if (lane < kWaves) S.wsum[lane] = vi - v;
        if (lane == kWaves - 1) S.k_total = vi;  // k' (Alg. 1 (k' sum))
    }
    __syncthreads();
    const uint64_t excl     = (uint64_t)S.wsum[wave] + (incl - c);
    const uint64_t k_actual = S.k_total;
    if (tid < P) {
        A.part_cnt[tid] = c;
        if (mode != kCtrlUpdate) A.part_off[tid] = excl < prm.cap ? excl : prm.cap;
    }
    if (mode == kCtrlSelect) {  // the gathered counts decide the rest, after the exchange
        if (tid == 0) {
            DevState *st = A.st;
            A.part_off[P]   = k_actual < prm.cap ? k_actual : prm.cap;
            st->own_actual  = k_actual;
            st->own_emitted = k_actual < prm.cap ? k_actual : prm.cap;
            st->delta_used  = delta;
            st->bad_index   = 0u;
        }
        return;
    }

    // Alg. 3 (averages ahead of the sweep) and the two overload tests.  This iteration's
    // counts are the next Allocate's partial-k vector (Alg. 1 (partial-k carry)); they
    // are integers, so their fp64 sum is k' exactly.  When pair i is inspected,
    // k[i] is its count, or its count +/- k_move if pair i-1 moved blocks, and
    // k[i+1] is still its count: quotients for the three cases, compared
    // against alpha and 1/alpha, go into six flag bits.
    const double sum      = (double)k_actual;
    const double pk_prev  = sum / (double)P;
    const double den_prev = sum / (double)prm.n_g;
    const double k_move   = (double)prm.blk_move * (double)prm.block_size * den_prev;
    if (tid < P) {
        uint32_t f = 0;
        if (k_actual) {  // nothing selected: det is 0/0 and no pair moves
            const double kc = (double)c;
            const double d0 = kc / pk_prev;
            const double dp = (kc + k_move) / pk_prev;
            const double dm = (kc - k_move) / pk_prev;
            f = (d0 > prm.alpha ? 1u : 0u) | (d0 < prm.inv_alpha ? 2u : 0u) |
                (dp > prm.alpha ? 4u : 0u) | (dp < prm.inv_alpha ? 8u : 0u) |
                (dm > prm.alpha ? 16u : 0u) | (dm < prm.inv_alpha ? 32u : 0u);
        }
        S.flags[tid] = (uint8_t)f;
    }
    __syncthreads();

    // decision table of pair (tid, tid+1) for the three incoming states
    const int64_t bm      = (int64_t)prm.blk_move;
    const int64_t min_blk = (int64_t)prm.min_blk;
    uint32_t table = 0;  // beyond the last pair: every state maps to "none"
    if (tid + 1 < P) {
        const uint32_t f_i     = S.flags[tid];
        const uint32_t f_n     = S.flags[tid + 1];
        const bool     det2_hi = f_n & 1u, det2_lo = f_n & 2u;
        const int64_t  part_n  = S.lpart[tid + 1];
#pragma unroll
        for (uint32_t st = 0; st < 3; ++st) {
            const uint32_t fi     = f_i >> (2u * st);
            const bool     det_hi = fi & 1u, det_lo = fi & 2u;
            const int64_t  part_i = (int64_t)part + (st == 1 ? bm : st == 2 ? -bm : 0);
            uint32_t act = 0;
            if (det_hi && det2_lo) {
                if (!(part_i - bm < min_blk)) act = 1;   // else "continue" (first min_blk guard)
            } else if (det_lo && det2_hi) {
                if (!(part_n - bm < min_blk)) act = 2;   // else "continue" (second min_blk guard)
            }
            table |= act << (2u * st);
        }
    }
    // inclusive scan of compositions: after it, `fun` maps the state entering
    // this wave's first pair to the state leaving pair tid
    uint32_t fun = table;
#pragma unroll
    for (uint32_t d = 1; d < 64; d <<= 1) {
        const uint32_t prev = __shfl_up(fun, d, 64);
        if (lane >= d) fun = compose(fun, prev);
    }
    if (lane == 63) S.wfun[wave] = fun;
    __syncthreads();
    if (tid == 0) {
        uint32_t stt = 0;  // pair 0 starts untouched
        for (uint32_t w = 0; w < kWaves; ++w) {
            S.wcarry[w] = stt;
            stt = (S.wfun[w] >> (2u * stt)) & 3u;
        }
    }
    __syncthreads();
    uint32_t before = __shfl_up(fun, 1, 64);
    if (lane == 0) before = kIdent;
    const uint32_t st_in = (before >> (2u * S.wcarry[wave])) & 3u;  // what pair tid-1 did
    const uint32_t act   = (table >> (2u * st_in)) & 3u;            // what pair tid does
    const uint64_t moved = __ballot(act != 0);
    if (lane == 0 && moved) atomicAdd(&S.n_moves, (uint32_t)__popcll(moved));
    if (tid < P) {
        const int32_t bmi = (int32_t)prm.blk_move;
        // the two block moves as seen from partition tid: it is the right side
        // of pair tid-1 and the left side of pair tid
        const int32_t d_in  = st_in == 1 ? bmi : st_in == 2 ? -bmi : 0;
        const int32_t d_out = act == 1 ? -bmi : act == 2 ? bmi : 0;
        A.nxt_part[tid] = part + d_in + d_out;
        A.nxt_pos[tid]  = pos - d_in;
    }
    __syncthreads();

    if (tid == 0) {
        DevState *st = A.st;
        // ---- Alg. 5: online threshold scaling ----
        const double exam = (double)k_actual / prm.k;
        float sf;
        if (exam > prm.beta)
            sf = prm.sf_hi;
        else if (exam > prm.inv_beta)
            sf = prm.sf_mid;
        else
            sf = prm.sf_lo;
        const float next = delta * sf;
        st->delta[A.parity ^ 1u] = next;  // the other slot: this iteration's compaction still reads delta[parity]
        st->delta_used = delta;
        st->delta_next = next;

        // ---- Eq. 2 / 5 / 6 ----
        uint64_t m_t = 0;
        for (uint32_t w = 0; w < kWaves; ++w) m_t = S.wmax[w] > m_t ? S.wmax[w] : m_t;
        uint64_t emitted = k_actual < prm.cap ? k_actual : prm.cap;
        if (mode == kCtrlFull) {
            A.part_off[P]   = emitted;
            st->own_actual  = k_actual;
            st->own_emitted = emitted;
        } else {
            // every worker's list is cut at the capacity on its own
            emitted = 0;
            for (uint32_t p = 0; p < P; ++p) emitted += S.cnt[p] < prm.cap ? S.cnt[p] : prm.cap;
        }
        st->k_actual      = k_actual;
        st->k_emitted     = emitted;
        st->overflow      = emitted < k_actual ? 1u : 0u;
        st->k_max_part    = m_t;
        st->density_error = fabs(prm.k - (double)k_actual) / (double)prm.n_g;
        st->traffic_ratio = k_actual ? (double)P * (double)m_t / (double)k_actual : 0.0;
        st->t     = t_done + 1;  // counted on the device so that a captured graph can be replayed
        st->moves = prm.blk_move ? S.n_moves : 0u;  // blk_move = 0: the pairs decide, nothing moves
    }
}

__device__ void finish_control(const FinishArgs &A, const CtrlParams &prm)
{
    __shared__ CtrlShared S;
    control_counts(A, prm, S);
    control_decide(A, prm, S, A.mode);
}

// ---- compaction: a workgroup takes 16 consecutive chunks, one wavefront per
// chunk, one lane per wave tile.  The output position of the chunk's first pair
// is the number of selected gradients in front of it: the workgroup sums the
// segment counters before its first chunk (all 1024 threads, counters sit in L2)
// and the wave totals inside the workgroup; a wave scan of the 64 tile counts
// then gives every lane the position of its tile's first pair.  Tiles, and the
// pairs staged inside a tile, are in index order, so the output is ascending. ----

// A flagged tile (more selected gradients than staging slots; its residual
// still holds acc): the whole wave re-reads its 1024 gradients, repeats the
// comparison with the threshold the streaming pass used, emits the pairs that
// fit the output and zeroes them in the residual.
template <bool NORM, int CMP>
__device__ __forceinline__ void compact_flagged_tile(const FinishArgs &A, uint32_t tile, uint64_t r0,
                                                     float delta, uint32_t lane, uint32_t n_g,
                                                     uint64_t cap, uint32_t e_lo, uint32_t e_hi,
                                                     float &spill)
{
    if (!NORM && r0 >= cap) return;  // nothing fits: the tile stays in the residual as it is
    float *__restrict__ e = A.e;
    const uint32_t gran0 = tile * kTileGran;
    float    v[kTileGran][4];
    uint32_t nib[kTileGran];
    if (gran0 + kTileGran <= (n_g >> 8)) {  // whole tile inside the vector: four float4 loads in flight
        f32x4 a[kTileGran];
#pragma unroll
        for (uint32_t u = 0; u < kTileGran; ++u)
            a[u] = *reinterpret_cast<const f32x4 *>(e + ((size_t)(gran0 + u) << 8) + lane * 4u);
#pragma unroll
        for (uint32_t u = 0; u < kTileGran; ++u) {
            v[u][0] = a[u].x; v[u][1] = a[u].y; v[u][2] = a[u].z; v[u][3] = a[u].w;
        }
    } else {
#pragma unroll
        for (uint32_t u = 0; u < kTileGran; ++u) {
            const uint64_t base = ((uint64_t)(gran0 + u) << 8) + lane * 4u;
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q) v[u][q] = base + q < n_g ? e[base + q] : 0.f;
        }
    }
#pragma unroll
    for (uint32_t u = 0; u < kTileGran; ++u) {
        const uint64_t base = ((uint64_t)(gran0 + u) << 8) + lane * 4u;
        nib[u] = 0;
        if (base >= e_lo && base < e_hi) {  // the streaming pass compared only these (a lane's four share a block)
#pragma unroll
            for (uint32_t q = 0; q < 4; ++q)
                if (base + q < n_g) nib[u] |= sel<CMP>(v[u][q], delta) << q;
        }
    }
    uint64_t running = r0;
#pragma unroll
    for (uint32_t u = 0; u < kTileGran; ++u) {
        const uint64_t base = ((uint64_t)(gran0 + u) << 8) + lane * 4u;
        uint32_t cu, below;
        granule_ranks(nib[u], cu, below);
        uint64_t r = running + below;
#pragma unroll
        for (uint32_t q = 0; q < 4; ++q) {
            if (nib[u] & (1u << q)) {
                if (r < cap) {
                    A.out_idx[r] = (uint32_t)(base + q);
                    A.out_val[r] = v[u][q];
                    e[base + q]  = 0.0f;  // +0 where sent (Alg. 1 (zeroing of the sent entries))
                } else if (NORM) {
                    spill += v[u][q] * v[u][q];  // selected but not emitted: stays in the residual
                }
                ++r;
            }
        }
        running += cu;
    }
}

template <bool NORM, int CMP>
__device__ void finish_compact(const FinishArgs &A, uint32_t n_g, uint64_t cap)
{
    constexpr uint32_t kWaves = kFinishWG / 64;
    __shared__ uint32_t red[kWaves];
    __shared__ uint32_t wtot[kWaves];
    __shared__ uint32_t s_incl[kWaves][64];  // per wave: running count of staged pairs over its tiles
    __shared__ uint32_t s_off[kWaves][64];   // first staging slot of each tile
    __shared__ uint32_t s_rel[kWaves][64];   // output position of each tile's first pair, minus the chunk's
    const uint32_t tid    = threadIdx.x;
    const uint32_t lane   = tid & 63u;
    const uint32_t wave   = tid >> 6;
    const uint32_t cs     = A.chunk_shift;             // log2(wave tiles per chunk)
    const uint32_t chunk0 = (blockIdx.x - 1u) * kWaves;
    const uint32_t chunk  = chunk0 + wave;
    const uint32_t tile   = (chunk << cs) + lane;

    // all first loads are requested before anything waits on them
    uint32_t word = 0;
    uint2    tab  = make_uint2(0u, 0u);
    const bool have_tile = chunk < A.n_chunks && lane < (1u << cs) && tile < A.n_tiles;
    if (have_tile) {
        word = A.tile_cnt[tile];
        tab  = A.slot_tab[tile];
    }
    float delta = 0.f;
    if (word & kFlag) delta = A.st->delta[A.parity];
    uint32_t s0 = 0, s1 = 0, s2 = 0, s3 = 0;
    {
        const uint32_t seg0 = (chunk0 << cs) >> A.seg_shift;  // segments in front of this workgroup
        uint32_t i = tid;
        for (; i + 3u * kFinishWG < seg0; i += 4u * kFinishWG) {
            s0 += A.seg_cnt[i];
            s1 += A.seg_cnt[i + kFinishWG];
            s2 += A.seg_cnt[i + 2u * kFinishWG];
            s3 += A.seg_cnt[i + 3u * kFinishWG];
        }
        for (; i < seg0; i += kFinishWG) s0 += A.seg_cnt[i];
    }
    uint32_t s = (s0 + s1) + (s2 + s3);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d, 64);

    const uint32_t c     = word & ~kFlag;                 // selected in this lane's tile
    const uint32_t cstg  = (word & kFlag) ? 0u : c;       // ... of which staged
    const uint32_t incl  = wave_incl_scan(c, lane);
    const uint32_t incls = wave_incl_scan(cstg, lane);
    const uint32_t tot   = __shfl(incl, 63, 64);
    const uint32_t tots  = __shfl(incls, 63, 64);
    s_incl[wave][lane] = incls;
    s_off[wave][lane]  = tab.x;
    s_rel[wave][lane]  = incl - c;
    if (lane == 0) {
        red[wave]  = s;
        wtot[wave] = tot;
    }
    __syncthreads();
    if (chunk >= A.n_chunks) return;
    uint64_t base = 0;  // selected gradients in front of this chunk
#pragma unroll
    for (uint32_t w = 0; w < kWaves; ++w) base += red[w] + (w < wave ? wtot[w] : 0u);

    {   // clean segment counters for the next iteration (a chunk holds whole segments)
        const uint32_t per_chunk = 1u << (cs - A.seg_shift);
        const uint32_t sg        = chunk * per_chunk + lane;
        if (lane < per_chunk && sg < A.n_segs) A.seg_cnt_next[sg] = 0u;
    }
    const uint64_t r0 = base + (incl - c);  // output position of this tile's first pair

    // Staging slots for the next iteration follow this iteration's counts: every
    // tile keeps slots_min slots and gets about two more per gradient it selected
    // now, as long as the pool's extra part lasts (it covers three times the
    // ranks the output can hold: tiles just beyond the capacity are the ones
    // that come within it next time).  Offsets are the running sum of the
    // sizes, taken from the same prefix that gives the output positions, and
    // rounded down to 16 pairs = 128 bytes, so two tiles never write into the
    // same cache line (partial writes to one line from different dies are slow).
    if (have_tile) {
        const uint64_t ex  = A.pool_extra;  // multiple of 16
        const uint64_t a2  = (2u * r0) & ~15ull, b2 = (2u * (r0 + c)) & ~15ull;
        const uint64_t lo2 = a2 < ex ? a2 : ex;
        const uint64_t hi2 = b2 < ex ? b2 : ex;
        A.slot_tab_next[tile] = make_uint2((uint32_t)((uint64_t)tile * A.slots_min + lo2),
                                           A.slots_min + (uint32_t)(hi2 - lo2));
    }

    if (tot == 0) return;
    float spill = 0.f;

    // Staged pairs of the whole chunk, copied by all lanes: pair number j of the
    // chunk (tiles in order, pairs in order inside a tile) belongs to the first
    // tile whose running staged count exceeds j.
    {
        const uint2 *__restrict__    stage   = A.stage;
        uint32_t *__restrict__       out_idx = A.out_idx;
        float *__restrict__          out_val = A.out_val;
        const uint32_t *__restrict__ incl_w  = s_incl[wave];
        const uint32_t *__restrict__ off_w = s_off[wave];
        const uint32_t *__restrict__ rel_w = s_rel[wave];
        // kCopy pairs per lane and trip.  The searches of one trip run side by side,
        // step by step (six LDS reads each, one after the other), and so do the loads
        // of the pairs they find.
        constexpr uint32_t kCopy = 8;
        for (uint32_t j0 = lane; j0 < tots; j0 += 64u * kCopy) {
            uint32_t pos[kCopy];
#pragma unroll
            for (uint32_t q = 0; q < kCopy; ++q) pos[q] = 0u;
            // first tile with incl_w[tile] > j: incl_w is non-decreasing over all 64
            // entries and incl_w[63] = tots > j, so the answer is in [0, 63]
#pragma unroll
            for (uint32_t step = 32u; step >= 1u; step >>= 1) {
#pragma unroll
                for (uint32_t q = 0; q < kCopy; ++q) {
                    const uint32_t j = j0 + q * 64u;
                    if (incl_w[pos[q] + step - 1u] <= j) pos[q] += step;
                }
            }
            uint2    pr[kCopy];
            uint32_t rr[kCopy];
#pragma unroll
            for (uint32_t q = 0; q < kCopy; ++q) {
                const uint32_t j = j0 + q * 64u;
                pr[q] = make_uint2(0u, 0u);
                rr[q] = 0;
                if (j < tots) {
                    const uint32_t t      = pos[q];
                    const uint32_t within = j - (t ? incl_w[t - 1u] : 0u);
                    pr[q] = stage[off_w[t] + within];
                    rr[q] = rel_w[t] + within;
                }
            }
#pragma unroll
            for (uint32_t q = 0; q < kCopy; ++q) {
                if (j0 + q * 64u < tots) {
                    const uint64_t r = base + rr[q];
                    if (r < cap) {
                        out_idx[r] = pr[q].x;
                        out_val[r] = __uint_as_float(pr[q].y);
                    } else {
                        // beyond the output capacity: not sent, so it goes back into the residual
                        const float v = __uint_as_float(pr[q].y);
                        A.e[pr[q].x] = v;
                        if (NORM) spill += v * v;
                    }
                }
            }
        }
    }

    uint64_t flagged = __ballot((word & kFlag) != 0);
    uint32_t e_lo = 0u, e_hi = 0xFFFFFFFFu;
    if (flagged && A.own_part != kAllParts)
        partition_elems(A.cur_part, A.cur_pos, A.own_part, A.block_size, n_g, e_lo, e_hi);
    while (flagged) {  // wave-uniform
        const uint32_t l = (uint32_t)__ffsll((unsigned long long)flagged) - 1u;
        flagged &= flagged - 1u;
        const uint32_t lo = __shfl((uint32_t)r0, l, 64), hi = __shfl((uint32_t)(r0 >> 32), l, 64);
        const float    dl = __shfl(delta, l, 64);
        compact_flagged_tile<NORM, CMP>(A, (chunk << cs) + l, ((uint64_t)hi << 32) | lo, dl, lane,
                                        n_g, cap, e_lo, e_hi, spill);
    }

    if (NORM) {
        double sq = (double)spill;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) sq += __shfl_xor(sq, d, 64);
        if (lane == 0 && sq != 0.0) atomicAdd(&A.err_slots[chunk % kErrSlots], sq);
    }
}

template <bool NORM, int CMP>
__global__ void __launch_bounds__(kFinishWG)
k_finish(FinishArgs A, CtrlParams prm)
{
    if (blockIdx.x == 0)
        finish_control(A, prm);
    else
        finish_compact<NORM, CMP>(A, (uint32_t)prm.n_g, prm.cap);
}

// ---------------------------------------------------------------------------
// Worker view, after the AllGather (Alg. 1: value gather and zeroing, then the
// k' sum, Estimate and the partial-k carry): one worker's residual meets the
// gathered index list of all workers.
//   blockIdx.y = r < P   rank r's part of the list: read acc at those indices
//                        into the value buffer (what the AllReduce will sum) and
//                        clear them.  The worker's own part was cleared by the
//                        streaming pass already: its values come from its list.
//   blockIdx.y = P       control: the gathered counts, moved from rank order
//                        to partition order (Alg. 3's re-indexing), drive
//                        Alg. 5 and Alg. 3 for the next iteration.
struct ExchangeArgs {
    const uint32_t *idx_all;  // P x stride: rank r's indices start at r * stride
    const uint64_t *counts;   // k_{r,t} by rank, not cut at the capacity
    float          *val_all;  // same layout as idx_all; 0 beyond each rank's list
    const float    *own_val;  // values of this worker's own list
    uint64_t        stride;
    uint32_t        rank;     // this worker
    uint32_t        t_mod_p;  // iteration mod P
};

template <bool NORM>
__global__ void __launch_bounds__(kFinishWG)
k_exchange(FinishArgs A, CtrlParams prm, ExchangeArgs X)
{
    const uint32_t P   = prm.n_parts;
    const uint32_t tid = threadIdx.x;
    if (blockIdx.y == P) {
        if (blockIdx.x != 0) return;
        __shared__ CtrlShared S;
        if (tid < P) {
            S.lpos[tid]  = A.cur_pos[tid];
            S.lpart[tid] = A.cur_part[tid];
            // rank tid selected partition (t mod P + tid) mod P (Alg. 3 (cyclic allocation))
            const uint64_t k_r = X.counts[tid];
            S.cnt[(X.t_mod_p + tid) % P] = (uint32_t)(k_r < prm.n_g ? k_r : prm.n_g);
        }
        __syncthreads();
        control_decide(A, prm, S, kCtrlUpdate);
        return;
    }
    const uint32_t r = blockIdx.y;
    const uint64_t q = (uint64_t)blockIdx.x * kFinishWG + tid;
    float sq = 0.f;
    if (q < X.stride) {
        uint64_t have = X.counts[r];
        have = have < prm.cap ? have : prm.cap;
        const uint64_t j = (uint64_t)r * X.stride + q;
        float v = 0.f;
        if (q < have) {
            if (r == X.rank) {
                v = X.own_val[q];
            } else {
                const uint32_t i = X.idx_all[j];
                if (i < prm.n_g) {
                    v = A.e[i];
                    A.e[i] = 0.0f;  // Alg. 1 (zeroing of the sent entries)
                    if (NORM) sq = v * v;
                } else {
                    atomicAdd(&A.st->bad_index, 1u);  // not a gradient index: skipped and reported
                }
            }
        }
        X.val_all[j] = v;  // Alg. 1 (value gather)
    }
    if (NORM) {
        // the streaming pass counted these entries as residual: take them out again
        double s = (double)sq;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d, 64);
        if ((tid & 63u) == 0 && s != 0.0) atomicAdd(&A.err_slots[(blockIdx.x + r) % kErrSlots], -s);
    }
}

// ---------------------------------------------------------------------------
// Alg. 1 (model update) on the selected entries only: x[idx] <- x[idx] - scale * g_t,
// one thread per entry of a rows x stride list (the layout of the exchange).
__global__ void __launch_bounds__(256)
k_apply(float *x, const uint32_t *idx, const float *val, const uint64_t *counts, uint64_t stride,
        uint64_t cap, uint32_t n_g, float scale, DevState *st)
{
#pragma clang fp contract(off)
    const uint32_t r = blockIdx.y;
    const uint64_t q = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= stride) return;
    uint64_t have = counts[r];
    have = have < cap ? have : cap;
    if (q >= have) return;
    const uint64_t j = (uint64_t)r * stride + q;
    const uint32_t i = idx[j];
    if (i >= n_g) {
        atomicAdd(&st->bad_index, 1u);
        return;
    }
    const float p = scale * val[j];  // rounded before the subtraction
    x[i] = x[i] - p;
}

// ---------------------------------------------------------------------------
// small set-up / read-out kernels

__global__ void k_fill_u32(uint32_t *p, uint32_t v, size_t n)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = v;
}

// Alg. 1's threshold and partition initialisation: delta_0 and Alg. 2's topology
// in closed form (the first `remainder` partitions hold quotient+1 blocks; positions are the exclusive
// prefix sum).  The uniform initial partial-k vector is not stored:
// with equal entries det = det2 for every pair, so the first Allocate moves
// nothing, and every later Allocate uses the counts of the step before it.
__global__ void k_init_state(DevState *st, int32_t *part0, int32_t *pos0, int32_t *part1,
                             int32_t *pos1, uint64_t *part_cnt, uint64_t *part_off,
                             double *err_slots, float delta0, uint32_t n_b, uint32_t P)
{
    const uint32_t tid = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t q = n_b / P, r = n_b % P;
    if (tid < P) {
        const int32_t part = (int32_t)(q + (tid < r ? 1u : 0u));
        const int32_t pos  = (int32_t)(tid * q + (tid < r ? tid : r));
        part0[tid] = part; pos0[tid] = pos;
        part1[tid] = part; pos1[tid] = pos;
        part_cnt[tid] = 0;
        part_off[tid] = 0;
    }
    if (tid == P) part_off[P] = 0;
    if (tid < 2 * kErrSlots) err_slots[tid] = 0.0;
    if (tid == 0) {
        st->delta[0] = delta0;
        st->delta[1] = delta0;
        st->delta_used = delta0;
        st->delta_next = delta0;
        st->overflow = 0; st->moves = 0; st->t = 0;
        st->k_actual = 0; st->k_emitted = 0; st->k_max_part = 0;
        st->density_error = 0.0; st->traffic_ratio = 0.0; st->err_norm = -1.0;
        st->own_actual = 0; st->own_emitted = 0; st->bad_index = 0; st->pad = 0;
    }
}

// Before the first iteration every wave tile has its slots_min staging slots.
__global__ void k_init_slot_tab(uint2 *tab0, uint2 *tab1, uint32_t n_tiles, uint32_t slots_min)
{
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n_tiles; i += gridDim.x * blockDim.x) {
        const uint2 v = make_uint2(i * slots_min, slots_min);
        tab0[i] = v;
        tab1[i] = v;
    }
}

// Resume: iteration counter and threshold as saved; statistics of "the last step" are cleared.
__global__ void k_restore_state(DevState *st, uint64_t t, float delta)
{
    st->delta[0] = delta;
    st->delta[1] = delta;
    st->delta_used = delta;
    st->delta_next = delta;
    st->overflow = 0; st->moves = 0; st->t = t;
    st->k_actual = 0; st->k_emitted = 0; st->k_max_part = 0;
    st->density_error = 0.0; st->traffic_ratio = 0.0; st->err_norm = -1.0;
    st->own_actual = 0; st->own_emitted = 0; st->bad_index = 0; st->pad = 0;
}

__global__ void k_norm_finalize(DevState *st, const double *err_slots)
{
    __shared__ double s[kErrSlots];
    s[threadIdx.x] = err_slots[threadIdx.x];
    __syncthreads();
    for (uint32_t d = kErrSlots / 2; d >= 1; d >>= 1) {
        if (threadIdx.x < d) s[threadIdx.x] += s[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) st->err_norm = sqrt(s[0] > 0.0 ? s[0] : s[0] == s[0] ? 0.0 : s[0]);
}

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
    uint32_t      own_part;  // partition the current selection pass compares, or kAllParts
    float        *d_residual;
    char         *ws;
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
// selected gradients in 1024 (density d), a power of two between 16 and 64
// (16 pairs = one 128-byte line).
uint32_t staging_slots(double density)
{
    const double want = 4.0 * density * (double)kTile + 4.0;
    uint32_t s = 16;
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
    uint32_t sh = kChunkShift;
    while (sh > 2 && (double)(1u << sh) * p_hit > 12.0) --sh;
    return sh;
}

// Wave tiles per compaction wavefront (a "chunk"): about 128 selected gradients
// per wavefront at the target density, between 4 and 64 tiles.
uint32_t chunk_shift_for(double density)
{
    const double per_tile = (double)kTile * density;
    uint32_t sh = kChunkShift;
    while (sh > 2 && (double)(1u << sh) * per_tile > 128.0) --sh;
    return sh;
}

Layout make_layout(const exdyna_config *c, uint64_t n_b, uint64_t cap)
{
    Layout L{};
    const size_t P = c->n_parts;
    L.n_tiles  = (c->n_g + kTile - 1) / kTile;
    L.chunk_shift = chunk_shift_for(c->density);
    L.n_chunks = (L.n_tiles + (1u << L.chunk_shift) - 1) >> L.chunk_shift;
    L.slots    = staging_slots(c->density);
    L.seg_shift = segment_shift(c->density);
    if (L.seg_shift > L.chunk_shift) L.seg_shift = L.chunk_shift;  // a chunk holds whole segments
    // When a block is a power-of-two number of tiles that is no coarser than that
    // segment size (and there are not too many blocks to sum over), let segments
    // be the blocks: the streaming pass then adds to one counter instead of two.
    L.one_counter = 0;
    for (uint32_t sh = 2; sh <= L.seg_shift; ++sh)
        if (c->block_size == (kTile << sh) && (sh == L.seg_shift || n_b <= 32768)) {
            L.seg_shift = sh;
            L.one_counter = 1;
        }
    L.n_segs   = (L.n_tiles + (1u << L.seg_shift) - 1) >> L.seg_shift;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    L.state     = take(sizeof(DevState));
    L.parts     = take(4 * P * sizeof(int32_t));             // slot0 part,pos ; slot1 part,pos
    L.part_cnt  = take(P * sizeof(uint64_t));
    L.part_off  = take((P + 1) * sizeof(uint64_t));
    L.blk_cnt   = take(2 * n_b * sizeof(uint32_t));           // two alternating counter arrays
    L.seg_cnt   = take(2 * L.n_segs * sizeof(uint32_t));      // likewise
    L.tile_cnt  = take(L.n_tiles * sizeof(uint32_t));
    L.err_slots = take(2 * kErrSlots * sizeof(double));
    // staging pool: slots for every tile plus two per pair for three output capacities
    {
        uint64_t extra = (6 * cap + 15) & ~15ull;
        const uint64_t fixed = (uint64_t)L.n_tiles * L.slots;
        if (fixed + extra > 0xFFFF0000ull) extra = (0xFFFF0000ull - fixed) & ~15ull;  // slot offsets are u32
        L.pool_extra = (uint32_t)extra;
        L.pool_pairs = fixed + extra;
    }
    L.slot_tab  = take(2 * L.n_tiles * sizeof(uint2));        // {first slot, slots} per tile, two parities
    L.stage     = take(L.pool_pairs * sizeof(uint2));
    L.out_idx   = take(cap * sizeof(uint32_t));
    L.out_val   = take(cap * sizeof(float));
    L.total     = off;
    return L;
}

bool ctx_ok(const exdyna_ctx *c) { return c && c->magic == kMagic; }

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
uint32_t *blk_cnt_of(exdyna_ctx *c, uint64_t t) { return at<uint32_t>(c, c->lay.blk_cnt) + (t & 1) * c->n_b; }
double *err_slots_of(exdyna_ctx *c, uint64_t t) { return at<double>(c, c->lay.err_slots) + (t & 1) * kErrSlots; }

uint2 *slot_tab_of(exdyna_ctx *c, uint64_t t) { return at<uint2>(c, c->lay.slot_tab) + (t & 1) * c->lay.n_tiles; }
uint32_t *seg_cnt_of(exdyna_ctx *c, uint64_t t) { return at<uint32_t>(c, c->lay.seg_cnt) + (t & 1) * c->lay.n_segs; }

template <int CMP, bool NORM, int GT, bool SCALE, bool GEN>
void launch_stream(exdyna_ctx *c, const void *g, float eta, hipStream_t s)
{
    StreamArgs A;
    A.g = g;
    A.eta = eta;
    A.e = c->d_residual;
    A.st = at<DevState>(c, c->lay.state);
    A.stage = at<uint2>(c, c->lay.stage);
    A.slot_tab = slot_tab_of(c, c->t);
    A.tile_cnt = at<uint32_t>(c, c->lay.tile_cnt);
    A.blk_cnt = blk_cnt_of(c, c->t);
    A.seg_cnt = c->lay.one_counter ? blk_cnt_of(c, c->t) : seg_cnt_of(c, c->t);
    A.seg_shift = c->lay.seg_shift;
    A.one_counter = c->lay.one_counter;
    A.err_slots = err_slots_of(c, c->t);
    A.n_g = (uint32_t)c->cfg.n_g;
    A.n_tiles = (uint32_t)c->lay.n_tiles;
    A.gran_per_blk = c->cfg.block_size / kGran;
    A.gpb_shift = 32;
    for (uint32_t sh = 0; sh < 32; ++sh)
        if ((1u << sh) == A.gran_per_blk) A.gpb_shift = sh;
    A.parity = (uint32_t)(c->t & 1);
    A.own_part = c->own_part;
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
    A.slot_tab = slot_tab_of(c, t);
    A.slot_tab_next = slot_tab_of(c, t + 1);
    A.tile_cnt = at<uint32_t>(c, c->lay.tile_cnt);
    A.blk_cnt = blk_cnt_of(c, t);
    A.seg_cnt = c->lay.one_counter ? blk_cnt_of(c, t) : seg_cnt_of(c, t);
    A.blk_cnt_next = blk_cnt_of(c, t + 1);
    A.seg_cnt_next = c->lay.one_counter ? blk_cnt_of(c, t + 1) : seg_cnt_of(c, t + 1);
    A.cur_part = slot_part(c, t);
    A.cur_pos = slot_pos(c, t);
    A.nxt_part = slot_part(c, t + 1);
    A.nxt_pos = slot_pos(c, t + 1);
    A.part_cnt = at<uint64_t>(c, c->lay.part_cnt);
    A.part_off = at<uint64_t>(c, c->lay.part_off);
    A.out_idx = at<uint32_t>(c, c->lay.out_idx);
    A.out_val = at<float>(c, c->lay.out_val);
    A.err_slots = err_slots_of(c, t);
    A.err_slots_next = err_slots_of(c, t + 1);
    A.n_tiles = (uint32_t)c->lay.n_tiles;
    A.n_chunks = (uint32_t)c->lay.n_chunks;
    A.n_segs = (uint32_t)c->lay.n_segs;
    A.seg_shift = c->lay.seg_shift;
    A.chunk_shift = c->lay.chunk_shift;
    A.slots_min = c->lay.slots;
    A.pool_extra = c->lay.pool_extra;
    A.parity = (uint32_t)(t & 1);
    A.mode = mode;
    A.own_part = c->own_part;
    A.block_size = c->cfg.block_size;
    return A;
}

template <bool NORM, int CMP>
void launch_finish(exdyna_ctx *c, uint32_t mode, hipStream_t s)
{
    const FinishArgs A = finish_args(c, mode);
    const uint32_t per_wg = kFinishWG / 64;
    const uint32_t grid = 1u + (uint32_t)((c->lay.n_chunks + per_wg - 1) / per_wg);
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
    const uint32_t P = c->cfg.n_parts;
    // Alg. 3 (cyclic allocation): the partition worker `rank` selects at iteration t
    c->own_part = worker_rank < 0 ? kAllParts : (uint32_t)((c->t % P + (uint64_t)worker_rank) % P);
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

// Iteration whose selection the getters describe: the last finished one, or the
// one whose worker-view selection is waiting for its exchange.
bool have_iteration(const exdyna_ctx *c) { return c->t + c->phase > 0; }
uint64_t last_iteration(const exdyna_ctx *c) { return c->t + c->phase - 1; }

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
    c->cfg = *cfg;
    c->lay = L;
    c->n_b = n_b;
    c->cap = cap;
    c->t = 0;
    c->phase = 0;
    c->rank = 0;
    c->own_part = kAllParts;
    c->d_residual = d_residual;
    c->ws = static_cast<char *>(d_workspace);
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
                       (size_t)(2 * n_b));
    hipLaunchKernelGGL(k_fill_u32, dim3(64), dim3(256), 0, s, at<uint32_t>(c, L.seg_cnt), 0u,
                       (size_t)(2 * L.n_segs));
    hipLaunchKernelGGL(k_fill_u32, dim3(256), dim3(256), 0, s, at<uint32_t>(c, L.tile_cnt), 0u,
                       L.n_tiles);
    hipLaunchKernelGGL(k_init_slot_tab, dim3(256), dim3(256), 0, s, slot_tab_of(c, 0), slot_tab_of(c, 1),
                       (uint32_t)L.n_tiles, L.slots);
    const uint32_t init_threads = (P + 1 > 2 * kErrSlots ? P + 1 : 2 * kErrSlots);
    hipLaunchKernelGGL(k_init_state, dim3((init_threads + 255) / 256), dim3(256), 0, s,
                       at<DevState>(c, L.state), slot_part(c, 0), slot_pos(c, 0), slot_part(c, 1),
                       slot_pos(c, 1), at<uint64_t>(c, L.part_cnt), at<uint64_t>(c, L.part_off),
                       at<double>(c, L.err_slots), cfg->threshold0, (uint32_t)n_b, P);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        delete c;
        return EXDYNA_EHIP;
    }
    c->magic = kMagic;
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
    X.own_val = at<float>(c, c->lay.out_val);
    X.stride = stride;
    X.rank = c->rank;
    X.t_mod_p = (uint32_t)(c->t % P);
    const uint64_t gx = (stride + kFinishWG - 1) / kFinishWG;
    const dim3 grid((uint32_t)(gx ? gx : 1), P + 1);
    if (c->cfg.want_err_norm)
        hipLaunchKernelGGL((k_exchange<true>), grid, dim3(kFinishWG), 0, s, A, c->prm, X);
    else
        hipLaunchKernelGGL((k_exchange<false>), grid, dim3(kFinishWG), 0, s, A, c->prm, X);
    HIP_TRY(c, hipGetLastError());
    c->t += 1;
    c->phase = 0;
    c->own_part = kAllParts;
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
    if (d_idx) *d_idx = at<uint32_t>(c, c->lay.out_idx);
    if (d_val) *d_val = at<float>(c, c->lay.out_val);
    if (d_part_off) *d_part_off = at<uint64_t>(c, c->lay.part_off);
    if (h_k_actual || h_k_emitted) {
        DevState st;
        HIP_TRY(c, hipMemcpyAsync(&st, at<DevState>(c, c->lay.state), sizeof st,
                                  hipMemcpyDeviceToHost, c->stream));
        HIP_TRY(c, hipStreamSynchronize(c->stream));
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
    HIP_TRY(c, hipMemcpyAsync(h_counts, blk_cnt_of(c, last_iteration(c)), c->n_b * sizeof(uint32_t),
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
                           at<DevState>(c, c->lay.state), err_slots_of(c, last_iteration(c)));
    DevState st;
    HIP_TRY(c, hipMemcpyAsync(&st, at<DevState>(c, c->lay.state), sizeof st, hipMemcpyDeviceToHost,
                              c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
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
void drop_events_fwd(exdyna_ctx *c);
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
        drop_events_fwd(c);
    }
    c->t = h.t;
    c->phase = 0;  // a selection waiting for its exchange is dropped
    c->own_part = kAllParts;
    const Layout &L = c->lay;
    HIP_TRY(c, hipMemcpyAsync(slot_part(c, c->t), part, 2 * P * sizeof(int32_t),
                              hipMemcpyHostToDevice, s));
    HIP_TRY(c, hipMemcpyAsync(slot_part(c, c->t + 1), part, 2 * P * sizeof(int32_t),
                              hipMemcpyHostToDevice, s));
    hipLaunchKernelGGL(k_restore_state, dim3(1), dim3(1), 0, s, at<DevState>(c, L.state), h.t, h.delta);
    hipLaunchKernelGGL(k_fill_u32, dim3(256), dim3(256), 0, s, at<uint32_t>(c, L.blk_cnt), 0u,
                       (size_t)(2 * c->n_b));
    hipLaunchKernelGGL(k_fill_u32, dim3(64), dim3(256), 0, s, at<uint32_t>(c, L.seg_cnt), 0u,
                       (size_t)(2 * L.n_segs));
    hipLaunchKernelGGL(k_fill_u32, dim3(64), dim3(256), 0, s, at<uint32_t>(c, L.err_slots), 0u,
                       (size_t)(2 * kErrSlots * 2));
    hipLaunchKernelGGL(k_init_slot_tab, dim3(256), dim3(256), 0, s, slot_tab_of(c, 0), slot_tab_of(c, 1),
                       (uint32_t)L.n_tiles, L.slots);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(s));  // h_state may be freed by the caller on return
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
}  // namespace

namespace {
void drop_events_fwd(exdyna_ctx *c) { drop_events(c); }
}  // namespace

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
    if (c->magic != kMagic) return EXDYNA_ESTATE;
    drop_events(c);
    c->magic = 0;
    delete c;
    return EXDYNA_OK;
}

}  // extern "C"
