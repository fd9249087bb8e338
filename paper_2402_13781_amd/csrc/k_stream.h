// The streaming pass: accumulate, compare, rank, stage, zeroed write-back.
#ifndef EXDYNA_K_STREAM_H
#define EXDYNA_K_STREAM_H

#include "device_common.h"

namespace {

// k_stream: error-feedback accumulate + compare + rank + stage + zeroed
// write-back.  Workgroup w streams gradients [4096 w, 4096 (w+1)); its wave v
// owns wave tile 4w + v = four consecutive granules.
struct StreamArgs {
    const void     *g;          // n_g gradients of the kernel's element type
    float           eta;        // learning rate (used by the scaled variants only)
    float          *e;
    DevState       *st;
    uint2          *stage;      // staging pool of (index, value bits) pairs: slots_min per tile ...
    uint2          *stage_extra;  // ... then the part handed out by the slot table
    const uint2    *slot_tab;   // per tile: {offset in the extra part, slots there | bits} for this iteration
    uint32_t       *tile_cnt;   // n_tiles: selected in the tile | kFlag (only counted) | kKept (staged, not zeroed)
    uint32_t        slots_min;  // fixed staging slots of every tile
    uint32_t        pack_off;   // the tile word also carries the offset of pairs staged in the extra part
    uint32_t       *blk_cnt;    // this iteration's per-block counters (zero on entry), 2^rep_shift to a block
    uint32_t       *seg_cnt;    // this iteration's per-segment counters (zero on entry)
    double         *err_slots;  // norm statistic: kErrSlots sums of unselected squares, then
                                // kErrSlots sums over selected entries left in the residual
    uint32_t        n_g, n_tiles, gran_per_blk, parity;
    uint32_t        gpb_shift;  // log2(gran_per_blk) when it is a power of two, else 32
    uint32_t        seg_shift;  // log2(wave tiles per segment counter), 2..6
    uint32_t        seg_only;   // blocks are whole segments: only the segment counters are added to
                                // (the finishing kernel sums a block's segments)
    uint32_t        rep_shift;  // otherwise: a block has 2^rep_shift counters, one per streaming workgroup
                                // in turn, so that no counter is added to by more than about four tiles
    // worker view (Alg. 1 (Sparsify)): compare only inside the partition that worker sel_rank
    // owns at this iteration (Alg. 3 (cyclic allocation), from the device's own iteration
    // counter); kAllParts = everywhere
    uint32_t        sel_rank;
    uint32_t        n_parts;
    const int32_t  *cur_part;
    const int32_t  *cur_pos;
    uint32_t        block_size;  // b (the generic variant counts and masks by element index)
};

// Alg. 3 (cyclic allocation): the partition worker `rank` selects at iteration t.
__device__ __forceinline__ uint32_t owned_partition(uint64_t t, uint32_t rank, uint32_t n_parts)
{
    return (uint32_t)((t % n_parts + rank) % n_parts);
}

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

// Norm statistic: a selected entry that this pass leaves in the residual (its tile is not
// zeroed in registers) goes into a separate fp64 sum, from which the placement subtracts
// exactly the same square when it emits the entry; infinities are counted instead.
__device__ __forceinline__ void left_selected(float v, double &sum, uint32_t &nonfinite)
{
    if (__builtin_isinf(v))
        ++nonfinite;
    else
        sum += (double)(v * v);
}

// A tile's selected gradients as (index, value bits) pairs, in index order, to dst[rank in
// the tile]: every lane writes its own (cu: selected per granule; below: those in the granule
// in front of this lane's).
__device__ __forceinline__ void put_pairs(uint2 *dst, const f32x4 (&a)[kTileGran], const uint32_t (&nib)[kTileGran],
                                          const uint32_t (&cu)[kTileGran], const uint32_t (&below)[kTileGran],
                                          uint32_t gran0, uint32_t lane)
{
    uint32_t pre = 0;
#pragma unroll
    for (uint32_t u = 0; u < kTileGran; ++u) {
        if (nib[u]) {
            uint32_t       r  = pre + below[u];
            const uint32_t i0 = ((gran0 + u) << 8) + lane * 4u;
            if (nib[u] & 1u) dst[r++] = make_uint2(i0, __float_as_uint(a[u].x));
            if (nib[u] & 2u) dst[r++] = make_uint2(i0 + 1u, __float_as_uint(a[u].y));
            if (nib[u] & 4u) dst[r++] = make_uint2(i0 + 2u, __float_as_uint(a[u].z));
            if (nib[u] & 8u) dst[r++] = make_uint2(i0 + 3u, __float_as_uint(a[u].w));
        }
        pre += cu[u];
    }
}

// GEN: block sizes that are multiples of 32 but not of 256.  Block and partition
// boundaries then fall inside granules (always between lanes: a lane's four
// gradients share a 32-aligned group), so the comparison is masked per lane
// and every lane adds its own selected gradients to its block's counter.
//
// What a tile does with its selected gradients follows its slot table entry, which the
// finishing kernel of the iteration before wrote from the tile's output rank then:
//   zero bit     stage the pairs, zero them in registers (rank well inside the capacity)
//   no bit       stage the pairs, leave the residual alone: the placement zeroes what it
//                emits (rank near the capacity: it may or may not fit)
//   count only   only count (rank far beyond the capacity)
// Up to slots_min pairs go to the tile's fixed slots (found without the table), more to its
// slots in the extra part of the pool if the table gave it enough.  A tile with more selected
// gradients than that is counted and flagged; the placement re-reads it from the residual if
// its rank turns out to lie within the capacity.
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
    float    nrm = 0.f;
    double   left = 0.0;
    uint32_t left_nf = 0;
    uint32_t g_lo = 0u, g_hi = 0xFFFFFFFFu;  // granules that are compared at all
    uint32_t e_lo = 0u, e_hi = 0xFFFFFFFFu;  // GEN: the same as a gradient range
    if (A.sel_rank != kAllParts) {
        const uint32_t own_part = owned_partition(A.st->t, A.sel_rank, A.n_parts);
        if (GEN)
            partition_elems(A.cur_part, A.cur_pos, own_part, A.block_size, A.n_g, e_lo, e_hi);
        else
            partition_granules(A.cur_part, A.cur_pos, own_part, A.gran_per_blk, g_lo, g_hi);
    }

    if (live) {
        f32x4    a[kTileGran];
        uint32_t nib[kTileGran];
        const uint2 tab = A.slot_tab[tile];  // requested with the data, used only if something is selected
        if (fast) {
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
            }
        } else {
            // the ragged end of the vector (its last wave tile): guarded scalar loads; what
            // lies beyond n_g reads as zero and is never compared
#pragma unroll
            for (uint32_t u = 0; u < kTileGran; ++u) {
                const uint64_t base = ((uint64_t)(gran0 + u) << 8) + lane * 4u;
                float    v[4];
                uint32_t f = 0;
#pragma unroll
                for (uint32_t q = 0; q < 4; ++q) {
                    v[q] = 0.f;
                    if (base + q < A.n_g) {
                        v[q] = accumulate<SCALE>(A.e[base + q], load_grad1<GT>(A.g, base + q), A.eta);
                        f |= sel<CMP>(v[q], delta) << q;
                    }
                }
                a[u].x = v[0]; a[u].y = v[1]; a[u].z = v[2]; a[u].w = v[3];
                nib[u] = f;
            }
        }
#pragma unroll
        for (uint32_t u = 0; u < kTileGran; ++u) {
            if (GEN) {
                const uint32_t i0 = ((gran0 + u) << 8) + lane * 4u;
                if (i0 < e_lo || i0 >= e_hi) nib[u] = 0u;
            } else if (gran0 + u < g_lo || gran0 + u >= g_hi) {
                nib[u] = 0u;  // wave-uniform: another worker's partition
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
            uint2 *slot = nullptr;  // wave-uniform
            if (!(tab.y & kCountOnly)) {
                if (total <= A.slots_min)
                    slot = A.stage + (size_t)tile * A.slots_min;
                else if (total <= (tab.y & kSlotMask)) {
                    slot = A.stage_extra + tab.x;
                    if (A.pack_off) word |= (tab.x >> 4) << kOffShift;  // offsets are multiples of 16
                }
            }
            if (slot) {
                // Staged: pairs in index order.  The lanes first put their pairs in rank order
                // into the wavefront's own piece of LDS (no barrier: a wavefront's LDS accesses
                // stay in program order), then lane j stores pair j: one store instruction per
                // 64 pairs to consecutive addresses.  Sixteen instructions with a lane or two
                // active each, one per gradient slot, cost the pass 2 % at one pair per tile.
                __shared__ uint2 sbuf[kWavesPerWG][kStageBuf];
                if (total <= kStageBuf) {  // wave-uniform
                    put_pairs(sbuf[wave], a, nib, cu, below, gran0, lane);
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    for (uint32_t j = lane; j < total; j += 64u) slot[j] = sbuf[wave][j];
                } else {
                    put_pairs(slot, a, nib, cu, below, gran0, lane);
                }
            } else {
                word |= kFlag;  // more than the slots hold (or no slots at all): counted only
            }
            if (slot && !(tab.y & kZeroBit)) word |= kKept;
            if (slot && (tab.y & kZeroBit)) {  // wave-uniform
                // the residual is zeroed where sent (+0), before its only store
#pragma unroll
                for (uint32_t u = 0; u < kTileGran; ++u) {
                    if (nib[u] & 1u) a[u].x = 0.f;
                    if (nib[u] & 2u) a[u].y = 0.f;
                    if (nib[u] & 4u) a[u].z = 0.f;
                    if (nib[u] & 8u) a[u].w = 0.f;
                }
            } else if (NORM) {
#pragma unroll
                for (uint32_t u = 0; u < kTileGran; ++u) {
                    if (nib[u] & 1u) left_selected(a[u].x, left, left_nf);
                    if (nib[u] & 2u) left_selected(a[u].y, left, left_nf);
                    if (nib[u] & 4u) left_selected(a[u].z, left, left_nf);
                    if (nib[u] & 8u) left_selected(a[u].w, left, left_nf);
                }
            }
            // (adds to one address serialise at the memory side, and a wavefront does not retire
            // before its add has returned: up to four tiles per counter -- the tiles of one
            // workgroup -- cost next to nothing, sixteen cost 4 % of the pass)
            const uint32_t rep = (tile >> 2) & ((1u << A.rep_shift) - 1u);  // this workgroup's counter of a block
            if (GEN) {
                const uint32_t first = gran0 << 8;
                const uint32_t last  = first + kTile - 1u < A.n_g ? first + kTile - 1u : A.n_g - 1u;
                const uint32_t b_lo = first / A.block_size, b_hi = last / A.block_size;  // wave-uniform
                if (b_lo == b_hi) {  // the whole tile inside one block: one add
                    if (lane == 0) atomicAdd(&A.blk_cnt[(b_lo << A.rep_shift) + rep], total);
                } else {
#pragma unroll
                    for (uint32_t u = 0; u < kTileGran; ++u)
                        if (nib[u])
                            atomicAdd(&A.blk_cnt[(((((gran0 + u) << 8) + lane * 4u) / A.block_size) << A.rep_shift) + rep],
                                      (uint32_t)__popc(nib[u]));
                }
                if (lane == 0) atomicAdd(&A.seg_cnt[tile >> A.seg_shift], total);
            } else if (lane == 0) {
                if (A.seg_only) {
                    atomicAdd(&A.seg_cnt[tile >> A.seg_shift], total);
                } else {
                    // per-block counters; consecutive granules of one block are added together
                    uint32_t blk = A.gpb_shift < 32u ? gran0 >> A.gpb_shift : gran0 / A.gran_per_blk;
                    uint32_t in_blk = gran0 - blk * A.gran_per_blk;  // granule's position inside its block
                    uint32_t run = cu[0];
#pragma unroll
                    for (uint32_t u = 1; u < kTileGran; ++u) {
                        if (++in_blk == A.gran_per_blk) {  // granule gran0 + u starts the next block
                            if (run) atomicAdd(&A.blk_cnt[(blk << A.rep_shift) + rep], run);
                            ++blk;
                            in_blk = 0;
                            run = 0;
                        }
                        run += cu[u];
                    }
                    if (run) atomicAdd(&A.blk_cnt[(blk << A.rep_shift) + rep], run);
                    atomicAdd(&A.seg_cnt[tile >> A.seg_shift], total);
                }
            }
        }

        if (fast) {
#pragma unroll
            for (uint32_t u = 0; u < kTileGran; ++u) {
                const size_t off = ((size_t)(gran0 + u) << 8) + lane * 4u;
                __builtin_nontemporal_store(a[u], reinterpret_cast<f32x4 *>(A.e + off));
            }
        } else {
#pragma unroll
            for (uint32_t u = 0; u < kTileGran; ++u) {
                const uint64_t base = ((uint64_t)(gran0 + u) << 8) + lane * 4u;
                if (base < A.n_g) A.e[base] = a[u].x;
                if (base + 1 < A.n_g) A.e[base + 1] = a[u].y;
                if (base + 2 < A.n_g) A.e[base + 2] = a[u].z;
                if (base + 3 < A.n_g) A.e[base + 3] = a[u].w;
            }
        }
        if (lane == 0) A.tile_cnt[tile] = word;
    }

    if (NORM) {
        __shared__ double   wsum[kWavesPerWG];
        __shared__ double   wleft[kWavesPerWG];
        __shared__ uint32_t wnf[kWavesPerWG];
        const double s = wave_sum((double)nrm);
        left    = wave_sum(left);
        left_nf = wave_sum(left_nf);
        if (lane == 0) {
            wsum[wave]  = s;
            wleft[wave] = left;
            wnf[wave]   = left_nf;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            // The two sums go to separate slots: what the placement subtracts later must meet
            // a sum of its own kind, not one already rounded together with many small squares.
            const double   tot  = wsum[0] + wsum[1] + wsum[2] + wsum[3];
            const double   totl = wleft[0] + wleft[1] + wleft[2] + wleft[3];
            const uint32_t nf   = wnf[0] + wnf[1] + wnf[2] + wnf[3];
            atomicAdd(&A.err_slots[blockIdx.x % kErrSlots], tot);
            if (totl != 0.0) atomicAdd(&A.err_slots[kErrSlots + blockIdx.x % kErrSlots], totl);
            if (nf) atomicAdd(&A.st->nf_sel[A.parity], nf);
        }
    }
}

}  // namespace

#endif  // EXDYNA_K_STREAM_H
