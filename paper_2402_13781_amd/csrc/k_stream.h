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
    if (A.sel_rank != kAllParts) {
        const uint32_t own_part = owned_partition(A.st->t, A.sel_rank, A.n_parts);
        if (GEN)
            partition_elems(A.cur_part, A.cur_pos, own_part, A.block_size, A.n_g, e_lo, e_hi);
        else
            partition_granules(A.cur_part, A.cur_pos, own_part, A.gran_per_blk, g_lo, g_hi);
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

}  // namespace

#endif  // EXDYNA_K_STREAM_H
