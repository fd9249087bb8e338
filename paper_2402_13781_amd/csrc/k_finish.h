// The finishing kernel: control workgroup (counts, Alg. 5, Alg. 3, statistics) and compaction.
#ifndef EXDYNA_K_FINISH_H
#define EXDYNA_K_FINISH_H

#include "device_common.h"
#include "k_stream.h"

namespace {

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
    uint32_t        sel_rank;        // worker view: the worker whose partition was compared; else kAllParts
    uint32_t        block_size;
    uint32_t        n_parts;
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
        st->padding       = (uint64_t)P * ((uint64_t)P * m_t - k_actual);  // sum of (m_t - k_p) over p, times P
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
    if (flagged && A.sel_rank != kAllParts)  // the iteration counter moves only after the exchange
        partition_elems(A.cur_part, A.cur_pos, owned_partition(A.st->t, A.sel_rank, A.n_parts),
                        A.block_size, n_g, e_lo, e_hi);
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

}  // namespace

#endif  // EXDYNA_K_FINISH_H
