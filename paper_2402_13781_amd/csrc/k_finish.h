// The finishing kernel: control workgroup (counts, Alg. 5, Alg. 3, statistics) and placement.
#ifndef EXDYNA_K_FINISH_H
#define EXDYNA_K_FINISH_H

#include "device_common.h"
#include "k_stream.h"

namespace {

struct FinishArgs {
    DevState       *st;
    float          *e;
    const uint2    *stage;           // staging pool: slots_min per tile ...
    const uint2    *stage_extra;     // ... then the part the slot table hands out
    const uint2    *slot_tab;        // this iteration's {offset in the extra part, slots | bits} per tile
    uint2          *slot_tab_next;   // the next iteration's, written here
    const uint32_t *tile_cnt;
    const uint32_t *blk_src;         // this iteration's counters that make up the block counts: per_blk
                                     // consecutive ones to a block (its segments' counters, or its own)
    uint32_t       *blk_clear;       // the other parity's block counters, cleared here (null: they are segment counters)
    uint32_t       *blk_out;         // receives the per-block counts (for the getters) when per_blk > 1
    const uint32_t *seg_cnt;         // this iteration's per-segment counters (complete)
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
    uint32_t        n_tiles, n_segs, n_groups, seg_shift, slots_min, pool_extra, parity;
    uint32_t        search_step;     // largest power of two below n_groups (0 if n_groups = 1)
    uint32_t        n_tile_wgs;      // placement workgroups 1 .. n_tile_wgs work by tile, the rest by output rank
    uint32_t        grp_shift;       // log2(segment counters per entry of the placement's offset table): 0, 2 or 4
    uint32_t        pack_off;        // tile words carry the extra-part offset of their pairs
    uint32_t        mode;            // kCtrlFull or kCtrlSelect
    uint32_t        sel_rank;        // worker view: the worker whose partition was compared; else kAllParts
    uint32_t        block_size;
    uint32_t        n_parts;
    uint32_t        per_blk;         // counters per block (>= 1)
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

// Selected gradients of blocks i0 + 64 q + lane, q < N (index clamped into [.., end) so that
// every load can be issued at once).  A block's count is the sum of per_blk consecutive
// counters: the counters of its segments when blocks are whole segments, else its own (one per
// streaming workgroup in turn).  M = per_blk when it is 1, 2, 4, 8 or 16 (one load per block
// and four counters, all of a trip's loads in flight before the first sum waits for one), 0 for
// any other number (counter by counter).
template <uint32_t M, uint32_t N>
__device__ __forceinline__ void block_counts(const FinishArgs &A, uint32_t i0, uint32_t end, uint32_t lane,
                                             uint32_t (&out)[N])
{
    if (M == 1u) {
#pragma unroll
        for (uint32_t q = 0; q < N; ++q) {
            const uint32_t i = i0 + q * 64u + lane;
            out[q] = A.blk_src[i < end ? i : 0u];
        }
    } else if (M == 2u) {
        uint2 raw[N];
#pragma unroll
        for (uint32_t q = 0; q < N; ++q) {
            const uint32_t i = i0 + q * 64u + lane;
            raw[q] = reinterpret_cast<const uint2 *>(A.blk_src)[i < end ? i : 0u];
        }
#pragma unroll
        for (uint32_t q = 0; q < N; ++q) out[q] = raw[q].x + raw[q].y;
    } else if (M >= 4u) {
        constexpr uint32_t V = M / 4u;  // loads of four counters per block
        uint4 raw[N][V ? V : 1];
#pragma unroll
        for (uint32_t q = 0; q < N; ++q) {
            const uint32_t i = i0 + q * 64u + lane;
#pragma unroll
            for (uint32_t v = 0; v < V; ++v)
                raw[q][v] = reinterpret_cast<const uint4 *>(A.blk_src)[(size_t)(i < end ? i : 0u) * V + v];
        }
#pragma unroll
        for (uint32_t q = 0; q < N; ++q) {
            out[q] = 0u;
#pragma unroll
            for (uint32_t v = 0; v < V; ++v) out[q] += (raw[q][v].x + raw[q][v].y) + (raw[q][v].z + raw[q][v].w);
        }
    } else {
        // any other number: the blocks side by side, counter by counter (the arrays are padded
        // with zeros to whole blocks)
        const uint32_t m = A.per_blk;
#pragma unroll
        for (uint32_t q = 0; q < N; ++q) out[q] = 0u;
        for (uint32_t j = 0; j < m; ++j) {
            uint32_t raw[N];
#pragma unroll
            for (uint32_t q = 0; q < N; ++q) {
                const uint32_t i = i0 + q * 64u + lane;
                raw[q] = A.blk_src[(size_t)(i < end ? i : 0u) * m + j];
            }
#pragma unroll
            for (uint32_t q = 0; q < N; ++q) out[q] += raw[q];
        }
    }
}

// Zeroes block i's counters of the other parity.
template <uint32_t M>
__device__ __forceinline__ void clear_block(const FinishArgs &A, uint32_t i)
{
    if (M == 1u) {
        A.blk_clear[i] = 0u;
    } else if (M == 2u) {
        reinterpret_cast<uint2 *>(A.blk_clear)[i] = make_uint2(0u, 0u);
    } else if (M >= 4u) {
#pragma unroll
        for (uint32_t v = 0; v < M / 4u; ++v)
            reinterpret_cast<uint4 *>(A.blk_clear)[(size_t)i * (M / 4u) + v] = make_uint4(0u, 0u, 0u, 0u);
    } else {
        for (uint32_t j = 0; j < A.per_blk; ++j) A.blk_clear[(size_t)i * A.per_blk + j] = 0u;
    }
}

// k_{p,t} from the per-block counts (Sec. 4.2: the workload of a partition).
// Each wave takes a contiguous run of the blocks, 64 at a time; a trip's slices are requested
// before anything waits on memory.  Also stores the block counts for the getters and clears
// the other parity's block counters and norm partials for the next iteration.
template <uint32_t M>
__device__ __forceinline__ void control_counts_impl(const FinishArgs &A, const CtrlParams &prm, CtrlShared &S)
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
    // slices per trip: 768 blocks per wave (12288 per trip of the workgroup), fewer when a block has many counters
    constexpr uint32_t kAhead = M == 8u ? 6u : M == 16u ? 3u : 12u;
    uint32_t cbuf[kAhead];
    block_counts<M>(A, beg, end, lane, cbuf);
    if (tid < P) {
        S.cnt[tid]   = 0u;
        S.lpos[tid]  = A.cur_pos[tid];
        S.lpart[tid] = A.cur_part[tid];
    }
    if (tid < 2 * kErrSlots) A.err_slots_next[tid] = 0.0;
    if (tid == 0) {
        A.st->nf_sel[A.parity ^ 1u]  = 0u;
        A.st->nf_emit[A.parity ^ 1u] = 0u;
    }
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
            if (i0 != beg) block_counts<M>(A, i0, end, lane, cbuf);
#pragma unroll
            for (uint32_t q = 0; q < kAhead; ++q) {
                const uint32_t s0 = i0 + q * 64u;  // first block of this slice
                const uint32_t i  = s0 + lane;
                uint32_t c = i < end ? cbuf[q] : 0u;
                if (i < end) {
                    if (M != 1u) A.blk_out[i] = c;         // the block's count, for the getters (one counter per block: it is the count)
                    if (A.blk_clear) clear_block<M>(A, i);  // clean block counters for the next iteration
                }
                while (next_start < s0 + 64u && next_start < end) {  // the slice reaches the next partition
                    acc += i < next_start ? c : 0u;
                    c = i < next_start ? 0u : c;
                    acc = wave_sum(acc);
                    if (lane == 0 && acc) atomicAdd(&S.cnt[pcur], acc);
                    acc = 0;
                    ++pcur;
                    next_start = pcur + 1 < P ? (uint32_t)S.lpos[pcur + 1] : 0xFFFFFFFFu;
                }
                acc += c;
            }
        }
        acc = wave_sum(acc);
        if (lane == 0 && acc) atomicAdd(&S.cnt[pcur], acc);
    }
    __syncthreads();
}

__device__ __forceinline__ void control_counts(const FinishArgs &A, const CtrlParams &prm, CtrlShared &S)
{
    switch (A.per_blk) {  // workgroup-uniform
    case 1u: control_counts_impl<1>(A, prm, S); break;
    case 2u: control_counts_impl<2>(A, prm, S); break;
    case 4u: control_counts_impl<4>(A, prm, S); break;
    case 8u: control_counts_impl<8>(A, prm, S); break;
    case 16u: control_counts_impl<16>(A, prm, S); break;
    default: control_counts_impl<0>(A, prm, S); break;
    }
}

// Everything that follows from the per-partition counts in S.cnt (S.lpos /
// S.lpart hold the topology they were counted with).  ONE_WAVE: P <= 64, the first wavefront
// does it alone and the workgroup barriers fall away (a wavefront's LDS accesses stay in
// program order); the caller has already sent the other wavefronts home.
template <bool ONE_WAVE>
__device__ __forceinline__ void ctrl_sync()
{
    if (ONE_WAVE)
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    else
        __syncthreads();
}

template <bool ONE_WAVE>
__device__ __forceinline__ void control_decide_impl(const FinishArgs &A, const CtrlParams &prm, CtrlShared &S, uint32_t mode,
                                    float delta_in, uint64_t t_in)
{
    constexpr uint32_t kWaves = ONE_WAVE ? 1u : kFinishWG / 64;
    constexpr uint32_t kIdent = 0u | (1u << 2) | (2u << 4);  // s -> s
    const uint32_t tid  = threadIdx.x;
    const uint32_t lane = tid & 63u;
    const uint32_t wave = tid >> 6;
    const uint32_t P    = prm.n_parts;

    // threshold and iteration counter of this iteration: requested by the caller before the
    // counting started, so that their latency is not added at the end
    const float    delta  = delta_in;
    const uint64_t t_done = t_in;
    if (tid == 0) S.n_moves = 0u;
    const int32_t part = tid < P ? S.lpart[tid] : 0;
    const int32_t pos  = tid < P ? S.lpos[tid] : 0;

    // exclusive scan and maximum of the P counts (P <= 1024 = one value per thread)
    const uint32_t c    = tid < P ? S.cnt[tid] : 0u;
    const uint32_t incl = wave_incl_scan(c, lane);
    const uint32_t mx = wave_max(c);
    if (lane == 63) S.wsum[wave] = incl;
    if (lane == 0) S.wmax[wave] = mx;
    ctrl_sync<ONE_WAVE>();
    if (wave == 0) {
        const uint32_t v  = lane < kWaves ? S.wsum[lane] : 0u;
        const uint32_t vi = wave_incl_scan(v, lane);
        if (lane < kWaves) S.wsum[lane] = vi - v;
        if (lane == kWaves - 1) S.k_total = vi;  // k' (Alg. 1 (k' sum))
    }
    ctrl_sync<ONE_WAVE>();
    const uint64_t excl     = (uint64_t)S.wsum[wave] + (incl - c);
    const uint64_t k_actual = S.k_total;
    if (tid < P) {
        A.part_cnt[tid] = c;
        if (mode != kCtrlUpdate) A.part_off[tid] = excl < prm.cap ? excl : prm.cap;
    }
    if (mode == kCtrlSelect) {  // the gathered counts decide the rest, after the exchange
        if (tid == 0) {
            DevState *st = A.st;
            st->k_hist[A.parity] = k_actual;
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
    ctrl_sync<ONE_WAVE>();

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
    struct OpCompose {
        __device__ __forceinline__ uint32_t operator()(uint32_t later, uint32_t earlier) const
        {
            return compose(later, earlier);
        }
    };
    const uint32_t fun = wave_scan(table, kIdent, OpCompose());
    if (lane == 63) S.wfun[wave] = fun;
    ctrl_sync<ONE_WAVE>();
    if (tid == 0) {
        uint32_t stt = 0;  // pair 0 starts untouched
        for (uint32_t w = 0; w < kWaves; ++w) {
            S.wcarry[w] = stt;
            stt = (S.wfun[w] >> (2u * stt)) & 3u;
        }
    }
    ctrl_sync<ONE_WAVE>();
    const uint32_t before = dpp_move<0x138, 0xF>(kIdent, fun);  // the lane below's; lane 0: identity
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
    ctrl_sync<ONE_WAVE>();

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
        if (mode == kCtrlFull) st->k_hist[A.parity] = k_actual;
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

__device__ __forceinline__ void control_decide(const FinishArgs &A, const CtrlParams &prm, CtrlShared &S, uint32_t mode,
                               float delta, uint64_t t_done)
{
    if (prm.n_parts <= 64u) {  // workgroup-uniform
        if (threadIdx.x < 64u) control_decide_impl<true>(A, prm, S, mode, delta, t_done);
    } else {
        control_decide_impl<false>(A, prm, S, mode, delta, t_done);
    }
}

__device__ __forceinline__ void finish_control(const FinishArgs &A, const CtrlParams &prm)
{
    __shared__ CtrlShared S;
    // requested before the counting starts (volatile: issued here, waited for where used)
    const float    delta  = *reinterpret_cast<const volatile float *>(&A.st->delta[A.parity]);
    const uint64_t t_done = *reinterpret_cast<const volatile uint64_t *>(&A.st->t);
    control_counts(A, prm, S);
    control_decide(A, prm, S, A.mode, delta, t_done);
}

// ---- placement: every other workgroup of k_finish ----
//
// A pair's output position is the number of selected gradients in front of it (partitions are
// contiguous and ascending, Sec. 4.1, so the per-partition lists in partition order are one
// ascending list).  Every placement workgroup first builds the same small table in LDS: the
// exclusive prefix of the segment counters, one entry per group of 1, 4 or 16 segments (at
// most 4096 entries).  With it
//   - some workgroups work by TILE: four consecutive wave tiles per thread.  The thread learns
//     its tiles' ranks, writes their slot table entries for the next iteration, and puts back
//     what the streaming pass zeroed although it lies beyond the capacity (rare);
//   - the others work by output RANK: windows of 1024 to 4096 consecutive output positions,
//     one to four per thread.  The thread finds the tile that holds its rank and copies that
//     one pair from the tile's staging slots.  However the selected gradients are spread over
//     the vector -- a sparse steady state, or a threshold transient that packs the whole
//     output into the first few per cent of the tiles -- every thread moves the same number
//     of pairs, and only ranks below min(k', capacity) cost anything.
// A flagged tile (not staged) inside the capacity is re-read from the residual by the wave
// that holds the rank of its first pair.

constexpr uint32_t kWinTiles = 4096;  // tile words (or segment counters) a rank workgroup spreads out in LDS at a time

struct alignas(16) PlaceShared {
    uint32_t grp[kMaxGroups];          // group sums, then exclusive offsets
    uint32_t wtot[kFinishWG / 64];
    uint32_t wbase[kFinishWG / 64];
    uint32_t total;
    uint32_t win[2];                   // the groups of a window's first and last rank
    uint32_t tpre[kWinTiles];          // a window's tiles (or segments): running (inclusive) count of selected gradients
    uint32_t tword[kWinTiles];         // ... and their tile words
};

// Sum of the 16 per-wave totals in front of wave `wave` (four LDS reads side by side instead
// of up to fifteen one after the other).
__device__ __forceinline__ uint32_t waves_before(const uint32_t *wtot, uint32_t wave)
{
    const uint4 *p = reinterpret_cast<const uint4 *>(wtot);
    const uint4 a = p[0], b = p[1], c = p[2], d = p[3];
    const uint32_t v[16] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w, c.x, c.y, c.z, c.w, d.x, d.y, d.z, d.w};
    uint32_t sum = 0;
#pragma unroll
    for (uint32_t w = 0; w < 16; ++w) sum += w < wave ? v[w] : 0u;
    return sum;
}

// Sums of the groups' segment counters into S.grp: thread tid takes counters 4 (tid + 1024 q)
// .. + 3 for q < N, which covers all n_vec <= 1024 N loads of four.
template <uint32_t N>
__device__ __forceinline__ void group_sums(const FinishArgs &A, PlaceShared &S, uint32_t n_vec)
{
    const uint4 *__restrict__ src = reinterpret_cast<const uint4 *>(A.seg_cnt);
    const uint32_t tid  = threadIdx.x;
    const uint32_t lane = tid & 63u;
    const uint32_t gs   = A.grp_shift;
    uint4 c[N];
#pragma unroll
    for (uint32_t q = 0; q < N; ++q) {  // index clamped, not a guarded load: all in flight together
        const uint32_t v = tid + q * kFinishWG;
        c[q] = src[v < n_vec ? v : 0u];
    }
#pragma unroll
    for (uint32_t q = 0; q < N; ++q) {
        const uint32_t v = tid + q * kFinishWG;
        if (v >= n_vec) c[q] = make_uint4(0u, 0u, 0u, 0u);
        if ((v & ~63u) < n_vec) {  // wave-uniform: this wave's slice holds counters
            if (gs == 0u) {  // every counter is a group
                if (4u * v + 0u < A.n_groups) S.grp[4u * v + 0u] = c[q].x;
                if (4u * v + 1u < A.n_groups) S.grp[4u * v + 1u] = c[q].y;
                if (4u * v + 2u < A.n_groups) S.grp[4u * v + 2u] = c[q].z;
                if (4u * v + 3u < A.n_groups) S.grp[4u * v + 3u] = c[q].w;
            } else {
                uint32_t x = (c[q].x + c[q].y) + (c[q].z + c[q].w);
                if (gs == 4u) {  // four lanes = one group
                    x += dpp_move<0xB1, 0xF>(0u, x);  // quad lanes 1 0 3 2
                    x += dpp_move<0x4E, 0xF>(0u, x);  // quad lanes 2 3 0 1
                    if ((lane & 3u) == 0u && (v >> 2) < A.n_groups) S.grp[v >> 2] = x;
                } else if (v < A.n_groups) {
                    S.grp[v] = x;
                }
            }
        }
    }
}

// Builds S.grp (exclusive prefix of the segment counters, one entry per group of 1, 4 or 16
// segments: A.grp_shift = 0, 2, 4) and S.total.
__device__ __forceinline__ void place_table(const FinishArgs &A, PlaceShared &S)
{
    constexpr uint32_t kWaves = kFinishWG / 64;
    const uint32_t tid  = threadIdx.x;
    const uint32_t lane = tid & 63u;
    const uint32_t wave = tid >> 6;
    // group sums: a lane takes four counters per load (the counter arrays are padded with
    // zeros to a multiple of 64), and a thread's loads are all requested before the first is
    // used: up to 8 (32768 counters) or up to 16 (65536)
    {
        const uint32_t n_vec = (A.n_segs + 3u) >> 2;
        if (n_vec <= 8u * kFinishWG)
            group_sums<8>(A, S, n_vec);
        else
            group_sums<16>(A, S, n_vec);
    }
    __syncthreads();
    // exclusive scan of the group sums, a run of consecutive groups per thread
    const uint32_t per = (A.n_groups + kFinishWG - 1u) / kFinishWG;  // <= kMaxGroups / 1024
    const uint32_t g0  = tid * per;
    uint32_t mine = 0;
    for (uint32_t q = 0; q < per; ++q)
        if (g0 + q < A.n_groups) mine += S.grp[g0 + q];
    const uint32_t incl = wave_incl_scan(mine, lane);
    if (lane == 63) S.wtot[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        const uint32_t w  = lane < kWaves ? S.wtot[lane] : 0u;
        const uint32_t wi = wave_incl_scan(w, lane);
        if (lane < kWaves) S.wbase[lane] = wi - w;
        if (lane == kWaves - 1) S.total = wi;
    }
    __syncthreads();
    uint32_t run = S.wbase[wave] + (incl - mine);
    for (uint32_t q = 0; q < per; ++q)
        if (g0 + q < A.n_groups) {
            const uint32_t c = S.grp[g0 + q];
            S.grp[g0 + q] = run;
            run += c;
        }
    __syncthreads();
}

// Where a staged tile's pairs are: in its fixed slots if they fit there, else in the extra part
// (at the offset the tile word carries, or the slot table's when the pool is too large for that).
__device__ __forceinline__ const uint2 *staged_pairs(const FinishArgs &A, uint32_t tile, uint32_t word)
{
    if ((word & kCountMask) <= A.slots_min) return A.stage + (size_t)tile * A.slots_min;
    if (A.pack_off) return A.stage_extra + ((size_t)(word >> kOffShift) << 4);
    return A.stage_extra + A.slot_tab[tile].x;
}

// ---- by tile: ranks, the next slot table, clean segment counters, put-backs ----
template <bool NORM>
__device__ __forceinline__ void place_tiles(const FinishArgs &A, PlaceShared &S, uint64_t cap, uint32_t wg, uint4 w4,
                            uint64_t prev, double &add)
{
    // how fast the selected count grows: this pass's total over the last pass's (prev), 1 .. 4
    uint64_t zero_below = cap;
    uint32_t slots_per8 = 32;  // extra staging slots per selected gradient, in eighths
    {
        const double   now  = (double)S.total;
        double growth = prev ? now / (double)prev : 1.0;
        // Four slots per pair: a tile with 6 to 16 pairs now (its fixed slots hold 16) then
        // has room for 32 or more, far outside the spread of its next count.  Two and a half
        // while the total shrinks: the same pool then reaches tiles ranked further out, which
        // is where the capacity's edge moves to.
        slots_per8 = growth < 0.9 ? 20u : 32u;
        growth = growth < 1.0 ? 1.0 : growth > 4.0 ? 4.0 : growth;
        zero_below = (uint64_t)((double)cap / (growth * 1.125));
    }
    const uint32_t tid  = threadIdx.x;
    const uint32_t lane = tid & 63u;
    const uint32_t wave = tid >> 6;
    const uint32_t sh   = A.seg_shift;
    constexpr uint32_t kBig = kFinishWG * kTilesPerThr;  // wave tiles per workgroup and round
    const uint32_t n_big = (A.n_tiles + kBig - 1u) / kBig;
    for (uint32_t big = wg; big < n_big; big += A.n_tile_wgs) {
        const uint32_t tile0 = (big * kFinishWG + tid) * kTilesPerThr;
        const uint32_t word[4] = {w4.x, w4.y, w4.z, w4.w};
        {   // the next round's tile words are requested before this round waits for anything
            const uint32_t nxt = ((big + A.n_tile_wgs) * kFinishWG + tid) * kTilesPerThr;
            if (big + A.n_tile_wgs < n_big && nxt < A.n_tiles)
                w4 = *reinterpret_cast<const uint4 *>(A.tile_cnt + nxt);
            else
                w4 = make_uint4(0u, 0u, 0u, 0u);
        }
        const uint32_t c4[4] = {word[0] & kCountMask, word[1] & kCountMask, word[2] & kCountMask,
                                word[3] & kCountMask};
        const uint32_t mine = (c4[0] + c4[1]) + (c4[2] + c4[3]);
        const uint32_t incl = wave_incl_scan(mine, lane);
        if (lane == 63) S.wtot[wave] = incl;
        __syncthreads();
        uint32_t r0 = S.grp[big * ((kBig >> sh) >> A.grp_shift)] + (incl - mine);  // a round starts on a group boundary
        r0 += waves_before(S.wtot, wave);
        __syncthreads();  // S.wtot is rewritten by the next round

        {   // a round holds whole segments: their counters of the other parity are cleared here
            const uint32_t per_big = kBig >> sh;
            for (uint32_t i = tid; i < per_big; i += kFinishWG) {
                const uint32_t sg = big * per_big + i;
                if (sg < A.n_segs) A.seg_cnt_next[sg] = 0u;
            }
        }
        // Staging slots for the next iteration follow this iteration's ranks and counts.
        // Beyond its fixed slots a tile gets four slots per gradient it selected now (two and
        // a half while the total is shrinking) in the extra part of the pool, at an
        // offset that is the running sum of those sizes (taken from the rank, rounded down to
        // 16 pairs = 128 bytes so that two tiles never share a cache line), for as long as
        // the extra part lasts: it covers at least one and a half output capacities.  A tile
        // ranked beyond that only counts; a tile whose pairs would still end within the
        // capacity if all ranks grew as the total just did (and an eighth more) may zero what
        // it stages.
        const uint64_t ex = A.pool_extra;  // multiple of 16
#pragma unroll
        for (uint32_t k = 0; k < kTilesPerThr; ++k) {
            const uint32_t tile = tile0 + k;
            const uint32_t c    = c4[k];
            if (tile < A.n_tiles) {
                const uint64_t a2 = (((uint64_t)r0 * slots_per8) >> 3) & ~15ull;
                const uint64_t b2 = ((((uint64_t)r0 + c) * slots_per8) >> 3) & ~15ull;
                uint2 nxt;
                if (a2 >= ex) {
                    nxt = make_uint2(0u, kCountOnly);
                } else {
                    const uint64_t hi2 = b2 < ex ? b2 : ex;
                    uint32_t       y   = (uint32_t)(hi2 - a2);
                    if ((uint64_t)r0 + c <= zero_below) y |= kZeroBit;
                    nxt = make_uint2((uint32_t)a2, y);
                }
                A.slot_tab_next[tile] = nxt;

                // zeroed in registers, yet beyond the capacity: not sent, so back into the residual
                if (c && !(word[k] & (kFlag | kKept)) && (uint64_t)r0 + c > cap) {
                    const uint32_t first = r0 < cap ? (uint32_t)(cap - r0) : 0u;
                    const uint2 *__restrict__ src = staged_pairs(A, tile, word[k]);
                    for (uint32_t j = first; j < c; ++j) {
                        const uint2 pr = src[j];
                        const float v  = __uint_as_float(pr.y);
                        A.e[pr.x] = v;
                        if (NORM) add += (double)(v * v);
                    }
                }
            }
            r0 += c;
        }
    }
}

// Wave-cooperative: re-read flagged tile `tile` (its residual still holds acc), repeat the
// comparison, and emit its selected gradients whose output rank lies below n_out; r0 is the
// rank of the tile's first selected gradient.  Emitted entries are zeroed in the residual
// (Alg. 1 (zeroing of the sent entries)), which is why ONE wave does the whole tile: a second
// wave re-reading it meanwhile would no longer find what the first has sent.
template <bool NORM, int CMP>
__device__ __forceinline__ void emit_flagged_tile(const FinishArgs &A, uint32_t tile, uint32_t r0,
                                                  uint32_t n_out, float delta,
                                                  uint32_t lane, uint32_t n_g, uint32_t e_lo,
                                                  uint32_t e_hi, double &sub, uint32_t &sub_nf)
{
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
    uint32_t running = r0;
#pragma unroll
    for (uint32_t u = 0; u < kTileGran; ++u) {
        const uint64_t base = ((uint64_t)(gran0 + u) << 8) + lane * 4u;
        uint32_t cu, below;
        granule_ranks(nib[u], cu, below);
        uint32_t r = running + below;
#pragma unroll
        for (uint32_t q = 0; q < 4; ++q) {
            if (nib[u] & (1u << q)) {
                if (r < n_out) {
                    A.out_idx[r] = (uint32_t)(base + q);
                    A.out_val[r] = v[u][q];
                    e[base + q]  = 0.0f;
                    if (NORM) left_selected(v[u][q], sub, sub_nf);
                }
                ++r;
            }
        }
        running += cu;
    }
}

// Group that holds output rank r: the last one whose offset is <= r (empty groups in front
// share the offset).
__device__ __forceinline__ uint32_t find_group(const FinishArgs &A, const PlaceShared &S, uint32_t r)
{
    uint32_t g = 0;
    for (uint32_t step = A.search_step; step; step >>= 1) {
        const uint32_t m = g + step;
        if (m < A.n_groups && S.grp[m] <= r) g = m;
    }
    return g;
}

// Segment that holds position rem of group g (groups of 4 or 16 segments): the group's
// counters, requested together, then one after the other.  rem becomes the position inside
// the segment.
__device__ __forceinline__ uint32_t find_segment(const FinishArgs &A, uint32_t g, uint32_t &rem)
{
    uint32_t seg = g << A.grp_shift;
    if (A.grp_shift) {  // workgroup-uniform
        const uint32_t n_vec = A.grp_shift == 4u ? 4u : 1u;
        const uint4 *p = reinterpret_cast<const uint4 *>(A.seg_cnt + seg);
        uint4 c4[4];
#pragma unroll
        for (uint32_t v = 0; v < 4; ++v) c4[v] = p[v < n_vec ? v : 0u];
        bool found = false;
#pragma unroll
        for (uint32_t v = 0; v < 4; ++v) {
            const uint32_t cc[4] = {c4[v].x, c4[v].y, c4[v].z, c4[v].w};
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k) {
                const bool here = !found && v < n_vec && rem < cc[k];
                found = found || here;
                if (!found && v < n_vec) {
                    rem -= cc[k];
                    ++seg;
                }
            }
        }
    }
    return seg;
}

// Tile that holds position rem of segment seg: the segment's tile words, 16 requested
// together, then one after the other.  rem becomes the position inside the tile.
__device__ __forceinline__ uint32_t find_tile(const FinishArgs &A, uint32_t seg, uint32_t &rem, uint32_t &word)
{
    const uint32_t sh     = A.seg_shift;
    const uint32_t n_vec  = sh >= 4u ? 4u : 1u << (sh - 2u);
    const uint32_t rounds = sh > 4u ? 1u << (sh - 4u) : 1u;
    uint32_t tile = seg << sh;
    bool found = false;
    word = 0;
    for (uint32_t round = 0; round < rounds && !found; ++round) {
        const uint4 *p = reinterpret_cast<const uint4 *>(A.tile_cnt + (seg << sh)) + round * 4u;
        uint4 c4[4];
#pragma unroll
        for (uint32_t v = 0; v < 4; ++v) c4[v] = p[v < n_vec ? v : 0u];
#pragma unroll
        for (uint32_t v = 0; v < 4; ++v) {
            const uint32_t ww[4] = {c4[v].x, c4[v].y, c4[v].z, c4[v].w};
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k) {
                const uint32_t cnt  = ww[k] & kCountMask;
                const bool     here = !found && v < n_vec && rem < cnt;
                if (here) word = ww[k];
                found = found || here;
                if (!found && v < n_vec) {
                    rem -= cnt;
                    ++tile;
                }
            }
        }
    }
    return tile;
}

// ---- by rank: a workgroup takes a window of consecutive output ranks, 1024 to 4096 of them
// (as many as it takes for all workgroups together to cover the output in one pass), one to
// four per thread.  Two threads look the window's first and last rank up in the table; the
// groups in between hold every pair of the window.  If their tile words fit (4096), the
// workgroup spreads the tiles' running counts out in LDS -- one coalesced load, one scan --
// and every thread finds its ranks' tiles there with a short binary search.  If only their
// segment counters fit (sparse selections: hundreds of tiles per output pair), the same is
// done with segments, and each thread then walks through its segment's tile words.  Beyond
// that every thread walks down all levels on its own.  Then the pairs are copied, all loads
// of a thread in flight together. ----
template <bool NORM, int CMP>
__device__ __forceinline__ void place_ranks(const FinishArgs &A, PlaceShared &S, uint32_t n_g, uint32_t n_out,
                            uint32_t wg, uint32_t n_wg, float delta, double &sub, uint32_t &sub_nf)
{
    constexpr uint32_t kMaxPer = 4;  // output ranks per thread and window
    const uint32_t tid  = threadIdx.x;
    const uint32_t lane = tid & 63u;
    const uint32_t wave = tid >> 6;
    const uint32_t sh   = A.seg_shift;
    const uint32_t gs   = A.grp_shift;
    uint32_t e_lo = 0u, e_hi = 0xFFFFFFFFu;
    if (A.sel_rank != kAllParts)  // the iteration counter moves only after the exchange
        partition_elems(A.cur_part, A.cur_pos, owned_partition(A.st->t, A.sel_rank, A.n_parts),
                        A.block_size, n_g, e_lo, e_hi);
    // ranks per thread: as many as it takes to cover the output in one pass, at most kMaxPer
    const uint64_t one_each = (uint64_t)n_wg * kFinishWG;
    const uint32_t per  = n_out > 3u * one_each ? 4u : n_out > 2u * one_each ? 3u : n_out > one_each ? 2u : 1u;
    const uint64_t span = (uint64_t)per * kFinishWG;
    for (uint64_t w0 = (uint64_t)wg * span; w0 < n_out; w0 += (uint64_t)n_wg * span) {  // workgroup-uniform
        const uint32_t w1 = w0 + span < n_out ? (uint32_t)(w0 + span) : n_out;  // the window is [w0, w1)
        // every thread looks at a few groups: the two that hold the window's ends report
        for (uint32_t g = tid; g < A.n_groups; g += kFinishWG) {
            const uint32_t lo = S.grp[g], hi = g + 1u < A.n_groups ? S.grp[g + 1u] : S.total;
            if (lo <= (uint32_t)w0 && (uint32_t)w0 < hi) S.win[0] = g;
            if (lo <= w1 - 1u && w1 - 1u < hi) S.win[1] = g;
        }
        __syncthreads();
        const uint32_t g_lo = S.win[0], n_grp = S.win[1] - g_lo + 1u;
        const uint32_t base = S.grp[g_lo];  // rank of the first pair of group g_lo
        // what is spread out: tile words if they fit, else segment counters, else nothing
        const bool by_tile = ((uint64_t)n_grp << (gs + sh)) <= kWinTiles;        // workgroup-uniform
        const bool by_seg  = !by_tile && ((uint64_t)n_grp << gs) <= kWinTiles;   // workgroup-uniform
        const uint32_t *src_cnt = by_tile ? A.tile_cnt + ((size_t)g_lo << (gs + sh)) : A.seg_cnt + (g_lo << gs);
        const uint32_t  n_ent   = by_tile ? n_grp << (gs + sh) : n_grp << gs;    // multiple of 4 when it is used
        const uint32_t  cmask   = by_tile ? kCountMask : 0xFFFFFFFFu;

        uint32_t tile[kMaxPer], within[kMaxPer], word[kMaxPer];
        bool     active[kMaxPer];
#pragma unroll
        for (uint32_t q = 0; q < kMaxPer; ++q) {
            active[q] = q < per && w0 + (uint64_t)q * kFinishWG + tid < w1;
            tile[q] = 0; within[q] = 0; word[q] = 0;
        }
        if (by_tile || by_seg) {
            // running counts of the window's tiles (segments), four per thread
            uint4 w4 = *reinterpret_cast<const uint4 *>(src_cnt + (4u * tid < n_ent ? 4u * tid : 0u));
            if (4u * tid >= n_ent) w4 = make_uint4(0u, 0u, 0u, 0u);
            const uint32_t c0 = w4.x & cmask, c1 = w4.y & cmask, c2 = w4.z & cmask, c3 = w4.w & cmask;
            const uint32_t incl = wave_incl_scan((c0 + c1) + (c2 + c3), lane);
            if (lane == 63) S.wtot[wave] = incl;
            __syncthreads();
            uint32_t run = incl - ((c0 + c1) + (c2 + c3));
            run += waves_before(S.wtot, wave);
            run += c0; S.tpre[4u * tid]      = run;
            run += c1; S.tpre[4u * tid + 1u] = run;
            run += c2; S.tpre[4u * tid + 2u] = run;
            run += c3; S.tpre[4u * tid + 3u] = run;
            if (by_tile) *reinterpret_cast<uint4 *>(&S.tword[4u * tid]) = w4;
            __syncthreads();
            // first entry whose running count exceeds the rank's position among the window's
            // groups: tpre is non-decreasing over all kWinTiles entries and the window's last
            // rank lies in its last group, so the answer is below n_ent
            uint32_t pos[kMaxPer], j[kMaxPer];
#pragma unroll
            for (uint32_t q = 0; q < kMaxPer; ++q) {
                pos[q] = active[q] ? (uint32_t)w0 + q * kFinishWG + tid - base : 0u;
                j[q]   = 0;
            }
            // the searches of a thread's ranks go side by side, step by step
#pragma unroll
            for (uint32_t step = kWinTiles / 2u; step >= 1u; step >>= 1) {
                uint32_t probe[kMaxPer];
#pragma unroll
                for (uint32_t q = 0; q < kMaxPer; ++q) probe[q] = S.tpre[j[q] + step - 1u];
#pragma unroll
                for (uint32_t q = 0; q < kMaxPer; ++q)
                    if (probe[q] <= pos[q]) j[q] += step;
            }
#pragma unroll
            for (uint32_t q = 0; q < kMaxPer; ++q) within[q] = pos[q] - (j[q] ? S.tpre[j[q] - 1u] : 0u);
            if (by_tile) {
#pragma unroll
                for (uint32_t q = 0; q < kMaxPer; ++q) {
                    tile[q] = (g_lo << (gs + sh)) + j[q];
                    word[q] = S.tword[j[q]];
                }
            } else {
#pragma unroll 1
                for (uint32_t q = 0; q < per; ++q) {
                    uint32_t rem = 0, wd = 0, t = 0, seg = 0;
#pragma unroll
                    for (uint32_t k = 0; k < kMaxPer; ++k)
                        if (k == q) {
                            rem = within[k];
                            seg = (g_lo << gs) + j[k];
                        }
                    if (active[q]) t = find_tile(A, seg, rem, wd);
#pragma unroll
                    for (uint32_t k = 0; k < kMaxPer; ++k)
                        if (k == q) {
                            tile[k] = t; within[k] = rem; word[k] = wd;
                        }
                }
            }
        } else {
#pragma unroll 1
            for (uint32_t q = 0; q < per; ++q) {
                const uint32_t r = (uint32_t)w0 + q * kFinishWG + tid;
                uint32_t rem = 0, wd = 0, t = 0;
                if (w0 + (uint64_t)q * kFinishWG + tid < w1) {
                    const uint32_t g = find_group(A, S, r);
                    rem = r - S.grp[g];
                    const uint32_t seg = find_segment(A, g, rem);
                    t = find_tile(A, seg, rem, wd);
                }
#pragma unroll
                for (uint32_t k = 0; k < kMaxPer; ++k)
                    if (k == q) {
                        tile[k] = t; within[k] = rem; word[k] = wd;
                    }
            }
        }
        // the pairs themselves: within is the position among the tile's staged pairs
        {
            const uint2 *src[kMaxPer];
            uint2        pr[kMaxPer];
#pragma unroll
            for (uint32_t q = 0; q < kMaxPer; ++q) {
                src[q] = nullptr;
                if (active[q] && !(word[q] & kFlag)) src[q] = staged_pairs(A, tile[q], word[q]) + within[q];
            }
#pragma unroll
            for (uint32_t q = 0; q < kMaxPer; ++q) pr[q] = src[q] ? *src[q] : make_uint2(0u, 0u);
#pragma unroll
            for (uint32_t q = 0; q < kMaxPer; ++q) {
                if (src[q]) {
                    const uint32_t r = (uint32_t)w0 + q * kFinishWG + tid;
                    // streamed out: nothing in this kernel reads them again, and what is not left
                    // dirty in L2 does not have to be written back when the kernel ends
                    __builtin_nontemporal_store(pr[q].x, &A.out_idx[r]);
                    __builtin_nontemporal_store(__uint_as_float(pr[q].y), &A.out_val[r]);
                    if (word[q] & kKept) {
                        // staged but left in the residual: zeroed now that it is sent
                        __builtin_nontemporal_store(0.0f, &A.e[pr[q].x]);
                        if (NORM) left_selected(__uint_as_float(pr[q].y), sub, sub_nf);
                    }
                }
            }
        }
        // Flagged tiles: the lane whose rank is a flagged tile's FIRST pair has its wave re-read
        // that tile and emit all of it (up to the capacity); the tile's other ranks, in this
        // wave or elsewhere, are left to that one wave.
#pragma unroll
        for (uint32_t q = 0; q < kMaxPer; ++q) {
            uint64_t pend = __ballot(active[q] && (word[q] & kFlag) != 0 && within[q] == 0u);
            while (pend) {  // wave-uniform
                const uint32_t l = (uint32_t)__ffsll((unsigned long long)pend) - 1u;
                pend &= pend - 1u;
                emit_flagged_tile<NORM, CMP>(A, wave_lane(tile[q], l),
                                             wave_lane((uint32_t)w0 + q * kFinishWG + tid, l), n_out, delta,
                                             lane, n_g, e_lo, e_hi, sub, sub_nf);
            }
        }
        __syncthreads();  // S.win, S.tpre, S.tword are rewritten by the next window
    }
}

template <bool NORM, int CMP>
__device__ __forceinline__ void finish_place(const FinishArgs &A, uint32_t n_g, uint64_t cap)
{
    constexpr uint32_t kWaves = kFinishWG / 64;
    __shared__ PlaceShared S;
    const uint32_t tid  = threadIdx.x;
    const uint32_t lane = tid & 63u;
    const uint32_t wave = tid >> 6;
    const uint32_t wg   = blockIdx.x - 1u;
    const bool by_tile  = wg < A.n_tile_wgs;  // workgroup-uniform

    // what the device state is asked for, and a tile workgroup's first tile words, are requested
    // before the table is built: every first touch of memory costs over a microsecond here
    // (volatile: issued here, in program order, and waited for only where the value is used)
    const float    delta  = *reinterpret_cast<const volatile float *>(&A.st->delta[A.parity]);
    const uint64_t k_prev = *reinterpret_cast<const volatile uint64_t *>(&A.st->k_hist[A.parity ^ 1u]);  // the control workgroup writes the other entry
    uint4 w4 = make_uint4(0u, 0u, 0u, 0u);
    if (by_tile) {
        const uint32_t tile0 = (wg * kFinishWG + tid) * kTilesPerThr;
        if (tile0 < A.n_tiles) w4 = *reinterpret_cast<const uint4 *>(A.tile_cnt + tile0);
    }
    place_table(A, S);
    const uint32_t total = S.total;                                  // selected by this pass
    const uint32_t n_out = total < cap ? total : (uint32_t)cap;      // pairs the output receives
    double   sub = 0.0, add = 0.0;   // norm statistic: squares leaving / re-entering the residual
    uint32_t sub_nf = 0;
    if (by_tile)
        place_tiles<NORM>(A, S, cap, wg, w4, k_prev, add);
    else
        place_ranks<NORM, CMP>(A, S, n_g, n_out, wg - A.n_tile_wgs, gridDim.x - 1u - A.n_tile_wgs, delta, sub,
                               sub_nf);

    if (NORM) {
        const double net = wave_sum(add - sub);
        sub_nf = wave_sum(sub_nf);
        if (lane == 0) {
            // into the slots that hold the squares of the selected entries the streaming pass left behind
            if (net != 0.0) atomicAdd(&A.err_slots[kErrSlots + (wg * kWaves + wave) % kErrSlots], net);
            if (sub_nf) atomicAdd(&A.st->nf_emit[A.parity], sub_nf);
        }
    }
}

template <bool NORM, int CMP>
__global__ void __launch_bounds__(kFinishWG)
k_finish(FinishArgs A, CtrlParams prm)
{
    if (blockIdx.x == 0)
        finish_control(A, prm);
    else
        finish_place<NORM, CMP>(A, (uint32_t)prm.n_g, prm.cap);
}

}  // namespace

#endif  // EXDYNA_K_FINISH_H
