// Small set-up and read-out kernels.
#ifndef EXDYNA_K_SETUP_H
#define EXDYNA_K_SETUP_H

#include "device_common.h"

namespace {

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
    if (tid < 4 * kErrSlots) err_slots[tid] = 0.0;
    if (tid == 0) {
        st->delta[0] = delta0;
        st->delta[1] = delta0;
        st->delta_used = delta0;
        st->delta_next = delta0;
        st->overflow = 0; st->moves = 0; st->t = 0;
        st->k_actual = 0; st->k_emitted = 0; st->k_max_part = 0;
        st->density_error = 0.0; st->traffic_ratio = 0.0; st->err_norm = -1.0;
        st->own_actual = 0; st->own_emitted = 0; st->bad_index = 0; st->pad = 0; st->padding = 0;
        st->nf_sel[0] = st->nf_sel[1] = 0; st->nf_emit[0] = st->nf_emit[1] = 0;
        st->k_hist[0] = st->k_hist[1] = 0;
    }
}

// Before the first iteration every wave tile has only its fixed staging slots and zeroes what
// it stages (nothing is known yet that would place a tile beyond the output capacity).
__global__ void k_init_slot_tab(uint2 *tab0, uint2 *tab1, uint32_t n_tiles)
{
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n_tiles; i += gridDim.x * blockDim.x) {
        const uint2 v = make_uint2(0u, kZeroBit);
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
    st->own_actual = 0; st->own_emitted = 0; st->bad_index = 0; st->pad = 0; st->padding = 0;
    st->nf_sel[0] = st->nf_sel[1] = 0; st->nf_emit[0] = st->nf_emit[1] = 0;
    st->k_hist[0] = st->k_hist[1] = 0;
}

// Eq. 1 from the partial sums of squares.  A selected infinity that stayed in the residual is
// not in the sums (it would cancel badly against the ones that were emitted): it is counted.
__global__ void k_norm_finalize(DevState *st, const double *err_slots, uint32_t parity)
{
    __shared__ double s[kErrSlots];
    // unselected squares, and what is left of the selected entries that stayed in the residual
    s[threadIdx.x] = err_slots[threadIdx.x] + err_slots[kErrSlots + threadIdx.x];
    __syncthreads();
    for (uint32_t d = kErrSlots / 2; d >= 1; d >>= 1) {
        if (threadIdx.x < d) s[threadIdx.x] += s[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        double sq = s[0] > 0.0 ? s[0] : s[0] == s[0] ? 0.0 : s[0];
        if (sq == sq && st->nf_sel[parity] > st->nf_emit[parity]) sq = INFINITY;
        st->err_norm = sqrt(sq);
    }
}

}  // namespace

#endif  // EXDYNA_K_SETUP_H
