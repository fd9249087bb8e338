// Worker view after the AllGather (gather, clear, replicated control) and the model update.
#ifndef EXDYNA_K_EXCHANGE_H
#define EXDYNA_K_EXCHANGE_H

#include "device_common.h"
#include "k_finish.h"

namespace {

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
        const float    delta  = A.st->delta[A.parity];
        const uint64_t t_done = A.st->t;  // read before this workgroup advances it
        if (tid < P) {
            const uint32_t t_mod_p = (uint32_t)(t_done % P);
            S.lpos[tid]  = A.cur_pos[tid];
            S.lpart[tid] = A.cur_part[tid];
            // rank tid selected partition (t mod P + tid) mod P (Alg. 3 (cyclic allocation))
            const uint64_t k_r = X.counts[tid];
            S.cnt[(t_mod_p + tid) % P] = (uint32_t)(k_r < prm.n_g ? k_r : prm.n_g);
        }
        __syncthreads();
        control_decide(A, prm, S, kCtrlUpdate, delta, t_done);
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
        const double s = wave_sum((double)sq);
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

}  // namespace

#endif  // EXDYNA_K_EXCHANGE_H
