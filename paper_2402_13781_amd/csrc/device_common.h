// Constants, device-resident state and wavefront helpers shared by all kernels.
#ifndef EXDYNA_DEVICE_COMMON_H
#define EXDYNA_DEVICE_COMMON_H

#include <hip/hip_runtime.h>

#include <cstdint>

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
    uint64_t padding;      // Eq. 4: P * (P * m_t - k')
};

struct CtrlParams {
    uint64_t n_g;
    uint64_t cap;
    double   k;          // d * n_g
    double   alpha, inv_alpha, beta, inv_beta;
    float    sf_hi, sf_mid, sf_lo;
    uint32_t n_b, n_parts, block_size, blk_move, min_blk;
};

typedef float f32x4 __attribute__((ext_vector_type(4)));

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

}  // namespace

#endif  // EXDYNA_DEVICE_COMMON_H
