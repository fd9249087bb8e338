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
constexpr uint32_t kStageBuf    = 256;   // pairs a wavefront of k_stream lines up in LDS before it stores them
constexpr uint32_t kSegShift    = 4;     // longer vectors: 16 wave tiles per segment counter, unless the density asks for fewer
constexpr uint32_t kMaxSegShift = 6;     // ... or the vector is so long (> 2 G gradients) that the group table asks for more
constexpr uint32_t kMaxFineSegs = 65536; // up to this many segments, a segment is the four tiles of one streaming workgroup
constexpr uint32_t kMaxGroups   = 4096;  // groups (of 1, 4 or 16 segments) a placement workgroup keeps offsets for: 16 KB of LDS
constexpr uint32_t kMaxParts    = 1024;
constexpr uint32_t kFinishWG    = 1024;  // k_finish: 16 waves
constexpr uint32_t kTilesPerThr = 4;     // placement by tile: consecutive wave tiles per thread
constexpr uint32_t kMaxTileWG   = 96;    // placement workgroups that work by tile ...
constexpr uint32_t kMaxPlaceWG  = 255;   // ... and in all: with the control workgroup, one per compute unit
constexpr uint32_t kErrSlots    = 256;
// tile word, written by the streaming pass: count (0..1024), what became of the selected
// gradients, and where in the extra part of the staging pool they are (in units of 16 pairs)
// when they did not fit the tile's fixed slots
constexpr uint32_t kCountMask   = 0x000007FFu;
constexpr uint32_t kKept        = 0x00000800u;  // staged, but left in the residual (not zeroed)
constexpr uint32_t kFlag        = 0x00001000u;  // only counted, not staged
constexpr uint32_t kOffShift    = 13;           // 19 bits: extra parts of up to 2^23 pairs
constexpr uint64_t kMaxPackedExtra = 1ull << 23;  // a larger extra part is addressed through the slot table
// slot table entry {.x = offset in the extra part of the staging pool, .y = slots there | bits}
constexpr uint32_t kZeroBit     = 0x80000000u;  // the streaming pass may zero what it stages
constexpr uint32_t kCountOnly   = 0x40000000u;  // do not stage at all, only count
constexpr uint32_t kSlotMask    = 0x00FFFFFFu;
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
    // norm statistic, by iteration parity: selected +-Inf entries that were left in the residual
    // by the streaming pass, and how many of them the placement then emitted
    uint32_t nf_sel[2];
    uint32_t nf_emit[2];
    uint64_t k_hist[2];    // selected count of the last two selection passes, by iteration parity
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

// Wavefront scans and reductions on the data-parallel-primitive path of the vector ALU
// (lane shifts inside 16-lane rows, then the last lane of a row broadcast to the rows after
// it): a few cycles per step, where a shuffle through the LDS crossbar costs about a hundred.
// A lane whose source lies outside its row, or whose row the step does not address, receives
// `ident`.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_move(uint32_t ident, uint32_t src)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)ident, (int)src, CTRL, ROW_MASK, 0xF, false);
}

// Inclusive scan over the 64 lanes with an associative op(later, earlier); ident is its
// neutral element.  Steps: row_shr 1, 2, 4, 8; row_bcast 15 into rows 1 and 3; row_bcast 31
// into rows 2 and 3.
template <class Op>
__device__ __forceinline__ uint32_t wave_scan(uint32_t x, uint32_t ident, Op op)
{
    x = op(x, dpp_move<0x111, 0xF>(ident, x));
    x = op(x, dpp_move<0x112, 0xF>(ident, x));
    x = op(x, dpp_move<0x114, 0xF>(ident, x));
    x = op(x, dpp_move<0x118, 0xF>(ident, x));
    x = op(x, dpp_move<0x142, 0xA>(ident, x));
    x = op(x, dpp_move<0x143, 0xC>(ident, x));
    return x;
}

struct OpAdd { __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a + b; } };
struct OpMax { __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a > b ? a : b; } };

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v, uint32_t /*lane*/)
{
    return wave_scan(v, 0u, OpAdd());
}

// value of lane `l` (the same l in every lane) in all lanes
__device__ __forceinline__ uint32_t wave_lane(uint32_t v, uint32_t l)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)l);
}

// sums / maximum over the 64 lanes, in all lanes
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) { return wave_lane(wave_scan(v, 0u, OpAdd()), 63); }
__device__ __forceinline__ uint32_t wave_max(uint32_t v) { return wave_lane(wave_scan(v, 0u, OpMax()), 63); }

__device__ __forceinline__ double wave_sum(double v)
{
    // the two 32-bit halves move through the same lane pattern; the additions are fp64
    auto shifted = [](double x, int step) -> double {
        const uint64_t b = (uint64_t)__double_as_longlong(x);
        uint32_t lo = (uint32_t)b, hi = (uint32_t)(b >> 32);
        switch (step) {
        case 0: lo = dpp_move<0x111, 0xF>(0u, lo); hi = dpp_move<0x111, 0xF>(0u, hi); break;
        case 1: lo = dpp_move<0x112, 0xF>(0u, lo); hi = dpp_move<0x112, 0xF>(0u, hi); break;
        case 2: lo = dpp_move<0x114, 0xF>(0u, lo); hi = dpp_move<0x114, 0xF>(0u, hi); break;
        case 3: lo = dpp_move<0x118, 0xF>(0u, lo); hi = dpp_move<0x118, 0xF>(0u, hi); break;
        case 4: lo = dpp_move<0x142, 0xA>(0u, lo); hi = dpp_move<0x142, 0xA>(0u, hi); break;
        default: lo = dpp_move<0x143, 0xC>(0u, lo); hi = dpp_move<0x143, 0xC>(0u, hi); break;
        }
        return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));  // +0.0 where nothing arrives
    };
#pragma unroll
    for (int step = 0; step < 6; ++step) v += shifted(v, step);
    const uint64_t b = (uint64_t)__double_as_longlong(v);
    const uint32_t lo = wave_lane((uint32_t)b, 63), hi = wave_lane((uint32_t)(b >> 32), 63);
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
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
