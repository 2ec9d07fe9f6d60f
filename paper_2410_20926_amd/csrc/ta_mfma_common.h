// Pieces shared by the bf16 MFMA kernels (forward and backward): vector types, the
// bf16 pack, the wave-level LDS ordering point, tile geometry and the host-side launch
// geometry.  Internal to the library.
#pragma once

#include "ta_internal.h"

namespace ta {
namespace mfma {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int kTile = 32;                                 // rows of one MFMA tile
constexpr float kLog2e = 1.4426950408889634f;

__device__ inline uint32_t pack_bf16x2(float lo, float hi) {      // v_cvt_pk_bf16_f32, round to nearest even
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ inline void lds_wave_sync() {
    // LDS operations of one wave complete in issue order; this only stops the compiler
    // from moving shared-memory accesses across the point where lanes exchange data.
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

__device__ inline f32x16 mma(const u32x4 a, const u32x4 b, const f32x16 c) {   // 32x32x16 bf16, fp32 accumulate
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

template <int D>
struct Geo {
    static constexpr int kChunks = D / 8;                 // 16-byte chunks per row
    static constexpr int kRowsPerPass = 64 / kChunks;     // rows one wave-wide load covers
    static constexpr int kPasses = kTile / kRowsPerPass;  // loads per lane per 32-row tile
    static constexpr int kPitch = D * 2 + 16;             // bytes, row-major bf16 transit rows
    static constexpr int kVPitch = D * 4 + 32;            // bytes, one interleaved row pair of V (4 pitches = 32 banks mod 64)
    static constexpr int kKSteps = D / 16;                // MFMA steps over the feature axis
    static constexpr int kDTiles = D / 32;                // 32-column tiles of an output
    static constexpr int kBufBytes = (kTile * kPitch > (kTile / 2) * kVPitch) ? kTile * kPitch : (kTile / 2) * kVPitch;
};

// Launch geometry computed on the host.
struct TileParams {
    int32_t fpt;          // fibres per 32-row tile (n <= 32), else 1
    int32_t qtiles;       // query tiles per fibre: 1 (n <= 32) or 2
    uint32_t tiles;       // units per (batch, head)
    uint32_t tiles_lo;    // gridDim.y; gridDim.z = B * ceil(tiles / tiles_lo)
    uint32_t tiles_hi;
    uint32_t q_row, k_row, v_row, o_row;   // token pitch of each tensor in BYTES
    float inv_n;          // 1 / n
};

// Fills tp for an axis of length p.n walked in `key_tiles` 32-key tiles; false when the
// grid would not fit.
inline bool make_tile_params(const HopParams& p, int key_tiles, TileParams* tp) {
    tp->fpt = key_tiles == 1 ? kTile / p.n : 1;
    tp->qtiles = key_tiles == 1 ? 1 : (p.n + kTile - 1) / kTile;
    const int64_t tiles = key_tiles == 1 ? (p.fibres + tp->fpt - 1) / tp->fpt : p.fibres * tp->qtiles;
    if (tiles <= 0 || tiles > 0x7fffffffLL) return false;
    tp->tiles = (uint32_t)tiles;
    tp->tiles_lo = (uint32_t)(tiles < 32768 ? tiles : 32768);
    tp->tiles_hi = (uint32_t)((tiles + tp->tiles_lo - 1) / tp->tiles_lo);
    if ((int64_t)p.B * tp->tiles_hi > 65535) return false;
    tp->q_row = (uint32_t)(p.q.st * 2);
    tp->k_row = (uint32_t)(p.k.st * 2);
    tp->v_row = (uint32_t)(p.vin.st * 2);
    tp->o_row = (uint32_t)(p.o.st * 2);
    tp->inv_n = 1.0f / (float)p.n;
    return true;
}

// Largest byte offset inside one (batch, head) slice must fit 32 bits.
inline bool fits_u32(const Tensor& t, int64_t N) { return (N - 1) * t.st * 2 + 512 < (int64_t)0xffffffffLL; }

}  // namespace mfma
}  // namespace ta
