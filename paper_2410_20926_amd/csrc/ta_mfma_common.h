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

// One lane's 16-byte chunk (8 features starting at byte `lbyte` of the row at `base + rowoff`).  NARROW:
// the row holds only `dbytes` bytes (at least 16; a head width that is a multiple of 4 but not of 8 features,
// or simply narrower than the tile) and starts on a multiple of 8 bytes: what lies outside the row reads as
// zero, so that the tile's extra features are zero in every operand.  One 16-byte request per lane (on an
// 8-byte boundary where the row starts on one) and no branch: a branch per request makes every request wait
// for the one before.  A chunk that would pass the end of the row is replaced by the row's last 16 bytes,
// whose second half is the chunk's first (the row's length is a multiple of 8).
template <bool NARROW, bool NT>
__device__ inline u32x4 load_chunk(const char* base, uint32_t rowoff, uint32_t lbyte, uint32_t dbytes) {
    if constexpr (!NARROW) {
        const u32x4* a = reinterpret_cast<const u32x4*>(base + (rowoff + lbyte));
        return NT ? __builtin_nontemporal_load(a) : *a;
    } else {
        const bool full = lbyte + 16 <= dbytes, tail = !full && lbyte + 8 <= dbytes;
        const u32x4* a = reinterpret_cast<const u32x4*>(base + (rowoff + (full ? lbyte : dbytes - 16)));
        u32x4 v = NT ? __builtin_nontemporal_load(a) : *a;
        if (tail) v = u32x4{v.z, v.w, 0u, 0u};
        if (!full && !tail) v = u32x4{0u, 0u, 0u, 0u};
        return v;
    }
}
// The same chunk for the row gathers, where the lanes of a row are consecutive lanes that hold consecutive chunks of
// the whole tile row (chunk = lane % 8 or lane % 16) and every lane of the wave takes part.  NARROW rows start on a
// multiple of 8 bytes; strided 8-byte halves (load_chunk) ask for every cache line twice and reach 3.5 TB/s in a plain
// streaming kernel on 200-byte rows, 16-byte requests on 16-byte boundaries 4.65 TB/s.  So a lane asks for the aligned
// 16 bytes that start at or 8 bytes before its chunk (those 8 bytes lie inside the tensor's span: the tensor itself
// starts on a 16-byte boundary), never for bytes past the end of the row, and a row that starts 8 bytes into an
// aligned unit takes the second half of each chunk from the next lane.  Rows are at least 16 bytes long.
template <bool NARROW, bool NT>
__device__ inline u32x4 gather_chunk(const char* base, uint32_t rowoff, uint32_t lbyte, uint32_t dbytes) {
    if constexpr (!NARROW) {
        return load_chunk<false, NT>(base, rowoff, lbyte, dbytes);
    } else {
        const char* row = base + rowoff;
        const uint32_t mis = (uint32_t)(reinterpret_cast<uintptr_t>(row) & 8u);
        const int32_t s = (int32_t)lbyte - (int32_t)mis;           // where this lane's aligned unit starts, relative to the row
        // One 16-byte request per lane and no branch (a branch per chunk would make every request wait for the one
        // before): a unit that would pass the end of the row is replaced by the row's last 16 bytes, whose second
        // half is the unit's first (the row's length is a multiple of 8, so exactly 8 bytes of the unit are inside).
        const bool full = s + 16 <= (int32_t)dbytes, tail = !full && s + 8 <= (int32_t)dbytes;
        const u32x4* src = reinterpret_cast<const u32x4*>(row + (full ? s : (int32_t)dbytes - 16));
        u32x4 a = NT ? __builtin_nontemporal_load(src) : *src;
        if (tail) a = u32x4{a.z, a.w, 0u, 0u};
        if (!full && !tail) a = u32x4{0u, 0u, 0u, 0u};
        // lane i takes the first half of lane i + 1's unit (row_shl:1 within 16 lanes; nothing comes in at the end)
        const uint32_t nx = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a.x, 0x101, 0xf, 0xf, true);
        const uint32_t ny = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a.y, 0x101, 0xf, 0xf, true);
        u32x4 out = mis ? u32x4{a.z, a.w, nx, ny} : a;
        if (lbyte + 8 > dbytes) { out.x = 0u; out.y = 0u; }
        if (lbyte + 16 > dbytes) { out.z = 0u; out.w = 0u; }
        return out;
    }
}
// A finished output row leaves its row-major LDS tile (`lds_chunk` = this lane's 16-byte chunk of it, `lbyte` bytes into
// the row).  NARROW: as 8-byte pieces that are contiguous within each store instruction (the lane that holds chunk c
// writes piece c of the row, then piece chunks + c), read from LDS in that order: the two halves of a chunk, 16 bytes
// apart from the next lane's, would leave every cache line half written by either instruction.
template <bool NARROW, int CHUNKS>
__device__ inline void store_row_chunk(char* base, uint32_t rowoff, const char* lds_chunk, uint32_t lbyte, uint32_t dbytes) {
    if constexpr (!NARROW) {
        __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(lds_chunk), reinterpret_cast<u32x4*>(base + (rowoff + lbyte)));
    } else {
        const uint32_t p0 = lbyte / 2, p1 = 8u * CHUNKS + lbyte / 2;   // byte offsets of the two pieces within the row
        const char* lds_row = lds_chunk - lbyte;
        // (through the cache, so that L2 can join a row's first and last line with the neighbouring heads' parts)
        if (p0 + 8 <= dbytes) *reinterpret_cast<u32x2*>(base + (rowoff + p0)) = *reinterpret_cast<const u32x2*>(lds_row + p0);
        if (p1 + 8 <= dbytes) *reinterpret_cast<u32x2*>(base + (rowoff + p1)) = *reinterpret_cast<const u32x2*>(lds_row + p1);
    }
}
template <bool NARROW>
__device__ inline void store_chunk(char* base, uint32_t rowoff, uint32_t lbyte, uint32_t dbytes, const u32x4 v) {
    if constexpr (!NARROW) {
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(base + (rowoff + lbyte)));
    } else {
        // a whole chunk in one store (on an 8-byte boundary where the row starts on one), the row's last 8 bytes on their own
        // (through the cache: a row's first and last cache line may be shared with the neighbouring heads' rows, and
        // L2 can put the parts together before the line goes to memory)
        char* a = base + (rowoff + lbyte);
        if (lbyte + 16 <= dbytes) *reinterpret_cast<u32x4*>(a) = v;
        else if (lbyte + 8 <= dbytes) *reinterpret_cast<u32x2*>(a) = u32x2{v.x, v.y};
    }
}

// ---- rotary encoding of a lane's 16-byte chunk (Sec. 3.2: per-axis positions) ----------------------
// A chunk is 4 interleaved feature pairs (2p, 2p+1), p = 4 * chunk + e.  rope_rates gives the turn of
// each of the lane's pairs per position step, in revolutions; rope_chunk turns the chunk of a row at
// position `pos` (by the negative angle when INVERSE: the transpose, what a gradient needs).  fp32
// throughout; the hardware sine and cosine take revolutions, reduced to [0, 1) first.
__device__ inline void rope_rates(const HopParams& p, int chunk, float (&rev)[4]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) rev[e] = __builtin_amdgcn_exp2f(p.rope_c0 * (float)(4 * chunk + e) + p.rope_c1);
}
__device__ inline void rope_sincos(float pos, const float (&rev)[4], float (&c)[4], float (&s)[4]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float t = __builtin_amdgcn_fractf(pos * rev[e]);
        s[e] = __builtin_amdgcn_sinf(t);
        c[e] = __builtin_amdgcn_cosf(t);
    }
}
template <bool INVERSE = false>
__device__ inline u32x4 rope_apply(const u32x4 x, const float (&c)[4], const float (&s)[4]) {
    u32x4 y;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float lo = bf16_lo(x[e]), hi = bf16_hi(x[e]);
        const float sn = INVERSE ? -s[e] : s[e];
        y[e] = pack_bf16x2(lo * c[e] - hi * sn, lo * sn + hi * c[e]);
    }
    return y;
}
__device__ inline u32x4 rope_chunk(const u32x4 x, float pos, const float (&rev)[4]) {
    float c[4], s[4];
    rope_sincos(pos, rev, c, s);
    return rope_apply(x, c, s);
}
// The same on 8 fp32 values (4 pairs) in registers, e.g. a gradient row chunk before it is rounded.
template <bool INVERSE>
__device__ inline void rope_apply_f32(float (&y)[8], const float (&c)[4], const float (&s)[4]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float lo = y[2 * e], hi = y[2 * e + 1];
        const float sn = INVERSE ? -s[e] : s[e];
        y[2 * e] = lo * c[e] - hi * sn;
        y[2 * e + 1] = lo * sn + hi * c[e];
    }
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

// Writes this lane's 16-byte chunks (rows i * kRowsPerPass + lrow) into a row-major tile.
template <int D>
__device__ inline void stage_rows(char* stg, const u32x4 (&raw)[Geo<D>::kPasses]) {
#pragma unroll
    for (int i = 0; i < Geo<D>::kPasses; ++i)
        *reinterpret_cast<u32x4*>(stg + i * Geo<D>::kRowsPerPass * Geo<D>::kPitch) = raw[i];
}

// Operand whose contraction index is the feature: lane (row r32, half hf) reads 8 features
// per 16-wide MFMA step.  Serves as A (rows = tile rows) or B (columns = tile rows).
template <int D>
__device__ inline void read_natural(const char* oprd, u32x4 (&op)[Geo<D>::kKSteps]) {
#pragma unroll
    for (int s = 0; s < Geo<D>::kKSteps; ++s) op[s] = *reinterpret_cast<const u32x4*>(oprd + s * 32);
}

// Operand whose contraction index is the tile row: for feature tile t and 16-row step s2,
// lane (feature 32 t + lane % 32, half hf) gets rows 16 s2 + 8 u + 4 hf + (0..3), u = 0, 1.
// ds_read_b64_tr_b16 works on groups of 16 lanes: lane L of a group supplies the address
// of 4 consecutive features of row (L / 4), at feature offset 4 (L % 4); lane L receives
// feature L of the group's 16, from the 4 rows.
template <int D>
__device__ inline void read_transposed(const char* trbase, u32x4 (&op)[Geo<D>::kDTiles][2]) {
#pragma unroll
    for (int t = 0; t < Geo<D>::kDTiles; ++t)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const char* a0 = trbase + (16 * s2) * Geo<D>::kPitch + 64 * t;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a0));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a0 + 8 * Geo<D>::kPitch));
            const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
            op[t][s2] = u32x4{l2.x, l2.y, h2.x, h2.y};
        }
}

// 16 accumulator values of one lane (rows 8 (r/4) + 4 hf + r % 4) -> two B operands.
__device__ inline void pack_rows(const float (&x)[16], u32x4 (&op)[2]) {
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
        op[s2] = u32x4{pack_bf16x2(x[8 * s2 + 0], x[8 * s2 + 1]), pack_bf16x2(x[8 * s2 + 2], x[8 * s2 + 3]),
                       pack_bf16x2(x[8 * s2 + 4], x[8 * s2 + 5]), pack_bf16x2(x[8 * s2 + 6], x[8 * s2 + 7])};
}

__device__ inline uint32_t range_mask(int lo, int hi) {   // bits [lo, hi), 0 <= lo, hi <= 32
    const uint32_t mh = hi >= 32 ? 0xffffffffu : ((1u << hi) - 1u);
    const uint32_t ml = lo >= 32 ? 0xffffffffu : ((1u << lo) - 1u);
    return mh & ~ml;
}

// Tile rows [lo, hi) visible from query row `row` of a fibre occupying tile rows [flo, fhi):
// the causal triangle and a band of width `window` (0 = none).  The same range, read the
// other way round (rows that see key `row`), is seen_range().
__device__ inline void visible_range(int row, int flo, int fhi, int causal, int window, int& lo, int& hi) {
    lo = flo;
    hi = causal ? row + 1 : fhi;
    if (window > 0) { lo = max(lo, row - window + 1); hi = min(hi, row + window); }
}
__device__ inline void seen_range(int row, int flo, int fhi, int causal, int window, int& lo, int& hi) {
    lo = causal ? row : flo;
    hi = fhi;
    if (window > 0) { lo = max(lo, row - window + 1); hi = min(hi, row + window); }
}

// The caller's bit table of the axis (row a, word j: keys 32 j .. 32 j + 31 visible from query
// position a), all ones when there is none.
// `fibre`: the fibre's number on this axis (used when every fibre has a table of its own).
__device__ inline uint32_t table_word(const HopParams& p, uint32_t fibre, int a, int j) {
    return p.mask ? p.mask[(int64_t)fibre * p.mask_fibre_words + a * p.mask_words + j] : 0xffffffffu;
}
// Its transpose for key position c of an axis of at most 32 positions: bit a = query
// position a sees key c.
__device__ inline uint32_t table_column(const HopParams& p, uint32_t fibre, int c) {
    if (!p.mask) return 0xffffffffu;
    const uint32_t* t = p.mask + (int64_t)fibre * p.mask_fibre_words;
    uint32_t col = 0;
    for (int a = 0; a < p.n; ++a) col |= ((t[a] >> c) & 1u) << a;
    return col;
}

// One key tile of an online softmax.  st: the scores S^T of the tile (lane = query row, 16 of its keys, the other 16
// in lane ^ 32); vis32: the keys of the tile this lane's row may attend (bit = key); sl2 = scale * log2(e) > 0.  Updates
// the running maximum m (log2 domain) and sum l, returns the un-normalised weights, rounded to bf16, as B operands, and
// the factor `corr` by which everything accumulated before this tile has to be multiplied.
// The maximum is taken over the raw scores and scaled once, and the scale goes into the exponent's multiply-add; a tile
// that every row of the wave sees completely (inside the causal triangle, no band, table or padding) skips the masking:
// the kernels that walk many tiles spend a good part of their time in this vector arithmetic.
__device__ inline void online_softmax_tile(const f32x16& st, uint32_t vis32, int hf, float sl2, float& m, float& l,
                                           u32x4 (&pop)[2], float& corr) {
    float e[16], tmax = -INFINITY;
    if (__all(vis32 == 0xffffffffu)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) { e[r] = st[r]; tmax = fmaxf(tmax, e[r]); }
    } else {
        const uint32_t vis = vis32 >> (4 * hf);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const bool ok = (vis >> (8 * (r / 4) + (r % 4))) & 1u;
            e[r] = ok ? st[r] : -INFINITY;
            tmax = fmaxf(tmax, e[r]);
        }
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    if (tmax != -INFINITY) tmax *= sl2;
    const float mnew = fmaxf(m, tmax);
    const float msafe = mnew == -INFINITY ? 0.f : mnew;
    corr = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - msafe);
    m = mnew;
    float psum = 0.f;
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
        uint32_t wds[4];
#pragma unroll
        for (int jp = 0; jp < 4; ++jp) {
            const int r = 8 * s2 + 2 * jp;
            const uint32_t pk = pack_bf16x2(__builtin_amdgcn_exp2f(fmaf(e[r], sl2, -msafe)), __builtin_amdgcn_exp2f(fmaf(e[r + 1], sl2, -msafe)));
            psum += bf16_lo(pk) + bf16_hi(pk);            // sum of the ROUNDED weights
            wds[jp] = pk;
        }
        pop[s2] = u32x4{wds[0], wds[1], wds[2], wds[3]};
    }
    psum += __shfl_xor(psum, 32);
    l = l * corr + psum;
}

// Workgroup numbering of the NARROW instantiations.  Rows that are not whole 64-byte pieces share their first and last
// piece with the neighbouring heads' rows.  Workgroup ids go round the 8 XCDs, so with the plain numbering (head block
// = blockIdx.x, fastest) neighbouring heads are written from different L2s and every shared piece reaches memory as two
// partial writes.  Here each XCD takes a contiguous run of the (blockIdx.y, blockIdx.x) sequence instead: neighbouring
// head blocks follow each other on one XCD, and their rows, stored through the cache, leave its L2 as whole lines
// (head width 100, 32 heads, 32k tokens: a backward hop 620 -> 400 us).  bx, by: the pair to use in place of
// blockIdx.x and blockIdx.y.
template <bool NARROW>
__device__ inline void workgroup_xy(uint32_t& bx, uint32_t& by) {
    bx = blockIdx.x; by = blockIdx.y;
    if constexpr (NARROW) {
        const uint32_t gx = gridDim.x, total = gx * gridDim.y;
        if (total % 8u == 0u) {
            const uint32_t lin = blockIdx.x + gx * blockIdx.y;
            const uint32_t seq = (lin & 7u) * (total / 8u) + (lin >> 3);
            bx = seq % gx;
            by = seq / gx;
        }
    }
}

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
