// bf16 MFMA per-axis attention backward for gfx950 (CDNA4): the derivative of one hop of
// Eq. 4 of arXiv 2410.20926 (the paper states only that a backward exists, Sec. 3.2).
//
// For one 32-row tile (floor(32 / n) fibres packed, block-diagonal mask) of one query head,
// with A the hop's attention, X the value input and G the upstream gradient:
//     P  = softmax(Q K^T * scale, mask)          dP = G X^T
//     dS = P o (dP - rowsum(P o dP))
//     dX = P^T G      dQ = dS K * scale      dK = dS^T Q * scale
// One wavefront handles one (tile, query head); a workgroup is the G <= 8 query heads that
// share a key/value head (8 of them at a time when there are more), so dK (and dX when the value input is V) are summed across the
// workgroup's waves in a fixed order through LDS: deterministic, no atomics.
//
// Layouts.  Every tensor tile goes ONCE into a row-major LDS transit buffer and is read
// back (a) row by row as an MFMA operand whose contraction runs over the features
// (S, dP) and (b) with ds_read_b64_tr_b16 as the transposed operand whose contraction runs
// over the tile rows (K^T for dQ, G^T for dX, Q^T for dK).  The 32x32 score products are
// formed in both orientations (S^T, dP^T: one query row per lane; S, dP: one key per lane)
// so that dS^T and P, dS come out of the accumulators directly in B-operand layout; row
// statistics cross from the first orientation to the second through 3 x 32 floats of LDS.
#include "ta_mfma_common.h"

namespace ta {
namespace {

using namespace mfma;

template <int D>
struct BGeo : Geo<D> {
    static constexpr int kBuf = kTile * Geo<D>::kPitch;   // one row-major bf16 tile; also 32 rows x 64 fp32 (+pad) for D = 128
    static constexpr int kFPitch = 64 * 4 + 16;           // bytes, fp32 half-tile rows (64 columns)
    static constexpr int kBufBytes = (kBuf > kTile * kFPitch) ? kBuf : kTile * kFPitch;
    static constexpr int kStats = 3 * kTile * 4;          // row max (log2 domain), 1/rowsum, delta
    static constexpr int kWaveBytes = kBufBytes + kStats + kTile * 16;
    static constexpr int kRedBytes = Geo<D>::kDTiles * 16 * 64 * 4;   // one fp32 accumulator set, lane-major
};

// The epilogue's lane -> (row, 16-byte chunk) mapping: pass i of feature half `half` covers
// row 8 i + lane / 8, chunk lane % 8 of the half (8 lanes x 16 B = 128 contiguous bytes).
template <int D>
__device__ inline uint32_t tile_out_offset(const u32x4* rowoff, int which, int half, int i, int lane) {
    const u32x4 off4 = rowoff[8 * i + (lane >> 3)];
    return (which == 0 ? off4.x : which == 1 ? off4.y : off4.z) + (half * 64 + (lane & 7) * 8) * 2;
}

// Requests the current contents of an output tile (for accumulate = 1) long before the
// epilogue needs them, in the epilogue's mapping.
// NARROW (here and below): rows hold only `dbytes` bytes and are 8-byte aligned; see load_chunk.
template <int D, bool NARROW = false>
__device__ inline void prefetch_tile(u32x4 (&old)[Geo<D>::kDTiles * 2], const u32x4* rowoff, int which, const char* gbase, int lane,
                                     uint32_t dbytes = 0) {
#pragma unroll
    for (int half = 0; half < Geo<D>::kDTiles / 2; ++half)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if constexpr (NARROW) {
                const uint32_t fbyte = (uint32_t)(half * 64 + (lane & 7) * 8) * 2;
                old[half * 4 + i] = load_chunk<true, true>(gbase, tile_out_offset<D>(rowoff, which, half, i, lane) - fbyte, fbyte, dbytes);
            } else {
                old[half * 4 + i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gbase + tile_out_offset<D>(rowoff, which, half, i, lane)));
            }
        }
}

// acc[t][r] holds (row = lane % 32, feature 32 t + 8 (r/4) + 4 hf + r % 4).  Multiplies by
// `mult`, optionally adds the tensor's previous contents (`old`, from prefetch_tile), rounds
// to bf16 and stores the rows with 16-byte stores; the transposition goes through LDS in
// fp32, 64 features at a time.
// No rotation of the stored rows.
struct NoRope {
    static constexpr bool on = false;
    __device__ float pos(int) const { return 0.f; }
    __device__ const HopParams* hop() const { return nullptr; }
};
// The rows are gradients with respect to rotary-encoded rows: tile row r sits at position pos(r) on the
// hop's axis and is turned back (the encoding's transpose) before anything is added to it.
template <typename PosFn>
struct UnRope {
    static constexpr bool on = true;
    const HopParams* p;
    PosFn fn;
    __device__ float pos(int r) const { return fn(r); }
    __device__ const HopParams* hop() const { return p; }
};
template <typename PosFn>
__device__ inline UnRope<PosFn> unrope(const HopParams* p, PosFn fn) { return UnRope<PosFn>{p, fn}; }

template <int D, bool NARROW = false, typename Enc = NoRope>
__device__ inline void store_tile(const f32x16 (&acc)[Geo<D>::kDTiles], float mult, char* buf, const u32x4* rowoff,
                                  int which, char* gbase, const u32x4 (&old)[Geo<D>::kDTiles * 2], bool add_old, int rows_valid, int lane,
                                  uint32_t dbytes = 0, const Enc enc = Enc{}) {
    using G = BGeo<D>;
    const int r32 = lane & 31, hf = lane >> 5;
#pragma unroll
    for (int half = 0; half < G::kDTiles / 2; ++half) {
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x16& a = acc[2 * half + t2];
                const f32x4 v = {a[4 * q4] * mult, a[4 * q4 + 1] * mult, a[4 * q4 + 2] * mult, a[4 * q4 + 3] * mult};
                *reinterpret_cast<f32x4*>(buf + r32 * G::kFPitch + (32 * t2 + 8 * q4 + 4 * hf) * 4) = v;
            }
        lds_wave_sync();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = 8 * i + (lane >> 3), cc = lane & 7;
            const f32x4 x0 = *reinterpret_cast<const f32x4*>(buf + row * G::kFPitch + cc * 32);
            const f32x4 x1 = *reinterpret_cast<const f32x4*>(buf + row * G::kFPitch + cc * 32 + 16);
            if (row < rows_valid) {
                float y[8] = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
                if constexpr (Enc::on) {
                    if (enc.hop()->rope) {
                        float rev[4], c[4], sn[4];
                        rope_rates(*enc.hop(), half * 8 + cc, rev);
                        rope_sincos(enc.pos(row), rev, c, sn);
                        rope_apply_f32<true>(y, c, sn);
                    }
                }
                if (add_old) {
                    const u32x4 o = old[half * 4 + i];
#pragma unroll
                    for (int e = 0; e < 4; ++e) { y[2 * e] += bf16_lo(o[e]); y[2 * e + 1] += bf16_hi(o[e]); }
                }
                const u32x4 packed = u32x4{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]), pack_bf16x2(y[4], y[5]), pack_bf16x2(y[6], y[7])};
                if constexpr (NARROW) {
                    const uint32_t fbyte = (uint32_t)(half * 64 + (lane & 7) * 8) * 2;
                    store_chunk<true>(gbase, tile_out_offset<D>(rowoff, which, half, i, lane) - fbyte, fbyte, dbytes, packed);
                } else {
                    __builtin_nontemporal_store(packed, reinterpret_cast<u32x4*>(gbase + tile_out_offset<D>(rowoff, which, half, i, lane)));
                }
            }
        }
        lds_wave_sync();
    }
}

// The same without previous contents to add: the values are rounded to bf16 BEFORE the
// transposition, which then moves half the bytes through LDS (one row-major bf16 tile).
template <int D, bool NARROW = false>
__device__ inline void store_tile_plain(const f32x16 (&acc)[Geo<D>::kDTiles], float mult, char* buf, const u32x4* rowoff,
                                        int which, char* gbase, int rows_valid, int lane, uint32_t dbytes = 0) {
    using G = BGeo<D>;
    const int r32 = lane & 31, hf = lane >> 5;
    const int lrow = lane / G::kChunks, lcol = lane % G::kChunks;
#pragma unroll
    for (int t = 0; t < G::kDTiles; ++t)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            u32x2 v;
            v.x = pack_bf16x2(acc[t][4 * q4] * mult, acc[t][4 * q4 + 1] * mult);
            v.y = pack_bf16x2(acc[t][4 * q4 + 2] * mult, acc[t][4 * q4 + 3] * mult);
            *reinterpret_cast<u32x2*>(buf + r32 * G::kPitch + (32 * t + 8 * q4 + 4 * hf) * 2) = v;
        }
    lds_wave_sync();
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i) {
        const int row = i * G::kRowsPerPass + lrow;
        if (row < rows_valid) {
            const u32x4 v = *reinterpret_cast<const u32x4*>(buf + row * G::kPitch + lcol * 16);
            const u32x4 off4 = rowoff[row];
            if constexpr (NARROW) store_chunk<true>(gbase, which == 0 ? off4.x : which == 1 ? off4.y : off4.z, (uint32_t)lcol * 16, dbytes, v);
            else __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(gbase + ((which == 0 ? off4.x : which == 1 ? off4.y : off4.z) + lcol * 16)));
        }
    }
    lds_wave_sync();
}

// Sum of acc over the workgroup's waves in wave order; the total ends in the LAST wave's
// registers.  `red` is a workgroup-shared fp32 area in lane-major layout.
template <int D>
__device__ inline void chain_sum(f32x16 (&acc)[Geo<D>::kDTiles], float* red, int w, int nw, int lane) {
    constexpr int kT = Geo<D>::kDTiles;
    for (int s = 0; s + 1 < nw; ++s) {
        if (w == s) {
#pragma unroll
            for (int t = 0; t < kT; ++t)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    f32x4* cell = reinterpret_cast<f32x4*>(red) + (t * 4 + q4) * 64 + lane;
                    f32x4 v = {acc[t][4 * q4], acc[t][4 * q4 + 1], acc[t][4 * q4 + 2], acc[t][4 * q4 + 3]};
                    if (s > 0) v += *cell;
                    *cell = v;
                }
        }
        __syncthreads();
    }
    if (nw > 1 && w == nw - 1) {
#pragma unroll
        for (int t = 0; t < kT; ++t)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 v = *(reinterpret_cast<const f32x4*>(red) + (t * 4 + q4) * 64 + lane);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[t][4 * q4 + e] += v[e];
            }
    }
    __syncthreads();                                      // red may be reused
}

// blockDim.x = 64 * G (G = query heads per key/value head: 1, 2, 4 or 8); grid = (Hkv, tiles_lo, B * tiles_hi).
// TABLE: the axis has a caller's bit table; MULTI: the group has more than 8 heads and this launch
// covers 8 of them (separate instantiations keep the common case free of both).
// ROPE: the hop scores with rotary-encoded Q and K (separate instantiations, so that the plain kernel carries none of it).
template <int D, bool TABLE, bool MULTI, bool NARROW, bool ROPE>
__global__ __launch_bounds__(512, 2) void mfma_bwd_kernel(BwdParams bp, TileParams tp) {
    using G = BGeo<D>;
    const HopParams& p = bp.hop;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw = MULTI ? bp.wg_heads : p.G;

    uint32_t bx, ty;
    workgroup_xy<NARROW>(bx, ty);
    const int g = (int)bx;
    const int h = g * p.G + (MULTI ? bp.head_base : 0) + w;
    const uint32_t zb = blockIdx.z / tp.tiles_hi;
    const uint32_t tt = (blockIdx.z - zb * tp.tiles_hi) * tp.tiles_lo + ty;
    if (tt >= tp.tiles) return;                           // whole workgroup leaves together
    const int b = (int)zb;
    const bool vin_is_o = (p.vin_heads == p.Hq);
    const int hv = vin_is_o ? h : g;
    const int n = p.n;

    float* red = reinterpret_cast<float*>(smem);          // workgroup-shared reduction area
    char* buf = smem + (nw > 1 ? G::kRedBytes : 0) + w * G::kWaveBytes;
    float* stats = reinterpret_cast<float*>(buf + G::kBufBytes);
    u32x4* rowoff = reinterpret_cast<u32x4*>(buf + G::kBufBytes + G::kStats);   // per row: byte offsets in (q, k, v_in, o) layouts

    const uint32_t f0 = tt * tp.fpt;
    const int rows_valid = (int)min((uint32_t)tp.fpt, (uint32_t)p.fibres - f0) * n;
    uint32_t real_rows;                                   // bit r: tile row r exists and its token is not padding
    {
        bool real = false;
        if (lane < kTile) {
            const uint32_t stride = (uint32_t)p.stride;
            const int rc = min(lane, rows_valid - 1);     // rows past the last fibre alias the last valid row: loads need no predicate
            const uint32_t fi = (uint32_t)((rc + 0.5f) * tp.inv_n);
            const uint32_t a = rc - fi * n;
            const uint32_t f = f0 + fi;
            const uint32_t outer = f / stride;
            const uint32_t tok = outer * stride * n + (f - outer * stride) + a * stride;
            rowoff[lane] = u32x4{tok * tp.q_row, tok * tp.k_row, tok * tp.v_row, tok * tp.o_row};
            real = lane < rows_valid && tok < (uint32_t)hop_valid_len(p, b);
        }
        real_rows = (uint32_t)__ballot(real);
    }
    lds_wave_sync();

    const char* qb = reinterpret_cast<const char*>(p.q.p) + ((int64_t)b * p.q.sb + (int64_t)h * p.q.sh) * 2;
    const char* kb = reinterpret_cast<const char*>(p.k.p) + ((int64_t)b * p.k.sb + (int64_t)g * p.k.sh) * 2;
    const char* xb = reinterpret_cast<const char*>(p.vin.p) + ((int64_t)b * p.vin.sb + (int64_t)hv * p.vin.sh) * 2;
    const char* gb = reinterpret_cast<const char*>(bp.d_o.p) + ((int64_t)b * bp.d_o.sb + (int64_t)h * bp.d_o.sh) * 2;
    char* dqb = reinterpret_cast<char*>(bp.dq.p) + ((int64_t)b * bp.dq.sb + (int64_t)h * bp.dq.sh) * 2;
    char* dkb = reinterpret_cast<char*>(bp.dk.p) + ((int64_t)b * bp.dk.sb + (int64_t)g * bp.dk.sh) * 2;
    char* dxb = reinterpret_cast<char*>(bp.d_vin.p) + ((int64_t)b * bp.d_vin.sb + (int64_t)hv * bp.d_vin.sh) * 2;

    const int lrow = lane / G::kChunks, lcol = lane % G::kChunks;
    const uint32_t lbyte = lcol * 16;
    const uint32_t dbytes = (uint32_t)p.D * 2;            // bytes of a row (less than the tile's when NARROW)
    const int r32 = lane & 31, hf = lane >> 5;

    // ---- gather Q, K, X, G rows: every load is issued before the first wait, in the order of first use
    //      (loads complete in order: Q and K can be staged while X and G are still on their way) ------------
    u32x4 qraw[G::kPasses], kraw[G::kPasses], xraw[G::kPasses], graw[G::kPasses];
    // Rows read by this wave alone are streamed; rows every wave of the group reads stay cached.
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i) qraw[i] = gather_chunk<NARROW, true>(qb, rowoff[i * G::kRowsPerPass + lrow].x, lbyte, dbytes);
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i) kraw[i] = gather_chunk<NARROW, false>(kb, rowoff[i * G::kRowsPerPass + lrow].y, lbyte, dbytes);
    if (vin_is_o) {                                        // one choice for all eight requests, not one per request
#pragma unroll
        for (int i = 0; i < G::kPasses; ++i) xraw[i] = gather_chunk<NARROW, true>(xb, rowoff[i * G::kRowsPerPass + lrow].z, lbyte, dbytes);
    } else {
#pragma unroll
        for (int i = 0; i < G::kPasses; ++i) xraw[i] = gather_chunk<NARROW, false>(xb, rowoff[i * G::kRowsPerPass + lrow].z, lbyte, dbytes);
    }
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i) graw[i] = gather_chunk<NARROW, true>(gb, rowoff[i * G::kRowsPerPass + lrow].w, lbyte, dbytes);
    __builtin_amdgcn_sched_barrier(0);

    // rotary encoding: Q and K rows are turned by their position on the axis before anything uses them;
    // dQ and dK below are gradients with respect to the turned rows and are turned back when stored
    auto row_pos = [&](int row) -> float {
        const int rc = min(row, rows_valid - 1);
        return (float)(rc - (int)((rc + 0.5f) * tp.inv_n) * n);
    };
    if constexpr (ROPE) {
        float rev[4];
        rope_rates(p, lcol, rev);
#pragma unroll
        for (int i = 0; i < G::kPasses; ++i) {
            float c[4], sn[4];
            rope_sincos(row_pos(i * G::kRowsPerPass + lrow), rev, c, sn);
            qraw[i] = rope_apply(qraw[i], c, sn);
            kraw[i] = rope_apply(kraw[i], c, sn);
        }
    }
    const auto enc = [&]() { if constexpr (ROPE) return unrope(&p, row_pos); else return NoRope{}; }();

    char* stg = buf + lrow * G::kPitch + lbyte;                              // row-major staging (this lane's chunk)
    const char* oprd = buf + r32 * G::kPitch + hf * 16;                      // natural operand reads
    const char* trbase = buf + (4 * hf + ((lane & 15) >> 2)) * G::kPitch     // transposed operand reads
                         + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;

    // ---- Q, K: natural operands for the scores, transposed operands for dK, dQ ----------
    u32x4 qop[G::kKSteps], kop[G::kKSteps], qT[G::kDTiles][2], kT[G::kDTiles][2];
    stage_rows<D>(stg, qraw);
    lds_wave_sync();
    read_natural<D>(oprd, qop);
    read_transposed<D>(trbase, qT);
    lds_wave_sync();
    stage_rows<D>(stg, kraw);
    lds_wave_sync();
    read_natural<D>(oprd, kop);
    read_transposed<D>(trbase, kT);
    lds_wave_sync();

    // sT[r]: query row r32, key 8 (r/4) + 4 hf + r % 4.   sN[r]: key r32, query row 8 (r/4) + 4 hf + r % 4.
    f32x16 sT = {}, sN = {};
#pragma unroll
    for (int s = 0; s < G::kKSteps; ++s) {
        sT = mma(kop[s], qop[s], sT);
        sN = mma(qop[s], kop[s], sN);
    }

    // ---- X, G: dP in both orientations; G^T for dX ---------------------------------------
    u32x4 xop[G::kKSteps], gop[G::kKSteps], gT[G::kDTiles][2];
    stage_rows<D>(stg, xraw);
    lds_wave_sync();
    read_natural<D>(oprd, xop);
    lds_wave_sync();
    stage_rows<D>(stg, graw);
    lds_wave_sync();
    read_natural<D>(oprd, gop);
    read_transposed<D>(trbase, gT);
    lds_wave_sync();
    f32x16 dpT = {}, dpN = {};
#pragma unroll
    for (int s = 0; s < G::kKSteps; ++s) {
        dpT = mma(xop[s], gop[s], dpT);
        dpN = mma(gop[s], xop[s], dpN);
    }

    // previous dQ (accumulate): requested now, consumed after the dQ products
    u32x4 oldq[G::kDTiles * 2] = {};
    if (bp.accumulate) prefetch_tile<D, NARROW>(oldq, rowoff, 0, dqb, lane, dbytes);

    // ---- softmax and dS, one query row per lane -------------------------------------------
    const float sl2 = p.scale * kLog2e;
    const bool row_real = (real_rows >> r32) & 1u;        // this lane's tile row exists and is not padding
    const int flo = (int)((min(r32, rows_valid - 1) + 0.5f) * tp.inv_n) * n;   // its fibre occupies tile rows [flo, fhi)
    const int fhi = flo + n;
    u32x4 dsTop[2];                                       // dS^T as B operands (contraction over keys)
    {
        int lo = 0, hi = 0;
        uint32_t tw = 0xffffffffu;
        if (row_real) { visible_range(r32, flo, fhi, p.causal, p.window, lo, hi); if (TABLE) tw = table_word(p, f0 + (uint32_t)(flo / n), r32 - flo, 0) << flo; }
        const uint32_t vis = (range_mask(lo, hi) & tw & real_rows) >> (4 * hf);
        float e[16], mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const bool ok = (vis >> (8 * (r / 4) + (r % 4))) & 1u;
            e[r] = ok ? sT[r] * sl2 : -INFINITY;
            mx = fmaxf(mx, e[r]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        if (mx == -INFINITY) mx = 0.f;
        float sum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) { e[r] = __builtin_amdgcn_exp2f(e[r] - mx); sum += e[r]; }
        sum += __shfl_xor(sum, 32);
        const float inv = sum > 0.f ? 1.f / sum : 0.f;
        float delta = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) { e[r] *= inv; delta += e[r] * dpT[r]; }
        delta += __shfl_xor(delta, 32);
#pragma unroll
        for (int r = 0; r < 16; ++r) e[r] *= (dpT[r] - delta);
        pack_rows(e, dsTop);
        // P = exp2(s - ref) with ref = max + log2(sum): one number per row instead of two
        if (lane < kTile) { stats[lane] = sum > 0.f ? mx + __builtin_amdgcn_logf(sum) : INFINITY; stats[kTile + lane] = delta; }
    }
    lds_wave_sync();

    // ---- the same, one key per lane: P and dS as B operands (contraction over query rows) --
    u32x4 pNop[2], dsNop[2];
    {
        // query rows that see this lane's key: its own fibre's rows, from itself on when causal
        int lo = 0, hi = 0;
        uint32_t tw = 0xffffffffu;
        if (row_real) { seen_range(r32, flo, fhi, p.causal, p.window, lo, hi); if (TABLE) tw = table_column(p, f0 + (uint32_t)(flo / n), r32 - flo) << flo; }
        const uint32_t vis = (range_mask(lo, hi) & tw & real_rows) >> (4 * hf);
        uint32_t pw[8], dw[8];                            // rounded in pairs as they are formed
        float slv = sl2;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const f32x4 m4 = *reinterpret_cast<const f32x4*>(stats + 8 * q4 + 4 * hf);
            const f32x4 d4 = *reinterpret_cast<const f32x4*>(stats + kTile + 8 * q4 + 4 * hf);
#pragma unroll
            for (int j = 0; j < 4; j += 2) {
                const int r = 4 * q4 + j;
                const bool ok0 = (vis >> (8 * q4 + j)) & 1u, ok1 = (vis >> (8 * q4 + j + 1)) & 1u;
                const float pv0 = ok0 ? __builtin_amdgcn_exp2f(sN[r] * slv - m4[j]) : 0.f;
                const float pv1 = ok1 ? __builtin_amdgcn_exp2f(sN[r + 1] * slv - m4[j + 1]) : 0.f;
                pw[r / 2] = pack_bf16x2(pv0, pv1);
                dw[r / 2] = pack_bf16x2(pv0 * (dpN[r] - d4[j]), pv1 * (dpN[r + 1] - d4[j + 1]));
            }
            // In the instantiations that are short of registers the next four rows start from a value that passes
            // through this statement together with the words just formed, so that the compiler cannot form all
            // sixteen weights first and hold them (it then spills); the plain kernel has room and is faster left alone.
            if constexpr (TABLE || MULTI || NARROW || ROPE)
                asm volatile("" : "+v"(pw[2 * q4]), "+v"(pw[2 * q4 + 1]), "+v"(dw[2 * q4]), "+v"(dw[2 * q4 + 1]), "+v"(slv));
        }
        pNop[0] = u32x4{pw[0], pw[1], pw[2], pw[3]};  pNop[1] = u32x4{pw[4], pw[5], pw[6], pw[7]};
        dsNop[0] = u32x4{dw[0], dw[1], dw[2], dw[3]}; dsNop[1] = u32x4{dw[4], dw[5], dw[6], dw[7]};
    }

    // ---- dQ^T = K^T dS^T : per head, stored at once -----------------------------------------
    f32x16 acc[G::kDTiles];
#pragma unroll
    for (int t = 0; t < G::kDTiles; ++t) {
        acc[t] = f32x16{};
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) acc[t] = mma(kT[t][s2], dsTop[s2], acc[t]);
    }
    store_tile<D, NARROW>(acc, p.scale, buf, rowoff, 0, dqb, oldq, bp.accumulate != 0, rows_valid, lane, dbytes, enc);

    // ---- dX^T = G^T P : per head, or summed over the group when the value input is V ------
#pragma unroll
    for (int t = 0; t < G::kDTiles; ++t) {
        acc[t] = f32x16{};
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) acc[t] = mma(gT[t][s2], pNop[s2], acc[t]);
    }
    if (vin_is_o) {
        store_tile_plain<D, NARROW>(acc, 1.f, buf, rowoff, 2, dxb, rows_valid, lane, dbytes);
    } else {
        if constexpr (MULTI) {
            u32x4 oldx[G::kDTiles * 2] = {};              // the sum of the group's earlier heads
            if (bp.acc_x && w == nw - 1) prefetch_tile<D, NARROW>(oldx, rowoff, 2, dxb, lane, dbytes);
            chain_sum<D>(acc, red, w, nw, lane);
            if (w == nw - 1) store_tile<D, NARROW>(acc, 1.f, buf, rowoff, 2, dxb, oldx, bp.acc_x != 0, rows_valid, lane, dbytes);
        } else {
            chain_sum<D>(acc, red, w, nw, lane);
            if (w == nw - 1) store_tile<D, NARROW>(acc, 1.f, buf, rowoff, 2, dxb, oldq, false, rows_valid, lane, dbytes);
        }
    }
    // previous dK (accumulate): only the wave that ends up with the group's sum needs it
    u32x4 oldk[G::kDTiles * 2] = {};
    const bool acc_k = MULTI ? bp.acc_k != 0 : bp.accumulate != 0;
    if (acc_k && w == nw - 1) prefetch_tile<D, NARROW>(oldk, rowoff, 1, dkb, lane, dbytes);

    // ---- dK^T = Q^T dS : summed over the group ----------------------------------------------
#pragma unroll
    for (int t = 0; t < G::kDTiles; ++t) {
        acc[t] = f32x16{};
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) acc[t] = mma(qT[t][s2], dsNop[s2], acc[t]);
    }
    chain_sum<D>(acc, red, w, nw, lane);
    if (w == nw - 1) store_tile<D, NARROW>(acc, p.scale, buf, rowoff, 1, dkb, oldk, acc_k, rows_valid, lane, dbytes, enc);
}

// ---------------------------------------------------------------------------------------
// Axes longer than one tile (32 < n <= kStreamMaxN): the same derivative, walked in 32 x 32
// blocks (query tile a, key tile c).  A wave is one query head of one fibre, the workgroup
// the heads of a key/value head, as above.  Nothing but the tensors themselves is kept
// between blocks: a block's operands are gathered again whenever it is visited (the fibre's
// rows stay in L2), and the row statistics of the fibre live in LDS.
//   for every query tile a:   sweep the key tiles once for the row statistics (running max,
//                             sum and sum of P o dP), once more for dQ_a = sum_c dS_ac K_c
//   for every key tile c:     sweep the query tiles for dX_c = sum_a P_ac^T G_a,
//                             and again for dK_c = sum_a dS_ac^T Q_a
// Blocks that the causal triangle or the band hides entirely are skipped.
constexpr int kStreamMaxN = 1024;
constexpr int kStreamMaxLds = 160 * 1024;              // LDS of one compute unit

struct StreamBwdParams {
    uint32_t q_row, k_row, v_row, o_row;   // token pitch in bytes of Q/dQ, K/dK, the value input and its gradient, dO
    uint32_t fibres_lo, fibres_hi;         // gridDim.y; gridDim.z = B * fibres_hi
    int32_t tiles;                         // ceil(n / 32)
};

// Keys 32 c .. 32 c + 31 that query row qr of the fibre may attend (bit = key), and query
// rows 32 a .. 32 a + 31 that may attend key kr (bit = query row).
__device__ inline uint32_t block_vis_keys(const HopParams& p, int64_t fibre, int qr, int c, int nreal) {
    if (qr >= nreal) return 0u;
    int lo, hi;
    visible_range(qr, 0, p.n, p.causal, p.window, lo, hi);
    hi = min(hi, nreal);
    uint32_t v = range_mask(min(max(lo - kTile * c, 0), kTile), min(max(hi - kTile * c, 0), kTile));
    if (p.mask) v &= p.mask[fibre * p.mask_fibre_words + qr * p.mask_words + c];
    return v;
}
__device__ inline uint32_t block_vis_rows(const HopParams& p, int64_t fibre, int kr, int a, int nreal) {
    if (kr >= nreal) return 0u;
    int lo, hi;
    seen_range(kr, 0, p.n, p.causal, p.window, lo, hi);
    hi = min(hi, nreal);
    uint32_t v = range_mask(min(max(lo - kTile * a, 0), kTile), min(max(hi - kTile * a, 0), kTile));
    if (p.mask) {
        const uint32_t* table = p.mask + fibre * p.mask_fibre_words;
        uint32_t col = 0;
#pragma unroll 1
        for (int q = 0; q < kTile; ++q) {                 // rare path: kept rolled, its 32 loads would otherwise claim registers in every kernel
            const int qr = kTile * a + q;
            if (qr < p.n) col |= ((table[qr * p.mask_words + (kr >> 5)] >> (kr & 31)) & 1u) << q;
        }
        v &= col;
    }
    return v;
}

// NARROW: the head is narrower than the D-wide tile; see load_chunk.
template <int D, bool NARROW>
__global__ __launch_bounds__(512, 2) void mfma_bwd_stream_kernel(BwdParams bp, StreamBwdParams sp) {
    using G = BGeo<D>;
    const HopParams& p = bp.hop;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw = bp.wg_heads;
    uint32_t bx, by;
    workgroup_xy<NARROW>(bx, by);
    const int g = (int)bx;
    const int h = g * p.G + bp.head_base + w;
    const uint32_t zb = blockIdx.z / sp.fibres_hi;
    const int64_t f = (int64_t)(blockIdx.z - zb * sp.fibres_hi) * sp.fibres_lo + by;
    if (f >= p.fibres) return;                            // whole workgroup leaves together
    const int b = (int)zb;
    const bool vin_is_o = (p.vin_heads == p.Hq);
    const int hv = vin_is_o ? h : g;
    const int n = p.n, T = sp.tiles;
    const uint32_t stride = (uint32_t)p.stride;
    const uint32_t tok0 = (uint32_t)fibre_base_token(f, p.stride, n);
    // rows of the fibre whose token is not padding form a prefix [0, nreal)
    const uint32_t vl = (uint32_t)hop_valid_len(p, b);
    const int nreal = tok0 >= vl ? 0 : (int)min((uint32_t)n, (vl - tok0 + stride - 1) / stride);

    const int wave_bytes = G::kBufBytes + kTile * 16 + 3 * kTile * T * 4;
    float* red = reinterpret_cast<float*>(smem);
    char* buf = smem + (nw > 1 ? G::kRedBytes : 0) + w * wave_bytes;
    u32x4* rowoff = reinterpret_cast<u32x4*>(buf + G::kBufBytes);
    float* stats = reinterpret_cast<float*>(buf + G::kBufBytes + kTile * 16);   // [tile][max | 1/sum | delta][32]

    const char* qb = reinterpret_cast<const char*>(p.q.p) + ((int64_t)b * p.q.sb + (int64_t)h * p.q.sh) * 2;
    const char* kb = reinterpret_cast<const char*>(p.k.p) + ((int64_t)b * p.k.sb + (int64_t)g * p.k.sh) * 2;
    const char* xb = reinterpret_cast<const char*>(p.vin.p) + ((int64_t)b * p.vin.sb + (int64_t)hv * p.vin.sh) * 2;
    const char* gb = reinterpret_cast<const char*>(bp.d_o.p) + ((int64_t)b * bp.d_o.sb + (int64_t)h * bp.d_o.sh) * 2;
    char* dqb = reinterpret_cast<char*>(bp.dq.p) + ((int64_t)b * bp.dq.sb + (int64_t)h * bp.dq.sh) * 2;
    char* dkb = reinterpret_cast<char*>(bp.dk.p) + ((int64_t)b * bp.dk.sb + (int64_t)g * bp.dk.sh) * 2;
    char* dxb = reinterpret_cast<char*>(bp.d_vin.p) + ((int64_t)b * bp.d_vin.sb + (int64_t)hv * bp.d_vin.sh) * 2;

    const int lrow = lane / G::kChunks, lcol = lane % G::kChunks;
    const uint32_t lbyte = lcol * 16;
    const uint32_t dbytes = (uint32_t)p.D * 2;            // bytes of a row (less than the tile's when NARROW)
    const int r32 = lane & 31, hf = lane >> 5;
    char* stg = buf + lrow * G::kPitch + lbyte;
    const char* oprd = buf + r32 * G::kPitch + hf * 16;
    const char* trbase = buf + (4 * hf + ((lane & 15) >> 2)) * G::kPitch + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
    const float sl2 = p.scale * kLog2e;

    // rows 32 t + .. of the fibre (clamped to the last one: padding rows of the last tile are
    // masked in the softmax and never stored)
    auto gather = [&](const char* base, uint32_t pitch, int t, u32x4 (&raw)[G::kPasses]) {
#pragma unroll
        for (int i = 0; i < G::kPasses; ++i) {
            const uint32_t rr = (uint32_t)min(kTile * t + i * G::kRowsPerPass + lrow, n - 1);
            raw[i] = gather_chunk<NARROW, false>(base, (tok0 + rr * stride) * pitch, lbyte, dbytes);
        }
    };
    // rotary encoding: every gathered Q or K tile is turned, row by row, by its position on the axis
    float rev[4];
    if (p.rope) rope_rates(p, lcol, rev);
    auto encode = [&](int t, u32x4 (&raw)[G::kPasses]) {
        if (p.rope) {
#pragma unroll
            for (int i = 0; i < G::kPasses; ++i) raw[i] = rope_chunk(raw[i], (float)min(kTile * t + i * G::kRowsPerPass + lrow, n - 1), rev);
        }
    };
    auto set_rowoff = [&](int t) {                        // byte offsets of the rows of tile t for the epilogue helpers
        lds_wave_sync();
        if (lane < kTile) {
            const uint32_t tok = tok0 + (uint32_t)min(kTile * t + lane, n - 1) * stride;
            rowoff[lane] = u32x4{tok * sp.q_row, tok * sp.k_row, tok * sp.v_row, tok * sp.o_row};
        }
        lds_wave_sync();
    };
    // key tiles that some row of query tile a sees, and query tiles with a row that sees some key of tile c
    auto key_tiles = [&](int a, int& cb, int& ce) {
        int lo, hi, lo2, hi2;
        visible_range(kTile * a, 0, n, p.causal, p.window, lo, hi);
        visible_range(min(kTile * a + kTile - 1, n - 1), 0, n, p.causal, p.window, lo2, hi2);
        cb = lo / kTile;
        ce = (hi2 + kTile - 1) / kTile;
    };
    auto row_tiles = [&](int c, int& ab, int& ae) {
        int lo, hi, lo2, hi2;
        seen_range(kTile * c, 0, n, p.causal, p.window, lo, hi);
        seen_range(min(kTile * c + kTile - 1, n - 1), 0, n, p.causal, p.window, lo2, hi2);
        ab = lo / kTile;
        ae = (hi2 + kTile - 1) / kTile;
    };

    // ===== query tiles: row statistics, then dQ =====================================================
    for (int a = 0; a < T; ++a) {
        u32x4 qop[G::kKSteps], gop[G::kKSteps];
        {
            u32x4 qraw[G::kPasses], graw[G::kPasses];
            gather(qb, sp.q_row, a, qraw);
            gather(gb, sp.o_row, a, graw);
            lds_wave_sync();
            encode(a, qraw);
            stage_rows<D>(stg, qraw);
            lds_wave_sync();
            read_natural<D>(oprd, qop);
            lds_wave_sync();
            stage_rows<D>(stg, graw);
            lds_wave_sync();
            read_natural<D>(oprd, gop);
            lds_wave_sync();
        }
        int cb, ce;
        key_tiles(a, cb, ce);
        const int qr = kTile * a + r32;                   // this lane's query row
        // ---- sweep 1: running max m (log2 domain), sum l and sum of e * dP ------------------------
        float m = -INFINITY, l = 0.f, dn = 0.f;
        for (int c = cb; c < ce; ++c) {
            u32x4 kraw[G::kPasses], xraw[G::kPasses], op[G::kKSteps];
            gather(kb, sp.k_row, c, kraw);
            gather(xb, sp.v_row, c, xraw);
            encode(c, kraw);
            stage_rows<D>(stg, kraw);
            lds_wave_sync();
            read_natural<D>(oprd, op);
            lds_wave_sync();
            f32x16 sT = {}, dpT = {};
#pragma unroll
            for (int s = 0; s < G::kKSteps; ++s) sT = mma(op[s], qop[s], sT);
            stage_rows<D>(stg, xraw);
            lds_wave_sync();
            read_natural<D>(oprd, op);
            lds_wave_sync();
#pragma unroll
            for (int s = 0; s < G::kKSteps; ++s) dpT = mma(op[s], gop[s], dpT);
            const uint32_t vis = block_vis_keys(p, f, qr, c, nreal) >> (4 * hf);
            float e[16], tmax = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const bool ok = (vis >> (8 * (r / 4) + (r % 4))) & 1u;
                e[r] = ok ? sT[r] * sl2 : -INFINITY;
                tmax = fmaxf(tmax, e[r]);
            }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            const float mnew = fmaxf(m, tmax);
            const float msafe = mnew == -INFINITY ? 0.f : mnew;
            const float corr = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - msafe);
            float ps = 0.f, pd = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float ev = __builtin_amdgcn_exp2f(e[r] - msafe);
                ps += ev;
                pd += ev * dpT[r];
            }
            ps += __shfl_xor(ps, 32);
            pd += __shfl_xor(pd, 32);
            l = l * corr + ps;
            dn = dn * corr + pd;
            m = mnew;
        }
        const float msafe = m == -INFINITY ? 0.f : m;
        const float inv = l > 0.f ? 1.f / l : 0.f;
        const float delta = dn * inv;
        if (lane < kTile) {
            stats[(3 * a + 0) * kTile + lane] = msafe;
            stats[(3 * a + 1) * kTile + lane] = inv;
            stats[(3 * a + 2) * kTile + lane] = delta;
        }
        // ---- sweep 2: dQ_a^T = sum_c K_c^T dS_ac^T ------------------------------------------------
        f32x16 acc[G::kDTiles];
#pragma unroll
        for (int t = 0; t < G::kDTiles; ++t) acc[t] = f32x16{};
        for (int c = cb; c < ce; ++c) {
            u32x4 kraw[G::kPasses], xraw[G::kPasses], op[G::kKSteps], kT[G::kDTiles][2];
            gather(xb, sp.v_row, c, xraw);
            stage_rows<D>(stg, xraw);
            gather(kb, sp.k_row, c, kraw);
            lds_wave_sync();
            read_natural<D>(oprd, op);
            lds_wave_sync();
            f32x16 sT = {}, dpT = {};
#pragma unroll
            for (int s = 0; s < G::kKSteps; ++s) dpT = mma(op[s], gop[s], dpT);
            encode(c, kraw);
            stage_rows<D>(stg, kraw);
            lds_wave_sync();
            read_natural<D>(oprd, op);
#pragma unroll
            for (int s = 0; s < G::kKSteps; ++s) sT = mma(op[s], qop[s], sT);
            read_transposed<D>(trbase, kT);                // K^T last: it lives only until the products below
            lds_wave_sync();
            const uint32_t vis = block_vis_keys(p, f, qr, c, nreal) >> (4 * hf);
            float e[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const bool ok = (vis >> (8 * (r / 4) + (r % 4))) & 1u;
                const float pv = ok ? __builtin_amdgcn_exp2f(sT[r] * sl2 - msafe) * inv : 0.f;
                e[r] = pv * (dpT[r] - delta);
            }
            u32x4 dsTop[2];
            pack_rows(e, dsTop);
#pragma unroll
            for (int t = 0; t < G::kDTiles; ++t)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) acc[t] = mma(kT[t][s2], dsTop[s2], acc[t]);
        }
        set_rowoff(a);
        u32x4 oldq[G::kDTiles * 2] = {};
        if (bp.accumulate) prefetch_tile<D, NARROW>(oldq, rowoff, 0, dqb, lane, dbytes);
        store_tile<D, NARROW>(acc, p.scale, buf, rowoff, 0, dqb, oldq, bp.accumulate != 0, min(kTile, n - kTile * a), lane, dbytes,
                              unrope(&p, [&](int r) { return (float)(kTile * a + r); }));
    }
    lds_wave_sync();

    // ===== key tiles: dX, then dK ===================================================================
    // P and dS of a block with one key per lane: lane = key row, registers = 16 of the 32 query rows
    for (int c = 0; c < T; ++c) {
        int ab, ae;
        row_tiles(c, ab, ae);
        const int kr = kTile * c + r32;                   // this lane's key row
        u32x4 kop[G::kKSteps];
        {
            u32x4 kraw[G::kPasses];
            gather(kb, sp.k_row, c, kraw);
            lds_wave_sync();
            encode(c, kraw);
            stage_rows<D>(stg, kraw);
            lds_wave_sync();
            read_natural<D>(oprd, kop);
            lds_wave_sync();
        }
        // ---- dX_c^T = sum_a G_a^T P_ac ---------------------------------------------------------------
        f32x16 acc[G::kDTiles];
#pragma unroll
        for (int t = 0; t < G::kDTiles; ++t) acc[t] = f32x16{};
        for (int a = ab; a < ae; ++a) {
            u32x4 qraw[G::kPasses], graw[G::kPasses], op[G::kKSteps], gT[G::kDTiles][2];
            gather(qb, sp.q_row, a, qraw);
            encode(a, qraw);
            stage_rows<D>(stg, qraw);
            gather(gb, sp.o_row, a, graw);
            lds_wave_sync();
            read_natural<D>(oprd, op);
            lds_wave_sync();
            f32x16 sN = {};
#pragma unroll
            for (int s = 0; s < G::kKSteps; ++s) sN = mma(op[s], kop[s], sN);
            stage_rows<D>(stg, graw);
            lds_wave_sync();
            read_transposed<D>(trbase, gT);
            lds_wave_sync();
            const uint32_t vis = block_vis_rows(p, f, kr, a, nreal) >> (4 * hf);
            float pr[16];
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 m4 = *reinterpret_cast<const f32x4*>(stats + (3 * a + 0) * kTile + 8 * q4 + 4 * hf);
                const f32x4 i4 = *reinterpret_cast<const f32x4*>(stats + (3 * a + 1) * kTile + 8 * q4 + 4 * hf);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int r = 4 * q4 + j;
                    const bool ok = (vis >> (8 * q4 + j)) & 1u;
                    pr[r] = ok ? __builtin_amdgcn_exp2f(sN[r] * sl2 - m4[j]) * i4[j] : 0.f;
                }
            }
            u32x4 pNop[2];
            pack_rows(pr, pNop);
#pragma unroll
            for (int t = 0; t < G::kDTiles; ++t)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) acc[t] = mma(gT[t][s2], pNop[s2], acc[t]);
        }
        set_rowoff(c);
        const int rows_c = min(kTile, n - kTile * c);
        u32x4 none[G::kDTiles * 2] = {};
        if (vin_is_o) {
            store_tile<D, NARROW>(acc, 1.f, buf, rowoff, 2, dxb, none, false, rows_c, lane, dbytes);
        } else {
            u32x4 oldx[G::kDTiles * 2] = {};
            if (bp.acc_x && w == nw - 1) prefetch_tile<D, NARROW>(oldx, rowoff, 2, dxb, lane, dbytes);
            chain_sum<D>(acc, red, w, nw, lane);
            if (w == nw - 1) store_tile<D, NARROW>(acc, 1.f, buf, rowoff, 2, dxb, oldx, bp.acc_x != 0, rows_c, lane, dbytes);
        }
        // ---- dK_c^T = sum_a Q_a^T dS_ac ---------------------------------------------------------------
        u32x4 xop[G::kKSteps];
        {
            u32x4 xraw[G::kPasses];
            gather(xb, sp.v_row, c, xraw);
            lds_wave_sync();
            stage_rows<D>(stg, xraw);
            lds_wave_sync();
            read_natural<D>(oprd, xop);
            lds_wave_sync();
        }
#pragma unroll
        for (int t = 0; t < G::kDTiles; ++t) acc[t] = f32x16{};
        for (int a = ab; a < ae; ++a) {
            u32x4 qraw[G::kPasses], graw[G::kPasses], op[G::kKSteps], qT[G::kDTiles][2];
            gather(gb, sp.o_row, a, graw);
            stage_rows<D>(stg, graw);
            gather(qb, sp.q_row, a, qraw);
            lds_wave_sync();
            read_natural<D>(oprd, op);
            lds_wave_sync();
            f32x16 sN = {}, dpN = {};
#pragma unroll
            for (int s = 0; s < G::kKSteps; ++s) dpN = mma(op[s], xop[s], dpN);
            encode(a, qraw);
            stage_rows<D>(stg, qraw);
            lds_wave_sync();
            read_natural<D>(oprd, op);
#pragma unroll
            for (int s = 0; s < G::kKSteps; ++s) sN = mma(op[s], kop[s], sN);
            read_transposed<D>(trbase, qT);
            lds_wave_sync();
            const uint32_t vis = block_vis_rows(p, f, kr, a, nreal) >> (4 * hf);
            float ds[16];
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 m4 = *reinterpret_cast<const f32x4*>(stats + (3 * a + 0) * kTile + 8 * q4 + 4 * hf);
                const f32x4 i4 = *reinterpret_cast<const f32x4*>(stats + (3 * a + 1) * kTile + 8 * q4 + 4 * hf);
                const f32x4 d4 = *reinterpret_cast<const f32x4*>(stats + (3 * a + 2) * kTile + 8 * q4 + 4 * hf);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int r = 4 * q4 + j;
                    const bool ok = (vis >> (8 * q4 + j)) & 1u;
                    const float pv = ok ? __builtin_amdgcn_exp2f(sN[r] * sl2 - m4[j]) * i4[j] : 0.f;
                    ds[r] = pv * (dpN[r] - d4[j]);
                }
            }
            u32x4 dsNop[2];
            pack_rows(ds, dsNop);
#pragma unroll
            for (int t = 0; t < G::kDTiles; ++t)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) acc[t] = mma(qT[t][s2], dsNop[s2], acc[t]);
        }
        lds_wave_sync();
        u32x4 oldk[G::kDTiles * 2] = {};
        if (bp.acc_k && w == nw - 1) prefetch_tile<D, NARROW>(oldk, rowoff, 1, dkb, lane, dbytes);   // only the wave that ends up with the sum
        chain_sum<D>(acc, red, w, nw, lane);
        if (w == nw - 1) store_tile<D, NARROW>(acc, p.scale, buf, rowoff, 1, dkb, oldk, bp.acc_k != 0, rows_c, lane, dbytes,
                                               unrope(&p, [&](int r) { return (float)(kTile * c + r); }));
        lds_wave_sync();
    }
}

// LDS of the two-tile kernel: shared K (and X) tiles, two reduction areas, statistics (room for three floats per row and
// tile; two are used: the softmax reference value and delta), one transit tile and one row table per wave.
template <int D>
constexpr size_t two_tile_lds(int gh, bool vs) {
    return (size_t)(vs ? 4 : 2) * kTile * Geo<D>::kPitch + (gh > 1 ? 2 * (size_t)BGeo<D>::kRedBytes : 0) + (size_t)gh * 2 * 3 * kTile * 4 +
           (size_t)2 * gh * BGeo<D>::kBufBytes + (size_t)2 * gh * kTile * 16;
}

// ---------------------------------------------------------------------------------------
// Axes of two tiles (32 < n <= 64), groups of 1, 2 or 4 query heads (a larger group that is a multiple of 4 goes 4
// heads per launch, the later launches adding to dK and to the group's dV): the same derivative with
// every tensor tile read from memory ONCE per fibre.  Two waves serve one query head of one
// fibre: wave (head, t) owns query tile t (the rows of dQ_t) and key tile t (the rows of dK_t
// and dX_t), and the two exchange their tiles through LDS.  The K tiles (and the X tiles when
// the value input is per key/value head, VS) are fetched once per workgroup into shared LDS
// tiles; every wave stages its own Q, X and G tile, one after the other, in its private
// transit tile, where its partner reads them as MFMA operands:
//   X staged   hold X_0, X_1 as operands
//   G staged   dP^T_tc = X_c G_t^T (rows of tile t, every visible key tile c),
//              dP_at = G_a X_t^T (keys of tile t, every query tile a that sees them)
//   Q staged   S^T_tc = K_c Q_t^T, S_at = Q_a K_t^T; row statistics of tile t -> LDS; dS^T_tc;
//              then, with the partner's statistics, P_at and dS_at; dK_t^T = sum_a Q_a^T dS_at
//   dQ_t^T = sum_c K_c^T dS^T_tc;  G staged again: dX_t^T = sum_a G_a^T P_at
// dK (and dX under VS) are summed over the heads in a fixed order, as in the one-tile kernel.
template <int D, int GH, bool VS>
__global__ __launch_bounds__(128 * GH, 2) void mfma_bwd2_kernel(BwdParams bp, StreamBwdParams sp) {
    using G = BGeo<D>;
    constexpr int kBuf = kTile * G::kPitch;
    constexpr int kWavesWg = 2 * GH;
    constexpr int kShare = 2 * G::kPasses / kWavesWg;     // load passes of the two shared tiles per wave
    static_assert((2 * G::kPasses) % kWavesWg == 0 && kShare >= 1, "the shared tiles split evenly over the waves");
    const HopParams& p = bp.hop;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int hl = w >> 1, t = w & 1;                     // head of the group; tile this wave owns
    const int g = blockIdx.x;
    const int h = g * p.G + bp.head_base + hl;            // a group of more than GH heads goes GH heads per launch
    const uint32_t zb = blockIdx.z / sp.fibres_hi;
    const int64_t f = (int64_t)(blockIdx.z - zb * sp.fibres_hi) * sp.fibres_lo + blockIdx.y;
    if (f >= p.fibres) return;                            // whole workgroup leaves together
    const int b = (int)zb;
    const int hv = VS ? g : h;
    const int n = p.n;
    const uint32_t stride = (uint32_t)p.stride;
    const uint32_t tok0 = (uint32_t)fibre_base_token(f, p.stride, n);
    const uint32_t vl = (uint32_t)hop_valid_len(p, b);
    const int nreal = tok0 >= vl ? 0 : (int)min((uint32_t)n, (vl - tok0 + stride - 1) / stride);

    // LDS: shared K tiles | shared X tiles (VS) | two reduction areas | statistics | private tiles | row tables
    char* sK = smem;
    char* sX = smem + 2 * kBuf;
    float* red = reinterpret_cast<float*>(smem + (VS ? 4 : 2) * kBuf) + (GH > 1 ? t * (G::kRedBytes / 4) : 0);
    float* stats = reinterpret_cast<float*>(smem + (VS ? 4 : 2) * kBuf + (GH > 1 ? 2 * G::kRedBytes : 0)) + hl * (2 * 3 * kTile);
    char* bufs = smem + (VS ? 4 : 2) * kBuf + (GH > 1 ? 2 * G::kRedBytes : 0) + GH * 2 * 3 * kTile * 4;
    char* buf = bufs + w * G::kBufBytes;                  // this wave's transit tile
    const char* pbuf = bufs + (w ^ 1) * G::kBufBytes;     // its partner's
    u32x4* rowoff = reinterpret_cast<u32x4*>(bufs + kWavesWg * G::kBufBytes) + w * kTile;

    const char* qb = reinterpret_cast<const char*>(p.q.p) + ((int64_t)b * p.q.sb + (int64_t)h * p.q.sh) * 2;
    const char* kb = reinterpret_cast<const char*>(p.k.p) + ((int64_t)b * p.k.sb + (int64_t)g * p.k.sh) * 2;
    const char* xb = reinterpret_cast<const char*>(p.vin.p) + ((int64_t)b * p.vin.sb + (int64_t)hv * p.vin.sh) * 2;
    const char* gb = reinterpret_cast<const char*>(bp.d_o.p) + ((int64_t)b * bp.d_o.sb + (int64_t)h * bp.d_o.sh) * 2;
    char* dqb = reinterpret_cast<char*>(bp.dq.p) + ((int64_t)b * bp.dq.sb + (int64_t)h * bp.dq.sh) * 2;
    char* dkb = reinterpret_cast<char*>(bp.dk.p) + ((int64_t)b * bp.dk.sb + (int64_t)g * bp.dk.sh) * 2;
    char* dxb = reinterpret_cast<char*>(bp.d_vin.p) + ((int64_t)b * bp.d_vin.sb + (int64_t)hv * bp.d_vin.sh) * 2;

    const int lrow = lane / G::kChunks, lcol = lane % G::kChunks;
    const uint32_t lbyte = lcol * 16;
    const int r32 = lane & 31, hf = lane >> 5;
    const float sl2 = p.scale * kLog2e;
    const int rows_t = min(kTile, n - kTile * t);         // rows of this wave's tile that exist

    // row table of this wave's tile for the epilogue helpers (rows past the fibre alias its last row)
    if (lane < kTile) {
        const uint32_t tok = tok0 + (uint32_t)min(kTile * t + lane, n - 1) * stride;
        rowoff[lane] = u32x4{tok * sp.q_row, tok * sp.k_row, tok * sp.v_row, tok * sp.o_row};
    }

    // ---- gather: own Q, G (and X) tile, this wave's share of the shared tiles: all requested at once ----
    // In the order of their first use (loads complete in order): the shared tiles and X, then G, then Q.
    u32x4 qraw[G::kPasses], graw[G::kPasses], xraw[VS ? 1 : G::kPasses], ksh[kShare], xsh[VS ? kShare : 1];
#pragma unroll
    for (int i = 0; i < kShare; ++i) {
        const int pidx = w * kShare + i;                  // pass pidx % kPasses of shared tile pidx / kPasses
        const uint32_t tok = tok0 + (uint32_t)min(kTile * (pidx / G::kPasses) + (pidx % G::kPasses) * G::kRowsPerPass + lrow, n - 1) * stride;
        ksh[i] = *reinterpret_cast<const u32x4*>(kb + (tok * sp.k_row + lbyte));
        if constexpr (VS) xsh[i] = *reinterpret_cast<const u32x4*>(xb + (tok * sp.v_row + lbyte));
    }
    uint32_t tokrow[G::kPasses];
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i) tokrow[i] = tok0 + (uint32_t)min(kTile * t + i * G::kRowsPerPass + lrow, n - 1) * stride;
    if constexpr (!VS) {
#pragma unroll
        for (int i = 0; i < G::kPasses; ++i) xraw[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xb + (tokrow[i] * sp.v_row + lbyte)));
    }
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i) graw[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gb + (tokrow[i] * sp.o_row + lbyte)));
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i) qraw[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(qb + (tokrow[i] * sp.q_row + lbyte)));
    __builtin_amdgcn_sched_barrier(0);

    // rotary encoding: Q and K rows are turned by their position on the axis before they enter LDS (K here, Q
    // where it is staged: its rows arrive last)
    float rev[4];
    if (p.rope) {
        rope_rates(p, lcol, rev);
#pragma unroll
        for (int i = 0; i < kShare; ++i) {
            const int pidx = w * kShare + i;
            ksh[i] = rope_chunk(ksh[i], (float)min(kTile * (pidx / G::kPasses) + (pidx % G::kPasses) * G::kRowsPerPass + lrow, n - 1), rev);
        }
    }

    const uint32_t stg = (uint32_t)(lrow * G::kPitch) + lbyte;                                   // row-major staging offset of this lane's chunk
    const uint32_t nat = (uint32_t)(r32 * G::kPitch + hf * 16);                                  // natural operand reads
    const uint32_t trn = (uint32_t)((4 * hf + ((lane & 15) >> 2)) * G::kPitch + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2);   // transposed operand reads

    // which blocks exist: key tiles some row of query tile t sees, query tiles with a row that sees a key of tile t
    bool visq[2], visk[2];
    {
        int lo, hi, lo2, hi2;
        visible_range(kTile * t, 0, n, p.causal, p.window, lo, hi);
        visible_range(min(kTile * t + kTile - 1, n - 1), 0, n, p.causal, p.window, lo2, hi2);
        visq[0] = lo < kTile && hi2 > 0;
        visq[1] = hi2 > kTile;
        seen_range(kTile * t, 0, n, p.causal, p.window, lo, hi);
        seen_range(min(kTile * t + kTile - 1, n - 1), 0, n, p.causal, p.window, lo2, hi2);
        visk[0] = lo < kTile && hi2 > 0;
        visk[1] = hi2 > kTile;
    }

    // ---- shared tiles into LDS; X staged ------------------------------------------------------------------
#pragma unroll
    for (int i = 0; i < kShare; ++i) {
        const int pidx = w * kShare + i;
        const uint32_t at = (uint32_t)((pidx / G::kPasses) * kBuf + ((pidx % G::kPasses) * G::kRowsPerPass) * G::kPitch) + stg;
        *reinterpret_cast<u32x4*>(sK + at) = ksh[i];
        if constexpr (VS) *reinterpret_cast<u32x4*>(sX + at) = xsh[i];
    }
    // X_0, X_1 as natural operands: held in registers when they pass through the transit tiles, read from the
    // shared tiles where needed otherwise
    u32x4 xn[VS ? 1 : 2][G::kKSteps];
    if constexpr (!VS) stage_rows<D>(buf + stg, xraw);
    __syncthreads();                                      // (1) shared tiles and every X tile are in place
    if constexpr (!VS) {
#pragma unroll
        for (int c = 0; c < 2; ++c) read_natural<D>((c == t ? buf : pbuf) + nat, xn[c]);
    }
    __syncthreads();                                      // (2) the X tiles have been read

    // ---- G staged: dP in both orientations --------------------------------------------------------------
    stage_rows<D>(buf + stg, graw);
    __syncthreads();                                      // (3)
    f32x16 dpT[2], dpN[2];                                // dpT[c]: rows of tile t x keys of tile c;  dpN[a]: keys of tile t x rows of tile a
    {
        u32x4 gn[G::kKSteps];
        read_natural<D>(buf + nat, gn);
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            dpT[c] = f32x16{};
            if (visq[c]) {
                if constexpr (VS) read_natural<D>(sX + c * kBuf + nat, xn[0]);
#pragma unroll
                for (int s = 0; s < G::kKSteps; ++s) dpT[c] = mma(xn[VS ? 0 : c][s], gn[s], dpT[c]);
            }
        }
        if constexpr (VS) read_natural<D>(sX + t * kBuf + nat, xn[0]);        // X of this wave's own tile
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            dpN[a] = f32x16{};
            if (visk[a]) {
                read_natural<D>((a == t ? buf : pbuf) + nat, gn);
#pragma unroll
                for (int s = 0; s < G::kKSteps; ++s) {
                    u32x4 xt;                             // t is the same in every lane: a select, not an indexed register
                    if constexpr (VS) xt = xn[0][s];
                    else xt = t ? xn[1][s] : xn[0][s];
                    dpN[a] = mma(gn[s], xt, dpN[a]);
                }
            }
        }
    }
    __syncthreads();                                      // (4) the G tiles have been read

    // ---- Q staged: scores in both orientations, statistics, dS ----------------------------------------
    if (p.rope) {
#pragma unroll
        for (int i = 0; i < G::kPasses; ++i) qraw[i] = rope_chunk(qraw[i], (float)min(kTile * t + i * G::kRowsPerPass + lrow, n - 1), rev);
    }
    stage_rows<D>(buf + stg, qraw);
    __syncthreads();                                      // (5)
    f32x16 sT[2];
    {
        u32x4 qn[G::kKSteps], kn[G::kKSteps];
        read_natural<D>(buf + nat, qn);
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            sT[c] = f32x16{};
            if (visq[c]) {
                read_natural<D>(sK + c * kBuf + nat, kn);
#pragma unroll
                for (int s = 0; s < G::kKSteps; ++s) sT[c] = mma(kn[s], qn[s], sT[c]);
            }
        }
    }
    // rows of tile t: masked softmax over both key tiles, delta, dS^T as B operands
    u32x4 dsT[2][2];
    {
        const int qr = kTile * t + r32;
        float e[2][16], mx = -INFINITY;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const uint32_t vis = visq[c] ? block_vis_keys(p, f, qr, c, nreal) >> (4 * hf) : 0u;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const bool ok = (vis >> (8 * (r / 4) + (r % 4))) & 1u;
                e[c][r] = ok ? sT[c][r] * sl2 : -INFINITY;
                mx = fmaxf(mx, e[c][r]);
            }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        if (mx == -INFINITY) mx = 0.f;
        float sum = 0.f;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) { e[c][r] = __builtin_amdgcn_exp2f(e[c][r] - mx); sum += e[c][r]; }
        sum += __shfl_xor(sum, 32);
        const float inv = sum > 0.f ? 1.f / sum : 0.f;
        float delta = 0.f;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) { e[c][r] *= inv; delta += e[c][r] * dpT[c][r]; }
        delta += __shfl_xor(delta, 32);
#pragma unroll
        for (int c = 0; c < 2; ++c) {
#pragma unroll
            for (int r = 0; r < 16; ++r) e[c][r] *= (dpT[c][r] - delta);
            pack_rows(e[c], dsT[c]);
        }
        if (lane < kTile) {                               // P = exp2(s - ref) with ref = max + log2(sum): one number instead of two
            float* st = stats + t * (3 * kTile);
            st[lane] = sum > 0.f ? mx + __builtin_amdgcn_logf(sum) : INFINITY; st[kTile + lane] = delta;
        }
    }
    __syncthreads();                                      // (6) both tiles' statistics are visible
    // keys of tile t: P and dS with one key per lane, as B operands
    u32x4 pN[2][2], dsN[2][2];
    {
        const int kr = kTile * t + r32;
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            // the scores with one key per lane: S_at = Q_a K_t^T, one query tile at a time (both at once would not fit)
            f32x16 sN = f32x16{};
            if (visk[a]) {
                u32x4 qn[G::kKSteps], kn[G::kKSteps];
                read_natural<D>(sK + t * kBuf + nat, kn);
                read_natural<D>((a == t ? buf : pbuf) + nat, qn);
#pragma unroll
                for (int s = 0; s < G::kKSteps; ++s) sN = mma(qn[s], kn[s], sN);
            }
            const uint32_t vis = visk[a] ? block_vis_rows(p, f, kr, a, nreal) >> (4 * hf) : 0u;
            const float* st = stats + a * (3 * kTile);
            uint32_t pw[8], dw[8];                        // rounded in pairs as they are formed: sixteen of each in fp32 do not fit
            float slv = sl2;
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 m4 = *reinterpret_cast<const f32x4*>(st + 8 * q4 + 4 * hf);
                const f32x4 d4 = *reinterpret_cast<const f32x4*>(st + kTile + 8 * q4 + 4 * hf);
#pragma unroll
                for (int j = 0; j < 4; j += 2) {
                    const int r = 4 * q4 + j;
                    const bool ok0 = (vis >> (8 * q4 + j)) & 1u, ok1 = (vis >> (8 * q4 + j + 1)) & 1u;
                    const float pv0 = ok0 ? __builtin_amdgcn_exp2f(sN[r] * slv - m4[j]) : 0.f;
                    const float pv1 = ok1 ? __builtin_amdgcn_exp2f(sN[r + 1] * slv - m4[j + 1]) : 0.f;
                    pw[r / 2] = pack_bf16x2(pv0, pv1);
                    dw[r / 2] = pack_bf16x2(pv0 * (dpN[a][r] - d4[j]), pv1 * (dpN[a][r + 1] - d4[j + 1]));
                }
                // The next four rows start from a value that passes through this statement together with the four words
                // just formed: the compiler cannot form all sixteen weights first (it did, and spilled them).
                asm volatile("" : "+v"(pw[2 * q4]), "+v"(pw[2 * q4 + 1]), "+v"(dw[2 * q4]), "+v"(dw[2 * q4 + 1]), "+v"(slv));
            }
            pN[a][0] = u32x4{pw[0], pw[1], pw[2], pw[3]};  pN[a][1] = u32x4{pw[4], pw[5], pw[6], pw[7]};
            dsN[a][0] = u32x4{dw[0], dw[1], dw[2], dw[3]}; dsN[a][1] = u32x4{dw[4], dw[5], dw[6], dw[7]};
        }
    }
    // the previous dQ rows are requested here: the product and the sum below give them time to arrive
    u32x4 oldq[G::kDTiles * 2] = {};
    if (bp.accumulate) prefetch_tile<D>(oldq, rowoff, 0, dqb, lane);
    // ---- dK_t^T = sum_a Q_a^T dS_at, while the Q tiles are still staged ----------------------------------
    f32x16 acc[G::kDTiles];
#pragma unroll
    for (int tt = 0; tt < G::kDTiles; ++tt) acc[tt] = f32x16{};
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        if (visk[a]) {
            u32x4 qT[G::kDTiles][2];
            read_transposed<D>((a == t ? buf : pbuf) + trn, qT);
#pragma unroll
            for (int tt = 0; tt < G::kDTiles; ++tt)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) acc[tt] = mma(qT[tt][s2], dsN[a][s2], acc[tt]);
        }
    }
    __syncthreads();                                      // (7) the Q tiles have been read: the transit tiles are free
    const auto enc = unrope(&p, [&](int r) { return (float)(kTile * t + r); });
    {
        u32x4 oldk[G::kDTiles * 2] = {};
        // the sum runs up the heads for tile 0 and down for tile 1, so that the two waves that end up with a
        // sum, and store it, are not the two waves of one head
        const int hc = t ? GH - 1 - hl : hl;
        const bool last = hc == GH - 1;                   // the wave that ends up with the group's sum
        if (bp.acc_k && last) prefetch_tile<D>(oldk, rowoff, 1, dkb, lane);
        if (GH > 1) chain_sum<D>(acc, red, hc, GH, lane);
        if (last) store_tile<D, false>(acc, p.scale, buf, rowoff, 1, dkb, oldk, bp.acc_k != 0, rows_t, lane, 0, enc);
    }
    // ---- dQ_t^T = sum_c K_c^T dS^T_tc ------------------------------------------------------------------------
    {
#pragma unroll
        for (int tt = 0; tt < G::kDTiles; ++tt) acc[tt] = f32x16{};
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            if (visq[c]) {
                u32x4 kT[G::kDTiles][2];
                read_transposed<D>(sK + c * kBuf + trn, kT);
#pragma unroll
                for (int tt = 0; tt < G::kDTiles; ++tt)
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) acc[tt] = mma(kT[tt][s2], dsT[c][s2], acc[tt]);
            }
        }
        store_tile<D, false>(acc, p.scale, buf, rowoff, 0, dqb, oldq, bp.accumulate != 0, rows_t, lane, 0, enc);
    }
    // ---- G staged again: dX_t^T = sum_a G_a^T P_at ---------------------------------------------------------
    lds_wave_sync();
    stage_rows<D>(buf + stg, graw);
    __syncthreads();                                      // (8)
#pragma unroll
    for (int tt = 0; tt < G::kDTiles; ++tt) acc[tt] = f32x16{};
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        if (visk[a]) {
            u32x4 gT[G::kDTiles][2];
            read_transposed<D>((a == t ? buf : pbuf) + trn, gT);
#pragma unroll
            for (int tt = 0; tt < G::kDTiles; ++tt)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) acc[tt] = mma(gT[tt][s2], pN[a][s2], acc[tt]);
        }
    }
    __syncthreads();                                      // (9) the G tiles have been read
    if (!VS) {
        store_tile_plain<D>(acc, 1.f, buf, rowoff, 2, dxb, rows_t, lane);
    } else {
        u32x4 oldx[G::kDTiles * 2] = {};                  // the sum of the group's earlier launches
        const int hc = t ? GH - 1 - hl : hl;
        if (bp.acc_x && hc == GH - 1) prefetch_tile<D>(oldx, rowoff, 2, dxb, lane);
        if (GH > 1) chain_sum<D>(acc, red, hc, GH, lane);
        if (hc == GH - 1) store_tile<D, false>(acc, 1.f, buf, rowoff, 2, dxb, oldx, bp.acc_x != 0, rows_t, lane);
    }
}

template <int D, int GH>
hipError_t launch_two_tile(const BwdParams& bp, hipStream_t s) {
    const HopParams& p = bp.hop;
    StreamBwdParams sp;
    sp.q_row = (uint32_t)(p.q.st * 2); sp.k_row = (uint32_t)(p.k.st * 2);
    sp.v_row = (uint32_t)(p.vin.st * 2); sp.o_row = (uint32_t)(bp.d_o.st * 2);
    sp.tiles = 2;
    sp.fibres_lo = (uint32_t)(p.fibres < 32768 ? p.fibres : 32768);
    sp.fibres_hi = (uint32_t)((p.fibres + sp.fibres_lo - 1) / sp.fibres_lo);
    if ((int64_t)p.B * sp.fibres_hi > 65535) return hipErrorInvalidValue;
    const bool vs = p.vin_heads != p.Hq;
    const size_t smem = two_tile_lds<D>(GH, vs);
    const void* kf = vs ? reinterpret_cast<const void*>(mfma_bwd2_kernel<D, GH, true>) : reinterpret_cast<const void*>(mfma_bwd2_kernel<D, GH, false>);
    if (smem > 64 * 1024) {
        const hipError_t e = allow_dynamic_lds(kf, (int)smem);
        if (e != hipSuccess) return e;
    }
    const dim3 grid((unsigned)p.Hkv, sp.fibres_lo, (unsigned)p.B * sp.fibres_hi);
    if (vs) hipLaunchKernelGGL((mfma_bwd2_kernel<D, GH, true>), grid, dim3(128 * GH), smem, s, bp, sp);
    else    hipLaunchKernelGGL((mfma_bwd2_kernel<D, GH, false>), grid, dim3(128 * GH), smem, s, bp, sp);
    return hipGetLastError();
}

template <int D, bool NARROW>
hipError_t launch_stream(const BwdParams& bp, hipStream_t s) {
    const HopParams& p = bp.hop;
    StreamBwdParams sp;
    sp.q_row = (uint32_t)(p.q.st * 2); sp.k_row = (uint32_t)(p.k.st * 2);
    sp.v_row = (uint32_t)(p.vin.st * 2); sp.o_row = (uint32_t)(bp.d_o.st * 2);
    sp.tiles = (p.n + kTile - 1) / kTile;
    sp.fibres_lo = (uint32_t)(p.fibres < 32768 ? p.fibres : 32768);
    sp.fibres_hi = (uint32_t)((p.fibres + sp.fibres_lo - 1) / sp.fibres_lo);
    if ((int64_t)p.B * sp.fibres_hi > 65535) return hipErrorInvalidValue;
    const size_t wave_bytes = (size_t)BGeo<D>::kBufBytes + kTile * 16 + (size_t)3 * kTile * sp.tiles * 4;
    const size_t smem = (size_t)(bp.wg_heads > 1 ? BGeo<D>::kRedBytes : 0) + (size_t)bp.wg_heads * wave_bytes;
    if (smem > kStreamMaxLds) return hipErrorInvalidValue;
    if (smem > 64 * 1024) {
        const hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(mfma_bwd_stream_kernel<D, NARROW>), kStreamMaxLds);
        if (e != hipSuccess) return e;
    }
    const dim3 grid((unsigned)p.Hkv, sp.fibres_lo, (unsigned)p.B * sp.fibres_hi);
    hipLaunchKernelGGL((mfma_bwd_stream_kernel<D, NARROW>), grid, dim3(64 * bp.wg_heads), smem, s, bp, sp);
    return hipGetLastError();
}

template <int D, bool NARROW>
hipError_t launch(const BwdParams& bp, const TileParams& tp, hipStream_t s) {
    const HopParams& p = bp.hop;
    const bool multi = p.G > bp.wg_heads, table = p.mask != nullptr;
    const size_t smem = (size_t)(bp.wg_heads > 1 ? BGeo<D>::kRedBytes : 0) + (size_t)bp.wg_heads * BGeo<D>::kWaveBytes;
    const dim3 grid((unsigned)p.Hkv, tp.tiles_lo, (unsigned)p.B * tp.tiles_hi);
    const dim3 block(64 * bp.wg_heads);
    const void* kf;
    if (p.rope) kf = multi ? (table ? (const void*)mfma_bwd_kernel<D, true, true, NARROW, true> : (const void*)mfma_bwd_kernel<D, false, true, NARROW, true>)
                           : (table ? (const void*)mfma_bwd_kernel<D, true, false, NARROW, true> : (const void*)mfma_bwd_kernel<D, false, false, NARROW, true>);
    else        kf = multi ? (table ? (const void*)mfma_bwd_kernel<D, true, true, NARROW, false> : (const void*)mfma_bwd_kernel<D, false, true, NARROW, false>)
                           : (table ? (const void*)mfma_bwd_kernel<D, true, false, NARROW, false> : (const void*)mfma_bwd_kernel<D, false, false, NARROW, false>);
    BwdParams bpc = bp;
    TileParams tpc = tp;
    void* args[2] = {&bpc, &tpc};
    if (smem > 64 * 1024) {
        const hipError_t e = allow_dynamic_lds(kf, (int)smem);
        if (e != hipSuccess) return e;
    }
    return hipLaunchKernel(kf, grid, block, args, smem, s);
}

}  // namespace

// 1: the one-tile kernel (n <= 32); 3: the two-tile kernel (32 < n <= 64, see there); 2: the blocked kernel (other axes up to kStreamMaxN); 0: none.
static int backward_variant(const BwdParams& bp, int dtype) {
    const HopParams& p = bp.hop;
    const bool full = p.D == 64 || p.D == 128;
    // other widths that are multiples of 4 ride in the next wider tile
    const bool narrow = !full && p.D % 4 == 0 && p.D >= 8 && p.D < 128;
    if (dtype != TA_BF16 || !(full || narrow) || p.n < 1 || p.n > kStreamMaxN) return 0;
    if (p.G < 1 || p.G > 256) return 0;                              // groups of more than 8 heads run 8 heads per launch
    const int64_t N = p.fibres * p.n;
    if (!(N < ((int64_t)1 << 31) && p.B <= 65535 && fits_u32(p.q, N) && fits_u32(p.k, N) && fits_u32(p.vin, N) &&
          fits_u32(bp.d_o, N) && fits_u32(bp.d_vin, N) && fits_u32(bp.dq, N) && fits_u32(bp.dk, N))) return 0;
    if (p.n <= kTile) {
        TileParams tp;
        HopParams hp = p;
        hp.o = bp.d_o;
        return make_tile_params(hp, 1, &tp) ? 1 : 0;
    }
    {   // the grid of the kernels below: (Hkv, fibres_lo, B * fibres_hi)
        const int64_t lo = p.fibres < 32768 ? p.fibres : 32768;
        if (p.fibres <= 0 || (int64_t)p.B * ((p.fibres + lo - 1) / lo) > 65535) return 0;
    }
    // two tiles, full-width heads, groups of 1, 2 or a multiple of 4 heads: every tile is read once per fibre and launch
    if (p.n <= 2 * kTile && full && (p.G == 1 || p.G == 2 || p.G % 4 == 0)) return 3;
    // the blocked kernel keeps three floats per row and head in LDS
    const size_t tiles = (size_t)(p.n + kTile - 1) / kTile;
    const size_t kbuf = p.D > 64 ? BGeo<128>::kBufBytes : BGeo<64>::kBufBytes;
    const size_t red = p.G > 1 ? (p.D > 64 ? BGeo<128>::kRedBytes : BGeo<64>::kRedBytes) : 0;
    const size_t wgh = p.G > 8 ? 8 : p.G;
    return red + wgh * (kbuf + kTile * 16 + 3 * kTile * tiles * 4) <= (size_t)kStreamMaxLds ? 2 : 0;
}

bool mfma_backward_supports(const BwdParams& bp, int dtype) { return backward_variant(bp, dtype) != 0; }
bool mfma_backward_is_blocked(const BwdParams& bp, int dtype) { return backward_variant(bp, dtype) == 2; }
bool mfma_backward_is_two_tile(const BwdParams& bp, int dtype) { return backward_variant(bp, dtype) == 3; }

hipError_t launch_mfma_backward(const BwdParams& user, hipStream_t s) {
    const int variant = backward_variant(user, TA_BF16);
    if (variant == 0) return hipErrorInvalidValue;
    HopParams hp = user.hop;
    hp.o = user.d_o;                                      // the table's fourth offset follows the O layout (dO)
    TileParams tp;
    if (variant == 1 && !make_tile_params(hp, 1, &tp)) return hipErrorInvalidValue;
    // A workgroup holds at most 8 heads.  A larger group goes 8 heads per launch, one launch after
    // the other on the stream: each later launch adds its heads' share to dK (and to the group's
    // dV), in a fixed order, so the result stays deterministic.
    BwdParams bp = user;
    const int G = user.hop.G;
    if (variant == 3) {                                   // groups of 1, 2 or 4 heads in one launch, larger ones 4 heads per launch
        const int gh = G >= 4 ? 4 : G;
        for (int base = 0; base < G; base += gh) {
            bp.wg_heads = gh; bp.head_base = base;
            bp.acc_k = base == 0 ? user.accumulate : 1;
            bp.acc_x = base == 0 ? 0 : 1;
            hipError_t e;
            if (bp.hop.D == 128) e = gh == 4 ? launch_two_tile<128, 4>(bp, s) : gh == 2 ? launch_two_tile<128, 2>(bp, s) : launch_two_tile<128, 1>(bp, s);
            else                 e = gh == 4 ? launch_two_tile<64, 4>(bp, s) : gh == 2 ? launch_two_tile<64, 2>(bp, s) : launch_two_tile<64, 1>(bp, s);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    for (int base = 0; base < G; base += 8) {
        bp.wg_heads = G - base > 8 ? 8 : G - base;
        bp.head_base = base;
        bp.acc_k = base == 0 ? user.accumulate : 1;
        bp.acc_x = base == 0 ? 0 : 1;
        hipError_t e;
        if (variant == 2) e = bp.hop.D == 128 ? launch_stream<128, false>(bp, s) : bp.hop.D == 64 ? launch_stream<64, false>(bp, s)
                            : bp.hop.D > 64 ? launch_stream<128, true>(bp, s) : launch_stream<64, true>(bp, s);
        else if (bp.hop.D == 128) e = launch<128, false>(bp, tp, s);
        else if (bp.hop.D == 64)  e = launch<64, false>(bp, tp, s);
        else                      e = bp.hop.D > 64 ? launch<128, true>(bp, tp, s) : launch<64, true>(bp, tp, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace ta
