// bf16 MFMA per-axis attention backward for gfx950 (CDNA4): the derivative of one hop of
// Eq. 4 of arXiv 2410.20926 (the paper states only that a backward exists, Sec. 3.2).
//
// For one 32-row tile (floor(32 / n) fibres packed, block-diagonal mask) of one query head,
// with A the hop's attention, X the value input and G the upstream gradient:
//     P  = softmax(Q K^T * scale, mask)          dP = G X^T
//     dS = P o (dP - rowsum(P o dP))
//     dX = P^T G      dQ = dS K * scale      dK = dS^T Q * scale
// One wavefront handles one (tile, query head); a workgroup is the G <= 8 query heads that
// share a key/value head, so dK (and dX when the value input is V) are summed across the
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
template <int D>
__device__ inline void prefetch_tile(u32x4 (&old)[Geo<D>::kDTiles * 2], const u32x4* rowoff, int which, const char* gbase, int lane) {
#pragma unroll
    for (int half = 0; half < Geo<D>::kDTiles / 2; ++half)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            old[half * 4 + i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gbase + tile_out_offset<D>(rowoff, which, half, i, lane)));
}

// acc[t][r] holds (row = lane % 32, feature 32 t + 8 (r/4) + 4 hf + r % 4).  Multiplies by
// `mult`, optionally adds the tensor's previous contents (`old`, from prefetch_tile), rounds
// to bf16 and stores the rows with 16-byte stores; the transposition goes through LDS in
// fp32, 64 features at a time.
template <int D>
__device__ inline void store_tile(const f32x16 (&acc)[Geo<D>::kDTiles], float mult, char* buf, const u32x4* rowoff,
                                  int which, char* gbase, const u32x4 (&old)[Geo<D>::kDTiles * 2], bool add_old, int rows_valid, int lane) {
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
                if (add_old) {
                    const u32x4 o = old[half * 4 + i];
#pragma unroll
                    for (int e = 0; e < 4; ++e) { y[2 * e] += bf16_lo(o[e]); y[2 * e + 1] += bf16_hi(o[e]); }
                }
                __builtin_nontemporal_store(
                    u32x4{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3]), pack_bf16x2(y[4], y[5]), pack_bf16x2(y[6], y[7])},
                    reinterpret_cast<u32x4*>(gbase + tile_out_offset<D>(rowoff, which, half, i, lane)));
            }
        }
        lds_wave_sync();
    }
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
// TABLE: the axis has a caller's bit table (a separate instantiation keeps the common case free of it).
template <int D, bool TABLE>
__global__ __launch_bounds__(512, 2) void mfma_bwd_kernel(BwdParams bp, TileParams tp) {
    using G = BGeo<D>;
    const HopParams& p = bp.hop;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw = p.G;

    const int g = blockIdx.x;
    const int h = g * p.G + w;
    const uint32_t zb = blockIdx.z / tp.tiles_hi;
    const uint32_t tt = (blockIdx.z - zb * tp.tiles_hi) * tp.tiles_lo + blockIdx.y;
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
            real = lane < rows_valid && tok < (uint32_t)p.valid_len;
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
    const int r32 = lane & 31, hf = lane >> 5;

    // ---- gather Q, K, X, G rows: every load is issued before the first wait ------------
    u32x4 qraw[G::kPasses], kraw[G::kPasses], xraw[G::kPasses], graw[G::kPasses];
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i) {
        const u32x4 off = rowoff[i * G::kRowsPerPass + lrow];
        // Rows read by this wave alone are streamed; rows every wave of the group reads stay cached.
        qraw[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(qb + (off.x + lbyte)));
        kraw[i] = *reinterpret_cast<const u32x4*>(kb + (off.y + lbyte));
        xraw[i] = vin_is_o ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xb + (off.z + lbyte)))
                           : *reinterpret_cast<const u32x4*>(xb + (off.z + lbyte));
        graw[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(gb + (off.w + lbyte)));
    }
    __builtin_amdgcn_sched_barrier(0);

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
    if (bp.accumulate) prefetch_tile<D>(oldq, rowoff, 0, dqb, lane);

    // ---- softmax and dS, one query row per lane -------------------------------------------
    const float sl2 = p.scale * kLog2e;
    const bool row_real = (real_rows >> r32) & 1u;        // this lane's tile row exists and is not padding
    const int flo = (int)((min(r32, rows_valid - 1) + 0.5f) * tp.inv_n) * n;   // its fibre occupies tile rows [flo, fhi)
    const int fhi = flo + n;
    u32x4 dsTop[2];                                       // dS^T as B operands (contraction over keys)
    {
        int lo = 0, hi = 0;
        uint32_t tw = 0xffffffffu;
        if (row_real) { visible_range(r32, flo, fhi, p.causal, p.window, lo, hi); if (TABLE) tw = table_word(p, r32 - flo, 0) << flo; }
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
        if (lane < kTile) { stats[lane] = mx; stats[kTile + lane] = inv; stats[2 * kTile + lane] = delta; }
    }
    lds_wave_sync();

    // ---- the same, one key per lane: P and dS as B operands (contraction over query rows) --
    u32x4 pNop[2], dsNop[2];
    {
        // query rows that see this lane's key: its own fibre's rows, from itself on when causal
        int lo = 0, hi = 0;
        uint32_t tw = 0xffffffffu;
        if (row_real) { seen_range(r32, flo, fhi, p.causal, p.window, lo, hi); if (TABLE) tw = table_column(p, r32 - flo) << flo; }
        const uint32_t vis = (range_mask(lo, hi) & tw & real_rows) >> (4 * hf);
        float pr[16], ds[16];
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const f32x4 m4 = *reinterpret_cast<const f32x4*>(stats + 8 * q4 + 4 * hf);
            const f32x4 i4 = *reinterpret_cast<const f32x4*>(stats + kTile + 8 * q4 + 4 * hf);
            const f32x4 d4 = *reinterpret_cast<const f32x4*>(stats + 2 * kTile + 8 * q4 + 4 * hf);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int r = 4 * q4 + j;
                const bool ok = (vis >> (8 * q4 + j)) & 1u;
                const float pv = ok ? __builtin_amdgcn_exp2f(sN[r] * sl2 - m4[j]) * i4[j] : 0.f;
                pr[r] = pv;
                ds[r] = pv * (dpN[r] - d4[j]);
            }
        }
        pack_rows(pr, pNop);
        pack_rows(ds, dsNop);
    }

    // ---- dQ^T = K^T dS^T : per head, stored at once -----------------------------------------
    f32x16 acc[G::kDTiles];
#pragma unroll
    for (int t = 0; t < G::kDTiles; ++t) {
        acc[t] = f32x16{};
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) acc[t] = mma(kT[t][s2], dsTop[s2], acc[t]);
    }
    store_tile<D>(acc, p.scale, buf, rowoff, 0, dqb, oldq, bp.accumulate != 0, rows_valid, lane);

    // ---- dX^T = G^T P : per head, or summed over the group when the value input is V ------
#pragma unroll
    for (int t = 0; t < G::kDTiles; ++t) {
        acc[t] = f32x16{};
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) acc[t] = mma(gT[t][s2], pNop[s2], acc[t]);
    }
    if (vin_is_o) {
        store_tile<D>(acc, 1.f, buf, rowoff, 2, dxb, oldq, false, rows_valid, lane);
    } else {
        chain_sum<D>(acc, red, w, nw, lane);
        if (w == nw - 1) store_tile<D>(acc, 1.f, buf, rowoff, 2, dxb, oldq, false, rows_valid, lane);
    }
    // previous dK (accumulate): only the wave that ends up with the group's sum needs it
    u32x4 oldk[G::kDTiles * 2] = {};
    if (bp.accumulate && w == nw - 1) prefetch_tile<D>(oldk, rowoff, 1, dkb, lane);

    // ---- dK^T = Q^T dS : summed over the group ----------------------------------------------
#pragma unroll
    for (int t = 0; t < G::kDTiles; ++t) {
        acc[t] = f32x16{};
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) acc[t] = mma(qT[t][s2], dsNop[s2], acc[t]);
    }
    chain_sum<D>(acc, red, w, nw, lane);
    if (w == nw - 1) store_tile<D>(acc, p.scale, buf, rowoff, 1, dkb, oldk, bp.accumulate != 0, rows_valid, lane);
}

template <int D>
hipError_t launch(const BwdParams& bp, const TileParams& tp, hipStream_t s) {
    const HopParams& p = bp.hop;
    const size_t smem = (size_t)(p.G > 1 ? BGeo<D>::kRedBytes : 0) + (size_t)p.G * BGeo<D>::kWaveBytes;
    const dim3 grid((unsigned)p.Hkv, tp.tiles_lo, (unsigned)p.B * tp.tiles_hi);
    if (p.mask) hipLaunchKernelGGL((mfma_bwd_kernel<D, true>), grid, dim3(64 * p.G), smem, s, bp, tp);
    else        hipLaunchKernelGGL((mfma_bwd_kernel<D, false>), grid, dim3(64 * p.G), smem, s, bp, tp);
    return hipGetLastError();
}

}  // namespace

bool mfma_backward_supports(const BwdParams& bp, int dtype) {
    const HopParams& p = bp.hop;
    if (dtype != TA_BF16 || (p.D != 64 && p.D != 128) || p.n < 1 || p.n > kTile) return false;
    if (p.G != 1 && p.G != 2 && p.G != 4 && p.G != 8) return false;
    const int64_t N = p.fibres * p.n;
    return N < ((int64_t)1 << 31) && p.B <= 65535 && fits_u32(p.q, N) && fits_u32(p.k, N) && fits_u32(p.vin, N) &&
           fits_u32(bp.d_o, N) && fits_u32(bp.d_vin, N) && fits_u32(bp.dq, N) && fits_u32(bp.dk, N);
}

hipError_t launch_mfma_backward(const BwdParams& bp, hipStream_t s) {
    if (!mfma_backward_supports(bp, TA_BF16)) return hipErrorInvalidValue;
    HopParams hp = bp.hop;
    hp.o = bp.d_o;                                        // the table's fourth offset follows the O layout (dO)
    TileParams tp;
    if (!make_tile_params(hp, 1, &tp)) return hipErrorInvalidValue;
    return bp.hop.D == 128 ? launch<128>(bp, tp, s) : launch<64>(bp, tp, s);
}

}  // namespace ta
