// bf16 MFMA per-axis attention forward for gfx950 (CDNA4), one hop of Eq. 4 of
// arXiv 2410.20926.
//
// Work unit: 32 query rows of one query head, handled by ONE wavefront with no workgroup
// barrier.  For an axis of length n <= 32 the 32 rows are floor(32 / n) mode-i fibres
// packed one after the other (rows past the last fibre are padding) and the mask is block
// diagonal (lower triangular inside a block for the causal variant).  For 32 < n <= 64 a
// fibre has two query tiles (two units) and each unit walks up to two 32-key tiles.
//
// Per wave:
//   1. gather: rows of Q, K and the value input come from HBM with 16-byte loads, 16
//      lanes per 256-byte row (D = 128), i.e. fully coalesced whatever the axis stride is;
//      every load of the unit is issued before the first use;
//   2. Q and K pass through an LDS transit buffer (padded rows) and come back in MFMA
//      operand layout;
//   3. S^T = K Q^T with v_mfma_f32_32x32x16_bf16: the accumulator then holds, per lane,
//      16 of the 32 keys of ONE query row (the other 16 are in lane^32), so the row
//      softmax needs in-lane reductions and a single cross-lane exchange;
//   4. the un-normalised probabilities, rounded to bf16, are already in B-operand
//      layout for O^T = V^T P^T (keys c and c + 8 share a 32-bit word); V goes through
//      LDS with rows c and c + 8 interleaved the same way, so that a 32-bit LDS read
//      yields the two keys of one feature column, which is the A-operand layout of V^T;
//   5. O^T is scaled by 1/rowsum in fp32, rounded to bf16, transposed through LDS and
//      stored with 16-byte coalesced stores (fold).
#include <type_traits>

#include "ta_mfma_common.h"

namespace ta {
namespace {

using namespace mfma;

constexpr int kWavesPerBlock = 4;

// KT = number of 32-key tiles a unit may walk (1: n <= 32, 2: n <= 64).
// NARROW: the head is narrower than the D-wide tile (p.D features of 2 bytes per row); see load_chunk.
// ROPE: the hop scores with rotary-encoded Q and K (instantiated separately: the plain kernels carry none of it).
template <int D, int KT, bool NARROW, bool ROPE>
__global__ __launch_bounds__(kWavesPerBlock * 64, 2) void mfma_fwd_kernel(HopParams p, TileParams tp) {
    using G = Geo<D>;
    constexpr int kRows = kTile * KT;                     // rows of the unit's fibre set that have a table entry
    constexpr int kWaveBytes = G::kBufBytes + kRows * 16;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // block -> (head block, tile, batch); heads fastest so that co-resident waves read
    // the same tokens (whole DRAM rows) and the four waves of a block share K
    uint32_t bx, by;
    workgroup_xy<NARROW>(bx, by);
    const int h = (int)bx * kWavesPerBlock + w;
    const uint32_t zb = blockIdx.z / tp.tiles_hi;
    const uint32_t tt = (blockIdx.z - zb * tp.tiles_hi) * tp.tiles_lo + by;
    if (h >= p.Hq || tt >= tp.tiles) return;              // no workgroup barrier below
    const int b = (int)zb;
    const int g = h / p.G;
    const int hv = (p.vin_heads == p.Hq) ? h : g;
    const int n = p.n;

    char* buf = smem + w * kWaveBytes;
    u32x4* rowoff = reinterpret_cast<u32x4*>(buf + G::kBufBytes);   // per row: byte offsets in (q, k, v_in, o)

    // fibre(s) and query tile of this unit
    uint32_t f0;
    int qt, rows_valid;                                   // rows_valid: rows of the table that exist
    if (KT == 1) {
        f0 = tt * tp.fpt;
        qt = 0;
        rows_valid = (int)min((uint32_t)tp.fpt, (uint32_t)p.fibres - f0) * n;
    } else {
        f0 = tt / tp.qtiles;
        qt = (int)(tt - f0 * tp.qtiles);
        rows_valid = n;
    }
    // byte offset of every row of the fibre set, clamped to the last valid row, so that
    // loads need no predicate (padding rows are masked in the softmax and never stored)
    uint64_t real_rows;                                   // bit r: table row r exists and its token is not padding
    {
        const uint32_t stride = (uint32_t)p.stride;
        const uint32_t vl = (uint32_t)hop_valid_len(p, b);
        bool real = false;
        if (lane < kRows) {
            const int rc = min(lane, rows_valid - 1);
            const uint32_t fi = (KT == 1) ? (uint32_t)((rc + 0.5f) * tp.inv_n) : 0u;
            const uint32_t a = rc - fi * n;
            const uint32_t f = f0 + fi;
            const uint32_t outer = f / stride;
            const uint32_t tok = outer * stride * n + (f - outer * stride) + a * stride;
            rowoff[lane] = u32x4{tok * tp.q_row, tok * tp.k_row, tok * tp.v_row, tok * tp.o_row};
            real = lane < rows_valid && tok < vl;
        }
        real_rows = __ballot(real);
    }
    lds_wave_sync();

    const char* qb = reinterpret_cast<const char*>(p.q.p) + ((int64_t)b * p.q.sb + (int64_t)h * p.q.sh) * 2;
    const char* kb = reinterpret_cast<const char*>(p.k.p) + ((int64_t)b * p.k.sb + (int64_t)g * p.k.sh) * 2;
    const char* vb = reinterpret_cast<const char*>(p.vin.p) + ((int64_t)b * p.vin.sb + (int64_t)hv * p.vin.sh) * 2;
    char* ob = reinterpret_cast<char*>(p.o.p) + ((int64_t)b * p.o.sb + (int64_t)h * p.o.sh) * 2;

    const int lrow = lane / G::kChunks;                   // row within a pass
    const int lcol = lane % G::kChunks;                   // 16-byte chunk within the row
    const uint32_t lbyte = lcol * 16;
    const uint32_t dbytes = (uint32_t)p.D * 2;           // bytes of a row (less than the tile's when NARROW)
    const int kt_end = (KT == 1) ? 1 : (p.causal ? qt + 1 : (n > kTile ? 2 : 1));   // key tiles this unit walks

    if (((real_rows >> (qt * kTile)) & 0xffffffffull) == 0) {
        // every query row of this unit is padding: zero rows out, nothing read
#pragma unroll
        for (int i = 0; i < G::kPasses; ++i) {
            const int row = qt * kTile + i * G::kRowsPerPass + lrow;
            if (row < rows_valid) store_chunk<NARROW>(ob, rowoff[row].w, lbyte, dbytes, u32x4{0u, 0u, 0u, 0u});
        }
        return;
    }

    // ---- 1. gather ---------------------------------------------------------------------
    // Lane (lrow, lcol) loads chunk lcol of rows i * kRowsPerPass + lrow of every tile.
    // Q, every K tile and the first V tile are requested here, before the first wait; a
    // second V tile is requested as soon as the first K tile has left its registers.
    // Rows that no other wave reads (Q always; K and V rows of a one-tile fibre whose head
    // is not shared by a group) are streamed past the caches, and so is O.
    const bool k_once = (KT == 1) && p.G == 1;
    const bool v_once = (KT == 1) && (p.G == 1 || p.vin_heads == p.Hq);
    u32x4 qreg[G::kPasses], kreg[KT][G::kPasses], vreg[KT][G::kPasses];
    uint32_t ooff[G::kPasses], voff[KT][G::kPasses];
    // (the choice between last-use and cached requests is made once, outside the loops: a choice per request is a branch
    // per request, and with narrow rows, whose chunks are put together from two lanes, every request then waits for the one before)
    auto gather_kv = [&](auto k_nt, auto v_nt) {
#pragma unroll
        for (int j = 0; j < KT; ++j) {
            if (j < kt_end) {
#pragma unroll
                for (int i = 0; i < G::kPasses; ++i) {
                    const u32x4 off = rowoff[j * kTile + i * G::kRowsPerPass + lrow];
                    kreg[j][i] = gather_chunk<NARROW, decltype(k_nt)::value>(kb, off.y, lbyte, dbytes);
                    voff[j][i] = off.z;
                    if (j == 0) vreg[j][i] = gather_chunk<NARROW, decltype(v_nt)::value>(vb, voff[j][i], lbyte, dbytes);
                    if (KT == 1) {
                        qreg[i] = gather_chunk<NARROW, true>(qb, off.x, lbyte, dbytes);
                        ooff[i] = off.w;
                    }
                }
            }
        }
    };
    if (k_once && v_once) gather_kv(std::true_type{}, std::true_type{});
    else if (v_once) gather_kv(std::false_type{}, std::true_type{});
    else gather_kv(std::false_type{}, std::false_type{});      // (k_once implies v_once)
    if (KT > 1) {
#pragma unroll
        for (int i = 0; i < G::kPasses; ++i) {
            const u32x4 off = rowoff[qt * kTile + i * G::kRowsPerPass + lrow];
            qreg[i] = gather_chunk<NARROW, true>(qb, off.x, lbyte, dbytes);
            ooff[i] = off.w;
        }
    }
    __builtin_amdgcn_sched_barrier(0);                    // keep these loads ahead of the first wait

    // ---- rotary encoding of the gathered Q and K rows, by their position on the axis -----
    float rev[4];
    auto row_pos = [&](int row) -> float {                // position on the axis of row `row` of the fibre set
        if (KT == 1) { const int rc = min(row, rows_valid - 1); return (float)(rc - (int)((rc + 0.5f) * tp.inv_n) * n); }
        return (float)min(row, n - 1);
    };
    if constexpr (ROPE) {
        rope_rates(p, lcol, rev);
#pragma unroll
        for (int i = 0; i < G::kPasses; ++i) {
            float c[4], sn[4];
            rope_sincos(row_pos(qt * kTile + i * G::kRowsPerPass + lrow), rev, c, sn);
            qreg[i] = rope_apply(qreg[i], c, sn);
            if (KT == 1) kreg[0][i] = rope_apply(kreg[0][i], c, sn);     // one tile: K's rows are Q's rows
        }
    }

    const int r32 = lane & 31;                            // tile row this lane owns in operands
    const int hf = lane >> 5;                             // which 8-wide half of a 16-wide MFMA step
    const char* oprd = buf + r32 * G::kPitch + hf * 16;   // operand read base
    char* stg = buf + lrow * G::kPitch + lbyte;           // row-major staging base

    // ---- 2. Q through LDS into B-operand layout -------------------------------------
    u32x4 qop[G::kKSteps];
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i)
        *reinterpret_cast<u32x4*>(stg + i * G::kRowsPerPass * G::kPitch) = qreg[i];
    lds_wave_sync();
#pragma unroll
    for (int s = 0; s < G::kKSteps; ++s) qop[s] = *reinterpret_cast<const u32x4*>(oprd + s * 32);
    lds_wave_sync();

    // ---- 3. per key tile: K through LDS, S^T = K Q^T ----------------------------------
    // st[j][r] = S[a = r32][c = 32 j + 8*(r/4) + 4*hf + r%4]
    f32x16 st[KT];
#pragma unroll
    for (int j = 0; j < KT; ++j) {
        st[j] = f32x16{};
        if (j < kt_end) {
            u32x4 kop[G::kKSteps];
            if constexpr (KT > 1 && ROPE) {
#pragma unroll
                for (int i = 0; i < G::kPasses; ++i) kreg[j][i] = rope_chunk(kreg[j][i], row_pos(j * kTile + i * G::kRowsPerPass + lrow), rev);
            }
#pragma unroll
            for (int i = 0; i < G::kPasses; ++i)
                *reinterpret_cast<u32x4*>(stg + i * G::kRowsPerPass * G::kPitch) = kreg[j][i];
            lds_wave_sync();
#pragma unroll
            for (int s = 0; s < G::kKSteps; ++s) kop[s] = *reinterpret_cast<const u32x4*>(oprd + s * 32);
            lds_wave_sync();
            if (KT > 1 && j == 0 && kt_end > 1) {         // K tile 0 is out of its registers: request V tile 1
#pragma unroll
                for (int i = 0; i < G::kPasses; ++i) vreg[1][i] = gather_chunk<NARROW, false>(vb, voff[1][i], lbyte, dbytes);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int s = 0; s < G::kKSteps; ++s)
                st[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kop[s]),
                                                                __builtin_bit_cast(bf16x8, qop[s]), st[j], 0, 0, 0);
        }
    }

    // ---- 4. masked row softmax over all key tiles ---------------------------------------
    // keys visible to this lane's query row: its own fibre's rows, up to itself when causal
    const int qrow = qt * kTile + r32;                    // row index in the fibre set
    uint32_t vis[KT];
    {
        int lo = 0, hi = 0;                               // visible keys = [lo, hi)
        uint32_t tw[KT];                                  // the axis table's words for this row, in tile-row coordinates
#pragma unroll
        for (int j = 0; j < KT; ++j) tw[j] = 0xffffffffu;
        if ((real_rows >> qrow) & 1) {
            const int fi = (KT == 1) ? (int)((qrow + 0.5f) * tp.inv_n) : 0;      // the row's fibre within the unit
            const int flo = fi * n;
            visible_range(qrow, flo, flo + n, p.causal, p.window, lo, hi);
#pragma unroll
            for (int j = 0; j < KT; ++j) tw[j] = (KT == 1) ? table_word(p, f0 + fi, qrow - flo, 0) << flo : table_word(p, f0, qrow, j);
        }
#pragma unroll
        for (int j = 0; j < KT; ++j)
            vis[j] = (range_mask(min(max(lo - 32 * j, 0), 32), min(max(hi - 32 * j, 0), 32)) & tw[j] & (uint32_t)(real_rows >> (32 * j))) >> (4 * hf);
    }
    const float sl2 = p.scale * kLog2e;
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < KT; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const bool ok = (vis[j] >> (8 * (r / 4) + (r % 4))) & 1u;
            st[j][r] = ok ? st[j][r] * sl2 : -INFINITY;
            mx = fmaxf(mx, st[j][r]);
        }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    if (mx == -INFINITY) mx = 0.f;                        // padding rows: everything masked
    uint32_t pop[KT][2][4];                               // P^T as B operands, 16 keys each
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < KT; ++j)
#pragma unroll
        for (int ri = 0; ri < 8; ++ri) {
            const int r = (ri / 4) * 8 + ri % 4;          // r pairs with r + 4: keys c and c + 8
            const float e0 = __builtin_amdgcn_exp2f(st[j][r] - mx);
            const float e1 = __builtin_amdgcn_exp2f(st[j][r + 4] - mx);
            const uint32_t pk = pack_bf16x2(e0, e1);
            sum += __uint_as_float(pk << 16) + __uint_as_float(pk & 0xffff0000u);   // sum of the ROUNDED weights
            pop[j][r / 8][r % 4] = pk;
        }
    sum += __shfl_xor(sum, 32);
    const float inv = sum > 0.f ? 1.f / sum : 0.f;

    // ---- per key tile: V through LDS (row pairs interleaved), O^T += V^T P^T -------------
    f32x16 ot[G::kDTiles];
#pragma unroll
    for (int t = 0; t < G::kDTiles; ++t) ot[t] = f32x16{};
#pragma unroll
    for (int j = 0; j < KT; ++j) {
        if (j < kt_end) {
            // rows rho and rho + 8 (rho mod 16 < 8) share a 32-bit word per column: slot
            // (rho / 16) * 8 + rho % 16 of the buffer
#pragma unroll
            for (int pi = 0; pi < G::kPasses / 2; ++pi) {
                constexpr int kStep = 8 / G::kRowsPerPass;                  // passes between rho and rho + 8
                const int i = (pi / kStep) * 2 * kStep + pi % kStep;        // passes whose rows have rho mod 16 < 8
                const int rho = i * G::kRowsPerPass;                        // + lrow
                const int slot = (rho / 16) * 8 + rho % 16;                 // + lrow
                const u32x4 x = vreg[j][i], y = vreg[j][i + kStep];
                const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
                uint32_t o[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    o[2 * e] = __builtin_amdgcn_perm(ys[e], xs[e], 0x05040100u);      // (x.lo, y.lo)
                    o[2 * e + 1] = __builtin_amdgcn_perm(ys[e], xs[e], 0x07060302u);  // (x.hi, y.hi)
                }
                char* dst = buf + (slot + lrow) * G::kVPitch + lcol * 32;
                *reinterpret_cast<u32x4*>(dst) = u32x4{o[0], o[1], o[2], o[3]};
                *reinterpret_cast<u32x4*>(dst + 16) = u32x4{o[4], o[5], o[6], o[7]};
            }
            lds_wave_sync();
#pragma unroll
            for (int t = 0; t < G::kDTiles; ++t) {
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    uint32_t a[4];
#pragma unroll
                    for (int jp = 0; jp < 4; ++jp)              // keys c = 16 s2 + 4 hf + jp and c + 8
                        a[jp] = *reinterpret_cast<const uint32_t*>(buf + (8 * s2 + 4 * hf + jp) * G::kVPitch + (32 * t + r32) * 4);
                    const u32x4 av = u32x4{a[0], a[1], a[2], a[3]};
                    const u32x4 bv = u32x4{pop[j][s2][0], pop[j][s2][1], pop[j][s2][2], pop[j][s2][3]};
                    ot[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av),
                                                                    __builtin_bit_cast(bf16x8, bv), ot[t], 0, 0, 0);
                }
            }
            lds_wave_sync();
        }
    }

    // ---- 5. normalise, round, transpose through LDS, store -------------------------------
#pragma unroll
    for (int t = 0; t < G::kDTiles; ++t)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            u32x2 v;
            v.x = pack_bf16x2(ot[t][4 * q4] * inv, ot[t][4 * q4 + 1] * inv);
            v.y = pack_bf16x2(ot[t][4 * q4 + 2] * inv, ot[t][4 * q4 + 3] * inv);
            *reinterpret_cast<u32x2*>(buf + r32 * G::kPitch + (32 * t + 8 * q4 + 4 * hf) * 2) = v;
        }
    lds_wave_sync();
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i) {
        const int row = qt * kTile + i * G::kRowsPerPass + lrow;
        if (row < rows_valid) {
            store_row_chunk<NARROW, G::kChunks>(ob, ooff[i], stg + i * G::kRowsPerPass * G::kPitch, lbyte, dbytes);
        }
    }
}

// ---------------------------------------------------------------------------------------
// Group-shared variant, for grouped-query heads with 4 (or a multiple of 4) query heads per
// key/value head: the 4 waves of a workgroup are 4 query heads of ONE group working on the
// same rows, so the K tile (and the V tile, when the value input is V) is fetched ONCE per
// workgroup - each wave loads a quarter of its rows - into a shared row-major LDS tile, and
// every wave reads its MFMA operands from there (K: row reads; V: ds_read_b64_tr_b16).
// This quarters the K/V traffic between L2 and the compute unit; a per-head value input
// (a previous O) still goes through the wave's private transit tile.
// VS: the value input is shared too (first hop).  Then the private tile only carries Q in and O
// out, one lane per row, and is used in two halves of 16 rows to halve its LDS footprint.
template <int D, int KT, bool VS, bool NARROW, bool ROPE>
__global__ __launch_bounds__(kWavesPerBlock * 64, 2) void mfma_fwd_shared_kernel(HopParams p, TileParams tp) {
    using G = Geo<D>;
    constexpr int kRows = kTile * KT;
    constexpr int kTileBytes = kTile * G::kPitch;                           // one row-major 32-row tile
    constexpr int kShare = G::kPasses / kWavesPerBlock;                     // load passes per wave per shared tile
    static_assert(G::kPasses % kWavesPerBlock == 0, "a shared tile must split evenly over the waves");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    uint32_t bx, by;
    workgroup_xy<NARROW>(bx, by);
    const int h = (int)bx * kWavesPerBlock + w;                             // host guarantees Hq % 4 == 0 and G % 4 == 0
    const uint32_t zb = blockIdx.z / tp.tiles_hi;
    const uint32_t tt = (blockIdx.z - zb * tp.tiles_hi) * tp.tiles_lo + by;
    if (tt >= tp.tiles) return;                                             // the whole workgroup leaves together
    const int b = (int)zb;
    const int g = h / p.G;
    constexpr bool v_shared = VS;
    constexpr int kHalves = VS ? 2 : 1;                                     // passes through the private tile per 32 rows
    constexpr int kHalfRows = kTile / kHalves;
    constexpr int kHalfPasses = G::kPasses / kHalves;
    const int hv = v_shared ? g : h;
    const int n = p.n;

    // LDS: [KT] shared K tiles | [KT] shared V tiles (only when v_shared) | row table | 4 private tiles.
    // The row table is the same for the 4 waves (same rows): each wave writes it, with identical values.
    char* sK = smem;
    char* sV = smem + KT * kTileBytes;
    u32x4* rowoff = reinterpret_cast<u32x4*>(smem + (v_shared ? 2 : 1) * KT * kTileBytes);
    char* buf = reinterpret_cast<char*>(rowoff + kRows) + w * (kTileBytes / kHalves);

    uint32_t f0;
    int qt, rows_valid;
    if (KT == 1) {
        f0 = tt * tp.fpt;
        qt = 0;
        rows_valid = (int)min((uint32_t)tp.fpt, (uint32_t)p.fibres - f0) * n;
    } else {
        f0 = tt / tp.qtiles;
        qt = (int)(tt - f0 * tp.qtiles);
        rows_valid = n;
    }
    uint64_t real_rows;                                   // bit r: table row r exists and its token is not padding
    {
        const uint32_t stride = (uint32_t)p.stride;
        const uint32_t vl = (uint32_t)hop_valid_len(p, b);
        bool real = false;
        if (lane < kRows) {
            const int rc = min(lane, rows_valid - 1);
            const uint32_t fi = (KT == 1) ? (uint32_t)((rc + 0.5f) * tp.inv_n) : 0u;
            const uint32_t a = rc - fi * n;
            const uint32_t f = f0 + fi;
            const uint32_t outer = f / stride;
            const uint32_t tok = outer * stride * n + (f - outer * stride) + a * stride;
            rowoff[lane] = u32x4{tok * tp.q_row, tok * tp.k_row, tok * tp.v_row, tok * tp.o_row};
            real = lane < rows_valid && tok < vl;
        }
        real_rows = __ballot(real);
    }
    lds_wave_sync();

    const char* qb = reinterpret_cast<const char*>(p.q.p) + ((int64_t)b * p.q.sb + (int64_t)h * p.q.sh) * 2;
    const char* kb = reinterpret_cast<const char*>(p.k.p) + ((int64_t)b * p.k.sb + (int64_t)g * p.k.sh) * 2;
    const char* vb = reinterpret_cast<const char*>(p.vin.p) + ((int64_t)b * p.vin.sb + (int64_t)hv * p.vin.sh) * 2;
    char* ob = reinterpret_cast<char*>(p.o.p) + ((int64_t)b * p.o.sb + (int64_t)h * p.o.sh) * 2;

    const int lrow = lane / G::kChunks, lcol = lane % G::kChunks;
    const uint32_t lbyte = lcol * 16;
    const uint32_t dbytes = (uint32_t)p.D * 2;           // bytes of a row (less than the tile's when NARROW)
    if (((real_rows >> (qt * kTile)) & 0xffffffffull) == 0) {
        // every query row of this unit is padding (the same in all four waves): zero rows out, nothing read
#pragma unroll
        for (int i = 0; i < G::kPasses; ++i) {
            const int row = qt * kTile + i * G::kRowsPerPass + lrow;
            if (row < rows_valid) store_chunk<NARROW>(ob, rowoff[row].w, lbyte, dbytes, u32x4{0u, 0u, 0u, 0u});
        }
        return;
    }
    const int kt_end = (KT == 1) ? 1 : (p.causal ? qt + 1 : (n > kTile ? 2 : 1));

    // ---- gather: Q (private), this wave's quarter of every K tile, and V: its quarter of
    //      every shared tile, or its own tiles when the value input is per head -------------
    u32x4 qreg[G::kPasses], ksh[KT][kShare], vsh[KT][kShare], vreg[KT][G::kPasses];
    uint32_t ooff[G::kPasses];
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i) {
        const u32x4 off = rowoff[qt * kTile + i * G::kRowsPerPass + lrow];
        qreg[i] = gather_chunk<NARROW, true>(qb, off.x, lbyte, dbytes);
        ooff[i] = off.w;
    }
#pragma unroll
    for (int j = 0; j < KT; ++j) {
        if (j < kt_end) {
#pragma unroll
            for (int i = 0; i < kShare; ++i) {
                const u32x4 off = rowoff[j * kTile + (w * kShare + i) * G::kRowsPerPass + lrow];
                ksh[j][i] = gather_chunk<NARROW, false>(kb, off.y, lbyte, dbytes);
                if (v_shared) vsh[j][i] = gather_chunk<NARROW, false>(vb, off.z, lbyte, dbytes);
            }
            if (!v_shared) {
#pragma unroll
                for (int i = 0; i < G::kPasses; ++i) {
                    const u32x4 off = rowoff[j * kTile + i * G::kRowsPerPass + lrow];
                    vreg[j][i] = (KT == 1) ? gather_chunk<NARROW, true>(vb, off.z, lbyte, dbytes)
                                           : gather_chunk<NARROW, false>(vb, off.z, lbyte, dbytes);   // with two query tiles a value tile is read twice: keep it cached
                }
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- rotary encoding of the gathered rows, by their position on the axis: Q (private) and this
    //      wave's quarter of every K tile, before they enter LDS ---------------------------------
    if constexpr (ROPE) {
        float rev[4];
        rope_rates(p, lcol, rev);
        auto row_pos = [&](int row) -> float {
            if (KT == 1) { const int rc = min(row, rows_valid - 1); return (float)(rc - (int)((rc + 0.5f) * tp.inv_n) * n); }
            return (float)min(row, n - 1);
        };
#pragma unroll
        for (int i = 0; i < G::kPasses; ++i) qreg[i] = rope_chunk(qreg[i], row_pos(qt * kTile + i * G::kRowsPerPass + lrow), rev);
#pragma unroll
        for (int j = 0; j < KT; ++j)
            if (j < kt_end) {
#pragma unroll
                for (int i = 0; i < kShare; ++i)
                    ksh[j][i] = rope_chunk(ksh[j][i], row_pos(j * kTile + (w * kShare + i) * G::kRowsPerPass + lrow), rev);
            }
    }

    const int r32 = lane & 31, hf = lane >> 5;
    char* stg = buf + lrow * G::kPitch + lbyte;
    const int opoff = r32 * G::kPitch + hf * 16;                            // natural operand read offset in a tile
    const int troff = (4 * hf + ((lane & 15) >> 2)) * G::kPitch + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;

    // ---- this wave's quarter of the shared tiles -> LDS; Q through the private tile -------
#pragma unroll
    for (int j = 0; j < KT; ++j) {
        if (j < kt_end) {
#pragma unroll
            for (int i = 0; i < kShare; ++i) {
                const int rowb = ((w * kShare + i) * G::kRowsPerPass + lrow) * G::kPitch + lbyte;
                *reinterpret_cast<u32x4*>(sK + j * kTileBytes + rowb) = ksh[j][i];
                if (v_shared) *reinterpret_cast<u32x4*>(sV + j * kTileBytes + rowb) = vsh[j][i];
            }
        }
    }
    u32x4 qop[G::kKSteps];
#pragma unroll
    for (int hs = 0; hs < kHalves; ++hs) {
        if (hs) lds_wave_sync();
#pragma unroll
        for (int i = 0; i < kHalfPasses; ++i)
            *reinterpret_cast<u32x4*>(stg + i * G::kRowsPerPass * G::kPitch) = qreg[hs * kHalfPasses + i];
        lds_wave_sync();
        if (r32 / kHalfRows == hs) read_natural<D>(buf + (r32 % kHalfRows) * G::kPitch + hf * 16, qop);
    }
    __syncthreads();                                                        // shared tiles complete

    // ---- S^T = K Q^T per key tile -----------------------------------------------------------
    f32x16 st[KT];
#pragma unroll
    for (int j = 0; j < KT; ++j) {
        st[j] = f32x16{};
        if (j < kt_end) {
            u32x4 kop[G::kKSteps];
            read_natural<D>(sK + j * kTileBytes + opoff, kop);
#pragma unroll
            for (int s = 0; s < G::kKSteps; ++s) st[j] = mma(kop[s], qop[s], st[j]);
        }
    }

    // ---- masked row softmax over all key tiles -------------------------------------------------
    const int qrow = qt * kTile + r32;
    int lo = 0, hi = 0;                                                     // visible keys = [lo, hi)
    uint32_t tw[KT];                                                        // the axis table's words for this row, in tile-row coordinates
#pragma unroll
    for (int j = 0; j < KT; ++j) tw[j] = 0xffffffffu;
    if ((real_rows >> qrow) & 1) {
        const int fi = (KT == 1) ? (int)((qrow + 0.5f) * tp.inv_n) : 0;          // the row's fibre within the unit
        const int flo = fi * n;
        visible_range(qrow, flo, flo + n, p.causal, p.window, lo, hi);
#pragma unroll
        for (int j = 0; j < KT; ++j) tw[j] = (KT == 1) ? table_word(p, f0 + fi, qrow - flo, 0) << flo : table_word(p, f0, qrow, j);
    }
    const float sl2 = p.scale * kLog2e;
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < KT; ++j) {
        const uint32_t vis = (range_mask(min(max(lo - 32 * j, 0), 32), min(max(hi - 32 * j, 0), 32)) & tw[j] & (uint32_t)(real_rows >> (32 * j))) >> (4 * hf);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const bool ok = (vis >> (8 * (r / 4) + (r % 4))) & 1u;
            st[j][r] = ok ? st[j][r] * sl2 : -INFINITY;
            mx = fmaxf(mx, st[j][r]);
        }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    if (mx == -INFINITY) mx = 0.f;
    u32x4 pop[KT][2];
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < KT; ++j)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            uint32_t wds[4];
#pragma unroll
            for (int jp = 0; jp < 4; ++jp) {
                const int r = 8 * s2 + 2 * jp;
                const uint32_t pk = pack_bf16x2(__builtin_amdgcn_exp2f(st[j][r] - mx), __builtin_amdgcn_exp2f(st[j][r + 1] - mx));
                sum += bf16_lo(pk) + bf16_hi(pk);                           // sum of the ROUNDED weights
                wds[jp] = pk;
            }
            pop[j][s2] = u32x4{wds[0], wds[1], wds[2], wds[3]};
        }
    sum += __shfl_xor(sum, 32);
    const float inv = sum > 0.f ? 1.f / sum : 0.f;

    // ---- O^T = V^T P^T per key tile ---------------------------------------------------------------
    f32x16 ot[G::kDTiles];
#pragma unroll
    for (int t = 0; t < G::kDTiles; ++t) ot[t] = f32x16{};
#pragma unroll
    for (int j = 0; j < KT; ++j) {
        if (j < kt_end) {
            u32x4 vT[G::kDTiles][2];
            if (v_shared) {
                read_transposed<D>(sV + j * kTileBytes + troff, vT);
            } else {
                lds_wave_sync();
                stage_rows<D>(stg, vreg[j]);
                lds_wave_sync();
                read_transposed<D>(buf + troff, vT);
            }
#pragma unroll
            for (int t = 0; t < G::kDTiles; ++t)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) ot[t] = mma(vT[t][s2], pop[j][s2], ot[t]);
        }
    }
    lds_wave_sync();

    // ---- normalise, round, transpose through the private tile, store ---------------------------------
#pragma unroll
    for (int hs = 0; hs < kHalves; ++hs) {
        if (r32 / kHalfRows == hs) {
#pragma unroll
            for (int t = 0; t < G::kDTiles; ++t)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    u32x2 v;
                    v.x = pack_bf16x2(ot[t][4 * q4] * inv, ot[t][4 * q4 + 1] * inv);
                    v.y = pack_bf16x2(ot[t][4 * q4 + 2] * inv, ot[t][4 * q4 + 3] * inv);
                    *reinterpret_cast<u32x2*>(buf + (r32 % kHalfRows) * G::kPitch + (32 * t + 8 * q4 + 4 * hf) * 2) = v;
                }
        }
        lds_wave_sync();
#pragma unroll
        for (int i = 0; i < kHalfPasses; ++i) {
            const int row = qt * kTile + (hs * kHalfPasses + i) * G::kRowsPerPass + lrow;
            if (row < rows_valid) {
                store_row_chunk<NARROW, G::kChunks>(ob, ooff[hs * kHalfPasses + i], stg + i * G::kRowsPerPass * G::kPitch, lbyte, dbytes);
            }
        }
        lds_wave_sync();
    }
}

template <int D, int KT, bool NARROW>
hipError_t launch_shared(const HopParams& p, const TileParams& tp, hipStream_t s) {
    const size_t tile = (size_t)kTile * Geo<D>::kPitch;
    const bool vs = p.vin_heads != p.Hq;
    const size_t smem = (vs ? 2 : 1) * KT * tile + (size_t)kTile * KT * 16 + kWavesPerBlock * (vs ? tile / 2 : tile);
    const dim3 grid((unsigned)(p.Hq / kWavesPerBlock), tp.tiles_lo, (unsigned)p.B * tp.tiles_hi);
    const void* kf = p.rope ? (vs ? (const void*)mfma_fwd_shared_kernel<D, KT, true, NARROW, true> : (const void*)mfma_fwd_shared_kernel<D, KT, false, NARROW, true>)
                            : (vs ? (const void*)mfma_fwd_shared_kernel<D, KT, true, NARROW, false> : (const void*)mfma_fwd_shared_kernel<D, KT, false, NARROW, false>);
    HopParams pc = p;
    TileParams tc = tp;
    void* args[2] = {&pc, &tc};
    return hipLaunchKernel(kf, grid, dim3(kWavesPerBlock * 64), args, smem, s);
}

template <int D, int KT, bool NARROW>
hipError_t launch(const HopParams& p, const TileParams& tp, hipStream_t s) {
    const size_t smem = (size_t)kWavesPerBlock * (Geo<D>::kBufBytes + kTile * KT * 16);
    const dim3 grid((unsigned)((p.Hq + kWavesPerBlock - 1) / kWavesPerBlock), tp.tiles_lo, (unsigned)p.B * tp.tiles_hi);
    const void* kf = p.rope ? (const void*)mfma_fwd_kernel<D, KT, NARROW, true> : (const void*)mfma_fwd_kernel<D, KT, NARROW, false>;
    HopParams pc = p;
    TileParams tc = tp;
    void* args[2] = {&pc, &tc};
    return hipLaunchKernel(kf, grid, dim3(kWavesPerBlock * 64), args, smem, s);
}

}  // namespace

bool mfma_forward_layout_ok(const HopParams& p) {
    const int64_t N = p.fibres * p.n;
    if (p.rope && p.n > 4096) return false;             // fp32 angles: positions beyond that lose too much of the turn
    return N < ((int64_t)1 << 31) && p.B <= 65535 && fits_u32(p.q, N) && fits_u32(p.k, N) && fits_u32(p.vin, N) &&
           fits_u32(p.o, N);
}

bool mfma_forward_supports(int32_t n, int32_t D, int dtype, int* kernel_id) {
    int kid = K_GENERIC;
    // head widths 64 and 128 fill a tile; any other multiple of 4 up to 128 rides in the next wider
    // tile with its extra features zero
    const bool full = D == 64 || D == 128, narrow = !full && D % 4 == 0 && D >= 8 && D < 128;
    if (dtype == TA_BF16 && n >= 1 && (full || narrow)) {
        if (n <= 32) kid = K_MFMA_BF16_N32;
        else if (n <= 64) kid = K_MFMA_BF16_N64;
        else kid = K_MFMA_BF16_STREAM;
    }
    if (kernel_id) *kernel_id = kid;
    return kid != K_GENERIC;
}

namespace {
template <int D, bool NARROW>
hipError_t launch_width(const HopParams& p, const TileParams& tp, int KT, hipStream_t s) {
    if (p.G % kWavesPerBlock == 0)                     // 4 query heads of a workgroup share their key/value head
        return KT == 1 ? launch_shared<D, 1, NARROW>(p, tp, s) : launch_shared<D, 2, NARROW>(p, tp, s);
    return KT == 1 ? launch<D, 1, NARROW>(p, tp, s) : launch<D, 2, NARROW>(p, tp, s);
}
}  // namespace

bool mfma_forward_feasible(const HopParams& p, int kernel_id) {
    if (kernel_id == K_MFMA_BF16_STREAM) return mfma_forward_stream_feasible(p);
    const int KT = kernel_id == K_MFMA_BF16_N32 ? 1 : (kernel_id == K_MFMA_BF16_N64 ? 2 : 0);
    if (KT == 0 || p.n < 1 || p.n > kTile * KT || p.D < 8 || p.D > 128 || p.D % 4 != 0 || !mfma_forward_layout_ok(p)) return false;
    TileParams tp;
    return make_tile_params(p, KT, &tp);
}

hipError_t launch_mfma_forward(const HopParams& p, int kernel_id, hipStream_t s) {
    if (kernel_id == K_MFMA_BF16_STREAM) return launch_mfma_forward_stream(p, s);
    if (!mfma_forward_feasible(p, kernel_id)) return hipErrorInvalidValue;
    const int KT = kernel_id == K_MFMA_BF16_N32 ? 1 : 2;
    TileParams tp;
    if (!make_tile_params(p, KT, &tp)) return hipErrorInvalidValue;
    if (p.D == 128) return launch_width<128, false>(p, tp, KT, s);
    if (p.D == 64) return launch_width<64, false>(p, tp, KT, s);
    return p.D > 64 ? launch_width<128, true>(p, tp, KT, s) : launch_width<64, true>(p, tp, KT, s);
}

}  // namespace ta
