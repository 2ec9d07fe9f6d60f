// bf16 MFMA per-axis attention forward for LONG axes (any axis length; used above 64) on
// gfx950: one hop of Eq. 4 of arXiv 2410.20926 with the keys of a fibre streamed in tiles
// of 32 and an online (running max / running sum) softmax, so that registers and LDS do not
// grow with the axis length.  The paper's own extrapolation recipe (Sec. 4.3) lengthens
// the first axis of a {32,32,32} model to reach 128k tokens; this kernel covers those axes.
//
// Work unit: 32 query rows of one fibre of one query head, one wavefront, no workgroup
// barrier.  Per 32-key tile: K tile -> LDS -> A operand, S^T = K Q^T, mask, running
// max/sum update, probabilities rounded to bf16 as the B operand, V tile -> LDS ->
// transposed read (ds_read_b64_tr_b16) as the A operand, O^T = corr * O^T + V^T P^T.
// The loads of tile j + 1 are issued as soon as tile j has left its registers.
#include "ta_mfma_common.h"
#include <type_traits>

namespace ta {
namespace {

using namespace mfma;

constexpr int kWavesPerBlock = 4;

struct StreamParams {
    uint32_t qtiles;          // 32-row query tiles per fibre = ceil(n / 32)
    uint32_t qchunk, qchunks; // chunked variant: query tiles per workgroup, workgroups per fibre
    uint32_t tiles;           // units per (batch, head block): fibres * qtiles, or fibres * qchunks
    uint32_t tiles_lo, tiles_hi;
    uint32_t q_row, k_row, v_row, o_row;       // token pitch in bytes
    uint32_t q_step, k_step, v_step, o_step;   // bytes between neighbouring rows of a fibre (stride * token pitch)
};

// NARROW (all three kernels): the head is narrower than the D-wide tile; see load_chunk.
template <int D, bool NARROW>
__global__ __launch_bounds__(kWavesPerBlock * 64, 2) void mfma_fwd_stream_kernel(HopParams p, StreamParams sp) {
    using G = Geo<D>;
    constexpr int kBuf = kTile * G::kPitch;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t bx, by;
    workgroup_xy<NARROW>(bx, by);
    const int h = (int)bx * kWavesPerBlock + w;
    const uint32_t zb = blockIdx.z / sp.tiles_hi;
    const uint32_t tt = (blockIdx.z - zb * sp.tiles_hi) * sp.tiles_lo + by;
    if (h >= p.Hq || tt >= sp.tiles) return;              // no workgroup barrier below
    const int b = (int)zb;
    const int g = h / p.G;
    const int hv = (p.vin_heads == p.Hq) ? h : g;
    const int n = p.n;
    char* buf = smem + w * kBuf;

    // heavier (later) query tiles of a fibre first: under the causal mask tile qt walks qt + 1 key tiles
    const uint32_t f = tt / sp.qtiles;
    const int qt = (int)(sp.qtiles - 1 - (tt - f * sp.qtiles));
    const uint32_t stride = (uint32_t)p.stride;
    const uint32_t outer = f / stride;
    const uint32_t tok0 = outer * stride * n + (f - outer * stride);       // first token of the fibre

    const char* qb = reinterpret_cast<const char*>(p.q.p) + ((int64_t)b * p.q.sb + (int64_t)h * p.q.sh) * 2 + tok0 * sp.q_row;
    const char* kb = reinterpret_cast<const char*>(p.k.p) + ((int64_t)b * p.k.sb + (int64_t)g * p.k.sh) * 2 + tok0 * sp.k_row;
    const char* vb = reinterpret_cast<const char*>(p.vin.p) + ((int64_t)b * p.vin.sb + (int64_t)hv * p.vin.sh) * 2 + tok0 * sp.v_row;
    char* ob = reinterpret_cast<char*>(p.o.p) + ((int64_t)b * p.o.sb + (int64_t)h * p.o.sh) * 2 + tok0 * sp.o_row;

    const int lrow = lane / G::kChunks, lcol = lane % G::kChunks;
    const uint32_t lbyte = lcol * 16;
    const uint32_t dbytes = (uint32_t)p.D * 2;            // bytes of a row (less than the tile's when NARROW)
    const int r32 = lane & 31, hf = lane >> 5;
    const int ktiles = (n + kTile - 1) / kTile;
    // key tiles that any row of this query tile can see (causal triangle, band)
    int jbeg = 0, jend = p.causal ? qt + 1 : ktiles;
    if (p.window > 0) {
        jbeg = max(0, qt * kTile - p.window + 1) / kTile;
        jend = min(jend, (qt * kTile + kTile - 1 + p.window - 1) / kTile + 1);
    }

    // rows past the end of the fibre alias its last row: loads need no predicate
    u32x4 qreg[G::kPasses], kreg[G::kPasses], vreg[G::kPasses];
    uint32_t ooff[G::kPasses];
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i) {
        const uint32_t rq = (uint32_t)min(qt * kTile + i * G::kRowsPerPass + lrow, n - 1);
        const uint32_t rk = (uint32_t)min(jbeg * kTile + i * G::kRowsPerPass + lrow, n - 1);
        qreg[i] = gather_chunk<NARROW, true>(qb, rq * sp.q_step, lbyte, dbytes);   // read by this wave alone
        kreg[i] = gather_chunk<NARROW, false>(kb, rk * sp.k_step, lbyte, dbytes);
        vreg[i] = gather_chunk<NARROW, false>(vb, rk * sp.v_step, lbyte, dbytes);
        ooff[i] = rq * sp.o_step + lbyte;
    }
    __builtin_amdgcn_sched_barrier(0);

    char* stg = buf + lrow * G::kPitch + lbyte;
    const char* oprd = buf + r32 * G::kPitch + hf * 16;
    const char* trbase = buf + (4 * hf + ((lane & 15) >> 2)) * G::kPitch + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;

    // rotary encoding: Q here, every K tile just before it enters LDS, each row by its position on the axis
    float rev[4];
    if (p.rope) {
        rope_rates(p, lcol, rev);
#pragma unroll
        for (int i = 0; i < G::kPasses; ++i) qreg[i] = rope_chunk(qreg[i], (float)min(qt * kTile + i * G::kRowsPerPass + lrow, n - 1), rev);
    }
    u32x4 qop[G::kKSteps];
    stage_rows<D>(stg, qreg);
    lds_wave_sync();
    read_natural<D>(oprd, qop);
    lds_wave_sync();

    // rows of the fibre whose token is not padding form a prefix [0, nreal)
    const uint32_t vl = (uint32_t)hop_valid_len(p, b);
    const int nreal = tok0 >= vl ? 0 : (int)min((uint32_t)n, (vl - tok0 + stride - 1) / stride);
    const int qrow = qt * kTile + r32;                    // this lane's query row in the fibre
    int klo = 0, khi = 0;                                 // it sees keys [klo, khi)
    if (qrow < nreal) {
        visible_range(qrow, 0, n, p.causal, p.window, klo, khi);
        khi = min(khi, nreal);
    }
    const float sl2 = p.scale * kLog2e;
    float m = -INFINITY, l = 0.f;
    f32x16 ot[G::kDTiles];
#pragma unroll
    for (int t = 0; t < G::kDTiles; ++t) ot[t] = f32x16{};

    for (int j = jbeg; j < jend; ++j) {
        // ---- K tile j: LDS transit, then request tile j + 1 into the same registers ------
        u32x4 kop[G::kKSteps];
        if (p.rope) {
#pragma unroll
            for (int i = 0; i < G::kPasses; ++i) kreg[i] = rope_chunk(kreg[i], (float)min(j * kTile + i * G::kRowsPerPass + lrow, n - 1), rev);
        }
        stage_rows<D>(stg, kreg);
        lds_wave_sync();
        read_natural<D>(oprd, kop);
        lds_wave_sync();
        if (j + 1 < jend) {
#pragma unroll
            for (int i = 0; i < G::kPasses; ++i) {
                const uint32_t rk = (uint32_t)min((j + 1) * kTile + i * G::kRowsPerPass + lrow, n - 1);
                kreg[i] = gather_chunk<NARROW, false>(kb, rk * sp.k_step, lbyte, dbytes);
            }
        }
        f32x16 st = {};
#pragma unroll
        for (int s = 0; s < G::kKSteps; ++s) st = mma(kop[s], qop[s], st);

        // ---- mask, running max and sum ------------------------------------------------------
        const uint32_t tw = qrow < nreal ? table_word(p, f, qrow, j) : 0u;
        const uint32_t vis32 = range_mask(min(max(klo - kTile * j, 0), kTile), min(max(khi - kTile * j, 0), kTile)) & tw;
        u32x4 pop[2];
        float corr;
        online_softmax_tile(st, vis32, hf, sl2, m, l, pop, corr);

        // ---- V tile j: LDS transit, transposed operands, then request tile j + 1 ------------
        u32x4 vT[G::kDTiles][2];
        stage_rows<D>(stg, vreg);
        lds_wave_sync();
        read_transposed<D>(trbase, vT);
        lds_wave_sync();
        if (j + 1 < jend) {
#pragma unroll
            for (int i = 0; i < G::kPasses; ++i) {
                const uint32_t rk = (uint32_t)min((j + 1) * kTile + i * G::kRowsPerPass + lrow, n - 1);
                vreg[i] = gather_chunk<NARROW, false>(vb, rk * sp.v_step, lbyte, dbytes);
            }
        }
#pragma unroll
        for (int t = 0; t < G::kDTiles; ++t) {
#pragma unroll
            for (int r = 0; r < 16; ++r) ot[t][r] *= corr;
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) ot[t] = mma(vT[t][s2], pop[s2], ot[t]);
        }
    }

    // ---- normalise, round, transpose through LDS, store -------------------------------------
    const float inv = l > 0.f ? 1.f / l : 0.f;
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
        if (row < n) {
            store_row_chunk<NARROW, G::kChunks>(ob, ooff[i] - lbyte, stg + i * G::kRowsPerPass * G::kPitch, lbyte, dbytes);
        }
    }
}

// Group-shared variant, for grouped-query heads with 4 (or a multiple of 4) query heads per
// key/value head: the 4 waves of a workgroup are 4 heads of one group working on the same
// query tile, so they walk the same key tiles.  Each wave fetches a quarter of every K tile
// (and of every V tile when the value input is per key/value head, VS) into a workgroup-shared,
// double-buffered LDS tile: K and V leave L2 once per workgroup instead of once per head, with
// one barrier per key tile.
template <int D, bool VS, bool NARROW>
__global__ __launch_bounds__(kWavesPerBlock * 64, 2) void mfma_fwd_stream_shared_kernel(HopParams p, StreamParams sp) {
    using G = Geo<D>;
    constexpr int kBuf = kTile * G::kPitch;
    constexpr int kMine = G::kPasses / kWavesPerBlock;    // passes of a shared tile this wave fetches
    static_assert(G::kPasses % kWavesPerBlock == 0, "a tile splits evenly over the waves");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t bx, by;
    workgroup_xy<NARROW>(bx, by);
    const int h = (int)bx * kWavesPerBlock + w;
    const uint32_t zb = blockIdx.z / sp.tiles_hi;
    const uint32_t tt = (blockIdx.z - zb * sp.tiles_hi) * sp.tiles_lo + by;
    if (tt >= sp.tiles) return;                           // whole workgroup leaves together (every head exists: 4 divides G)
    const int b = (int)zb;
    const int g = h / p.G;
    const int hv = VS ? g : h;
    const int n = p.n;
    char* sK = smem;                                      // two K tiles
    char* sV = smem + 2 * kBuf;                           // two V tiles (VS only)
    char* buf = smem + (VS ? 4 : 2) * kBuf + w * kBuf;    // this wave's own transit tile

    const uint32_t f = tt / sp.qtiles;
    const int qt = (int)(sp.qtiles - 1 - (tt - f * sp.qtiles));
    const uint32_t stride = (uint32_t)p.stride;
    const uint32_t outer = f / stride;
    const uint32_t tok0 = outer * stride * n + (f - outer * stride);

    const char* qb = reinterpret_cast<const char*>(p.q.p) + ((int64_t)b * p.q.sb + (int64_t)h * p.q.sh) * 2 + tok0 * sp.q_row;
    const char* kb = reinterpret_cast<const char*>(p.k.p) + ((int64_t)b * p.k.sb + (int64_t)g * p.k.sh) * 2 + tok0 * sp.k_row;
    const char* vb = reinterpret_cast<const char*>(p.vin.p) + ((int64_t)b * p.vin.sb + (int64_t)hv * p.vin.sh) * 2 + tok0 * sp.v_row;
    char* ob = reinterpret_cast<char*>(p.o.p) + ((int64_t)b * p.o.sb + (int64_t)h * p.o.sh) * 2 + tok0 * sp.o_row;

    const int lrow = lane / G::kChunks, lcol = lane % G::kChunks;
    const uint32_t lbyte = lcol * 16;
    const uint32_t dbytes = (uint32_t)p.D * 2;            // bytes of a row (less than the tile's when NARROW)
    const int r32 = lane & 31, hf = lane >> 5;
    const int ktiles = (n + kTile - 1) / kTile;
    int jbeg = 0, jend = p.causal ? qt + 1 : ktiles;
    if (p.window > 0) {
        jbeg = max(0, qt * kTile - p.window + 1) / kTile;
        jend = min(jend, (qt * kTile + kTile - 1 + p.window - 1) / kTile + 1);
    }

    // This wave's quarters of the next three key tiles travel in three register sets (tile t in
    // set (t - jbeg) % 3): a tile is requested three steps before it is used, which covers the
    // memory latency that one step of compute does not.
    u32x4 qreg[G::kPasses], vreg[VS ? 1 : G::kPasses];
    u32x4 kp[3][kMine], vp[3][VS ? kMine : 1];
    uint32_t ooff[G::kPasses];
    // `set` is the same in every lane; the unrolled comparison turns it into scalar branches
    // around code with fixed register names (no indexed registers)
    auto load_shared = [&](int set, int j) {
#pragma unroll
        for (int sidx = 0; sidx < 3; ++sidx)
            if (set == sidx) {
#pragma unroll
                for (int i = 0; i < kMine; ++i) {
                    const uint32_t rk = (uint32_t)min(j * kTile + (w * kMine + i) * G::kRowsPerPass + lrow, n - 1);
                    kp[sidx][i] = gather_chunk<NARROW, false>(kb, rk * sp.k_step, lbyte, dbytes);
                    if (VS) vp[sidx][i] = gather_chunk<NARROW, false>(vb, rk * sp.v_step, lbyte, dbytes);
                }
            }
    };
    float rev[4];                                         // rotary encoding: turn rates of this lane's four feature pairs
    if (p.rope) rope_rates(p, lcol, rev);
    auto write_shared = [&](int set, int slot, int j) {    // j: the key tile the registers hold (its rows' positions, for the encoding)
#pragma unroll
        for (int sidx = 0; sidx < 3; ++sidx)
            if (set == sidx) {
#pragma unroll
                for (int i = 0; i < kMine; ++i) {
                    const uint32_t at = (uint32_t)(slot * kBuf + ((w * kMine + i) * G::kRowsPerPass + lrow) * G::kPitch) + lbyte;
                    const u32x4 kv = p.rope ? rope_chunk(kp[sidx][i], (float)min(j * kTile + (w * kMine + i) * G::kRowsPerPass + lrow, n - 1), rev) : kp[sidx][i];
                    *reinterpret_cast<u32x4*>(sK + at) = kv;
                    if (VS) *reinterpret_cast<u32x4*>(sV + at) = vp[sidx][i];
                }
            }
    };
    auto load_own_v = [&](int j) {                        // a per-head value tile is this wave's alone
#pragma unroll
        for (int i = 0; i < (VS ? 0 : G::kPasses); ++i) {
            const uint32_t rk = (uint32_t)min(j * kTile + i * G::kRowsPerPass + lrow, n - 1);
            vreg[i] = gather_chunk<NARROW, false>(vb, rk * sp.v_step, lbyte, dbytes);
        }
    };
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i) {
        const uint32_t rq = (uint32_t)min(qt * kTile + i * G::kRowsPerPass + lrow, n - 1);
        qreg[i] = gather_chunk<NARROW, true>(qb, rq * sp.q_step, lbyte, dbytes);
        ooff[i] = rq * sp.o_step + lbyte;
    }
    load_shared(0, jbeg);
    if (jbeg + 1 < jend) load_shared(1, jbeg + 1);
    if (jbeg + 2 < jend) load_shared(2, jbeg + 2);
    if (!VS) load_own_v(jbeg);
    __builtin_amdgcn_sched_barrier(0);

    char* stg = buf + lrow * G::kPitch + lbyte;
    const uint32_t oprd = (uint32_t)(r32 * G::kPitch + hf * 16);
    const uint32_t troff = (uint32_t)((4 * hf + ((lane & 15) >> 2)) * G::kPitch + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2);

    if (p.rope) {
#pragma unroll
        for (int i = 0; i < G::kPasses; ++i) qreg[i] = rope_chunk(qreg[i], (float)min(qt * kTile + i * G::kRowsPerPass + lrow, n - 1), rev);
    }
    u32x4 qop[G::kKSteps];
    stage_rows<D>(stg, qreg);
    lds_wave_sync();
    read_natural<D>(buf + oprd, qop);
    lds_wave_sync();
    write_shared(0, 0, jbeg);
    if (jbeg + 3 < jend) load_shared(0, jbeg + 3);

    const uint32_t vl = (uint32_t)hop_valid_len(p, b);
    const int nreal = tok0 >= vl ? 0 : (int)min((uint32_t)n, (vl - tok0 + stride - 1) / stride);
    const int qrow = qt * kTile + r32;
    int klo = 0, khi = 0;
    if (qrow < nreal) {
        visible_range(qrow, 0, n, p.causal, p.window, klo, khi);
        khi = min(khi, nreal);
    }
    const float sl2 = p.scale * kLog2e;
    float m = -INFINITY, l = 0.f;
    f32x16 ot[G::kDTiles];
#pragma unroll
    for (int t = 0; t < G::kDTiles; ++t) ot[t] = f32x16{};

    // one key tile; `next_set` (a constant at every call site) names the registers of tile j + 1
    auto step = [&](int j, auto next_set_tag) {
        constexpr int next_set = decltype(next_set_tag)::value;
        const int slot = (j - jbeg) & 1;
        __syncthreads();                                  // tile j is complete; nobody reads the other slot any more
        u32x4 kop[G::kKSteps];
        read_natural<D>(sK + slot * kBuf + oprd, kop);
        f32x16 st = {};
#pragma unroll
        for (int s = 0; s < G::kKSteps; ++s) st = mma(kop[s], qop[s], st);

        const uint32_t tw = qrow < nreal ? table_word(p, f, qrow, j) : 0u;
        const uint32_t vis32 = range_mask(min(max(klo - kTile * j, 0), kTile), min(max(khi - kTile * j, 0), kTile)) & tw;
        u32x4 pop[2];
        float corr;
        online_softmax_tile(st, vis32, hf, sl2, m, l, pop, corr);

        u32x4 vT[G::kDTiles][2];
        if constexpr (VS) {
            read_transposed<D>(sV + slot * kBuf + troff, vT);
        } else {
            stage_rows<D>(stg, vreg);
            lds_wave_sync();
            read_transposed<D>(buf + troff, vT);
            lds_wave_sync();
            if (j + 1 < jend) load_own_v(j + 1);
        }
#pragma unroll
        for (int t = 0; t < G::kDTiles; ++t) {
#pragma unroll
            for (int r = 0; r < 16; ++r) ot[t][r] *= corr;
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) ot[t] = mma(vT[t][s2], pop[s2], ot[t]);
        }
        if (j + 1 < jend) {                               // the other slot was last read before this iteration's barrier
            write_shared(next_set, slot ^ 1, j + 1);
            if (j + 4 < jend) load_shared(next_set, j + 4);
        }
    };
    for (int j = jbeg; j < jend; j += 3) {                // three steps per trip: the register sets get fixed names
        step(j, std::integral_constant<int, 1>{});
        if (j + 1 < jend) step(j + 1, std::integral_constant<int, 2>{});
        if (j + 2 < jend) step(j + 2, std::integral_constant<int, 0>{});
    }

    const float inv = l > 0.f ? 1.f / l : 0.f;
    lds_wave_sync();
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
        if (row < n) {
            store_row_chunk<NARROW, G::kChunks>(ob, ooff[i] - lbyte, stg + i * G::kRowsPerPass * G::kPitch, lbyte, dbytes);
        }
    }
}

// The group-shared variant for axes of up to 4 tiles (n <= 128), where one query tile is only
// a few steps of work and a workgroup per query tile spends most of its life waiting for its
// first rows.  Here a workgroup takes all query tiles of a fibre, the heaviest first, and
// treats their (query tile, key tile) steps as ONE sequence: the quarters of a key tile are
// requested three steps before the step that uses them and the rows of the next query tile while
// the current one is being worked on, across query-tile boundaries, so that only the first
// step of a workgroup waits for memory with nothing else to do.

template <int D, bool VS, bool NARROW>
__global__ __launch_bounds__(kWavesPerBlock * 64, 2) void mfma_fwd_stream_chunked_kernel(HopParams p, StreamParams sp) {
    using G = Geo<D>;
    constexpr int kBuf = kTile * G::kPitch;
    constexpr int kMine = G::kPasses / kWavesPerBlock;    // passes of a shared tile this wave fetches
    static_assert(G::kPasses % kWavesPerBlock == 0, "a tile splits evenly over the waves");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t bx, by;
    workgroup_xy<NARROW>(bx, by);
    const int h = (int)bx * kWavesPerBlock + w;
    const uint32_t zb = blockIdx.z / sp.tiles_hi;
    const uint32_t tt = (blockIdx.z - zb * sp.tiles_hi) * sp.tiles_lo + by;
    if (tt >= sp.tiles) return;                           // whole workgroup leaves together (every head exists: 4 divides G)
    const int b = (int)zb;
    const int g = h / p.G;
    const int hv = VS ? g : h;
    const int n = p.n;
    char* sK = smem;                                      // two K tiles
    char* sV = smem + 2 * kBuf;                           // two V tiles (VS only)
    char* buf = smem + (VS ? 4 : 2) * kBuf + w * kBuf;    // this wave's own transit tile

    // unit -> (fibre, chunk of query tiles); later (heavier, under the causal mask) chunks first
    const uint32_t f = tt / sp.qchunks;
    const int chunk = (int)(sp.qchunks - 1 - (tt - f * sp.qchunks));
    const int ktiles = (n + kTile - 1) / kTile;
    const int qt_hi = min((chunk + 1) * (int)sp.qchunk, ktiles) - 1, qt_lo = chunk * (int)sp.qchunk;   // query tiles qt_hi down to qt_lo
    const uint32_t stride = (uint32_t)p.stride;
    const uint32_t outer = f / stride;
    const uint32_t tok0 = outer * stride * n + (f - outer * stride);

    const char* qb = reinterpret_cast<const char*>(p.q.p) + ((int64_t)b * p.q.sb + (int64_t)h * p.q.sh) * 2 + tok0 * sp.q_row;
    const char* kb = reinterpret_cast<const char*>(p.k.p) + ((int64_t)b * p.k.sb + (int64_t)g * p.k.sh) * 2 + tok0 * sp.k_row;
    const char* vb = reinterpret_cast<const char*>(p.vin.p) + ((int64_t)b * p.vin.sb + (int64_t)hv * p.vin.sh) * 2 + tok0 * sp.v_row;
    char* ob = reinterpret_cast<char*>(p.o.p) + ((int64_t)b * p.o.sb + (int64_t)h * p.o.sh) * 2 + tok0 * sp.o_row;

    const int lrow = lane / G::kChunks, lcol = lane % G::kChunks;
    const uint32_t lbyte = lcol * 16;
    const uint32_t dbytes = (uint32_t)p.D * 2;            // bytes of a row (less than the tile's when NARROW)
    const int r32 = lane & 31, hf = lane >> 5;
    // key tiles [jb, je) that some row of query tile qt can see (causal triangle, band)
    auto key_tiles = [&](int qt, int& jb, int& je) {
        jb = 0;
        je = p.causal ? qt + 1 : ktiles;
        if (p.window > 0) {
            jb = max(0, qt * kTile - p.window + 1) / kTile;
            je = min(je, (qt * kTile + kTile - 1 + p.window - 1) / kTile + 1);
        }
    };
    // position in the sequence of steps: query tile qt (descending), key tile j (ascending)
    struct Cursor { int qt, j, je; };
    auto cursor_begin = [&](Cursor& c) { c.qt = qt_hi; key_tiles(c.qt, c.j, c.je); };
    auto cursor_next = [&](Cursor& c) {                   // returns false past the last step
        if (++c.j < c.je) return true;
        if (--c.qt < qt_lo) return false;
        key_tiles(c.qt, c.j, c.je);
        return true;
    };

    // This wave's quarters of the next three key tiles travel in three register sets (the tile
    // of step t in set t % 3).
    u32x4 qreg[G::kPasses], vreg[VS ? 1 : G::kPasses];
    u32x4 kp[3][kMine], vp[3][VS ? kMine : 1];
    auto load_shared = [&](auto set_tag, int j) {
        constexpr int set = decltype(set_tag)::value;
#pragma unroll
        for (int i = 0; i < kMine; ++i) {
            const uint32_t rk = (uint32_t)min(j * kTile + (w * kMine + i) * G::kRowsPerPass + lrow, n - 1);
            kp[set][i] = gather_chunk<NARROW, false>(kb, rk * sp.k_step, lbyte, dbytes);
            if (VS) vp[set][i] = gather_chunk<NARROW, false>(vb, rk * sp.v_step, lbyte, dbytes);
        }
    };
    float rev[4];                                         // rotary encoding: turn rates of this lane's four feature pairs
    if (p.rope) rope_rates(p, lcol, rev);
    auto write_shared = [&](auto set_tag, int slot, int j) {   // j: the key tile the registers hold (its rows' positions, for the encoding)
        constexpr int set = decltype(set_tag)::value;
#pragma unroll
        for (int i = 0; i < kMine; ++i) {
            const uint32_t at = (uint32_t)(slot * kBuf + ((w * kMine + i) * G::kRowsPerPass + lrow) * G::kPitch) + lbyte;
            const u32x4 kv = p.rope ? rope_chunk(kp[set][i], (float)min(j * kTile + (w * kMine + i) * G::kRowsPerPass + lrow, n - 1), rev) : kp[set][i];
            *reinterpret_cast<u32x4*>(sK + at) = kv;
            if (VS) *reinterpret_cast<u32x4*>(sV + at) = vp[set][i];
        }
    };
    auto load_own_v = [&](int j) {                        // a per-head value tile is this wave's alone
#pragma unroll
        for (int i = 0; i < (VS ? 0 : G::kPasses); ++i) {
            const uint32_t rk = (uint32_t)min(j * kTile + i * G::kRowsPerPass + lrow, n - 1);
            vreg[i] = gather_chunk<NARROW, false>(vb, rk * sp.v_step, lbyte, dbytes);
        }
    };
    auto load_q = [&](int qt) {
#pragma unroll
        for (int i = 0; i < G::kPasses; ++i) {
            const uint32_t rq = (uint32_t)min(qt * kTile + i * G::kRowsPerPass + lrow, n - 1);
            qreg[i] = gather_chunk<NARROW, true>(qb, rq * sp.q_step, lbyte, dbytes);
        }
    };
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    using S2 = std::integral_constant<int, 2>;

    Cursor cur, ahead;                                    // the step being worked on; the step whose tile is requested next
    cursor_begin(cur);
    ahead = cur;
    bool more_ahead = true;
    load_q(cur.qt);
    load_shared(S0{}, ahead.j);
    more_ahead = cursor_next(ahead);
    if (more_ahead) { load_shared(S1{}, ahead.j); more_ahead = cursor_next(ahead); }
    if (more_ahead) { load_shared(S2{}, ahead.j); more_ahead = cursor_next(ahead); }
    if (!VS) load_own_v(cur.j);
    __builtin_amdgcn_sched_barrier(0);

    char* stg = buf + lrow * G::kPitch + lbyte;
    const uint32_t oprd = (uint32_t)(r32 * G::kPitch + hf * 16);
    const uint32_t troff = (uint32_t)((4 * hf + ((lane & 15) >> 2)) * G::kPitch + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2);
    const uint32_t vl = (uint32_t)hop_valid_len(p, b);
    const int nreal = tok0 >= vl ? 0 : (int)min((uint32_t)n, (vl - tok0 + stride - 1) / stride);
    const float sl2 = p.scale * kLog2e;

    write_shared(S0{}, 0, cur.j);
    if (more_ahead) { load_shared(S0{}, ahead.j); more_ahead = cursor_next(ahead); }

    // per query tile
    u32x4 qop[G::kKSteps];
    int klo = 0, khi = 0;
    float m = -INFINITY, l = 0.f;
    f32x16 ot[G::kDTiles];
    int t = 0;                                            // step number: slot t & 1, register set t % 3
    bool more = true, first_of_tile = true;

    // one step; `next_set` (a constant at every call site) names the registers of the next step's tile
    auto step = [&](auto next_set_tag) {
        const int slot = t & 1;
        const int qt = cur.qt, j = cur.j;
        const int qrow = qt * kTile + r32;
        if (first_of_tile) {
            first_of_tile = false;
            // first step of a query tile: its rows become the B operand, the next query tile's rows are requested
            lds_wave_sync();
            if (p.rope) {
#pragma unroll
                for (int i = 0; i < G::kPasses; ++i) qreg[i] = rope_chunk(qreg[i], (float)min(qt * kTile + i * G::kRowsPerPass + lrow, n - 1), rev);
            }
            stage_rows<D>(stg, qreg);
            lds_wave_sync();
            read_natural<D>(buf + oprd, qop);
            lds_wave_sync();
            if (qt > qt_lo) load_q(qt - 1);
            klo = 0; khi = 0;
            if (qrow < nreal) {
                visible_range(qrow, 0, n, p.causal, p.window, klo, khi);
                khi = min(khi, nreal);
            }
            m = -INFINITY; l = 0.f;
#pragma unroll
            for (int tt2 = 0; tt2 < G::kDTiles; ++tt2) ot[tt2] = f32x16{};
        }
        __syncthreads();                                  // this step's tile is complete; nobody reads the other slot any more
        u32x4 kop[G::kKSteps];
        read_natural<D>(sK + slot * kBuf + oprd, kop);
        f32x16 st = {};
#pragma unroll
        for (int s = 0; s < G::kKSteps; ++s) st = mma(kop[s], qop[s], st);

        const uint32_t tw = qrow < nreal ? table_word(p, f, qrow, j) : 0u;
        const uint32_t vis32 = range_mask(min(max(klo - kTile * j, 0), kTile), min(max(khi - kTile * j, 0), kTile)) & tw;
        u32x4 pop[2];
        float corr;
        online_softmax_tile(st, vis32, hf, sl2, m, l, pop, corr);

        // the next step (if any): needed below for the per-head value tile and for the end of this query tile
        Cursor nxt = cur;
        const bool has_next = cursor_next(nxt);
        const bool last_of_tile = !has_next || nxt.qt != qt;

        u32x4 vT[G::kDTiles][2];
        if constexpr (VS) {
            read_transposed<D>(sV + slot * kBuf + troff, vT);
        } else {
            stage_rows<D>(stg, vreg);
            lds_wave_sync();
            read_transposed<D>(buf + troff, vT);
            lds_wave_sync();
            if (has_next) load_own_v(nxt.j);
        }
#pragma unroll
        for (int tt2 = 0; tt2 < G::kDTiles; ++tt2) {
#pragma unroll
            for (int r = 0; r < 16; ++r) ot[tt2][r] *= corr;
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) ot[tt2] = mma(vT[tt2][s2], pop[s2], ot[tt2]);
        }
        if (has_next) {                                   // the other slot was last read before this step's barrier
            write_shared(next_set_tag, slot ^ 1, nxt.j);
            if (more_ahead) { load_shared(next_set_tag, ahead.j); more_ahead = cursor_next(ahead); }
        }
        if (last_of_tile) {                               // normalise, round, transpose through the own tile, store
            const float inv = l > 0.f ? 1.f / l : 0.f;
            lds_wave_sync();
#pragma unroll
            for (int tt2 = 0; tt2 < G::kDTiles; ++tt2)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    u32x2 v;
                    v.x = pack_bf16x2(ot[tt2][4 * q4] * inv, ot[tt2][4 * q4 + 1] * inv);
                    v.y = pack_bf16x2(ot[tt2][4 * q4 + 2] * inv, ot[tt2][4 * q4 + 3] * inv);
                    *reinterpret_cast<u32x2*>(buf + r32 * G::kPitch + (32 * tt2 + 8 * q4 + 4 * hf) * 2) = v;
                }
            lds_wave_sync();
#pragma unroll
            for (int i = 0; i < G::kPasses; ++i) {
                const int row = qt * kTile + i * G::kRowsPerPass + lrow;
                if (row < n) {
                    store_row_chunk<NARROW, G::kChunks>(ob, (uint32_t)row * sp.o_step, stg + i * G::kRowsPerPass * G::kPitch, lbyte, dbytes);
                }
            }
        }
        if (last_of_tile) first_of_tile = true;
        cur = nxt;
        more = has_next;
        ++t;
    };
    while (more) {                                        // three steps per trip: the register sets get fixed names
        step(S1{});
        if (more) step(S2{});
        if (more) step(S0{});
    }
}

template <int D, bool VS, bool NARROW>
hipError_t launch_shared(const HopParams& p, const StreamParams& sp, hipStream_t s) {
    const size_t smem = (size_t)((VS ? 4 : 2) + kWavesPerBlock) * kTile * Geo<D>::kPitch;
    const dim3 grid((unsigned)(p.Hq / kWavesPerBlock), sp.tiles_lo, (unsigned)p.B * sp.tiles_hi);
    if (smem > 64 * 1024) {
        const void* kf = sp.qchunk > 1 ? reinterpret_cast<const void*>(mfma_fwd_stream_chunked_kernel<D, VS, NARROW>)
                                       : reinterpret_cast<const void*>(mfma_fwd_stream_shared_kernel<D, VS, NARROW>);
        const hipError_t e = allow_dynamic_lds(kf, (int)smem);
        if (e != hipSuccess) return e;
    }
    if (sp.qchunk > 1) hipLaunchKernelGGL((mfma_fwd_stream_chunked_kernel<D, VS, NARROW>), grid, dim3(kWavesPerBlock * 64), smem, s, p, sp);
    else               hipLaunchKernelGGL((mfma_fwd_stream_shared_kernel<D, VS, NARROW>), grid, dim3(kWavesPerBlock * 64), smem, s, p, sp);
    return hipGetLastError();
}

template <int D, bool NARROW>
hipError_t launch(const HopParams& p, const StreamParams& sp, hipStream_t s) {
    const size_t smem = (size_t)kWavesPerBlock * kTile * Geo<D>::kPitch;
    const dim3 grid((unsigned)((p.Hq + kWavesPerBlock - 1) / kWavesPerBlock), sp.tiles_lo, (unsigned)p.B * sp.tiles_hi);
    hipLaunchKernelGGL((mfma_fwd_stream_kernel<D, NARROW>), grid, dim3(kWavesPerBlock * 64), smem, s, p, sp);
    return hipGetLastError();
}

}  // namespace

// Launch geometry of the streaming kernels; false when the shape or the grid does not fit.
static bool stream_params(const HopParams& p, StreamParams* spp) {
    if (p.n < 1 || p.D < 8 || p.D > 128 || p.D % 4 != 0 || !mfma_forward_layout_ok(p)) return false;
    StreamParams& sp = *spp;
    const bool shared = p.G % kWavesPerBlock == 0;        // the 4 waves of a workgroup are 4 heads of one group
    sp.qtiles = (uint32_t)((p.n + kTile - 1) / kTile);
    sp.qchunk = (shared && sp.qtiles <= 4) ? sp.qtiles : 1u;   // short axes: one workgroup walks all query tiles of a fibre
    sp.qchunks = (sp.qtiles + sp.qchunk - 1) / sp.qchunk;
    const int64_t tiles = p.fibres * sp.qchunks;
    if (tiles <= 0 || tiles > 0x7fffffffLL) return false;
    sp.tiles = (uint32_t)tiles;
    sp.tiles_lo = (uint32_t)(tiles < 32768 ? tiles : 32768);
    sp.tiles_hi = (uint32_t)((tiles + sp.tiles_lo - 1) / sp.tiles_lo);
    if ((int64_t)p.B * sp.tiles_hi > 65535) return false;
    sp.q_row = (uint32_t)(p.q.st * 2);
    sp.k_row = (uint32_t)(p.k.st * 2);
    sp.v_row = (uint32_t)(p.vin.st * 2);
    sp.o_row = (uint32_t)(p.o.st * 2);
    sp.q_step = (uint32_t)(p.stride * p.q.st * 2);
    sp.k_step = (uint32_t)(p.stride * p.k.st * 2);
    sp.v_step = (uint32_t)(p.stride * p.vin.st * 2);
    sp.o_step = (uint32_t)(p.stride * p.o.st * 2);
    return true;
}

bool mfma_forward_stream_feasible(const HopParams& p) {
    StreamParams sp;
    return stream_params(p, &sp);
}

hipError_t launch_mfma_forward_stream(const HopParams& p, hipStream_t s) {
    StreamParams sp;
    if (!stream_params(p, &sp)) return hipErrorInvalidValue;
    const bool shared = p.G % kWavesPerBlock == 0;
    const bool vs = p.vin_heads != p.Hq;
    if (p.D == 128) return shared ? (vs ? launch_shared<128, true, false>(p, sp, s) : launch_shared<128, false, false>(p, sp, s)) : launch<128, false>(p, sp, s);
    if (p.D == 64) return shared ? (vs ? launch_shared<64, true, false>(p, sp, s) : launch_shared<64, false, false>(p, sp, s)) : launch<64, false>(p, sp, s);
    if (p.D > 64) return shared ? (vs ? launch_shared<128, true, true>(p, sp, s) : launch_shared<128, false, true>(p, sp, s)) : launch<128, true>(p, sp, s);
    return shared ? (vs ? launch_shared<64, true, true>(p, sp, s) : launch_shared<64, false, true>(p, sp, s)) : launch<64, true>(p, sp, s);
}

}  // namespace ta
