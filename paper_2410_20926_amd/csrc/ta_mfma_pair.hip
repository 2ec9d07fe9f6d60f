// Two consecutive hops of Algorithm 1 in one kernel: the hop along the second-innermost
// tensor axis followed by the hop along the innermost one (Eq. 4 twice, with the same Q and
// K), for 32 x 32 slabs, bf16, head width 128 or 64, with every per-axis mask of the single-hop kernels.  The intermediate value tensor of the pair
// never leaves the chip, and Q, K, the value input and the output each cross HBM once.
//
// A slab is the 1,024 consecutive tokens (i, j), i on the outer of the two axes, j on the
// inner one, of one (batch, head).  One workgroup of 8 waves owns one slab:
//
//   phase A  scores of both hops.  The slab's Q and K rows enter LDS 32 features at a time
//            (each row is read from HBM once, by the wave that owns its i); a wave
//            accumulates S^T = K Q^T for its 4 "column" fibres (j fixed, the first hop) and
//            its 4 "row" fibres (i fixed, the second hop) over the 4 feature chunks, then
//            does the masked row softmax of each in registers and keeps the rounded
//            probabilities as MFMA B operands.
//   phase B  values, 64 features at a time: the value input's rows enter LDS, every column
//            fibre replaces its rows by P1 X in place, then every row fibre computes P2 (P1 X)
//            from them and stores its output rows.
//
// Workgroups are numbered so that the query heads of one key/value head run on the same
// XCD at the same time and share its K rows through that XCD's L2.
#include "ta_mfma_common.h"

namespace ta {

using namespace mfma;

namespace {

constexpr int kN = 32;                       // both axis lengths
constexpr int kSlab = kN * kN;               // tokens per slab
constexpr int kWaves = 8;                    // waves per workgroup; wave w owns i (and j) in [4 w, 4 w + 4)
constexpr int kOwn = kN / kWaves;            // fibres of each kind per wave
constexpr int kCA = 32;                      // features per phase-A chunk (64 bytes of a row)
constexpr int kCB = 64;                      // features per phase-B chunk (128 bytes of a row)
constexpr int kARow = kCA * 2;               // bytes of one token's phase-A chunk row (half a 128-byte line)
constexpr int kAK = kN * kARow;              // within an i-block: the 32 Q rows, then the 32 K rows
constexpr int kABlock = 2 * kAK + 16;        // i-block pitch; the odd number of 16-byte units spreads a column fibre over the banks
constexpr int kABytes = kN * kABlock;
constexpr int kBPitch = kCB * 2 + 16;        // phase-B row pitch
constexpr int kBRowsPerI = kN + 1;           // one spare row slot per i keeps column fibres off a single bank group
constexpr int kBBytes = kN * kBRowsPerI * kBPitch;
constexpr int kLdsBytes = (kABytes > kBBytes) ? kABytes : kBBytes;

struct PairParams {
    Tensor q, k, vin, o;
    void* mid;                               // nullptr, or an O-shaped tensor that receives the output of the first hop
    int32_t B, Hq, Hkv, G, vin_heads, causal;
    float scale;
    int32_t window1, window2;                // band widths on the outer / inner axis, 0 = none
    const uint32_t* mask1;                   // bit tables of the outer / inner axis (32 words) or nullptr
    const uint32_t* mask2;
    uint32_t mask1_fibre, mask2_fibre;       // words from one fibre's table to the next (32), or 0: one table for the axis
    uint32_t slabs;                          // slabs per batch element
    uint32_t groups;                         // B * slabs * Hkv
    uint32_t q_row, k_row, v_row, o_row;     // token pitch of each tensor in bytes
    int64_t valid_len;                       // tokens at or past it (per batch element) are padding; N when there is none
    const int64_t* valid_lens;               // device: one such length per batch element (combined with valid_len), or nullptr
    uint32_t dbytes;                         // bytes of a row (2 * head width)
    float rope_c0, rope_c1;                  // rotary encoding inside the hops: pair p of a row at position a turns by a * exp2(rope_c0 * p + rope_c1) revolutions
};

// Phase-A LDS layout.  Token (i, j)'s 64-byte chunk row of Q sits at i * kABlock + j * 64, that
// of K kAK bytes further; inside a row the four 16-byte units are rotated by j / 2, so that
// unit u is at position (u + j / 2) mod 4.  Consecutive j (a row fibre) then alternate between
// the halves of a 128-byte line and walk through the units; consecutive i (a column fibre) are
// an odd number of units apart: both access patterns cover all banks.

// Narrow heads (rows of `dbytes` < 2 kD bytes, 8-byte aligned, at least 16 bytes): the 16-byte chunk at `addr`, which
// starts `at` bytes into its row; what lies outside the row reads as zero and is not written.  One 16-byte request
// per lane and no branch (with a branch per request every request waits for the one before): a chunk that would pass
// the end of the row is replaced by the row's last 16 bytes, whose second half is the chunk's first.
template <bool NT>
__device__ inline u32x4 narrow_load(const char* addr, uint32_t at, uint32_t dbytes) {
    const bool full = at + 16 <= dbytes, tail = !full && at + 8 <= dbytes;
    const u32x4* a = reinterpret_cast<const u32x4*>(full ? addr : addr + ((int32_t)dbytes - 16 - (int32_t)at));
    u32x4 v = NT ? __builtin_nontemporal_load(a) : *a;
    if (tail) v = u32x4{v.z, v.w, 0u, 0u};
    if (!full && !tail) v = u32x4{0u, 0u, 0u, 0u};
    return v;
}
__device__ inline void narrow_store(char* addr, uint32_t at, uint32_t dbytes, const u32x4 v) {
    // a whole chunk in one store, the row's last 8 bytes on their own; through the cache (see the kernel's numbering)
    if (at + 16 <= dbytes) *reinterpret_cast<u32x4*>(addr) = v;
    else if (at + 8 <= dbytes) *reinterpret_cast<u32x2*>(addr) = u32x2{v.x, v.y};
}

// Masked row softmax of one 32 x 32 score tile held as S^T (lane = query row, 16 keys per
// lane, the other 16 in lane ^ 32).  Returns the rounded, un-normalised probabilities as
// two B operands and 1 / (their row sum).
// Positions at or past `nreal` of the fibre are padding: never a key, and a padded row sees nothing.
__device__ inline void softmax_tile(const f32x16& st, int r32, int hf, int causal, int window, const uint32_t* table,
                                    int nreal, float sl2, u32x4 (&pop)[2], float& inv) {
    int lo, hi;
    visible_range(r32, 0, kN, causal, window, lo, hi);
    uint32_t vis = r32 < nreal ? range_mask(lo, min(hi, nreal)) : 0u;
    if (table) vis &= table[r32];
    vis >>= 4 * hf;
    float e[16], mx = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const bool ok = (vis >> (8 * (r / 4) + (r % 4))) & 1u;
        e[r] = ok ? st[r] * sl2 : -INFINITY;
        mx = fmaxf(mx, e[r]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    if (mx == -INFINITY) mx = 0.f;
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
        uint32_t wds[4];
#pragma unroll
        for (int jp = 0; jp < 4; ++jp) {
            const int r = 8 * s2 + 2 * jp;
            wds[jp] = pack_bf16x2(__builtin_amdgcn_exp2f(e[r] - mx), __builtin_amdgcn_exp2f(e[r + 1] - mx));
        }
        pop[s2] = u32x4{wds[0], wds[1], wds[2], wds[3]};
    }
    // The sum of the ROUNDED weights of a row comes from the matrix unit, which is idle here: a tile of ones times the
    // weights puts the sum over all 32 keys of query row r32 into every accumulator of the lane.
    const uint32_t ones = 0x3f803f80u;
    f32x16 rs = {};
    rs = mma(u32x4{ones, ones, ones, ones}, pop[0], rs);
    rs = mma(u32x4{ones, ones, ones, ones}, pop[1], rs);
    const float sum = rs[0];
    inv = sum > 0.f ? 1.f / sum : 0.f;
}

// One fibre's value update on a 64-feature chunk resident in LDS: rows at `fb + r * rs`.
// Reads the rows as transposed operands, forms (P X)^T, scales by `inv`, rounds and writes
// the rows back in place.  The rows belong to this wave alone while it runs.
__device__ inline void update_fibre(char* lds, uint32_t fb, uint32_t rs, const u32x4 (&pop)[2], float inv, int lane) {
    const int r32 = lane & 31, hf = lane >> 5;
    const uint32_t trow = 4 * hf + ((lane & 15) >> 2);
    const uint32_t tcol = (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
    f32x16 ot[kCB / 32];
#pragma unroll
    for (int t = 0; t < kCB / 32; ++t) {
        ot[t] = f32x16{};
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const char* a0 = lds + fb + (16 * s2 + trow) * rs + tcol + 64 * t;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a0));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a0 + 8 * rs));
            const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
            ot[t] = mma(u32x4{l2.x, l2.y, h2.x, h2.y}, pop[s2], ot[t]);
        }
    }
    lds_wave_sync();                                      // every lane has its operands before a row is overwritten
#pragma unroll
    for (int t = 0; t < kCB / 32; ++t)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            u32x2 v;
            v.x = pack_bf16x2(ot[t][4 * q4] * inv, ot[t][4 * q4 + 1] * inv);
            v.y = pack_bf16x2(ot[t][4 * q4 + 2] * inv, ot[t][4 * q4 + 3] * inv);
            *reinterpret_cast<u32x2*>(lds + fb + r32 * rs + (32 * t + 8 * q4 + 4 * hf) * 2) = v;
        }
}

// MID: the intermediate O (the first hop's output) is written out as well, for a backward pass.
// kD: tile width, 128 (two 128-byte lines per row, four score chunks, two value chunks) or 64.
// NARROW: the head is narrower than the tile (p.dbytes bytes per row, a multiple of 8); the tile's
// extra features are zero.
// ROPE: both hops score with Q and K rotated by the position on their own axis (Sec. 3.2).  A token's rows
// are needed in two versions then, turned by i for the first hop and by j for the second, so the turn is
// applied to the MFMA operands after they have been read from LDS, where a lane holds four feature pairs of
// the fibre row r32, whose position is r32 in either kind of fibre.  The sine and cosine of the lane's
// angles are rounded to bf16 and the turn is two bf16 dot products per pair (v_dot2_f32_bf16: exact
// products, fp32 sums), so a turned pair is exact up to 2^-9 of its size before its own rounding to bf16.
template <int kD, bool MID, bool NARROW, bool ROPE>
__global__ __launch_bounds__(64 * kWaves, 2) void mfma_fwd_pair_kernel(PairParams p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r32 = lane & 31, hf = lane >> 5;

    // workgroup -> (key/value group gi, head of the group hg): the heads of one group are 8
    // workgroup ids apart, i.e. on the same XCD when workgroup ids go round the 8 XCDs, and are
    // dispatched one after the other there: they run at the same time and share their K rows
    // through that XCD's L2.
    const bool vin_is_o = (p.vin_heads == p.Hq);
    const uint32_t span = 8u * (uint32_t)p.G;
    uint32_t blk = blockIdx.x / span, rem = blockIdx.x - blk * span;
    uint32_t hg = rem >> 3, gi = blk * 8u + (rem & 7u);
    if constexpr (NARROW) {
        // Narrow rows share their first and last cache line with the neighbouring heads' rows: every XCD takes a
        // contiguous run of the (slab, head) sequence, so that neighbouring heads are written, through the cache, from
        // one L2 and reach memory as whole lines (see workgroup_xy).  The grid is a multiple of 8 workgroups.
        const uint32_t seq = (blockIdx.x & 7u) * (gridDim.x / 8u) + (blockIdx.x >> 3);
        gi = seq / (uint32_t)p.G;
        hg = seq - gi * (uint32_t)p.G;
    }
    if (gi >= p.groups) return;                           // whole workgroup leaves together
    const uint32_t g = gi % (uint32_t)p.Hkv;
    const uint32_t sl = (gi / (uint32_t)p.Hkv) % p.slabs;
    const uint32_t b = gi / ((uint32_t)p.Hkv * p.slabs);
    const uint32_t h = g * (uint32_t)p.G + hg;
    const uint32_t hv = vin_is_o ? h : g;
    const int64_t tok0 = (int64_t)sl * kSlab;
    const char* qb = reinterpret_cast<const char*>(p.q.p) + ((int64_t)b * p.q.sb + (int64_t)h * p.q.sh) * 2 + tok0 * p.q_row;
    const char* kb = reinterpret_cast<const char*>(p.k.p) + ((int64_t)b * p.k.sb + (int64_t)g * p.k.sh) * 2 + tok0 * p.k_row;
    const char* xb = reinterpret_cast<const char*>(p.vin.p) + ((int64_t)b * p.vin.sb + (int64_t)hv * p.vin.sh) * 2 + tok0 * p.v_row;
    char* ob = reinterpret_cast<char*>(p.o.p) + ((int64_t)b * p.o.sb + (int64_t)h * p.o.sh) * 2 + tok0 * p.o_row;
    char* mb = reinterpret_cast<char*>(p.mid) + ((int64_t)b * p.o.sb + (int64_t)h * p.o.sh) * 2 + tok0 * p.o_row;

    int64_t valid_len = p.valid_len;                      // this batch element's padding length
    if (p.valid_lens) {
        const int64_t x = p.valid_lens[b];
        valid_len = x < valid_len ? (x < 0 ? 0 : x) : valid_len;
    }
    if (valid_len <= tok0) {                              // the whole slab is padding: its outputs are zero, nothing is read
        constexpr int kLanesPerRow = kD / 8, kRowsPerPass = 64 / kLanesPerRow;
#pragma unroll 4
        for (int pp = 0; pp < kOwn * kN / kRowsPerPass; ++pp) {
            const uint32_t t = (uint32_t)(w * (kOwn * kN) + pp * kRowsPerPass + lane / kLanesPerRow);
            const uint32_t off = t * p.o_row + (uint32_t)((lane % kLanesPerRow) * 16);
            if constexpr (NARROW) {
                narrow_store(ob + off, (uint32_t)((lane % kLanesPerRow) * 16), p.dbytes, u32x4{0u, 0u, 0u, 0u});
                if (MID) narrow_store(mb + off, (uint32_t)((lane % kLanesPerRow) * 16), p.dbytes, u32x4{0u, 0u, 0u, 0u});
            } else {
                __builtin_nontemporal_store(u32x4{0u, 0u, 0u, 0u}, reinterpret_cast<u32x4*>(ob + off));
                if (MID) __builtin_nontemporal_store(u32x4{0u, 0u, 0u, 0u}, reinterpret_cast<u32x4*>(mb + off));
            }
        }
        return;
    }

    // ===== phase A ==================================================================================
    // Loads: 4 lanes per row (16-byte unit ua), 16 rows per pass, 8 passes = this wave's 128 tokens.
    // Both halves of a 128-byte line of Q are requested together (the second waits in registers
    // for the next chunk), so that no line is fetched twice; K, which the other heads of the
    // group read as well, comes 64 bytes per chunk and finds its second half in L2.  The Q loads
    // of the second line are issued in two halves, one after each chunk write of the first line,
    // which keeps the bytes in flight even.
    const int ua = lane & 3, ja = lane >> 2;
    const uint32_t qoff = (uint32_t)(w * (kOwn * kN) + ja) * p.q_row + (uint32_t)(ua * 16);
    const uint32_t koff = (uint32_t)(w * (kOwn * kN) + ja) * p.k_row + (uint32_t)(ua * 16);
    u32x4 q0[8], q1[8], r0[8], r1[8], kreg[8];           // first / second halves of line 0 and of line 1; one chunk of K
    auto load_q = [&](u32x4 (&lo)[8], u32x4 (&hi)[8], int line, int pp_begin, int pp_end) {
#pragma unroll
        for (int pp = pp_begin; pp < pp_end; ++pp) {
            const char* row = qb + (size_t)(16u * pp) * p.q_row + line * 128;
            if constexpr (NARROW) {
                lo[pp] = narrow_load<true>(row + qoff, (uint32_t)(line * 128 + ua * 16), p.dbytes);
                hi[pp] = narrow_load<true>(row + 64 + qoff, (uint32_t)(line * 128 + 64 + ua * 16), p.dbytes);
            } else {
                lo[pp] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row + qoff));
                hi[pp] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row + 64 + qoff));
            }
        }
    };
    auto load_k = [&](int c) {
#pragma unroll
        for (int pp = 0; pp < 8; ++pp)
            if constexpr (NARROW) kreg[pp] = narrow_load<false>(kb + (size_t)(16u * pp) * p.k_row + c * kARow + koff, (uint32_t)(c * kARow + ua * 16), p.dbytes);
            else kreg[pp] = *reinterpret_cast<const u32x4*>(kb + (size_t)(16u * pp) * p.k_row + c * kARow + koff);
    };
    load_q(q0, q1, 0, 0, 8);
    load_k(0);
    __builtin_amdgcn_sched_barrier(0);

    // LDS addresses (see the layout above): what depends on the lane or the wave sits in a few
    // registers, the rest are instruction offsets
    const uint32_t wr_a = (uint32_t)(w * kOwn * kABlock + ja * kARow + ((ua + (lane >> 3)) & 3) * 16);
    uint32_t col_a[4], row_a[2];                          // column fibre j = 4 w + f, step s: col_a[(f >> 1) + 2 s] + f * 64
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) col_a[kk] = (uint32_t)(r32 * kABlock + w * (kOwn * kARow) + ((hf + 2 * w + kk) & 3) * 16);
#pragma unroll
    for (int s = 0; s < 2; ++s)                           // row fibre i = 4 w + f, step s: row_a[s] + f * kABlock
        row_a[s] = (uint32_t)(w * kOwn * kABlock + r32 * kARow + ((hf + (r32 >> 1) + 2 * s) & 3) * 16);

    f32x16 sc[kOwn], sr[kOwn];                            // S^T of the column fibres j = 4 w + f and the row fibres i = 4 w + f
#pragma unroll
    for (int f = 0; f < kOwn; ++f) { sc[f] = f32x16{}; sr[f] = f32x16{}; }
    auto write_chunk = [&](const u32x4 (&qv)[8]) {
#pragma unroll
        for (int pp = 0; pp < 8; ++pp) {
            char* dst = lds + wr_a + (pp >> 1) * kABlock + (pp & 1) * (16 * kARow);
            *reinterpret_cast<u32x4*>(dst) = qv[pp];
            *reinterpret_cast<u32x4*>(dst + kAK) = kreg[pp];
        }
    };
    auto scores = [&](int c) {                            // c: the 32-feature chunk in LDS
        if constexpr (!ROPE) {
#pragma unroll
            for (int f = 0; f < kOwn; ++f)
#pragma unroll
                for (int s = 0; s < kCA / 16; ++s) {
                    const char* ac = lds + col_a[((f >> 1) + 2 * s) & 3] + f * kARow;
                    const char* ar = lds + row_a[s] + f * kABlock;
                    sc[f] = mma(*reinterpret_cast<const u32x4*>(ac + kAK), *reinterpret_cast<const u32x4*>(ac), sc[f]);
                    sr[f] = mma(*reinterpret_cast<const u32x4*>(ar + kAK), *reinterpret_cast<const u32x4*>(ar), sr[f]);
                    __builtin_amdgcn_sched_barrier(0);    // keeps the operand reads from piling up in registers
                }
        } else {
#pragma unroll
            for (int s = 0; s < kCA / 16; ++s) {
                // this lane's operand words of step s are the feature pairs 16 c + 8 s + 4 hf + e of row r32
                bf16x2 ce[4], co[4];                      // (cos, -sin) and (sin, cos) of each pair's angle
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float rate = __builtin_amdgcn_exp2f(p.rope_c0 * (float)(16 * c + 8 * s + 4 * hf + e) + p.rope_c1);
                    const float tt = __builtin_amdgcn_fractf((float)r32 * rate);
                    const float sn = __builtin_amdgcn_sinf(tt), cs = __builtin_amdgcn_cosf(tt);
                    ce[e] = __builtin_bit_cast(bf16x2, pack_bf16x2(cs, -sn));
                    co[e] = __builtin_bit_cast(bf16x2, pack_bf16x2(sn, cs));
                }
                // The three-operand form of the bf16 dot product with a literal zero to add to (the compiler's own
                // choice, the two-operand accumulating form, needs a register cleared first for every product).
                // A dot product's result may be read by another vector instruction only three wait states later,
                // and its register be overwritten by one only four later: the eight products of an operand are
                // issued back to back and one s_nop of four wait states follows the last.
                auto turn = [&](const u32x4 x) {
                    float e0, o0, e1, o1, e2, o2, e3, o3;
                    asm("v_dot2_f32_bf16 %0, %8, %12, 0\n\t"
                        "v_dot2_f32_bf16 %1, %8, %13, 0\n\t"
                        "v_dot2_f32_bf16 %2, %9, %14, 0\n\t"
                        "v_dot2_f32_bf16 %3, %9, %15, 0\n\t"
                        "v_dot2_f32_bf16 %4, %10, %16, 0\n\t"
                        "v_dot2_f32_bf16 %5, %10, %17, 0\n\t"
                        "v_dot2_f32_bf16 %6, %11, %18, 0\n\t"
                        "v_dot2_f32_bf16 %7, %11, %19, 0\n\t"
                        "s_nop 3"
                        : "=&v"(e0), "=&v"(o0), "=&v"(e1), "=&v"(o1), "=&v"(e2), "=&v"(o2), "=&v"(e3), "=&v"(o3)
                        : "v"(x.x), "v"(x.y), "v"(x.z), "v"(x.w),
                          "v"(__builtin_bit_cast(uint32_t, ce[0])), "v"(__builtin_bit_cast(uint32_t, co[0])),
                          "v"(__builtin_bit_cast(uint32_t, ce[1])), "v"(__builtin_bit_cast(uint32_t, co[1])),
                          "v"(__builtin_bit_cast(uint32_t, ce[2])), "v"(__builtin_bit_cast(uint32_t, co[2])),
                          "v"(__builtin_bit_cast(uint32_t, ce[3])), "v"(__builtin_bit_cast(uint32_t, co[3])));
                    return u32x4{pack_bf16x2(e0, o0), pack_bf16x2(e1, o1), pack_bf16x2(e2, o2), pack_bf16x2(e3, o3)};
                };
#pragma unroll
                for (int f = 0; f < kOwn; ++f) {
                    const char* ac = lds + col_a[((f >> 1) + 2 * s) & 3] + f * kARow;
                    const char* ar = lds + row_a[s] + f * kABlock;
                    sc[f] = mma(turn(*reinterpret_cast<const u32x4*>(ac + kAK)), turn(*reinterpret_cast<const u32x4*>(ac)), sc[f]);
                    sr[f] = mma(turn(*reinterpret_cast<const u32x4*>(ar + kAK)), turn(*reinterpret_cast<const u32x4*>(ar)), sr[f]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };
    static_assert(kD == 4 * kCA || kD == 2 * kCA, "one or two 128-byte lines per row");
    write_chunk(q0);                                      // chunk 0
    if constexpr ((ROPE || NARROW) && kD == 4 * kCA) {
        // With the encoding (or narrow rows, read in 8-byte pieces) the score steps need a dozen registers more, and the requests below, as many as the plain kernel
        // keeps in flight, no longer fit: the compiler spilled three of them as they were issued and waited for every load
        // in flight to do so, three times per slab.  Here at most 80 registers of requests are in flight during a score
        // step: Q's second line comes two passes early and six late (both halves of a line still together: requested
        // apart, the second half found its line gone from L2 and fetched it again), and the third K chunk, an L2 hit, is
        // requested only after the second score step.
        __builtin_amdgcn_sched_barrier(0);
        load_k(1);
        load_q(r0, r1, 1, 0, 2);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        scores(0);
        __syncthreads();
        write_chunk(q1);                                  // chunk 1
        load_q(r0, r1, 1, 2, 8);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        scores(1);
        load_k(2);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        write_chunk(r0);                                  // chunk 2
        load_k(3);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        scores(2);
        __syncthreads();
        write_chunk(r1);                                  // chunk 3
    } else {
    load_k(1);
    if (kD == 4 * kCA) load_q(r0, r1, 1, 0, 4);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    scores(0);
    __syncthreads();
    write_chunk(q1);                                      // chunk 1
    if (kD == 4 * kCA) {
        load_k(2);
        load_q(r0, r1, 1, 4, 8);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        scores(1);
        __syncthreads();
        write_chunk(r0);                                  // chunk 2
        load_k(3);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        scores(2);
        __syncthreads();
        write_chunk(r1);                                  // chunk 3
    }
    }

    // value rows of the first phase-B chunk (8 lanes per row (unit ub), 8 rows per pass, 16 passes):
    // half of them are requested here, the other half once the column tiles' accumulators are gone
    const int ub = lane & 7;
    const uint32_t tok_b = (uint32_t)(w * (kOwn * kN) + (lane >> 3));        // + 8 * pass
    u32x4 xreg[16];
    auto load_x = [&](int c, int pp_begin, int pp_end) {
#pragma unroll
        for (int pp = pp_begin; pp < pp_end; ++pp) {
            const uint32_t t = tok_b + 8u * pp;
            const u32x4* src = reinterpret_cast<const u32x4*>(xb + (t * p.v_row + (uint32_t)(c * (kCB * 2) + ub * 16)));
            if constexpr (NARROW) {
                const uint32_t at = (uint32_t)(c * (kCB * 2) + ub * 16);
                xreg[pp] = narrow_load<true>(reinterpret_cast<const char*>(src), at, p.dbytes);   // (a per-group V too: one choice per request would be a branch per request)
            } else {
                xreg[pp] = vin_is_o ? __builtin_nontemporal_load(src) : *src;   // a per-group V is read by every head of the group
            }
        }
    };
    load_x(0, 0, 8);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    scores(kD / kCA - 1);

    // softmax of the 8 tiles; `left` = real (unpadded) tokens from the slab's first token on
    const float sl2 = p.scale * kLog2e;
    const int64_t left = valid_len - tok0;
    u32x4 p1[kOwn][2], p2[kOwn][2];
    float inv1[kOwn], inv2[kOwn];
#pragma unroll
    for (int f = 0; f < kOwn; ++f) {                      // column fibre j = 4 w + f: slab rows i with token 32 i + j < left
        const int64_t room = left - (w * kOwn + f);
        // (the column fibre's number on the outer axis: slab, then column)
        const uint32_t* table = p.mask1 ? p.mask1 + (size_t)(sl * kN + w * kOwn + f) * p.mask1_fibre : nullptr;
        softmax_tile(sc[f], r32, hf, p.causal, p.window1, table, room <= 0 ? 0 : (int)min((int64_t)kN, (room + kN - 1) / kN), sl2, p1[f], inv1[f]);
    }
    load_x(0, 8, 16);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int f = 0; f < kOwn; ++f) {                      // row fibre i = 4 w + f: columns j with token 32 i + j < left
        const int64_t room = left - (int64_t)(w * kOwn + f) * kN;
        const uint32_t* table = p.mask2 ? p.mask2 + (size_t)(sl * kN + w * kOwn + f) * p.mask2_fibre : nullptr;   // (slab, then row)
        softmax_tile(sr[f], r32, hf, p.causal, p.window2, table, room <= 0 ? 0 : (int)min((int64_t)kN, room), sl2, p2[f], inv2[f]);
    }

    // ===== phase B ==================================================================================
    __syncthreads();                                      // phase A's LDS contents are dead
#pragma unroll
    for (int c = 0; c < kD / kCB; ++c) {
        // this wave's rows (i in [4 w, 4 w + 4)) are its own at this point: no barrier before the write
#pragma unroll
        for (int pp = 0; pp < 16; ++pp) {
            const uint32_t t = tok_b + 8u * pp;
            *reinterpret_cast<u32x4*>(lds + ((t >> 5) * kBRowsPerI + (t & 31)) * kBPitch + ub * 16) = xreg[pp];
        }
        if (c + 1 < kD / kCB) { load_x(c + 1, 0, 16); __builtin_amdgcn_sched_barrier(0); }
        __syncthreads();
        // first hop: column fibres j = 4 w + f, rows i = 0..31 one slab row apart
#pragma unroll
        for (int f = 0; f < kOwn; ++f)
            update_fibre(lds, (uint32_t)((w * kOwn + f) * kBPitch), (uint32_t)(kBRowsPerI * kBPitch), p1[f], inv1[f], lane);
        __syncthreads();
        // second hop: row fibres i = 4 w + f, rows j = 0..31 adjacent; then the rows go out
#pragma unroll
        for (int f = 0; f < kOwn; ++f) {
            const uint32_t fb = (uint32_t)((w * kOwn + f) * kBRowsPerI * kBPitch);
            if (MID) {
#pragma unroll
                for (int pp = 0; pp < 4; ++pp) {
                    const uint32_t t = tok_b + (uint32_t)(f * kN + 8 * pp);
                    const u32x4 v = *reinterpret_cast<const u32x4*>(lds + fb + (t & 31) * kBPitch + ub * 16);
                    if constexpr (NARROW) narrow_store(mb + (t * p.o_row + (uint32_t)(c * (kCB * 2) + ub * 16)), (uint32_t)(c * (kCB * 2) + ub * 16), p.dbytes, v);
                    else __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(mb + (t * p.o_row + (uint32_t)(c * (kCB * 2) + ub * 16))));
                }
            }
            update_fibre(lds, fb, (uint32_t)kBPitch, p2[f], inv2[f], lane);
            lds_wave_sync();
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) {
                const uint32_t t = tok_b + (uint32_t)(f * kN + 8 * pp);       // token (i = 4 w + f, j = 8 pp + lane / 8)
                const u32x4 v = *reinterpret_cast<const u32x4*>(lds + fb + (t & 31) * kBPitch + ub * 16);
                if constexpr (NARROW) narrow_store(ob + (t * p.o_row + (uint32_t)(c * (kCB * 2) + ub * 16)), (uint32_t)(c * (kCB * 2) + ub * 16), p.dbytes, v);
                else __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(ob + (t * p.o_row + (uint32_t)(c * (kCB * 2) + ub * 16))));
            }
        }
        lds_wave_sync();                                  // the stores' LDS reads precede the next chunk's writes
    }
}

// The instantiation for a tile width (128 or 64), with or without the intermediate output, narrow rows, the encoding.
template <int kD>
const void* pair_kernel_of_width(bool mid, bool narrow, bool rope) {
    if (rope) return narrow ? (mid ? (const void*)mfma_fwd_pair_kernel<kD, true, true, true> : (const void*)mfma_fwd_pair_kernel<kD, false, true, true>)
                            : (mid ? (const void*)mfma_fwd_pair_kernel<kD, true, false, true> : (const void*)mfma_fwd_pair_kernel<kD, false, false, true>);
    return narrow ? (mid ? (const void*)mfma_fwd_pair_kernel<kD, true, true, false> : (const void*)mfma_fwd_pair_kernel<kD, false, true, false>)
                  : (mid ? (const void*)mfma_fwd_pair_kernel<kD, true, false, false> : (const void*)mfma_fwd_pair_kernel<kD, false, false, false>);
}
const void* pair_kernel_of(bool wide, bool mid, bool narrow, bool rope) {
    return wide ? pair_kernel_of_width<128>(mid, narrow, rope) : pair_kernel_of_width<64>(mid, narrow, rope);
}

bool pair_params(const HopParams& h1, const HopParams& h2, PairParams* pp) {
    if (h1.n != kN || h2.n != kN || h1.D < 8 || h1.D > 128 || h1.D % 4 != 0 || h2.stride != 1 || h1.stride != kN) return false;
    const int64_t N = h1.fibres * h1.n;
    if (!fits_u32(h1.q, kSlab) || !fits_u32(h1.k, kSlab) || !fits_u32(h1.vin, kSlab) || !fits_u32(h1.o, kSlab)) return false;
    if (N % kSlab != 0 || h1.G < 1 || h1.G > 64) return false;
    const int64_t slabs = N / kSlab;
    const int64_t groups = (int64_t)h1.B * slabs * h1.Hkv;
    if (groups > (int64_t)1 << 24) return false;
    pp->q = h1.q; pp->k = h1.k; pp->vin = h1.vin; pp->o = h1.o;
    pp->B = h1.B; pp->Hq = h1.Hq; pp->Hkv = h1.Hkv; pp->G = h1.G; pp->vin_heads = h1.vin_heads; pp->causal = h1.causal;
    pp->scale = h1.scale;
    pp->window1 = h1.window; pp->window2 = h2.window;
    pp->mask1 = h1.mask; pp->mask2 = h2.mask;
    pp->mask1_fibre = (uint32_t)h1.mask_fibre_words; pp->mask2_fibre = (uint32_t)h2.mask_fibre_words;
    pp->valid_len = h1.valid_len;
    pp->valid_lens = h1.valid_lens;
    pp->dbytes = (uint32_t)h1.D * 2;
    pp->rope_c0 = h1.rope_c0; pp->rope_c1 = h1.rope_c1;
    pp->slabs = (uint32_t)slabs;
    pp->groups = (uint32_t)groups;
    pp->q_row = (uint32_t)(h1.q.st * 2); pp->k_row = (uint32_t)(h1.k.st * 2);
    pp->v_row = (uint32_t)(h1.vin.st * 2); pp->o_row = (uint32_t)(h1.o.st * 2);
    return true;
}

}  // namespace

bool mfma_pair_supports(const HopParams& h1, const HopParams& h2, int dtype) {
    PairParams pp;
    return dtype == TA_BF16 && pair_params(h1, h2, &pp);
}

hipError_t launch_mfma_forward_pair(const HopParams& h1, const HopParams& h2, void* o_mid, hipStream_t s) {
    PairParams pp;
    if (!pair_params(h1, h2, &pp)) return hipErrorInvalidValue;
    pp.mid = o_mid;
    const bool wide = h1.D > 64, narrow = h1.D != 64 && h1.D != 128, mid = o_mid != nullptr, rope = h1.rope != 0;
    const void* kf = pair_kernel_of(wide, mid, narrow, rope);
    const hipError_t e = allow_dynamic_lds(kf, kLdsBytes);
    if (e != hipSuccess) return e;
    const uint32_t span = 8u * (uint32_t)pp.G;
    const uint32_t grid = ((pp.groups + 7u) / 8u) * span;
    void* args[1] = {&pp};
    return hipLaunchKernel(kf, dim3(grid), dim3(64 * kWaves), args, kLdsBytes, s);
}

}  // namespace ta
