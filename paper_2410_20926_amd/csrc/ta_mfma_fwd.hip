// bf16 MFMA per-axis attention forward for gfx950 (CDNA4), one hop of Eq. 4 of
// arXiv 2410.20926.
//
// Work unit: one 32-row "tile" of one query head: floor(32 / n) mode-i fibres packed one
// after the other (rows past the last fibre are padding), handled by ONE wavefront with
// no workgroup barrier.  Fibres in a tile never see each other: the mask is block
// diagonal (and lower triangular inside a block for the causal variant).
//
// Per wave:
//   1. gather: rows of Q, K and the value input come from HBM with 16-byte loads, 16
//      lanes per 256-byte row, i.e. fully coalesced whatever the axis stride is;
//   2. Q and K pass through an LDS transit buffer (padded rows) and come back in MFMA
//      operand layout;
//   3. S^T = K Q^T with v_mfma_f32_32x32x16_bf16: the accumulator then holds, per lane,
//      16 of the 32 keys of ONE query row (the other 16 are in lane^32), so the row
//      softmax needs in-lane reductions and a single cross-lane exchange;
//   4. the un-normalised probabilities, rounded to bf16, are already in B-operand
//      layout for O^T = V^T P^T; V goes through LDS with pairs of rows interleaved so
//      that a 32-bit LDS read yields two consecutive keys of one feature column, which
//      is the A-operand layout of V^T;
//   5. O^T is scaled by 1/rowsum in fp32, rounded to bf16, transposed through LDS and
//      stored with 16-byte coalesced stores (fold).
#include "ta_internal.h"

namespace ta {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kWavesPerBlock = 4;
constexpr int kTile = 32;
constexpr float kLog2e = 1.4426950408889634f;

__device__ inline uint32_t bf16_rne(float x) {           // finite inputs only
    uint32_t u = __float_as_uint(x);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ inline uint32_t pack_bf16x2(float lo, float hi) { return bf16_rne(lo) | (bf16_rne(hi) << 16); }

__device__ inline void lds_wave_sync() {
    // LDS operations of one wave complete in issue order; this only stops the compiler
    // from moving shared-memory accesses across the point where lanes exchange data.
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <int D>
struct Geo {
    static constexpr int kChunks = D / 8;                 // 16-byte chunks per row
    static constexpr int kRowsPerPass = 64 / kChunks;     // rows one wave-wide load covers
    static constexpr int kPasses = kTile / kRowsPerPass;  // loads per lane per 32-row tile
    static constexpr int kPitch = D * 2 + 16;             // bytes, Q/K/O transit rows
    static constexpr int kVPitch = D * 4 + 64;            // bytes, one interleaved row pair of V
    static constexpr int kVPasses = (kTile / 2) / kRowsPerPass;
    static constexpr int kKSteps = D / 16;                // MFMA steps over the feature axis
    static constexpr int kDTiles = D / 32;                // 32-column tiles of the output
    static constexpr int kBufBytes = (kTile * kPitch > (kTile / 2) * kVPitch) ? kTile * kPitch : (kTile / 2) * kVPitch;
    static constexpr int kWaveBytes = kBufBytes + kTile * 8;   // + row -> element-offset table
};

// One tile per wave.  `fpt` = fibres per tile, `tiles` = tiles per (batch, head).
template <int D>
__global__ __launch_bounds__(kWavesPerBlock * 64) void mfma_fwd_tile32(HopParams p, int fpt, int64_t tiles, int64_t units) {
    using G = Geo<D>;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int64_t unit = (int64_t)blockIdx.x * kWavesPerBlock + w;
    if (unit >= units) return;                            // no workgroup barrier below

    char* buf = smem + w * G::kWaveBytes;
    int64_t* rowtok = reinterpret_cast<int64_t*>(buf + G::kBufBytes);

    // unit -> (batch, tile, head): heads fastest, so the waves of a block share K
    const int h = (int)(unit % p.Hq);
    const int64_t rest = unit / p.Hq;
    const int64_t tt = rest % tiles;
    const int b = (int)(rest / tiles);
    const int g = h / p.G;
    const int hv = (p.vin_heads == p.Hq) ? h : g;
    const int n = p.n;
    const int64_t f0 = tt * fpt;
    const int nf = (int)min((int64_t)fpt, p.fibres - f0);
    const int rows_valid = nf * n;

    // token of every tile row (lanes 0..31), shared through LDS
    if (lane < kTile) {
        const int fi = lane / n;
        const int a = lane - fi * n;
        int64_t tok = 0;
        if (lane < rows_valid) tok = fibre_base_token(f0 + fi, p.stride, n) + (int64_t)a * p.stride;
        rowtok[lane] = tok;
    }
    lds_wave_sync();

    const uint16_t* qb = reinterpret_cast<const uint16_t*>(p.q.p) + (int64_t)b * p.q.sb + (int64_t)h * p.q.sh;
    const uint16_t* kb = reinterpret_cast<const uint16_t*>(p.k.p) + (int64_t)b * p.k.sb + (int64_t)g * p.k.sh;
    const uint16_t* vb = reinterpret_cast<const uint16_t*>(p.vin.p) + (int64_t)b * p.vin.sb + (int64_t)hv * p.vin.sh;
    uint16_t* ob = reinterpret_cast<uint16_t*>(p.o.p) + (int64_t)b * p.o.sb + (int64_t)h * p.o.sh;

    const int lrow = lane / G::kChunks;                   // row within a pass
    const int lcol = lane % G::kChunks;                   // 16-byte chunk within the row

    // ---- 1. gather Q, K, V rows (all loads issued before any use) ------------------
    uint4 qreg[G::kPasses], kreg[G::kPasses], vreg[2 * G::kVPasses];
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i) {
        const int row = i * G::kRowsPerPass + lrow;
        const int64_t tok = rowtok[row];
        qreg[i] = make_uint4(0, 0, 0, 0);
        kreg[i] = make_uint4(0, 0, 0, 0);
        if (row < rows_valid) {
            qreg[i] = *reinterpret_cast<const uint4*>(qb + tok * p.q.st + lcol * 8);
            kreg[i] = *reinterpret_cast<const uint4*>(kb + tok * p.k.st + lcol * 8);
        }
    }
#pragma unroll
    for (int i = 0; i < G::kVPasses; ++i) {
        const int pr = i * G::kRowsPerPass + lrow;        // row pair
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int row = 2 * pr + e;
            vreg[2 * i + e] = make_uint4(0, 0, 0, 0);
            if (row < rows_valid)
                vreg[2 * i + e] = *reinterpret_cast<const uint4*>(vb + rowtok[row] * p.vin.st + lcol * 8);
        }
    }

    const int r32 = lane & 31;                            // tile row this lane owns in operands
    const int hf = lane >> 5;                             // which 8-wide half of a 16-wide MFMA step

    // ---- 2. Q through LDS into B-operand layout -------------------------------------
    uint4 qop[G::kKSteps], kop[G::kKSteps];
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i)
        *reinterpret_cast<uint4*>(buf + (i * G::kRowsPerPass + lrow) * G::kPitch + lcol * 16) = qreg[i];
    lds_wave_sync();
#pragma unroll
    for (int s = 0; s < G::kKSteps; ++s)
        qop[s] = *reinterpret_cast<const uint4*>(buf + r32 * G::kPitch + (2 * s + hf) * 16);
    lds_wave_sync();
    // ---- K through LDS into A-operand layout ----------------------------------------
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i)
        *reinterpret_cast<uint4*>(buf + (i * G::kRowsPerPass + lrow) * G::kPitch + lcol * 16) = kreg[i];
    lds_wave_sync();
#pragma unroll
    for (int s = 0; s < G::kKSteps; ++s)
        kop[s] = *reinterpret_cast<const uint4*>(buf + r32 * G::kPitch + (2 * s + hf) * 16);
    lds_wave_sync();

    // ---- 3. S^T = K Q^T : acc[r] = S[a = r32][c = 8*(r/4) + 4*hf + r%4] ---------------
    f32x16 st = {};
#pragma unroll
    for (int s = 0; s < G::kKSteps; ++s)
        st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kop[s]), __builtin_bit_cast(bf16x8, qop[s]), st, 0, 0, 0);

    // ---- V through LDS, row pairs interleaved (overlaps the MFMAs above) --------------
#pragma unroll
    for (int i = 0; i < G::kVPasses; ++i) {
        const uint4 x = vreg[2 * i], y = vreg[2 * i + 1];
        const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
        uint32_t o[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            o[2 * j] = (xs[j] & 0xffffu) | (ys[j] << 16);
            o[2 * j + 1] = (xs[j] >> 16) | (ys[j] & 0xffff0000u);
        }
        char* dst = buf + (i * G::kRowsPerPass + lrow) * G::kVPitch + lcol * 32;
        *reinterpret_cast<uint4*>(dst) = make_uint4(o[0], o[1], o[2], o[3]);
        *reinterpret_cast<uint4*>(dst + 16) = make_uint4(o[4], o[5], o[6], o[7]);
    }
    lds_wave_sync();

    // ---- 4. masked row softmax --------------------------------------------------------
    // keys visible to query row r32: its own fibre's rows, up to itself when causal
    uint32_t vis = 0;
    if (r32 < rows_valid) {
        const int fi = r32 / n;
        const int lo = fi * n;
        const int hi = p.causal ? r32 + 1 : lo + n;
        vis = (hi >= 32 ? 0xffffffffu : ((1u << hi) - 1u)) & ~((1u << lo) - 1u);
    }
    const uint32_t vish = vis >> (4 * hf);
    const float sl2 = p.scale * kLog2e;
    float mx = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const bool ok = (vish >> (8 * (r / 4) + (r % 4))) & 1u;
        st[r] = ok ? st[r] * sl2 : -INFINITY;
        mx = fmaxf(mx, st[r]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    if (mx == -INFINITY) mx = 0.f;                        // padding rows: everything masked
    uint32_t pop[2][4];                                   // P^T as two B operands (16 keys each)
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
        const float e0 = __builtin_amdgcn_exp2f(st[r] - mx);
        const float e1 = __builtin_amdgcn_exp2f(st[r + 1] - mx);
        const uint32_t pk = pack_bf16x2(e0, e1);
        sum += __uint_as_float(pk << 16) + __uint_as_float(pk & 0xffff0000u);
        pop[r / 8][(r % 8) / 2] = pk;
    }
    sum += __shfl_xor(sum, 32);
    const float inv = sum > 0.f ? 1.f / sum : 0.f;

    // ---- O^T = V^T P^T ------------------------------------------------------------------
    f32x16 ot[G::kDTiles];
#pragma unroll
    for (int t = 0; t < G::kDTiles; ++t) {
        ot[t] = f32x16{};
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            uint32_t a[4];
#pragma unroll
            for (int jp = 0; jp < 4; ++jp) {
                const int cp = 8 * s2 + 4 * (jp / 2) + 2 * hf + (jp % 2);      // row pair holding keys c, c+1
                a[jp] = *reinterpret_cast<const uint32_t*>(buf + cp * G::kVPitch + (32 * t + r32) * 4);
            }
            const uint4 av = make_uint4(a[0], a[1], a[2], a[3]);
            const uint4 bv = make_uint4(pop[s2][0], pop[s2][1], pop[s2][2], pop[s2][3]);
            ot[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, bv), ot[t], 0, 0, 0);
        }
    }
    lds_wave_sync();

    // ---- 5. normalise, round, transpose through LDS, store -------------------------------
#pragma unroll
    for (int t = 0; t < G::kDTiles; ++t)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            uint2 v;
            v.x = pack_bf16x2(ot[t][4 * q4] * inv, ot[t][4 * q4 + 1] * inv);
            v.y = pack_bf16x2(ot[t][4 * q4 + 2] * inv, ot[t][4 * q4 + 3] * inv);
            *reinterpret_cast<uint2*>(buf + r32 * G::kPitch + (32 * t + 8 * q4 + 4 * hf) * 2) = v;
        }
    lds_wave_sync();
#pragma unroll
    for (int i = 0; i < G::kPasses; ++i) {
        const int row = i * G::kRowsPerPass + lrow;
        if (row < rows_valid) {
            const uint4 v = *reinterpret_cast<const uint4*>(buf + row * G::kPitch + lcol * 16);
            *reinterpret_cast<uint4*>(ob + rowtok[row] * p.o.st + lcol * 8) = v;
        }
    }
}

}  // namespace

bool mfma_forward_supports(int32_t n, int32_t D, int dtype, int* kernel_id) {
    int kid = K_GENERIC;
    if (dtype == TA_BF16 && (D == 64 || D == 128) && n >= 1 && n <= 32) kid = K_MFMA_BF16_N32;
    if (kernel_id) *kernel_id = kid;
    return kid != K_GENERIC;
}

hipError_t launch_mfma_forward(const HopParams& p, int kernel_id, hipStream_t s) {
    if (kernel_id != K_MFMA_BF16_N32 || p.n < 1 || p.n > kTile || (p.D != 64 && p.D != 128)) return hipErrorInvalidValue;
    const int fpt = kTile / p.n;
    const int64_t tiles = (p.fibres + fpt - 1) / fpt;
    const int64_t units = (int64_t)p.B * p.Hq * tiles;
    const int64_t blocks = (units + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (p.D == 128) {
        const size_t smem = (size_t)kWavesPerBlock * Geo<128>::kWaveBytes;
        hipLaunchKernelGGL(mfma_fwd_tile32<128>, dim3((unsigned)blocks), dim3(kWavesPerBlock * 64), smem, s, p, fpt, tiles, units);
    } else {
        const size_t smem = (size_t)kWavesPerBlock * Geo<64>::kWaveBytes;
        hipLaunchKernelGGL(mfma_fwd_tile32<64>, dim3((unsigned)blocks), dim3(kWavesPerBlock * 64), smem, s, p, fpt, tiles, units);
    }
    return hipGetLastError();
}

}  // namespace ta
