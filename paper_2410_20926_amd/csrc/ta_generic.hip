// Generic per-axis attention kernels (forward and backward) for gfx950.
//
// These cover every shape the library accepts - any axis length, head width up to 256,
// fp32 or bf16 storage - with fp32 arithmetic on the vector ALUs and a streaming
// (online) softmax over key tiles.  They are the fp32 path and the fallback for shapes
// the MFMA kernels do not take; they are written for clarity, not speed.
//
// One hop follows Eq. 4 of arXiv 2410.20926: for every mode-i fibre (n rows, row pitch
// `stride` tokens) A = softmax(Q_i K_i^T * scale, mask), O_i = A * Vin_i.
#include "ta_internal.h"

namespace ta {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kQB = 16;            // query rows per forward block (4 per wave)

__device__ inline float to_f32(float x) { return x; }
__device__ inline float to_f32(uint16_t x) { return __uint_as_float(((uint32_t)x) << 16); }

__device__ inline void from_f32(float* dst, float x) { *dst = x; }
__device__ inline void from_f32(uint16_t* dst, float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) {            // NaN stays NaN
        *dst = (uint16_t)((u >> 16) | 0x40u);
        return;
    }
    u += 0x7fffu + ((u >> 16) & 1u);                  // round to nearest, ties to even
    *dst = (uint16_t)(u >> 16);
}

__device__ inline float wave_max(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ inline float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

template <typename T>
__device__ inline const T* row_ptr(const Tensor& t, int64_t b, int64_t tok, int64_t h) {
    return reinterpret_cast<const T*>(t.p) + b * t.sb + tok * t.st + h * t.sh;
}
template <typename T>
__device__ inline T* row_ptr_w(const Tensor& t, int64_t b, int64_t tok, int64_t h) {
    return reinterpret_cast<T*>(t.p) + b * t.sb + tok * t.st + h * t.sh;
}

// Rotary encoding inside a hop (Sec. 3.2, per-axis positions): sine and cosine of the angle by
// which feature pair (2 pr, 2 pr + 1) of a row at position a on the hop's axis is turned,
// a * base^(-2 pr / D), formed in double precision.
__device__ inline void rope_angle(const HopParams& p, int a, int pr, double* sn, double* cs) {
    const double ang = (double)a * exp2(-(2.0 * pr / (double)p.D) * (double)p.rope_log2_base);
    sincos(ang, sn, cs);
}

// Element d of a row of Q or K at position a: as stored, or turned when the hop encodes positions.
template <typename T>
__device__ inline float enc_load(const HopParams& p, bool rope, const T* row, int d, int a) {
    const float x = to_f32(row[d]);
    if (!rope) return x;
    const float y = to_f32(row[d ^ 1]);                // the other feature of the pair
    double sn, cs;
    rope_angle(p, a, d >> 1, &sn, &cs);
    return (float)((d & 1) ? (double)y * sn + (double)x * cs : (double)x * cs - (double)y * sn);
}

// A gradient element with respect to a turned row, taken back to the row as stored (the turn's
// transpose): `x` is this lane's element d, the pair's other element sits in lane ^ 1.  Every
// lane of the wave must call it.
__device__ inline float enc_grad(const HopParams& p, float x, int d, int a) {
    if (!p.rope) return x;
    const float y = __shfl_xor(x, 1);
    double sn, cs;
    rope_angle(p, a, d >> 1, &sn, &cs);
    return (float)((d & 1) ? (double)x * cs - (double)y * sn : (double)x * cs + (double)y * sn);
}

// Copy `rows` rows of D elements (row r at token tok0 + (r0 + r) * stride) into an LDS
// tile of pitch `pitch` floats; rows at or past n are zero-filled.  With `rope` (a hop that
// encodes positions, Q and K tiles) every row is turned by its position r0 + r on the axis.
template <typename T>
__device__ inline void load_tile(float* tile, int pitch, int rows, int r0, const Tensor& t,
                                 int64_t b, int64_t tok0, int64_t stride, int64_t h, int n, int D,
                                 const HopParams* rope = nullptr) {
    for (int idx = threadIdx.x; idx < rows * D; idx += kThreads) {
        const int r = idx / D, d = idx - r * D;
        const int a = r0 + r;
        float x = 0.f;
        if (a < n) {
            const T* row = row_ptr<T>(t, b, tok0 + (int64_t)a * stride, h);
            x = rope ? enc_load<T>(*rope, true, row, d, a) : to_f32(row[d]);
        }
        tile[r * pitch + d] = x;
    }
}

// M_i[a][c] of this hop: causal triangle, band of width `window`, the caller's bit table, and
// padding (rows whose token is at or past valid_len neither see nor are seen).
__device__ inline bool visible(const HopParams& p, int64_t tok0, int a, int c) {
    if (p.causal && c > a) return false;
    if (p.window > 0 && (a - c >= p.window || c - a >= p.window)) return false;
    if (p.mask && a < p.n && c < p.n && !((p.mask[(int64_t)a * p.mask_words + (c >> 5)] >> (c & 31)) & 1u)) return false;
    return tok0 + (int64_t)(a > c ? a : c) * p.stride < p.valid_len;
}

// ------------------------------------------------------------------------------------
// Forward.  Block = (batch, query head, fibre, block of 16 query rows); wave w owns rows
// 4w..4w+3 of the block.  Keys are streamed in tiles of TK rows through LDS; lane
// (c, half) forms half of the dot product q_a . k_c, a lane owns output columns
// lane, lane+64, ...
template <typename T>
__global__ __launch_bounds__(kThreads) void generic_forward_kernel(HopParams p, int TK, int qblocks) {
    extern __shared__ float smem[];
    const int D = p.D, n = p.n;
    float* Qs = smem;                       // [kQB][D]
    float* Ks = Qs + kQB * D;               // [TK][D+1]
    float* Vs = Ks + TK * (D + 1);          // [TK][D]

    int64_t bid = blockIdx.x;
    const int qb = (int)(bid % qblocks); bid /= qblocks;
    const int64_t f = bid % p.fibres; bid /= p.fibres;
    const int h = (int)(bid % p.Hq);
    const int b = (int)(bid / p.Hq);
    const int g = h / p.G;
    const int hv = (p.vin_heads == p.Hq) ? h : g;
    const int64_t tok0 = fibre_base_token(f, p.stride, n);
    if (p.mask) p.mask += f * p.mask_fibre_words;          // this fibre's table (the same one when the axis has a single table)
    p.valid_len = hop_valid_len(p, b);                  // this batch element's padding length
    const HopParams* enc = p.rope ? &p : nullptr;       // the hop turns Q and K rows by their position

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int c_l = lane & 31, hh = lane >> 5;
    const int ncol = (D + 63) / 64;
    const int dh = D / 2;

    load_tile<T>(Qs, D, kQB, qb * kQB, p.q, b, tok0, p.stride, h, n, D, enc);

    float m[4], l[4], acc[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        m[r] = -INFINITY; l[r] = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[r][j] = 0.f;
    }
    const int a_last = min(n - 1, qb * kQB + kQB - 1);
    const int kend = p.causal ? a_last + 1 : n;         // keys past the block's last row are masked
    for (int k0 = 0; k0 < kend; k0 += TK) {
        __syncthreads();
        load_tile<T>(Ks, D + 1, TK, k0, p.k, b, tok0, p.stride, g, n, D, enc);
        load_tile<T>(Vs, D, TK, k0, p.vin, b, tok0, p.stride, hv, n, D);
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int a = qb * kQB + w * 4 + r;
            if (a >= n) continue;
            const float* qrow = Qs + (w * 4 + r) * D;
            const float* krow = Ks + c_l * (D + 1);
            float part = 0.f;
            if (c_l < TK)
                for (int d = hh * dh; d < (hh + 1) * dh; ++d) part += qrow[d] * krow[d];
            float s = part + __shfl_xor(part, 32);
            const int c = k0 + c_l;
            const bool valid = (c_l < TK) && (c < n) && visible(p, tok0, a, c);
            s = valid ? s * p.scale : -INFINITY;
            const float tmax = wave_max(s);
            if (tmax == -INFINITY) continue;            // nothing visible in this tile
            const float mn = fmaxf(m[r], tmax);
            const float pr = valid ? expf(s - mn) : 0.f;
            const float corr = expf(m[r] - mn);
            l[r] = l[r] * corr + wave_sum(hh == 0 ? pr : 0.f);
            m[r] = mn;
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[r][j] *= corr;
            for (int cc = 0; cc < TK; ++cc) {
                const float pc = __shfl(pr, cc);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int col = lane + 64 * j;
                    if (j < ncol && col < D) acc[r][j] += pc * Vs[cc * D + col];
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int a = qb * kQB + w * 4 + r;
        if (a >= n) continue;
        T* orow = row_ptr_w<T>(p.o, b, tok0 + (int64_t)a * p.stride, h);
        const float inv = l[r] > 0.f ? 1.f / l[r] : 0.f;   // a padded row sees nothing: zero output
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = lane + 64 * j;
            if (j < ncol && col < D) from_f32(orow + col, acc[r][j] * inv);
        }
    }
}

// ------------------------------------------------------------------------------------
// Backward.  Block = (batch, key/value head, fibre); it walks the G query heads of the
// group so that dK (and dV when the value input is V) are summed inside the block,
// without atomics.
//   Phase A (per head, one query row per wave at a time): recompute the row's softmax
//   statistics and output (as the forward does), delta_a = dO_a . O_a, then
//   dS = A o (dA - delta) and dQ_a = dS K * scale.
//   Phase B (one key per wave at a time): dK_c = sum_h sum_a dS[a,c] q_a * scale and
//   d(value input)_c = sum_a A[a,c] dO_a, using the statistics of phase A.
template <typename T>
__global__ __launch_bounds__(kThreads) void generic_backward_kernel(BwdParams bp, int TK) {
    extern __shared__ float smem[];
    HopParams& p = bp.hop;
    const int D = p.D, n = p.n, G = p.G;
    const int pitch = D + 1;
    float* st_m = smem;                     // [G][n] row max
    float* st_l = st_m + G * n;             // [G][n] row sum
    float* st_d = st_l + G * n;             // [G][n] delta
    float* tA = st_d + G * n;               // [TK][D+1]
    float* tB = tA + TK * pitch;            // [TK][D+1]
    float* rowbuf = tB + TK * pitch;        // [kWaves][2][D]

    int64_t bid = blockIdx.x;
    const int64_t f = bid % p.fibres; bid /= p.fibres;
    const int g = (int)(bid % p.Hkv);
    const int b = (int)(bid / p.Hkv);
    const int64_t tok0 = fibre_base_token(f, p.stride, n);
    if (p.mask) p.mask += f * p.mask_fibre_words;          // this fibre's table (the same one when the axis has a single table)
    const bool vin_is_o = (p.vin_heads == p.Hq);
    p.valid_len = hop_valid_len(p, b);                  // this batch element's padding length
    const HopParams* enc = p.rope ? &p : nullptr;       // the hop turns Q and K rows by their position

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int c_l = lane & 31, hh = lane >> 5;
    const int dh = D / 2;
    float* r0 = rowbuf + (w * 2 + 0) * D;
    float* r1 = rowbuf + (w * 2 + 1) * D;

    // ---------------- phase A ----------------
    for (int hl = 0; hl < G; ++hl) {
        const int h = g * G + hl;
        const int hv = vin_is_o ? h : g;
        for (int rb = 0; rb * kWaves < n; ++rb) {
            const int a = rb * kWaves + w;
            const bool active = a < n;
            __syncthreads();
            if (active) {
                const T* qrow = row_ptr<T>(p.q, b, tok0 + (int64_t)a * p.stride, h);
                const T* grow = row_ptr<T>(bp.d_o, b, tok0 + (int64_t)a * p.stride, h);
                for (int d = lane; d < D; d += 64) { r0[d] = enc_load<T>(p, p.rope != 0, qrow, d, a); r1[d] = to_f32(grow[d]); }
            }
            float m = -INFINITY, l = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
            const int kend = p.causal ? min(n, rb * kWaves + kWaves) : n;
            // pass 1: statistics and the row of O
            for (int k0 = 0; k0 < kend; k0 += TK) {
                __syncthreads();
                load_tile<T>(tA, pitch, TK, k0, p.k, b, tok0, p.stride, g, n, D, enc);
                load_tile<T>(tB, pitch, TK, k0, p.vin, b, tok0, p.stride, hv, n, D);
                __syncthreads();
                if (!active) continue;
                float part = 0.f;
                if (c_l < TK)
                    for (int d = hh * dh; d < (hh + 1) * dh; ++d) part += r0[d] * tA[c_l * pitch + d];
                float s = part + __shfl_xor(part, 32);
                const int c = k0 + c_l;
                const bool valid = (c_l < TK) && (c < n) && visible(p, tok0, a, c);
                s = valid ? s * p.scale : -INFINITY;
                const float tmax = wave_max(s);
                if (tmax == -INFINITY) continue;
                const float mn = fmaxf(m, tmax);
                const float pr = valid ? expf(s - mn) : 0.f;
                const float corr = expf(m - mn);
                l = l * corr + wave_sum(hh == 0 ? pr : 0.f);
                m = mn;
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[j] *= corr;
                for (int cc = 0; cc < TK; ++cc) {
                    const float pc = __shfl(pr, cc);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int col = lane + 64 * j;
                        if (col < D) acc[j] += pc * tB[cc * pitch + col];
                    }
                }
            }
            float delta = 0.f;
            const float invl = l > 0.f ? 1.f / l : 0.f;  // l == 0: a padded row
            if (active) {
                float part = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int col = lane + 64 * j;
                    if (col < D) part += r1[col] * (acc[j] * invl);
                }
                delta = wave_sum(part);
                if (lane == 0) { st_m[hl * n + a] = m; st_l[hl * n + a] = l; st_d[hl * n + a] = delta; }
            }
            // pass 2: dS and dQ_a
            float dqa[4] = {0.f, 0.f, 0.f, 0.f};
            for (int k0 = 0; k0 < kend; k0 += TK) {
                __syncthreads();
                load_tile<T>(tA, pitch, TK, k0, p.k, b, tok0, p.stride, g, n, D, enc);
                load_tile<T>(tB, pitch, TK, k0, p.vin, b, tok0, p.stride, hv, n, D);
                __syncthreads();
                if (!active) continue;
                float ps = 0.f, pa = 0.f;
                if (c_l < TK)
                    for (int d = hh * dh; d < (hh + 1) * dh; ++d) {
                        ps += r0[d] * tA[c_l * pitch + d];
                        pa += r1[d] * tB[c_l * pitch + d];
                    }
                const float s = (ps + __shfl_xor(ps, 32)) * p.scale;
                const float dA = pa + __shfl_xor(pa, 32);
                const int c = k0 + c_l;
                const bool valid = (c_l < TK) && (c < n) && visible(p, tok0, a, c);
                const float pr = valid ? expf(s - m) * invl : 0.f;
                const float dS = valid ? pr * (dA - delta) : 0.f;
                for (int cc = 0; cc < TK; ++cc) {
                    const float x = __shfl(dS, cc);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int col = lane + 64 * j;
                        if (col < D) dqa[j] += x * tA[cc * pitch + col];
                    }
                }
            }
            if (active) {
                T* dqrow = row_ptr_w<T>(bp.dq, b, tok0 + (int64_t)a * p.stride, h);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int col = lane + 64 * j;
                    float x = enc_grad(p, dqa[j] * p.scale, col, a);   // back to the row as stored (all lanes take part)
                    if (col < D) {
                        if (bp.accumulate) x += to_f32(dqrow[col]);
                        from_f32(dqrow + col, x);
                    }
                }
            }
        }
    }

    // ---------------- phase B ----------------
    for (int kb = 0; kb * kWaves < n; ++kb) {
        const int c = kb * kWaves + w;
        const bool active = c < n;
        float accK[4] = {0.f, 0.f, 0.f, 0.f}, accX[4] = {0.f, 0.f, 0.f, 0.f};
        for (int hl = 0; hl < G; ++hl) {
            const int h = g * G + hl;
            const int hv = vin_is_o ? h : g;
            __syncthreads();
            if (active) {
                const T* krow = row_ptr<T>(p.k, b, tok0 + (int64_t)c * p.stride, g);
                const T* xrow = row_ptr<T>(p.vin, b, tok0 + (int64_t)c * p.stride, hv);
                for (int d = lane; d < D; d += 64) { r0[d] = enc_load<T>(p, p.rope != 0, krow, d, c); r1[d] = to_f32(xrow[d]); }
            }
            if (vin_is_o) { accX[0] = accX[1] = accX[2] = accX[3] = 0.f; }
            const int qstart = p.causal ? (kb * kWaves / TK) * TK : 0;   // rows before the block's first key see none of its keys
            for (int q0 = qstart; q0 < n; q0 += TK) {
                __syncthreads();
                load_tile<T>(tA, pitch, TK, q0, p.q, b, tok0, p.stride, h, n, D, enc);
                load_tile<T>(tB, pitch, TK, q0, bp.d_o, b, tok0, p.stride, h, n, D);
                __syncthreads();
                if (!active) continue;
                float ps = 0.f, pa = 0.f;
                if (c_l < TK)
                    for (int d = hh * dh; d < (hh + 1) * dh; ++d) {
                        ps += tA[c_l * pitch + d] * r0[d];
                        pa += tB[c_l * pitch + d] * r1[d];
                    }
                const float s = (ps + __shfl_xor(ps, 32)) * p.scale;
                const float dA = pa + __shfl_xor(pa, 32);
                const int a = q0 + c_l;
                const bool valid = (c_l < TK) && (a < n) && visible(p, tok0, a, c);
                float pr = 0.f, dS = 0.f;
                if (valid) {
                    pr = expf(s - st_m[hl * n + a]) / st_l[hl * n + a];
                    dS = pr * (dA - st_d[hl * n + a]);
                }
                for (int aa = 0; aa < TK; ++aa) {
                    const float xs = __shfl(dS, aa);
                    const float xp = __shfl(pr, aa);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int col = lane + 64 * j;
                        if (col < D) {
                            accK[j] += xs * tA[aa * pitch + col];
                            accX[j] += xp * tB[aa * pitch + col];
                        }
                    }
                }
            }
            if (active && vin_is_o) {
                T* dx = row_ptr_w<T>(bp.d_vin, b, tok0 + (int64_t)c * p.stride, h);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int col = lane + 64 * j;
                    if (col < D) from_f32(dx + col, accX[j]);
                }
            }
        }
        if (active) {
            T* dkrow = row_ptr_w<T>(bp.dk, b, tok0 + (int64_t)c * p.stride, g);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = lane + 64 * j;
                float x = enc_grad(p, accK[j] * p.scale, col, c);     // back to the row as stored (all lanes take part)
                if (col < D) {
                    if (bp.accumulate) x += to_f32(dkrow[col]);
                    from_f32(dkrow + col, x);
                }
            }
            if (!vin_is_o) {
                T* dx = row_ptr_w<T>(bp.d_vin, b, tok0 + (int64_t)c * p.stride, g);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int col = lane + 64 * j;
                    if (col < D) from_f32(dx + col, accX[j]);
                }
            }
        }
    }
}

inline int tile_rows(int D) { return D <= 128 ? 32 : 16; }

}  // namespace

bool generic_forward_supports(const HopParams& p) {
    const int64_t qblocks = (p.n + kQB - 1) / kQB;
    const int64_t per_seq = p.fibres * qblocks;
    return per_seq > 0 && per_seq <= 0x7fffffffLL / ((int64_t)p.B * p.Hq);
}

hipError_t launch_generic_forward(const HopParams& p, int dtype, hipStream_t s) {
    if (!generic_forward_supports(p)) return hipErrorInvalidValue;
    const int TK = tile_rows(p.D);
    const int qblocks = (p.n + kQB - 1) / kQB;
    const int64_t blocks = (int64_t)p.B * p.Hq * p.fibres * qblocks;
    const size_t smem = sizeof(float) * ((size_t)kQB * p.D + (size_t)TK * (p.D + 1) + (size_t)TK * p.D);
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dtype == TA_F32)
        hipLaunchKernelGGL(generic_forward_kernel<float>, dim3((unsigned)blocks), dim3(kThreads), smem, s, p, TK, qblocks);
    else
        hipLaunchKernelGGL(generic_forward_kernel<uint16_t>, dim3((unsigned)blocks), dim3(kThreads), smem, s, p, TK, qblocks);
    return hipGetLastError();
}

static size_t backward_smem(int32_t n, int32_t G, int32_t D) {
    const int TK = tile_rows(D);
    return sizeof(float) * ((size_t)3 * G * n + (size_t)2 * TK * (D + 1) + (size_t)kWaves * 2 * D);
}

bool generic_backward_supports(const HopParams& p) {
    return backward_smem(p.n, p.G, p.D) <= 64 * 1024 && p.fibres > 0 && p.fibres <= 0x7fffffffLL / ((int64_t)p.B * p.Hkv);
}

hipError_t launch_generic_backward(const BwdParams& bp, int dtype, hipStream_t s) {
    const HopParams& p = bp.hop;
    if (!generic_backward_supports(p)) return hipErrorInvalidValue;
    const int TK = tile_rows(p.D);
    const int64_t blocks = (int64_t)p.B * p.Hkv * p.fibres;
    const size_t smem = backward_smem(p.n, p.G, p.D);
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dtype == TA_F32)
        hipLaunchKernelGGL(generic_backward_kernel<float>, dim3((unsigned)blocks), dim3(kThreads), smem, s, bp, TK);
    else
        hipLaunchKernelGGL(generic_backward_kernel<uint16_t>, dim3((unsigned)blocks), dim3(kThreads), smem, s, bp, TK);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// Plain copy: 16 bytes per lane, streaming (non-temporal) loads and stores, four workgroups per
// compute unit walking the buffer 4 KB at a time.  It measures the copy rate the memory reaches
// and calibrates the traffic counters (it moves a known number of bytes).
namespace {
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16) {
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += step)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}
}  // namespace

// A streaming kernel with a given mix of reads and writes: per unit of 4 KB (256 lanes of 16 bytes) it reads R
// blocks and writes W blocks, all loads of a unit in flight together.  It shows what the memory gives a kernel that
// does nothing but move that mix of bytes.
namespace {
template <int R, int W>
__global__ __launch_bounds__(256) void stream_mix_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t units) {
    for (size_t u = blockIdx.x; u < units; u += gridDim.x) {
        u32x4 v[R];
#pragma unroll
        for (int r = 0; r < R; ++r) v[r] = __builtin_nontemporal_load(src + (u * R + r) * 256 + threadIdx.x);
        u32x4 x = v[0];
#pragma unroll
        for (int r = 1; r < R; ++r) x ^= v[r];
#pragma unroll
        for (int w = 0; w < W; ++w) __builtin_nontemporal_store(x + (uint32_t)w, dst + (u * W + w) * 256 + threadIdx.x);
    }
}
template <int R, int W>
hipError_t launch_mix(const void* src, void* dst, size_t units, hipStream_t s) {
    const unsigned blocks = (unsigned)(units < 256 * 16 ? units : 256 * 16);
    hipLaunchKernelGGL((stream_mix_kernel<R, W>), dim3(blocks), dim3(256), 0, s, reinterpret_cast<const u32x4*>(src), reinterpret_cast<u32x4*>(dst), units);
    return hipGetLastError();
}
}  // namespace

hipError_t launch_stream_mix(const void* src, void* dst, size_t units, int reads, int writes, hipStream_t s) {
    if (units == 0) return hipSuccess;
    if (reads == 1 && writes == 1) return launch_mix<1, 1>(src, dst, units, s);
    if (reads == 3 && writes == 2) return launch_mix<3, 2>(src, dst, units, s);
    if (reads == 2 && writes == 1) return launch_mix<2, 1>(src, dst, units, s);
    if (reads == 9 && writes == 4) return launch_mix<9, 4>(src, dst, units, s);
    if (reads == 3 && writes == 1) return launch_mix<3, 1>(src, dst, units, s);
    if (reads == 4 && writes == 3) return launch_mix<4, 3>(src, dst, units, s);
    return hipErrorInvalidValue;
}

// The fused pair's traffic in the pair's access pattern, without its arithmetic (see ta_stream_slabs in the header).
namespace {
constexpr int kSlabTokens = 1024;
constexpr int kRowBytes = 256;

// One workgroup of 256 lanes per (slab, query head); workgroup ids as in the pair kernel: the heads of a key/value
// head are 8 ids apart.  PIECE = 128: 8 lanes per row, a line of every row, then the other line; 256: 16 lanes per row.
template <int PIECE>
__global__ __launch_bounds__(256) void stream_slab_kernel(const char* __restrict__ q, const char* __restrict__ k, const char* __restrict__ x,
                                                          char* __restrict__ o, uint32_t groups, int Hq, int Hkv) {
    const int G = Hq / Hkv;
    const uint32_t span = 8u * (uint32_t)G;
    const uint32_t blk = blockIdx.x / span, rem = blockIdx.x - blk * span;
    const uint32_t hg = rem >> 3, gi = blk * 8u + (rem & 7u);
    if (gi >= groups) return;
    const uint32_t g = gi % (uint32_t)Hkv, sl = gi / (uint32_t)Hkv, h = g * (uint32_t)G + hg;
    const size_t qp = (size_t)Hq * kRowBytes, kp = (size_t)Hkv * kRowBytes;
    const char* qb = q + (size_t)sl * kSlabTokens * qp + (size_t)h * kRowBytes;
    const char* kb = k + (size_t)sl * kSlabTokens * kp + (size_t)g * kRowBytes;
    const char* xb = x + (size_t)sl * kSlabTokens * qp + (size_t)h * kRowBytes;
    char* ob = o + (size_t)sl * kSlabTokens * qp + (size_t)h * kRowBytes;
    constexpr int kLanes = PIECE / 16, kRows = 256 / kLanes, kPieces = kRowBytes / PIECE;
    const int lane = (int)threadIdx.x % kLanes, row0 = (int)threadIdx.x / kLanes;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (int piece = 0; piece < kPieces; ++piece)
        for (int r = row0; r < kSlabTokens; r += 4 * kRows) {
            u32x4 v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(qb + (size_t)(r + kRows * j) * qp + piece * PIECE + lane * 16));
#pragma unroll
            for (int j = 0; j < 4; ++j) acc ^= v[j];
        }
    for (int piece = 0; piece < kPieces; ++piece)
        for (int r = row0; r < kSlabTokens; r += 4 * kRows) {
            u32x4 v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = *reinterpret_cast<const u32x4*>(kb + (size_t)(r + kRows * j) * kp + piece * PIECE + lane * 16);   // shared with the group's other heads through L2
#pragma unroll
            for (int j = 0; j < 4; ++j) acc ^= v[j];
        }
    // a value that is zero whenever q and k are: the loads above cannot be dropped, and o = x then
    const uint32_t fold = acc.x | acc.y | acc.z | acc.w;
    for (int piece = 0; piece < kPieces; ++piece)
        for (int r = row0; r < kSlabTokens; r += 4 * kRows) {
            u32x4 v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xb + (size_t)(r + kRows * j) * qp + piece * PIECE + lane * 16));
#pragma unroll
            for (int j = 0; j < 4; ++j) __builtin_nontemporal_store(v[j] ^ fold, reinterpret_cast<u32x4*>(ob + (size_t)(r + kRows * j) * qp + piece * PIECE + lane * 16));
        }
}

// One workgroup per (slab, key/value head): the whole head group of a token, G * 256 bytes, at once; K once.
__global__ __launch_bounds__(256) void stream_slab_group_kernel(const char* __restrict__ q, const char* __restrict__ k, const char* __restrict__ x,
                                                                char* __restrict__ o, uint32_t groups, int Hq, int Hkv) {
    const uint32_t gi = blockIdx.x;
    if (gi >= groups) return;
    const int G = Hq / Hkv;
    const uint32_t g = gi % (uint32_t)Hkv, sl = gi / (uint32_t)Hkv;
    const size_t qp = (size_t)Hq * kRowBytes, kp = (size_t)Hkv * kRowBytes;
    const size_t gbytes = (size_t)G * kRowBytes;          // bytes of a token's head group
    const char* qb = q + (size_t)sl * kSlabTokens * qp + g * gbytes;
    const char* kb = k + (size_t)sl * kSlabTokens * kp + (size_t)g * kRowBytes;
    const char* xb = x + (size_t)sl * kSlabTokens * qp + g * gbytes;
    char* ob = o + (size_t)sl * kSlabTokens * qp + g * gbytes;
    const uint32_t per_tok = (uint32_t)(gbytes / 16);       // 16-byte units of a token's head group
    const uint32_t units = (uint32_t)kSlabTokens * per_tok;
    u32x4 acc = {0u, 0u, 0u, 0u};
    if (256u % per_tok == 0u) {
        // the usual group sizes (1, 2, 4, 8, 16 heads): a pass of the 256 lanes covers 256 / per_tok whole tokens, eight
        // passes are in flight per lane
        const uint32_t step = 256u / per_tok;
        const uint32_t tok0 = threadIdx.x / per_tok, off = (threadIdx.x % per_tok) * 16u;
        for (uint32_t r = tok0; r < (uint32_t)kSlabTokens; r += 8 * step) {
            u32x4 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(qb + (size_t)(r + j * step) * qp + off));
#pragma unroll
            for (int j = 0; j < 8; ++j) acc ^= v[j];
        }
        for (int r = (int)threadIdx.x / 16; r < kSlabTokens; r += 4 * 16) {
            u32x4 v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kb + (size_t)(r + 16 * j) * kp + ((int)threadIdx.x % 16) * 16));
#pragma unroll
            for (int j = 0; j < 4; ++j) acc ^= v[j];
        }
        const uint32_t fold = acc.x | acc.y | acc.z | acc.w;
        for (uint32_t r = tok0; r < (uint32_t)kSlabTokens; r += 8 * step) {
            u32x4 v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xb + (size_t)(r + j * step) * qp + off));
#pragma unroll
            for (int j = 0; j < 8; ++j) __builtin_nontemporal_store(v[j] ^ fold, reinterpret_cast<u32x4*>(ob + (size_t)(r + j * step) * qp + off));
        }
        return;
    }
    // any other group size: unit u = (token, unit within the group), one unit per lane and trip
    for (uint32_t u = threadIdx.x; u < units; u += 256)
        acc ^= __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(qb + (size_t)(u / per_tok) * qp + (u % per_tok) * 16));
    for (int r = (int)threadIdx.x / 16; r < kSlabTokens; r += 16)
        acc ^= __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kb + (size_t)r * kp + ((int)threadIdx.x % 16) * 16));
    const uint32_t fold = acc.x | acc.y | acc.z | acc.w;
    for (uint32_t u = threadIdx.x; u < units; u += 256) {
        const size_t at = (size_t)(u / per_tok) * qp + (u % per_tok) * 16;
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(xb + at));
        __builtin_nontemporal_store(v ^ fold, reinterpret_cast<u32x4*>(ob + at));
    }
}
}  // namespace

hipError_t launch_stream_slabs(const void* q, const void* k, const void* x, void* o, int64_t tokens, int Hq, int Hkv, int granule, hipStream_t s) {
    if (tokens == 0) return hipSuccess;
    const int64_t groups = tokens / kSlabTokens * Hkv;
    const int G = Hq / Hkv;
    if (groups > (int64_t)1 << 24 || (granule != 3 && ((groups + 7) / 8) * 8 * G > 0x7fffffffLL)) return hipErrorInvalidValue;
    const char* qc = static_cast<const char*>(q);
    const char* kc = static_cast<const char*>(k);
    const char* xc = static_cast<const char*>(x);
    char* oc = static_cast<char*>(o);
    const unsigned grid = (unsigned)(((groups + 7) / 8) * 8 * G);
    if (granule == 1) hipLaunchKernelGGL((stream_slab_kernel<128>), dim3(grid), dim3(256), 0, s, qc, kc, xc, oc, (uint32_t)groups, Hq, Hkv);
    else if (granule == 2) hipLaunchKernelGGL((stream_slab_kernel<256>), dim3(grid), dim3(256), 0, s, qc, kc, xc, oc, (uint32_t)groups, Hq, Hkv);
    else if (granule == 3) hipLaunchKernelGGL(stream_slab_group_kernel, dim3((unsigned)groups), dim3(256), 0, s, qc, kc, xc, oc, (uint32_t)groups, Hq, Hkv);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_copy(const void* src, void* dst, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 4) blocks = 256 * 4;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                       reinterpret_cast<const u32x4*>(src), reinterpret_cast<u32x4*>(dst), n16);
    return hipGetLastError();
}

}  // namespace ta
