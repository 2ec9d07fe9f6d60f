// Tensorized rotary position encoding for gfx950 (arXiv 2410.20926, Sec. 3.2: the position of
// a token is the vector of its tensor coordinates, and rotary embedding is applied with
// per-axis positions).  Elementwise and HBM-bound: one 16-byte chunk per lane, read once,
// written once.  The paper gives no formula; the mechanics are the rotary embedding's own
// (feature pair (2p, 2p+1) of a block of width W turned by pos * base^(-2p/W)) and the choice
// of `pos` per feature is: axis >= 0 - the whole vector uses coordinate j_axis; axis = -1 -
// m consecutive blocks of width 2*floor(D/(2m)), block i using coordinate j_i, the left-over
// features unchanged.
#include "ta_internal.h"

namespace ta {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline float lo_bf16(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float hi_bf16(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ inline uint32_t to_bf16(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Rotation (cos, sin) for feature pair starting at even feature f of token `tok`.
__device__ inline void pair_rotation(const RopeParams& rp, uint32_t tok, int f, float& c, float& s) {
    int axis = rp.axis, width, p;
    if (axis >= 0) {
        width = rp.D & ~1;
        p = f >> 1;
        if (f >= width) { c = 1.f; s = 0.f; return; }
    } else {
        width = 2 * (rp.D / (2 * rp.order));
        axis = width > 0 ? f / width : rp.order;
        if (axis >= rp.order) { c = 1.f; s = 0.f; return; }
        p = (f - axis * width) >> 1;
    }
    const uint32_t pos = (tok / rp.strides[axis]) % rp.dims[axis];
    // angle in double: fp32 would lose ~1e-5 rad at positions in the hundreds
    double ang = (double)pos * exp2(-(2.0 * p / width) * (double)rp.log2_base);
    if (rp.inverse) ang = -ang;
    double sd, cd;
    sincos(ang, &sd, &cd);
    c = (float)cd;
    s = (float)sd;
}

// One work item = one 16-byte chunk position of one token: its rotations are computed once
// and applied to that chunk of every head (the angles do not depend on the head, and their
// double-precision sine and cosine cost far more than the memory traffic of one chunk).
template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(RopeParams rp) {
    constexpr int E = 16 / sizeof(T);                     // features per 16-byte chunk
    constexpr int P = E / 2;                              // rotary pairs per chunk
    constexpr int kBatch = 8;                             // heads in flight per lane
    const int chunks = rp.D / E;                          // D is a multiple of 8
    const uint64_t total = (uint64_t)rp.B * rp.N * chunks;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (uint64_t)gridDim.x * blockDim.x) {
        const int ch = (int)(i % chunks);
        const uint64_t r = i / chunks;
        const uint32_t tok = (uint32_t)(r % rp.N);
        const int b = (int)(r / rp.N);
        float c[P], s[P];
#pragma unroll
        for (int k = 0; k < P; ++k) pair_rotation(rp, tok, ch * E + 2 * k, c[k], s[k]);
        const int64_t off0 = (int64_t)b * rp.x.sb + (int64_t)tok * rp.x.st + ch * E;
        for (int h0 = 0; h0 < rp.H; h0 += kBatch) {
            u32x4 in[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j)
                if (h0 + j < rp.H) in[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(reinterpret_cast<const T*>(rp.x.p) + off0 + (int64_t)(h0 + j) * rp.x.sh));
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                if (h0 + j >= rp.H) continue;
                const uint32_t iw[4] = {in[j].x, in[j].y, in[j].z, in[j].w};
                uint32_t ow[4];
                if (sizeof(T) == 2) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {         // one pair per 32-bit word
                        const float e = lo_bf16(iw[k]), o = hi_bf16(iw[k]);
                        ow[k] = to_bf16(e * c[k % P] - o * s[k % P]) | (to_bf16(e * s[k % P] + o * c[k % P]) << 16);
                    }
                } else {
#pragma unroll
                    for (int k = 0; k < 2; ++k) {         // one pair per two words
                        const float e = __uint_as_float(iw[2 * k]), o = __uint_as_float(iw[2 * k + 1]);
                        ow[2 * k] = __float_as_uint(e * c[k] - o * s[k]);
                        ow[2 * k + 1] = __float_as_uint(e * s[k] + o * c[k]);
                    }
                }
                __builtin_nontemporal_store(u32x4{ow[0], ow[1], ow[2], ow[3]},
                                            reinterpret_cast<u32x4*>(reinterpret_cast<T*>(rp.y.p) + off0 + (int64_t)(h0 + j) * rp.x.sh));
            }
        }
    }
}

}  // namespace

hipError_t launch_rope(const RopeParams& rp, int dtype, hipStream_t s) {
    const uint64_t total = (uint64_t)rp.B * rp.N * (rp.D / (dtype == TA_F32 ? 4 : 8));
    if (total == 0) return hipSuccess;
    uint64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    if (dtype == TA_F32) hipLaunchKernelGGL(rope_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, s, rp);
    else hipLaunchKernelGGL(rope_kernel<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, s, rp);
    return hipGetLastError();
}

}  // namespace ta
