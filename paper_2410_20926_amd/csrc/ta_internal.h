// Internal declarations shared by the host API and the HIP kernel files.
// Nothing here is part of the C ABI (see include/tensattn.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tensattn.h"

namespace ta {

// A strided [B, N, H, D] tensor: element (b, t, h, x) at p + b*sb + t*st + h*sh + x (elements).
struct Tensor {
    void* p;
    int64_t sb, st, sh;
};

// One hop of Eq. 4: attention along one tensor axis, every other axis batched.
struct HopParams {
    Tensor q, k, vin, o;     // forward: o is written.  backward: see BwdParams
    int32_t B, Hq, Hkv, G;   // G = Hq / Hkv
    int32_t D;               // head width
    int32_t n;               // axis length n_i
    int32_t vin_heads;       // Hkv (value input is V) or Hq (value input is a previous O)
    int32_t causal;
    int64_t stride;          // tokens between neighbours along the axis
    int64_t fibres;          // N / n_i
    float scale;
    int32_t window;          // band width on this axis, 0 = none
    int64_t valid_len;       // tokens at or past it are padding; equals N when there is none
    const uint32_t* mask;    // device table of this axis (n rows of mask_words words, bit c of row a = visible) or nullptr
    int32_t mask_words;      // ceil(n / 32)
    int64_t mask_fibre_words;   // words from one fibre's table to the next one's (n * mask_words), or 0: one table for every fibre
    const int64_t* valid_lens;   // device, one padding length per batch element (clamped to [0, N], combined with valid_len), or nullptr
    int64_t N;               // tokens per batch element
    // Rotary encoding inside the hop: Q and K rows are turned by their position a on this axis before
    // the scores, feature pair (2p, 2p+1) by a * base^(-2p/D) radians.
    int32_t rope;            // 0: off
    float rope_c0, rope_c1;  // that angle in REVOLUTIONS is a * exp2(rope_c0 * p + rope_c1)
    float rope_log2_base;    // log2(base), for kernels that form the angle in double precision
};

// Padding length of batch element b: min(valid_len, valid_lens[b]) clamped to [0, N].
__device__ inline int64_t hop_valid_len(const HopParams& p, int b) {
    int64_t v = p.valid_len;
    if (p.valid_lens) {
        const int64_t x = p.valid_lens[b];
        v = x < v ? x : v;
        v = v < 0 ? 0 : v;
    }
    return v;
}

struct BwdParams {
    HopParams hop;           // hop.o is unused
    Tensor d_o;              // upstream gradient, O layout, Hq heads
    Tensor d_vin;            // gradient of the value input, vin layout/heads
    Tensor dq;               // Q layout
    Tensor dk;               // key/value layout
    int32_t accumulate;      // 0: overwrite dq, dk; 1: add
    // set by the MFMA launcher: groups of more than 8 query heads are run 8 heads per launch
    int32_t wg_heads;        // heads (= waves) per workgroup
    int32_t head_base;       // first head of the group this launch covers
    int32_t acc_k, acc_x;    // add to dk / to the group-summed d_vin (every launch after a group's first)
};

// Tensorized rotary position encoding of one [B, N, H, D] tensor (x -> y, same layout).
struct RopeParams {
    Tensor x, y;
    int32_t B, H, D, order;
    uint32_t N;
    uint32_t dims[TA_MAX_ORDER], strides[TA_MAX_ORDER];   // axis lengths and token strides
    int32_t axis;            // 0..order-1: every feature uses that coordinate; -1: one feature block per axis
    int32_t inverse;         // rotate by the negative angle
    float log2_base;
};

// First token of fibre f: fibres enumerate (outer, inner) with inner fastest, so that
// consecutive fibres are neighbouring tokens.
__host__ __device__ inline int64_t fibre_base_token(int64_t f, int64_t stride, int32_t n) {
    const int64_t outer = f / stride;
    const int64_t inner = f - outer * stride;
    return outer * stride * n + inner;
}

enum KernelId : int {
    K_NONE = -1,             // no kernel's launch geometry fits the shape
    K_GENERIC = 0,
    K_MFMA_BF16_N32 = 2,
    K_MFMA_BF16_N64 = 3,
    K_MFMA_BF16_STREAM = 4,
};

// Launchers and their feasibility predicates.  The API layer asks the predicates once, when the
// plan is made, and only launches what they accepted; a launcher repeats its own geometry checks
// and returns hipErrorInvalidValue rather than launch a grid its kernel does not fit.  Each
// launcher returns the hipError_t of the launch.
hipError_t launch_generic_forward(const HopParams& p, int dtype, hipStream_t s);
hipError_t launch_generic_backward(const BwdParams& p, int dtype, hipStream_t s);
bool       generic_forward_supports(const HopParams& p);
bool       generic_backward_supports(const HopParams& p);   // the row statistics fit LDS and the grid fits
hipError_t launch_mfma_forward(const HopParams& p, int kernel_id, hipStream_t s);
hipError_t launch_mfma_forward_stream(const HopParams& p, hipStream_t s);
bool       mfma_forward_supports(int32_t n, int32_t D, int dtype, int* kernel_id);
bool       mfma_forward_layout_ok(const HopParams& p);   // strides and sizes fit the kernel's 32-bit row offsets
bool       mfma_forward_feasible(const HopParams& p, int kernel_id);   // layout_ok and the launch grid fits
bool       mfma_forward_stream_feasible(const HopParams& p);
bool       mfma_backward_supports(const BwdParams& bp, int dtype);
bool       mfma_backward_is_blocked(const BwdParams& bp, int dtype);   // the variant for axes longer than one tile
bool       mfma_backward_is_two_tile(const BwdParams& bp, int dtype);  // the variant for axes of two tiles
hipError_t launch_mfma_backward(const BwdParams& bp, hipStream_t s);
// Fused pair of hops (axes h1 then h2 = the two innermost axes) in one kernel.
bool       mfma_pair_supports(const HopParams& h1, const HopParams& h2, int dtype);
hipError_t launch_mfma_forward_pair(const HopParams& h1, const HopParams& h2, void* o_mid, hipStream_t s);   // o_mid: nullptr or O-shaped, gets h1's output
hipError_t launch_rope(const RopeParams& rp, int dtype, hipStream_t s);
// Allows `kernel` to be launched with up to `bytes` of dynamic LDS (more than 64 KB has to be
// allowed once per device and kernel).  Remembers what it has set; callable from any thread.
hipError_t allow_dynamic_lds(const void* kernel, int bytes);
hipError_t launch_copy(const void* src, void* dst, size_t bytes, hipStream_t s);
// Streaming kernel that reads `reads` and writes `writes` blocks of 4 KB per unit; hipErrorInvalidValue for a mix it has no instantiation for.
hipError_t launch_stream_mix(const void* src, void* dst, size_t units, int reads, int writes, hipStream_t s);
hipError_t launch_stream_slabs(const void* q, const void* k, const void* x, void* o, int64_t tokens, int Hq, int Hkv, int granule, hipStream_t s);

}  // namespace ta
