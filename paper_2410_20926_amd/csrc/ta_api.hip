// Host side of the C ABI declared in include/tensattn.h: plan construction and
// validation, the cost model, argument checks, and the per-hop / multi-hop drivers.
// All device work happens in the kernel files; this file only enqueues launches.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>

#include "ta_internal.h"

struct ta_plan {
    ta_desc_t desc;              // as given, with defaults resolved
    int32_t order;
    int32_t dims[TA_MAX_ORDER];
    int64_t strides[TA_MAX_ORDER];   // token stride per axis (row-major reshape)
    int32_t hop_axis[TA_MAX_ORDER];  // axis executed at each hop position
    int64_t N;
    int32_t G;
    int32_t elem;                // bytes per element
    float scale;
    int64_t qs[3], kvs[3], os[3];    // resolved element strides (batch, token, head)
    int64_t o_span;              // elements from the first to one past the last element of an O tensor
    size_t o_buf_bytes;          // bytes of one inter-hop O buffer, rounded up to 256
    // decisions per (axis, value-input kind), made once in ta_plan_create so that no call
    // can fail on geometry after an earlier hop has been enqueued
    int kernel_id[TA_MAX_ORDER][2];  // forward kernel (ta::KernelId), or ta::K_NONE when no kernel's grid fits
    int bwd_id[TA_MAX_ORDER][2];     // backward variant (BwdId)
    bool pair[TA_MAX_ORDER][2];      // the fused pair (axis, axis + 1) is available
};

// Workspace of ta_multihop_forward_static: device memory that belongs to the library's code
// object, one copy per GPU, present from the moment the library is loaded on that GPU until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[TA_STATIC_WORKSPACE_BYTES];

namespace {

// Device address of `scratch` on the current device, looked up once per device.
ta_status_t static_workspace(void** out) {
    static std::mutex mu;
    static void* ptr[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return TA_ERR_DEVICE;
    if (dev < 0 || dev >= 64) return TA_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return TA_ERR_DEVICE;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return TA_OK;
}

enum BwdId : int { BWD_NONE = 0, BWD_MFMA_N32 = 1, BWD_MFMA_BLOCKED = 2, BWD_GENERIC = 3, BWD_MFMA_N64 = 4 };

thread_local char g_detail[256] = "";

ta_status_t fail(ta_status_t st, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
ta_status_t fail(ta_status_t st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_detail, sizeof(g_detail), fmt, ap);
    va_end(ap);
    return st;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Byte range [lo, hi) touched by a strided [B, N, H, D] tensor.
struct Range { uintptr_t lo, hi; };
Range span_of(const void* p, const int64_t s[3], int64_t B, int64_t N, int64_t H, int64_t D, int elem) {
    const int64_t last = (B - 1) * s[0] + (N - 1) * s[1] + (H - 1) * s[2] + D;
    const uintptr_t lo = reinterpret_cast<uintptr_t>(p);
    return {lo, lo + (uintptr_t)last * (uintptr_t)elem};
}
inline bool overlaps(Range a, Range b) { return a.lo < b.hi && b.lo < a.hi; }

bool strides_ok(const int64_t s[3], int64_t B, int64_t N, int64_t H, int64_t D) {
    // every stride positive, a multiple of 8 elements (16-byte rows; of 4 when the head width is only a
    // multiple of 4, whose rows the kernels read in 8-byte pieces; of 2 otherwise: generic kernels only), rows disjoint:
    // sort the three (stride, extent) pairs and require stride_k >= extent_{k-1} * stride_{k-1}.
    int64_t st[3] = {s[0], s[1], s[2]};
    int64_t ex[3] = {B, N, H};
    for (int i = 0; i < 3; ++i)
        if (st[i] <= 0 || (st[i] % (D % 8 == 0 ? 8 : D % 4 == 0 ? 4 : 2)) != 0) return false;
    for (int i = 0; i < 3; ++i)                           // the tensor's span in elements stays far below 2^63
        if (st[i] > ((int64_t)1 << 56) / ex[i]) return false;
    for (int i = 0; i < 3; ++i)
        for (int j = i + 1; j < 3; ++j)
            if (st[j] < st[i]) { int64_t t = st[i]; st[i] = st[j]; st[j] = t; t = ex[i]; ex[i] = ex[j]; ex[j] = t; }
    int64_t need = D;
    for (int i = 0; i < 3; ++i) {
        if (ex[i] > 1 && st[i] < need) return false;
        need = st[i] * ex[i];
    }
    return true;
}

void resolve_strides(const int64_t in[3], int64_t out[3], int64_t N, int64_t H, int64_t D) {
    if (in[0] == 0 && in[1] == 0 && in[2] == 0) {
        out[2] = D; out[1] = H * D; out[0] = N * H * D;
    } else {
        out[0] = in[0]; out[1] = in[1]; out[2] = in[2];
    }
}

ta::Tensor make_tensor(const void* p, const int64_t s[3]) {
    return ta::Tensor{const_cast<void*>(p), s[0], s[1], s[2]};
}

ta::HopParams hop_params(const ta_plan* pl, int axis, const void* q, const void* k, const void* vin,
                         int vin_kind, void* o) {
    ta::HopParams hp;
    hp.q = make_tensor(q, pl->qs);
    hp.k = make_tensor(k, pl->kvs);
    hp.vin = make_tensor(vin, vin_kind == TA_VIN_KV ? pl->kvs : pl->os);
    hp.o = make_tensor(o, pl->os);
    hp.B = pl->desc.batch; hp.Hq = pl->desc.n_q_heads; hp.Hkv = pl->desc.n_kv_heads; hp.G = pl->G;
    hp.D = pl->desc.head_dim;
    hp.n = pl->dims[axis];
    hp.vin_heads = vin_kind == TA_VIN_KV ? pl->desc.n_kv_heads : pl->desc.n_q_heads;
    hp.causal = pl->desc.causal;
    hp.stride = pl->strides[axis];
    hp.fibres = pl->N / pl->dims[axis];
    hp.scale = pl->scale;
    hp.window = pl->desc.window[axis];
    hp.valid_len = pl->desc.valid_len > 0 ? pl->desc.valid_len : pl->N;
    hp.mask = static_cast<const uint32_t*>(pl->desc.axis_mask[axis]);
    hp.mask_words = (pl->dims[axis] + 31) / 32;
    hp.mask_fibre_words = (hp.mask && pl->desc.axis_mask_per_fibre[axis]) ? (int64_t)pl->dims[axis] * hp.mask_words : 0;
    hp.valid_lens = pl->desc.valid_lens;
    hp.N = pl->N;
    hp.rope = pl->desc.rope;
    // pair p of a row at position a turns by a * base^(-2p/D) radians = a * exp2(c0 * p + c1) revolutions
    const double log2_base = log2(pl->desc.rope_base > 0.f ? (double)pl->desc.rope_base : 10000.0);
    hp.rope_log2_base = (float)log2_base;
    hp.rope_c0 = (float)(-2.0 * log2_base / (double)pl->desc.head_dim);
    hp.rope_c1 = (float)(-log2(2.0 * M_PI));
    return hp;
}

ta::BwdParams bwd_params(const ta_plan* pl, int axis, const void* q, const void* k, const void* vin, int vin_kind,
                         const void* d_o, void* d_vin, void* dq, void* dk, int accumulate) {
    ta::BwdParams bp;
    bp.hop = hop_params(pl, axis, q, k, vin, vin_kind, nullptr);
    bp.d_o = make_tensor(d_o, pl->os);
    bp.d_vin = make_tensor(d_vin, vin_kind == TA_VIN_KV ? pl->kvs : pl->os);
    bp.dq = make_tensor(dq, pl->qs);
    bp.dk = make_tensor(dk, pl->kvs);
    bp.accumulate = accumulate;
    bp.wg_heads = 0; bp.head_base = 0; bp.acc_k = 0; bp.acc_x = 0;
    return bp;
}

// Byte ranges of the plan's tensor kinds.
Range q_span(const ta_plan* pl, const void* p) {
    return span_of(p, pl->qs, pl->desc.batch, pl->N, pl->desc.n_q_heads, pl->desc.head_dim, pl->elem);
}
Range kv_span(const ta_plan* pl, const void* p) {
    return span_of(p, pl->kvs, pl->desc.batch, pl->N, pl->desc.n_kv_heads, pl->desc.head_dim, pl->elem);
}
Range o_span(const ta_plan* pl, const void* p) {
    return span_of(p, pl->os, pl->desc.batch, pl->N, pl->desc.n_q_heads, pl->desc.head_dim, pl->elem);
}
Range vin_span(const ta_plan* pl, const void* p, int vin) { return vin == TA_VIN_KV ? kv_span(pl, p) : o_span(pl, p); }

const char* forward_kernel_name(const ta_plan* pl, int axis, int vin) {
    switch (pl->kernel_id[axis][vin]) {
        case ta::K_NONE: return "unsupported";
        case ta::K_GENERIC: return "generic";
        // with 4 (or a multiple of 4) query heads per key/value head the group-shared variant runs;
        // its instantiation that also shares the value tile (value input per key/value head) is "_kv"
        case ta::K_MFMA_BF16_N32: return pl->G % 4 != 0 ? "mfma_bf16_n32" : vin == TA_VIN_KV ? "mfma_bf16_n32_shared_kv" : "mfma_bf16_n32_shared";
        case ta::K_MFMA_BF16_N64: return pl->G % 4 != 0 ? "mfma_bf16_n64" : vin == TA_VIN_KV ? "mfma_bf16_n64_shared_kv" : "mfma_bf16_n64_shared";
        case ta::K_MFMA_BF16_STREAM: return pl->G % 4 != 0 ? "mfma_bf16_stream" : vin == TA_VIN_KV ? "mfma_bf16_stream_shared_kv" : "mfma_bf16_stream_shared";
    }
    return nullptr;
}

// The enqueue steps proper.  Arguments have been validated by the caller; the only failure left
// is HIP refusing the launch.
ta_status_t enqueue_forward(const ta_plan* pl, int axis, const void* q, const void* k, const void* v_in, int vin,
                            void* o_out, hipStream_t stream) {
    const ta::HopParams hp = hop_params(pl, axis, q, k, v_in, vin, o_out);
    const int kid = pl->kernel_id[axis][vin];
    const hipError_t e = kid == ta::K_GENERIC ? ta::launch_generic_forward(hp, pl->desc.dtype, stream)
                                              : ta::launch_mfma_forward(hp, kid, stream);
    if (e != hipSuccess) return fail(TA_ERR_DEVICE, "forward launch failed (axis %d): %s", axis, hipGetErrorString(e));
    return TA_OK;
}

ta_status_t enqueue_pair(const ta_plan* pl, int axis, const void* q, const void* k, const void* v_in, int vin,
                         void* o_mid, void* o_out, hipStream_t stream) {
    const ta::HopParams h1 = hop_params(pl, axis, q, k, v_in, vin, o_out);
    const ta::HopParams h2 = hop_params(pl, axis + 1, q, k, v_in, vin, o_out);
    const hipError_t e = ta::launch_mfma_forward_pair(h1, h2, o_mid, stream);
    if (e != hipSuccess) return fail(TA_ERR_DEVICE, "fused forward launch failed (axes %d, %d): %s", axis, axis + 1, hipGetErrorString(e));
    return TA_OK;
}

ta_status_t enqueue_backward(const ta_plan* pl, int axis, const void* q, const void* k, const void* v_in, int vin,
                             const void* d_o, void* d_v_in, void* dq, void* dk, int accumulate, hipStream_t stream) {
    const ta::BwdParams bp = bwd_params(pl, axis, q, k, v_in, vin, d_o, d_v_in, dq, dk, accumulate);
    const int id = pl->bwd_id[axis][vin];
    const hipError_t e = id == BWD_GENERIC ? ta::launch_generic_backward(bp, pl->desc.dtype, stream)
                                           : ta::launch_mfma_backward(bp, stream);
    if (e != hipSuccess) return fail(TA_ERR_DEVICE, "backward launch failed (axis %d): %s", axis, hipGetErrorString(e));
    return TA_OK;
}

ta_status_t unsupported_forward(const ta_plan* pl, int axis) {
    return fail(TA_ERR_UNSUPPORTED, "forward: no kernel's launch grid fits axis %d (length %d) of this plan", axis, pl->dims[axis]);
}
ta_status_t unsupported_backward(const ta_plan* pl, int axis) {
    return fail(TA_ERR_UNSUPPORTED, "backward: axis %d of length %d with %d heads per group exceeds every kernel's limit",
                axis, pl->dims[axis], pl->G);
}

ta_status_t check_axis_vin(const ta_plan* pl, int axis, int vin) {
    if (!pl) return fail(TA_ERR_NULL, "plan is NULL");
    if (axis < 0 || axis >= pl->order) return fail(TA_ERR_INVALID_ARG, "axis %d out of range [0, %d)", axis, pl->order);
    if (vin != TA_VIN_KV && vin != TA_VIN_O) return fail(TA_ERR_INVALID_ARG, "vin must be TA_VIN_KV or TA_VIN_O");
    return TA_OK;
}

}  // namespace

extern "C" {

const char* ta_status_string(ta_status_t st) {
    switch (st) {
        case TA_OK: return "TA_OK";
        case TA_ERR_NULL: return "TA_ERR_NULL";
        case TA_ERR_INVALID_ARG: return "TA_ERR_INVALID_ARG";
        case TA_ERR_SHAPE: return "TA_ERR_SHAPE";
        case TA_ERR_UNSUPPORTED: return "TA_ERR_UNSUPPORTED";
        case TA_ERR_ALIAS: return "TA_ERR_ALIAS";
        case TA_ERR_WORKSPACE: return "TA_ERR_WORKSPACE";
        case TA_ERR_DEVICE: return "TA_ERR_DEVICE";
        case TA_ERR_NOMEM: return "TA_ERR_NOMEM";
    }
    return "TA_ERR_?";
}

const char* ta_last_error_detail(void) { return g_detail; }

void ta_version(int* major, int* minor) {
    if (major) *major = 0;
    if (minor) *minor = 7;
}

ta_status_t ta_plan_create(const ta_desc_t* d, ta_plan_t** out) {
    g_detail[0] = 0;
    if (!d || !out) return fail(TA_ERR_NULL, "desc or out_plan is NULL");
    *out = nullptr;
    if (d->order < 1 || d->order > TA_MAX_ORDER) return fail(TA_ERR_SHAPE, "order %d not in 1..%d", d->order, TA_MAX_ORDER);
    if (d->batch < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->head_dim < 1)
        return fail(TA_ERR_SHAPE, "batch, head counts and head_dim must be >= 1");
    if (d->n_q_heads % d->n_kv_heads != 0)
        return fail(TA_ERR_SHAPE, "n_q_heads %d is not a multiple of n_kv_heads %d", d->n_q_heads, d->n_kv_heads);
    if (d->dtype != TA_F32 && d->dtype != TA_BF16) return fail(TA_ERR_INVALID_ARG, "unknown dtype %d", d->dtype);
    if (d->causal != 0 && d->causal != 1) return fail(TA_ERR_INVALID_ARG, "causal must be 0 or 1");
    if (!(d->scale >= 0.f) || isinf(d->scale)) return fail(TA_ERR_INVALID_ARG, "scale must be finite and >= 0");
    int64_t N = 1;
    for (int i = 0; i < d->order; ++i) {
        if (d->dims[i] < 1) return fail(TA_ERR_SHAPE, "dims[%d] = %d < 1", i, d->dims[i]);
        if ((int64_t)d->dims[i] > ((int64_t)1 << 40) / N) return fail(TA_ERR_SHAPE, "sequence length exceeds 2^40 tokens");
        N *= d->dims[i];
    }
    for (int i = 0; i < d->order; ++i)
        if (d->window[i] < 0) return fail(TA_ERR_INVALID_ARG, "window[%d] = %d is negative", i, d->window[i]);
    for (int i = 0; i < d->order; ++i)
        if (reinterpret_cast<uintptr_t>(d->axis_mask[i]) % 4 != 0) return fail(TA_ERR_INVALID_ARG, "axis_mask[%d] is not 4-byte aligned", i);
    if (reinterpret_cast<uintptr_t>(d->valid_lens) % 8 != 0) return fail(TA_ERR_INVALID_ARG, "valid_lens is not 8-byte aligned");
    if (d->rope != 0 && d->rope != 1) return fail(TA_ERR_INVALID_ARG, "rope must be 0 or 1");
    for (int i = 0; i < d->order && i < TA_MAX_ORDER; ++i)
        if (d->axis_mask_per_fibre[i] != 0 && d->axis_mask_per_fibre[i] != 1)
            return fail(TA_ERR_INVALID_ARG, "axis_mask_per_fibre entries must be 0 or 1");
    if (!(d->rope_base >= 0.f) || isinf(d->rope_base)) return fail(TA_ERR_INVALID_ARG, "rope_base must be finite and >= 0");
    if (d->valid_len < 0) return fail(TA_ERR_INVALID_ARG, "valid_len is negative");
    if (d->valid_len > N) return fail(TA_ERR_SHAPE, "valid_len %lld exceeds the sequence length %lld", (long long)d->valid_len, (long long)N);
    if (d->head_dim % 2 != 0 || d->head_dim > 256)
        return fail(TA_ERR_UNSUPPORTED, "head_dim %d: need an even width, at most 256", d->head_dim);

    ta_plan* pl = new (std::nothrow) ta_plan;
    if (!pl) return fail(TA_ERR_NOMEM, "out of host memory");
    memset(pl, 0, sizeof(*pl));
    pl->desc = *d;
    pl->order = d->order;
    pl->N = N;
    pl->G = d->n_q_heads / d->n_kv_heads;
    pl->elem = d->dtype == TA_F32 ? 4 : 2;
    pl->scale = d->scale > 0.f ? d->scale : (float)(1.0 / sqrt((double)d->head_dim));
    for (int i = 0; i < d->order; ++i) pl->dims[i] = d->dims[i];
    pl->strides[d->order - 1] = 1;
    for (int i = d->order - 2; i >= 0; --i) pl->strides[i] = pl->strides[i + 1] * pl->dims[i + 1];

    // hop order: all -1 = Algorithm 1's order, else a permutation of the axes
    bool all_default = true;
    for (int i = 0; i < d->order; ++i) all_default = all_default && d->hop_order[i] == -1;
    if (all_default) {
        for (int i = 0; i < d->order; ++i) pl->hop_axis[i] = i;
    } else {
        bool seen[TA_MAX_ORDER] = {false};
        for (int i = 0; i < d->order; ++i) {
            const int a = d->hop_order[i];
            if (a < 0 || a >= d->order || seen[a]) {
                delete pl;
                return fail(TA_ERR_INVALID_ARG, "hop_order is not a permutation of 0..%d", d->order - 1);
            }
            seen[a] = true;
            pl->hop_axis[i] = a;
        }
    }

    const int64_t D = d->head_dim;
    resolve_strides(d->q_strides, pl->qs, N, d->n_q_heads, D);
    resolve_strides(d->kv_strides, pl->kvs, N, d->n_kv_heads, D);
    resolve_strides(d->o_strides, pl->os, N, d->n_q_heads, D);
    if (!strides_ok(pl->qs, d->batch, N, d->n_q_heads, D) || !strides_ok(pl->kvs, d->batch, N, d->n_kv_heads, D) ||
        !strides_ok(pl->os, d->batch, N, d->n_q_heads, D)) {
        delete pl;
        return fail(TA_ERR_SHAPE, "strides must be positive multiples of 8 elements (of 4 or 2 when head_dim is only a multiple of 4 or 2) describing non-overlapping rows");
    }
    pl->o_span = (d->batch - 1) * pl->os[0] + (N - 1) * pl->os[1] + (d->n_q_heads - 1) * pl->os[2] + D;
    pl->o_buf_bytes = (((size_t)pl->o_span * pl->elem) + 255) & ~(size_t)255;

    // every per-hop decision is taken here, against the launchers' own feasibility predicates
    for (int i = 0; i < d->order; ++i)
        for (int vin = 0; vin < 2; ++vin) {
            const ta::HopParams hp = hop_params(pl, i, nullptr, nullptr, nullptr, vin, nullptr);
            int kid = ta::K_GENERIC;
            ta::mfma_forward_supports(pl->dims[i], d->head_dim, d->dtype, &kid);
            if (kid != ta::K_GENERIC && !ta::mfma_forward_feasible(hp, kid)) kid = ta::K_GENERIC;
            if (kid == ta::K_GENERIC && !ta::generic_forward_supports(hp)) kid = ta::K_NONE;
            pl->kernel_id[i][vin] = kid;
            const ta::BwdParams bp = bwd_params(pl, i, nullptr, nullptr, nullptr, vin, nullptr, nullptr, nullptr, nullptr, 0);
            if (ta::mfma_backward_supports(bp, d->dtype))
                pl->bwd_id[i][vin] = ta::mfma_backward_is_blocked(bp, d->dtype) ? BWD_MFMA_BLOCKED
                                   : ta::mfma_backward_is_two_tile(bp, d->dtype) ? BWD_MFMA_N64 : BWD_MFMA_N32;
            else
                pl->bwd_id[i][vin] = ta::generic_backward_supports(hp) ? BWD_GENERIC : BWD_NONE;
            pl->pair[i][vin] = false;
            if (i + 1 < d->order) {
                const ta::HopParams h2 = hop_params(pl, i + 1, nullptr, nullptr, nullptr, vin, nullptr);
                pl->pair[i][vin] = ta::mfma_pair_supports(hp, h2, d->dtype);
            }
        }
    *out = pl;
    return TA_OK;
}

void ta_plan_destroy(ta_plan_t* pl) { delete pl; }

int64_t ta_plan_seq_len(const ta_plan_t* pl) { return pl ? pl->N : -1; }
int64_t ta_plan_axis_stride(const ta_plan_t* pl, int axis) {
    return (pl && axis >= 0 && axis < pl->order) ? pl->strides[axis] : -1;
}
int64_t ta_plan_axis_fibres(const ta_plan_t* pl, int axis) {
    return (pl && axis >= 0 && axis < pl->order) ? pl->N / pl->dims[axis] : -1;
}
int ta_plan_hop_axis(const ta_plan_t* pl, int pos) {
    return (pl && pos >= 0 && pos < pl->order) ? pl->hop_axis[pos] : -1;
}
const char* ta_plan_hop_kernel(const ta_plan_t* pl, int axis, int vin) {
    if (!pl || axis < 0 || axis >= pl->order || (vin != 0 && vin != 1)) return nullptr;
    return forward_kernel_name(pl, axis, vin);
}

const char* ta_plan_hop_backward_kernel(const ta_plan_t* pl, int axis, int vin) {
    if (!pl || axis < 0 || axis >= pl->order || (vin != 0 && vin != 1)) return nullptr;
    switch (pl->bwd_id[axis][vin]) {
        case BWD_MFMA_N32: return "mfma_bf16_bwd_n32";
        case BWD_MFMA_BLOCKED: return "mfma_bf16_bwd_blocked";
        case BWD_MFMA_N64: return "mfma_bf16_bwd_n64";
        case BWD_GENERIC: return "generic";
    }
    return "unsupported";
}

static bool pair_ok(const ta_plan* pl, int axis, int vin) {
    return axis >= 0 && axis + 1 < pl->order && pl->pair[axis][vin];
}

const char* ta_plan_pair_kernel(const ta_plan_t* pl, int axis, int vin) {
    if (!pl || axis < 0 || axis >= pl->order || (vin != 0 && vin != 1)) return nullptr;
    return pair_ok(pl, axis, vin) ? "mfma_bf16_pair_n32" : "unsupported";
}

double ta_plan_pair_bytes(const ta_plan_t* pl, int axis, int vin) {
    // one pass: Q, K and the value input read once, O written once
    return ta_plan_hop_bytes(pl, axis, vin, 0, 0);
}

int ta_plan_fused_position(const ta_plan_t* pl) {
    if (!pl || pl->order < 2) return -1;
    const int m = pl->order;
    if (pl->hop_axis[m - 2] != m - 2 || pl->hop_axis[m - 1] != m - 1) return -1;
    // Rows that are not a whole number of 64-byte pieces (head widths that are not a multiple of 32) straddle the pieces
    // the pair moves them in, and the pair is then slower than the two hops it replaces (head width 100, 32 heads, 32k
    // tokens: 499 us against 2 x 195 us): the multi-hop call runs those hops on their own.  ta_axis_pair_attn_forward
    // still accepts such widths.
    if (pl->desc.head_dim % 32 != 0) return -1;
    return pair_ok(pl, m - 2, m == 2 ? TA_VIN_KV : TA_VIN_O) ? m - 2 : -1;
}

double ta_plan_hop_bytes(const ta_plan_t* pl, int axis, int vin, int backward, int accumulate) {
    if (!pl || axis < 0 || axis >= pl->order || (vin != 0 && vin != 1)) return -1.0;
    const double per_head = (double)pl->desc.batch * (double)pl->N * pl->desc.head_dim * pl->elem;
    const double Hq = pl->desc.n_q_heads, Hkv = pl->desc.n_kv_heads;
    const double Hvin = vin == TA_VIN_KV ? Hkv : Hq;
    if (!backward) return per_head * (Hq + Hkv + Hvin + Hq);
    // reads Q, K, value input, dO; writes d(value input), dQ, dK; accumulate re-reads dQ, dK
    double heads = Hq + Hkv + Hvin + Hq + Hvin + Hq + Hkv;
    if (accumulate) heads += Hq + Hkv;
    return per_head * heads;
}

double ta_plan_hop_flops(const ta_plan_t* pl, int axis, int backward) {
    if (!pl || axis < 0 || axis >= pl->order) return -1.0;
    const double fwd = 4.0 * pl->desc.batch * pl->desc.n_q_heads * (double)pl->N * pl->dims[axis] * pl->desc.head_dim;
    return backward ? 2.5 * fwd : fwd;
}

size_t ta_plan_workspace_bytes(const ta_plan_t* pl, int save_for_backward) {
    if (!pl || pl->order <= 1) return 0;
    // hops that write an intermediate O: all but the last, and one fewer when the last two run fused
    const int writers = pl->order - 1 - (!save_for_backward && ta_plan_fused_position(pl) >= 0 ? 1 : 0);
    const int nbuf = save_for_backward ? writers : (writers < 2 ? writers : 2);
    return (size_t)nbuf * pl->o_buf_bytes;
}

size_t ta_plan_backward_scratch_bytes(const ta_plan_t* pl) {
    if (!pl) return 0;
    return 2 * pl->o_buf_bytes;
}

ta_status_t ta_axis_attn_forward(const ta_plan_t* pl, int axis, const void* q, const void* k, const void* v_in,
                                 int vin, void* o_out, void* stream) {
    g_detail[0] = 0;
    ta_status_t st = check_axis_vin(pl, axis, vin);
    if (st != TA_OK) return st;
    if (!q || !k || !v_in || !o_out) return fail(TA_ERR_NULL, "q, k, v_in or o_out is NULL");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v_in) || !aligned16(o_out))
        return fail(TA_ERR_INVALID_ARG, "device pointers must be 16-byte aligned");
    const Range ro = o_span(pl, o_out);
    if (overlaps(ro, q_span(pl, q)) || overlaps(ro, kv_span(pl, k)) || overlaps(ro, vin_span(pl, v_in, vin)))
        return fail(TA_ERR_ALIAS, "o_out overlaps an input");
    if (pl->kernel_id[axis][vin] == ta::K_NONE) return unsupported_forward(pl, axis);
    return enqueue_forward(pl, axis, q, k, v_in, vin, o_out, (hipStream_t)stream);
}

ta_status_t ta_axis_pair_attn_forward(const ta_plan_t* pl, int axis, const void* q, const void* k, const void* v_in,
                                      int vin, void* o_mid, void* o_out, void* stream) {
    g_detail[0] = 0;
    ta_status_t st = check_axis_vin(pl, axis, vin);
    if (st != TA_OK) return st;
    if (axis + 1 >= pl->order) return fail(TA_ERR_INVALID_ARG, "axis %d has no inner neighbour", axis);
    if (!q || !k || !v_in || !o_out) return fail(TA_ERR_NULL, "q, k, v_in or o_out is NULL");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v_in) || !aligned16(o_out) || !aligned16(o_mid))
        return fail(TA_ERR_INVALID_ARG, "device pointers must be 16-byte aligned");
    const Range ro = o_span(pl, o_out), rq = q_span(pl, q), rk = kv_span(pl, k), rv = vin_span(pl, v_in, vin);
    if (overlaps(ro, rq) || overlaps(ro, rk) || overlaps(ro, rv))
        return fail(TA_ERR_ALIAS, "o_out overlaps an input");
    if (o_mid) {
        const Range rm = o_span(pl, o_mid);
        if (overlaps(rm, rq) || overlaps(rm, rk) || overlaps(rm, rv) || overlaps(rm, ro))
            return fail(TA_ERR_ALIAS, "o_mid overlaps an input or o_out");
    }
    if (!pair_ok(pl, axis, vin))
        return fail(TA_ERR_UNSUPPORTED, "no fused kernel for axes %d and %d of this plan (needs bf16, head_dim a multiple of 4 up to 128 and the two innermost axes, both of length 32)", axis, axis + 1);
    return enqueue_pair(pl, axis, q, k, v_in, vin, o_mid, o_out, (hipStream_t)stream);
}

ta_status_t ta_axis_attn_backward(const ta_plan_t* pl, int axis, const void* q, const void* k, const void* v_in,
                                  int vin, const void* d_o, void* d_v_in, void* dq, void* dk, int accumulate,
                                  void* stream) {
    g_detail[0] = 0;
    ta_status_t st = check_axis_vin(pl, axis, vin);
    if (st != TA_OK) return st;
    if (!q || !k || !v_in || !d_o || !d_v_in || !dq || !dk) return fail(TA_ERR_NULL, "a tensor pointer is NULL");
    if (accumulate != 0 && accumulate != 1) return fail(TA_ERR_INVALID_ARG, "accumulate must be 0 or 1");
    const void* ptrs[7] = {q, k, v_in, d_o, d_v_in, dq, dk};
    for (const void* p : ptrs)
        if (!aligned16(p)) return fail(TA_ERR_INVALID_ARG, "device pointers must be 16-byte aligned");
    const Range in[4] = {q_span(pl, q), kv_span(pl, k), vin_span(pl, v_in, vin), o_span(pl, d_o)};
    const Range outr[3] = {vin_span(pl, d_v_in, vin), q_span(pl, dq), kv_span(pl, dk)};
    for (int i = 0; i < 3; ++i) {
        for (int j = 0; j < 4; ++j)
            if (overlaps(outr[i], in[j])) return fail(TA_ERR_ALIAS, "a gradient output overlaps an input");
        for (int j = i + 1; j < 3; ++j)
            if (overlaps(outr[i], outr[j])) return fail(TA_ERR_ALIAS, "gradient outputs overlap each other");
    }
    if (pl->bwd_id[axis][vin] == BWD_NONE) return unsupported_backward(pl, axis);
    return enqueue_backward(pl, axis, q, k, v_in, vin, d_o, d_v_in, dq, dk, accumulate, (hipStream_t)stream);
}

// Everything ta_multihop_forward checks, shared with its no-allocation form: all of it happens
// before the first launch.
static ta_status_t check_multihop_forward(const ta_plan* pl, const void* q, const void* k, const void* v, void* o,
                                          const void* workspace, size_t workspace_bytes, size_t need) {
    if (!q || !k || !v || !o) return fail(TA_ERR_NULL, "q, k, v or o is NULL");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o))
        return fail(TA_ERR_INVALID_ARG, "device pointers must be 16-byte aligned");
    const Range ro = o_span(pl, o), rq = q_span(pl, q), rk = kv_span(pl, k), rv = kv_span(pl, v);
    if (overlaps(ro, rq) || overlaps(ro, rk) || overlaps(ro, rv)) return fail(TA_ERR_ALIAS, "o overlaps an input");
    if (need > 0) {
        if (!workspace) return fail(TA_ERR_NULL, "workspace is NULL but %zu bytes are needed", need);
        if (workspace_bytes < need) return fail(TA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
        if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return fail(TA_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
        const Range rw = {reinterpret_cast<uintptr_t>(workspace), reinterpret_cast<uintptr_t>(workspace) + need};
        if (overlaps(rw, rq) || overlaps(rw, rk) || overlaps(rw, rv) || overlaps(rw, ro))
            return fail(TA_ERR_ALIAS, "workspace overlaps a tensor");
    }
    const int fused = ta_plan_fused_position(pl);
    for (int pos = 0; pos < pl->order && pos != fused; ++pos)
        if (pl->kernel_id[pl->hop_axis[pos]][pos == 0 ? TA_VIN_KV : TA_VIN_O] == ta::K_NONE) return unsupported_forward(pl, pl->hop_axis[pos]);
    return TA_OK;
}

static ta_status_t run_multihop_forward(const ta_plan* pl, const void* q, const void* k, const void* v, void* o,
                                        char* ws, int save_for_backward, hipStream_t stream) {
    const int m = pl->order;
    const void* cur = v;
    int cur_kind = TA_VIN_KV;
    const int fused = ta_plan_fused_position(pl);
    for (int pos = 0; pos < m; ++pos) {
        if (pos == fused)                                  // the last two hops in one launch; the O between them is only written for a backward
            return enqueue_pair(pl, pl->hop_axis[pos], q, k, cur, cur_kind,
                                save_for_backward ? ws + (size_t)pos * pl->o_buf_bytes : nullptr, o, stream);
        void* dst;
        if (pos == m - 1) dst = o;
        else if (save_for_backward) dst = ws + (size_t)pos * pl->o_buf_bytes;
        else dst = ws + (size_t)(pos & 1) * pl->o_buf_bytes;
        ta_status_t st = enqueue_forward(pl, pl->hop_axis[pos], q, k, cur, cur_kind, dst, stream);
        if (st != TA_OK) return st;
        cur = dst;
        cur_kind = TA_VIN_O;
    }
    return TA_OK;
}

ta_status_t ta_multihop_forward(const ta_plan_t* pl, const void* q, const void* k, const void* v, void* o,
                                void* workspace, size_t workspace_bytes, int save_for_backward, void* stream) {
    g_detail[0] = 0;
    if (!pl) return fail(TA_ERR_NULL, "plan is NULL");
    const size_t need = ta_plan_workspace_bytes(pl, save_for_backward);
    const ta_status_t st = check_multihop_forward(pl, q, k, v, o, workspace, workspace_bytes, need);
    if (st != TA_OK) return st;
    return run_multihop_forward(pl, q, k, v, o, static_cast<char*>(workspace), save_for_backward, (hipStream_t)stream);
}

ta_status_t ta_multihop_forward_static(const ta_plan_t* pl, const void* q, const void* k, const void* v, void* o,
                                       void* stream) {
    g_detail[0] = 0;
    if (!pl) return fail(TA_ERR_NULL, "plan is NULL");
    const size_t need = ta_plan_workspace_bytes(pl, 0);
    if (need > (size_t)TA_STATIC_WORKSPACE_BYTES)
        return fail(TA_ERR_WORKSPACE, "the inter-hop tensors of this plan need %zu bytes, the library's own workspace holds %zu",
                    need, (size_t)TA_STATIC_WORKSPACE_BYTES);
    void* ws = nullptr;
    if (static_workspace(&ws) != TA_OK) return fail(TA_ERR_DEVICE, "the address of the library's own workspace could not be obtained on the current device");
    const ta_status_t st = check_multihop_forward(pl, q, k, v, o, ws, (size_t)TA_STATIC_WORKSPACE_BYTES, need);
    if (st != TA_OK) return st;
    return run_multihop_forward(pl, q, k, v, o, static_cast<char*>(ws), 0, (hipStream_t)stream);
}

ta_status_t ta_multihop_backward(const ta_plan_t* pl, const void* q, const void* k, const void* v, const void* d_o,
                                 const void* workspace, size_t workspace_bytes, void* dq, void* dk, void* dv,
                                 void* scratch, size_t scratch_bytes, void* stream) {
    g_detail[0] = 0;
    if (!pl) return fail(TA_ERR_NULL, "plan is NULL");
    if (!q || !k || !v || !d_o || !dq || !dk || !dv) return fail(TA_ERR_NULL, "a tensor pointer is NULL");
    const void* ptrs[7] = {q, k, v, d_o, dq, dk, dv};
    for (const void* p : ptrs)
        if (!aligned16(p)) return fail(TA_ERR_INVALID_ARG, "device pointers must be 16-byte aligned");
    const int m = pl->order;
    const size_t need_ws = ta_plan_workspace_bytes(pl, 1);
    const size_t need_sc = m > 1 ? ta_plan_backward_scratch_bytes(pl) : 0;
    if (need_ws > 0) {
        if (!workspace) return fail(TA_ERR_NULL, "workspace is NULL");
        if (workspace_bytes < need_ws) return fail(TA_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need_ws);
        if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return fail(TA_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    }
    if (need_sc > 0) {
        if (!scratch) return fail(TA_ERR_NULL, "scratch is NULL");
        if (scratch_bytes < need_sc) return fail(TA_ERR_WORKSPACE, "scratch has %zu bytes, %zu needed", scratch_bytes, need_sc);
        if ((reinterpret_cast<uintptr_t>(scratch) & 255u) != 0) return fail(TA_ERR_INVALID_ARG, "scratch must be 256-byte aligned");
    }
    // no output may overlap an input, the saved tensors, the scratch or another output
    const Range in[4] = {q_span(pl, q), kv_span(pl, k), kv_span(pl, v), o_span(pl, d_o)};
    const Range outr[3] = {q_span(pl, dq), kv_span(pl, dk), kv_span(pl, dv)};
    const uintptr_t wlo = reinterpret_cast<uintptr_t>(workspace), slo = reinterpret_cast<uintptr_t>(scratch);
    const Range rw = {wlo, wlo + need_ws}, rs = {slo, slo + need_sc};
    for (int i = 0; i < 3; ++i) {
        for (int j = 0; j < 4; ++j)
            if (overlaps(outr[i], in[j])) return fail(TA_ERR_ALIAS, "a gradient output overlaps an input");
        for (int j = i + 1; j < 3; ++j)
            if (overlaps(outr[i], outr[j])) return fail(TA_ERR_ALIAS, "gradient outputs overlap each other");
        if (need_ws > 0 && overlaps(outr[i], rw)) return fail(TA_ERR_ALIAS, "a gradient output overlaps the workspace");
        if (need_sc > 0 && overlaps(outr[i], rs)) return fail(TA_ERR_ALIAS, "a gradient output overlaps the scratch");
    }
    if (need_sc > 0) {
        for (int j = 0; j < 4; ++j)
            if (overlaps(rs, in[j])) return fail(TA_ERR_ALIAS, "scratch overlaps an input");
        if (need_ws > 0 && overlaps(rs, rw)) return fail(TA_ERR_ALIAS, "scratch overlaps the workspace");
    }
    for (int pos = 0; pos < m; ++pos)
        if (pl->bwd_id[pl->hop_axis[pos]][pos == 0 ? TA_VIN_KV : TA_VIN_O] == BWD_NONE) return unsupported_backward(pl, pl->hop_axis[pos]);

    const char* ws = static_cast<const char*>(workspace);
    char* sc = static_cast<char*>(scratch);
    const void* grad = d_o;
    for (int pos = m - 1; pos >= 0; --pos) {
        const void* x = pos == 0 ? v : ws + (size_t)(pos - 1) * pl->o_buf_bytes;
        const int kind = pos == 0 ? TA_VIN_KV : TA_VIN_O;
        void* gprev = pos == 0 ? dv : sc + (size_t)(pos & 1) * pl->o_buf_bytes;
        ta_status_t st = enqueue_backward(pl, pl->hop_axis[pos], q, k, x, kind, grad, gprev, dq, dk, pos == m - 1 ? 0 : 1,
                                          (hipStream_t)stream);
        if (st != TA_OK) return st;
        grad = gprev;
    }
    return TA_OK;
}

ta_status_t ta_rope_apply(const ta_plan_t* pl, int which, int axis, float base, int inverse, const void* x, void* y,
                          void* stream) {
    g_detail[0] = 0;
    if (!pl) return fail(TA_ERR_NULL, "plan is NULL");
    if (!x || !y) return fail(TA_ERR_NULL, "x or y is NULL");
    if (which != 0 && which != 1) return fail(TA_ERR_INVALID_ARG, "which must be 0 (Q layout) or 1 (key/value layout)");
    if (axis < -1 || axis >= pl->order) return fail(TA_ERR_INVALID_ARG, "axis %d out of range [-1, %d)", axis, pl->order);
    if (!(base >= 0.f) || isinf(base)) return fail(TA_ERR_INVALID_ARG, "base must be finite and >= 0");
    if (!aligned16(x) || !aligned16(y)) return fail(TA_ERR_INVALID_ARG, "device pointers must be 16-byte aligned");
    if (pl->N >= ((int64_t)1 << 31)) return fail(TA_ERR_UNSUPPORTED, "sequence length %lld is too long for the encoding kernel", (long long)pl->N);
    const ta_desc_t& d = pl->desc;
    if (d.head_dim % 8 != 0) return fail(TA_ERR_UNSUPPORTED, "the encoding kernel needs head_dim to be a multiple of 8, got %d", d.head_dim);
    const int64_t* st = which == 0 ? pl->qs : pl->kvs;
    const int H = which == 0 ? d.n_q_heads : d.n_kv_heads;
    if (x != y && overlaps(span_of(x, st, d.batch, pl->N, H, d.head_dim, pl->elem), span_of(y, st, d.batch, pl->N, H, d.head_dim, pl->elem)))
        return fail(TA_ERR_ALIAS, "y overlaps x without being x");
    ta::RopeParams rp;
    rp.x = make_tensor(x, st);
    rp.y = make_tensor(y, st);
    rp.B = d.batch; rp.H = H; rp.D = d.head_dim; rp.order = pl->order; rp.N = (uint32_t)pl->N;
    for (int i = 0; i < TA_MAX_ORDER; ++i) {
        rp.dims[i] = i < pl->order ? (uint32_t)pl->dims[i] : 1u;
        rp.strides[i] = i < pl->order ? (uint32_t)pl->strides[i] : 1u;
    }
    rp.axis = axis;
    rp.inverse = inverse != 0;
    rp.log2_base = (float)log2(base > 0.f ? (double)base : 10000.0);
    hipError_t e = ta::launch_rope(rp, d.dtype, (hipStream_t)stream);
    if (e != hipSuccess) return fail(TA_ERR_DEVICE, "encoding launch failed: %s", hipGetErrorString(e));
    return TA_OK;
}

ta_status_t ta_stream_mix(const void* src, void* dst, size_t units, int reads, int writes, void* stream) {
    g_detail[0] = 0;
    if (!src || !dst) return fail(TA_ERR_NULL, "src or dst is NULL");
    if (!aligned16(src) || !aligned16(dst)) return fail(TA_ERR_INVALID_ARG, "stream mix needs 16-byte alignment");
    if (units > ((size_t)1 << 40) / 4096 / 16) return fail(TA_ERR_INVALID_ARG, "too many units");
    hipError_t e = ta::launch_stream_mix(src, dst, units, reads, writes, (hipStream_t)stream);
    if (e == hipErrorInvalidValue) return fail(TA_ERR_UNSUPPORTED, "no streaming kernel for %d reads : %d writes (1:1, 3:2, 2:1, 9:4, 3:1, 4:3)", reads, writes);
    if (e != hipSuccess) return fail(TA_ERR_DEVICE, "stream mix launch failed: %s", hipGetErrorString(e));
    return TA_OK;
}

ta_status_t ta_stream_slabs(const void* q, const void* k, const void* x, void* o, int64_t tokens, int n_q_heads,
                            int n_kv_heads, int granule, void* stream) {
    g_detail[0] = 0;
    if (!q || !k || !x || !o) return fail(TA_ERR_NULL, "q, k, x or o is NULL");
    if (!aligned16(q) || !aligned16(k) || !aligned16(x) || !aligned16(o)) return fail(TA_ERR_INVALID_ARG, "slab streaming needs 16-byte alignment");
    if (tokens < 0 || tokens % 1024 != 0 || tokens > ((int64_t)1 << 32)) return fail(TA_ERR_INVALID_ARG, "tokens must be a multiple of 1024, at most 2^32");
    if (n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads != 0 || n_q_heads > 1024)
        return fail(TA_ERR_INVALID_ARG, "head counts: 1 <= n_kv_heads, n_q_heads a multiple of it, at most 1024");
    if (granule < 1 || granule > 3) return fail(TA_ERR_INVALID_ARG, "granule must be 1, 2 or 3");
    hipError_t e = ta::launch_stream_slabs(q, k, x, o, tokens, n_q_heads, n_kv_heads, granule, (hipStream_t)stream);
    if (e == hipErrorInvalidValue) return fail(TA_ERR_INVALID_ARG, "too many slabs for one launch");
    if (e != hipSuccess) return fail(TA_ERR_DEVICE, "slab streaming launch failed: %s", hipGetErrorString(e));
    return TA_OK;
}

ta_status_t ta_copy_bytes(const void* src, void* dst, size_t bytes, void* stream) {
    g_detail[0] = 0;
    if (!src || !dst) return fail(TA_ERR_NULL, "src or dst is NULL");
    if (bytes % 16 != 0 || !aligned16(src) || !aligned16(dst)) return fail(TA_ERR_INVALID_ARG, "copy needs 16-byte alignment and size");
    hipError_t e = ta::launch_copy(src, dst, bytes, (hipStream_t)stream);
    if (e != hipSuccess) return fail(TA_ERR_DEVICE, "copy launch failed: %s", hipGetErrorString(e));
    return TA_OK;
}

}  // extern "C"

namespace ta {

hipError_t allow_dynamic_lds(const void* kernel, int bytes) {
    struct Entry { int dev; const void* kernel; int bytes; };
    static std::mutex mu;
    static Entry done[256];
    static int n_done = 0;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < n_done; ++i)
        if (done[i].dev == dev && done[i].kernel == kernel && done[i].bytes >= bytes) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    if (n_done < 256) done[n_done++] = Entry{dev, kernel, bytes};   // a full table only costs repeated (idempotent) calls
    return hipSuccess;
}

}  // namespace ta
