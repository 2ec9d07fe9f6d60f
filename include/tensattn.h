/*
 * tensattn.h - C ABI of the MI355X (gfx950) Tensorized Attention library.
 *
 * Tensorized attention (arXiv 2410.20926, Sec. 3.2) views a length-N sequence of
 * queries, keys and values as an order-m tensor, N = n_1 * ... * n_m, and runs
 * softmax attention along one tensor axis at a time (Eq. 4), all other axes acting
 * as batch; Algorithm 1 chains one such hop per axis, starting from O = V and always
 * using the same Q and K.
 *
 * Conventions shared by every call
 *  - Device buffers are caller-owned DEVICE pointers, 16-byte aligned, holding
 *    elements of the plan's dtype.  The library never allocates, frees or keeps
 *    device memory, never synchronises, and only enqueues work on `stream`
 *    (a hipStream_t passed as void*; NULL = the default stream).  Inputs are never
 *    written.  Descriptors and plans are HOST memory.
 *  - Tensor layout: element (b, t, h, x) of a tensor with heads H lives at
 *    b*stride[0] + t*stride[1] + h*stride[2] + x  (strides in ELEMENTS, feature axis
 *    contiguous).  All-zero strides mean dense [B, N, H, D].
 *  - Tensor reshape is row-major: token t = sum_i j_i * stride_i, the first axis is
 *    the slowest (Sec. 4.3: with {32,32,32} one more step on the first axis is 1,024
 *    more tokens).  Axes are numbered from 0 here.
 *  - Grouped-query heads: query head h uses key/value head h / (n_q_heads / n_kv_heads).
 *  - Every call returns a ta_status_t; nothing aborts, throws or prints.  Every check of a
 *    call (arguments, aliasing, kernel availability and launch geometry of EVERY hop it runs)
 *    happens before its first launch: on any status but TA_ERR_DEVICE nothing has been
 *    enqueued.  TA_ERR_DEVICE means HIP itself refused a launch; hops before it may have
 *    been enqueued.  ta_last_error_detail() gives a thread-local message.
 *    Kernel faults that happen asynchronously surface at the caller's next
 *    synchronisation, as with any HIP launch.
 */
#ifndef TENSATTN_H
#define TENSATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TA_MAX_ORDER 8

typedef enum {
    TA_OK = 0,
    TA_ERR_NULL = 1,          /* a required pointer is NULL */
    TA_ERR_INVALID_ARG = 2,   /* bad enum, axis out of range, misaligned pointer ... */
    TA_ERR_SHAPE = 3,         /* inconsistent sizes (heads not divisible, dims < 1, overflow ...) */
    TA_ERR_UNSUPPORTED = 4,   /* valid request this build has no kernel for */
    TA_ERR_ALIAS = 5,         /* an output overlaps an input */
    TA_ERR_WORKSPACE = 6,     /* workspace too small */
    TA_ERR_DEVICE = 7,        /* HIP reported a launch error */
    TA_ERR_NOMEM = 8          /* host memory for a plan could not be allocated */
} ta_status_t;

typedef enum { TA_F32 = 0, TA_BF16 = 1 } ta_dtype_t;

/* Which tensor a hop reads as its value input (Algorithm 1 initialises O = V, so
 * the first executed hop reads V, which has n_kv_heads heads and the key/value
 * layout; every later hop reads a previous O, with n_q_heads heads and O's layout). */
typedef enum { TA_VIN_KV = 0, TA_VIN_O = 1 } ta_vin_t;

/* Problem descriptor (Algorithm 1's inputs: Q, K, V in R^{n_1 x .. x n_m}, with a
 * feature axis, and the per-axis mask M_i).  Plain data; copied by ta_plan_create. */
typedef struct ta_desc_t {
    int32_t batch;                    /* B >= 1 */
    int32_t n_q_heads;                /* H_q >= 1 */
    int32_t n_kv_heads;               /* H_kv >= 1, divides H_q */
    int32_t head_dim;                 /* D, the d under the square root of Eq. 1 */
    int32_t order;                    /* m, 1..TA_MAX_ORDER */
    int32_t dims[TA_MAX_ORDER];       /* n_1..n_m, each >= 1; N = their product */
    int32_t dtype;                    /* ta_dtype_t of every tensor */
    int32_t causal;                   /* 0: no mask; 1: M_i[a][c] = (c <= a) on every axis */
    float   scale;                    /* logit scale; 0 means 1/sqrt(head_dim) (Eq. 1) */
    int32_t hop_order[TA_MAX_ORDER];  /* permutation of 0..m-1; all -1 = Algorithm 1's order 0,1,..,m-1 */
    int64_t q_strides[3];             /* (batch, token, head) strides of Q, dQ; all 0 = dense [B,N,H_q,D] */
    int64_t kv_strides[3];            /* of K, V, dK, dV; all 0 = dense [B,N,H_kv,D] */
    int64_t o_strides[3];             /* of O, dO and every inter-hop O; all 0 = dense [B,N,H_q,D] */
    /* Further per-axis masks M_i (Eq. 3 admits any; Sec. 2.1 mentions sparsity masks).  All of
     * them, and `causal`, are intersected; a row left with no visible key gives a zero output
     * row and takes no gradient. */
    int32_t window[TA_MAX_ORDER];     /* w_i > 0: on axis i key c is visible from row a only if |a - c| < w_i
                                         (together with c <= a when causal); 0 = no band on that axis */
    int64_t valid_len;                /* L in 1..N: tokens t >= L of every batch element are padding - never
                                         attended to, and their own outputs and gradients are zero; 0 = none */
    const void* axis_mask[TA_MAX_ORDER]; /* DEVICE pointers, or NULL for no table on that axis.  Table of axis i:
                                         n_i rows of ceil(n_i / 32) uint32 words, row-major; bit (c % 32) of
                                         word c / 32 of row a is 1 iff query position a may attend key
                                         position c on that axis (the same table for every head and
                                         batch element).  4-byte aligned, caller-owned, read-only, and must
                                         stay valid and unchanged while the plan is in use; entries at or
                                         beyond `order` are ignored. */
    const int64_t* valid_lens;        /* DEVICE pointer to B lengths, or NULL.  Eq. 3's M_i is one table per fibre;
                                         this is its everyday case, sequences of different lengths in one batch:
                                         batch element b is padded from token valid_lens[b] on (values are clamped
                                         to 0..N; 0 = the whole element is padding; combined with valid_len by
                                         taking the smaller).  8-byte aligned, caller-owned, read when a kernel
                                         runs: it may change between calls, not while one is in flight. */
    /* Tensorized positional encoding inside the hops (Sec. 3.2: a token's position is the vector of its
     * tensor coordinates, and the rotary encoding is applied per axis).  With rope = 1 the hop along axis i
     * scores with Q and K rotated by their coordinate j_i on that axis - feature pair (2p, 2p+1) turned by
     * j_i * rope_base^(-2p / head_dim) radians - so that its attention depends on j_i - k_i; the kernels turn
     * the rows between the global load and the matrix cores, and the backward turns dQ and dK back: no
     * encoded copy of Q or K ever exists in memory.  Values are not encoded.  Pairs are INTERLEAVED
     * neighbours; a model whose rotary pairs are (p, p + head_dim/2) gets the same scores by permuting the
     * columns of its query and key projections once (scores are invariant under a common feature
     * permutation).  Which features take which axis is not in the paper: this per-hop form is a reading.
     * The matrix-core kernels take it for axes of up to 4,096 positions (fp32 angles); longer axes, and
     * fp32 tensors, run on the generic kernels (double-precision angles).  The fused pair of hops takes it
     * too: there a token's rows are turned by one axis position for the first hop and by the other for
     * the second, with the rotation's cosines and sines rounded to bf16. */
    int32_t rope;                     /* 0 or 1 */
    float   rope_base;                /* the base; 0 means 10000 */
    int32_t axis_mask_per_fibre[TA_MAX_ORDER]; /* 0: axis_mask[i] is one table for every fibre of axis i (above);
                                         1: it holds one such table per fibre (Eq. 3: M_i has an n_i x n_i table for every
                                         choice of the other coordinates), N / n_i tables one after the other, the fibres
                                         numbered by their coordinates on the other axes read as one row-major number
                                         (the first token of fibre f is (f / stride_i) * stride_i * n_i + f % stride_i).
                                         The tables are shared by heads and batch elements. */
} ta_desc_t;

typedef struct ta_plan ta_plan_t;     /* opaque, immutable, host-only, shareable between threads */

/* ---- tensorize / plan (Sec. 3.1 "order-m tensorization ... achieved by reshaping";
 *      App. C.1).  Host only; touches no device memory. ------------------------------ */

/* Validates `desc`, derives per-axis token strides and fibre counts and picks a kernel
 * per hop.  Errors: NULL -> TA_ERR_NULL; order, dims, heads, head_dim, strides
 * inconsistent, valid_len > N -> TA_ERR_SHAPE; bad dtype / hop_order / negative window or
 * valid_len, misaligned axis_mask -> TA_ERR_INVALID_ARG; a shape no
 * kernel covers (head_dim odd or above 256) -> TA_ERR_UNSUPPORTED.  The matrix-core kernels take
 * head_dim 64 and 128 and any other multiple of 4 up to 128; the rest runs on the generic kernels. */
ta_status_t ta_plan_create(const ta_desc_t* desc, ta_plan_t** out_plan);
void        ta_plan_destroy(ta_plan_t* plan);                 /* NULL-safe */

int64_t ta_plan_seq_len(const ta_plan_t* plan);               /* N; -1 on NULL */
int64_t ta_plan_axis_stride(const ta_plan_t* plan, int axis); /* tokens between neighbours on `axis`; -1 on error */
int64_t ta_plan_axis_fibres(const ta_plan_t* plan, int axis); /* N / n_axis per (batch, head); -1 on error */
int     ta_plan_hop_axis(const ta_plan_t* plan, int hop_position); /* axis run at position 0..m-1; -1 on error */
/* Name of the kernel variant the plan chose for the forward hop on `axis` with value
 * input `vin` ("mfma_bf16_n32", "mfma_bf16_n64", "mfma_bf16_stream", their group-shared forms
 * "..._shared" and, when the value input is per key/value head, "..._shared_kv", "generic"); NULL on
 * error.  Static storage. */
const char* ta_plan_hop_kernel(const ta_plan_t* plan, int axis, int vin);
/* Same for the backward of that hop ("mfma_bf16_bwd_n32", "mfma_bf16_bwd_blocked" for axes of 33 to
 * 1024 positions, "generic", or "unsupported" when
 * ta_axis_attn_backward would return TA_ERR_UNSUPPORTED); NULL on error. */
const char* ta_plan_hop_backward_kernel(const ta_plan_t* plan, int axis, int vin);

/* Cost model of one hop (App. C.2, Table 5, with the fibre count N/n_i that Eq. 4
 * implies).  Bytes are ALGORITHMIC HBM bytes: each of Q, K, value-input read once,
 * O written once, K and V counted once per key/value head:
 *   B*N*D*elem*(H_q + H_kv + H_vin + H_q),  H_vin = H_kv for TA_VIN_KV else H_q.
 * Backward (backward != 0): reads Q, K, value-input, dO; writes d(value-input); dQ and
 * dK written (accumulate = 0) or read and written (accumulate = 1).
 * FLOPs are the dense executed count 4*B*H_q*N*n_axis*D (forward; 2.5x for backward).
 * Both return -1.0 on error. */
double ta_plan_hop_bytes(const ta_plan_t* plan, int axis, int vin, int backward, int accumulate);
double ta_plan_hop_flops(const ta_plan_t* plan, int axis, int backward);

/* Workspace for ta_multihop_forward, in bytes (0 when m == 1):
 * save_for_backward == 0: two ping-pong inter-hop O buffers (one when only one hop writes an
 *   intermediate O, none when none does: fused, the last two hops keep theirs on chip);
 * save_for_backward != 0: m-1 retained inter-hop O buffers, O_1..O_{m-1}, in hop order.
 * Each buffer is a dense or o_strides-shaped O tensor rounded up to 256 bytes. */
size_t ta_plan_workspace_bytes(const ta_plan_t* plan, int save_for_backward);
/* Scratch for ta_multihop_backward, in bytes: two ping-pong gradient buffers of O's size. */
size_t ta_plan_backward_scratch_bytes(const ta_plan_t* plan);

/* ---- per-axis attention, forward (Eq. 4; the loop body of Algorithm 1) --------------
 * o_out[fibre rows] = softmax(Q_i K_i^T * scale o M_i) * v_in[fibre rows] for every
 * mode-`axis` fibre of every (batch, head).  q: Q layout; k: key/value layout; v_in:
 * key/value layout with n_kv_heads (vin = TA_VIN_KV) or O layout with n_q_heads
 * (TA_VIN_O); o_out: O layout.  o_out must not overlap q, k or v_in (TA_ERR_ALIAS).
 * Asynchronous on `stream`. */
ta_status_t ta_axis_attn_forward(const ta_plan_t* plan, int axis,
                                 const void* q, const void* k, const void* v_in, int vin,
                                 void* o_out, void* stream);

/* ---- two hops of Algorithm 1 in one launch ---------------------------------------------
 * The hop along `axis` followed by the hop along `axis + 1` (Eq. 4 twice with the same Q, K):
 * the same result as two ta_axis_attn_forward calls up to the rounding of the intermediate
 * O, which stays on chip.  Arguments as ta_axis_attn_forward; `o_mid` is NULL, or an O-shaped
 * tensor that receives the output of the first of the two hops as well (what a backward
 * pass needs); it must not overlap anything else.  Available when `axis + 1` is the
 * innermost axis, both axes have length 32, dtype is bf16 and head_dim a multiple of 4 up to 128;
 * otherwise
 * TA_ERR_UNSUPPORTED (ta_plan_pair_kernel tells beforehand). */
ta_status_t ta_axis_pair_attn_forward(const ta_plan_t* plan, int axis,
                                      const void* q, const void* k, const void* v_in, int vin,
                                      void* o_mid, void* o_out, void* stream);
/* "mfma_bf16_pair_n32" or "unsupported"; NULL on error. */
const char* ta_plan_pair_kernel(const ta_plan_t* plan, int axis, int vin);
/* Algorithmic HBM bytes of the fused pair: Q, K, value input read once, O written once. */
double      ta_plan_pair_bytes(const ta_plan_t* plan, int axis, int vin);
/* Hop position at which ta_multihop_forward switches to the fused pair for the last two
 * hops, or -1 when it runs every hop on its own (no fused kernel for the plan, a hop order other than the
 * default, or a head width that is not a multiple of 32, for which the pair is slower than the two hops). */
int         ta_plan_fused_position(const ta_plan_t* plan);

/* ---- per-axis attention, backward (the paper gives none: Sec. 3.2 only states that a
 *      backward exists; this is the derivative of the hop above) -----------------------
 * With A the hop's attention, X = v_in, G = d_o:
 *   d_v_in = A^T G;  dS = A o (G X^T - rowsum(A o G X^T));
 *   dq (+)= dS K * scale;  dk (+)= sum over the query heads of the group of dS^T Q * scale.
 * d_v_in has v_in's layout and head count; for TA_VIN_KV it is summed over the query
 * heads that share the key/value head.  accumulate = 0 overwrites dq, dk; 1 adds to
 * them.  dq: Q layout; dk: key/value layout.  Outputs must not overlap inputs or each
 * other.  Deterministic (no atomics). */
ta_status_t ta_axis_attn_backward(const ta_plan_t* plan, int axis,
                                  const void* q, const void* k, const void* v_in, int vin,
                                  const void* d_o, void* d_v_in, void* dq, void* dk,
                                  int accumulate, void* stream);

/* ---- full multi-hop forward (Algorithm 1) --------------------------------------------
 * O_0 = V; one hop per axis in the plan's hop order; o receives the last hop's output.
 * `workspace` (device, >= ta_plan_workspace_bytes(plan, save_for_backward), 256-byte
 * aligned; may be NULL when that size is 0) holds the inter-hop O tensors; with
 * save_for_backward they stay valid for ta_multihop_backward.  TA_ERR_WORKSPACE when
 * too small. */
ta_status_t ta_multihop_forward(const ta_plan_t* plan,
                                const void* q, const void* k, const void* v, void* o,
                                void* workspace, size_t workspace_bytes,
                                int save_for_backward, void* stream);

/* ---- the multi-hop forward for callers that cannot allocate -------------------------------
 * For code under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc:
 * ta_multihop_forward with save_for_backward = 0, except that the inter-hop O tensors live in
 * device memory that is part of the library itself (a fixed array of TA_STATIC_WORKSPACE_BYTES
 * bytes in the library's code object; every GPU the library runs on holds its own copy until
 * the process ends) instead of a caller's workspace.  The call allocates and frees nothing.
 * Plans whose ta_plan_workspace_bytes(plan, 0) exceeds TA_STATIC_WORKSPACE_BYTES are refused
 * with TA_ERR_WORKSPACE (64 MiB holds e.g. one intermediate O of 8,192 tokens x 32 heads x 128
 * bf16 features, which is all a three-hop plan with a fused last pair needs).  All calls on one
 * GPU share that GPU's array: calls that overlap in time on one GPU (different streams or
 * threads) race; calls that follow one another on a stream do not, and nothing needs clearing
 * in between, since every hop overwrites an intermediate tensor before the next hop reads it.
 * The first call on a device looks up the array's address on that device, with that device
 * current; make it outside a stream capture.  Results are identical to ta_multihop_forward's. */
#define TA_STATIC_WORKSPACE_BYTES (64u << 20)
ta_status_t ta_multihop_forward_static(const ta_plan_t* plan,
                                       const void* q, const void* k, const void* v, void* o,
                                       void* stream);

/* ---- full multi-hop backward ----------------------------------------------------------
 * Gradients of sum(O * d_o) w.r.t. Q, K, V: hops undone in reverse order, dq and dk
 * accumulated over hops (first processed hop overwrites), dv = gradient reaching O_0.
 * `workspace` is the one a save_for_backward forward filled for the same q, k, v;
 * `scratch` (device, >= ta_plan_backward_scratch_bytes, 256-byte aligned) is
 * overwritten. */
ta_status_t ta_multihop_backward(const ta_plan_t* plan,
                                 const void* q, const void* k, const void* v, const void* d_o,
                                 const void* workspace, size_t workspace_bytes,
                                 void* dq, void* dk, void* dv,
                                 void* scratch, size_t scratch_bytes, void* stream);

/* ---- tensorized positional encoding (Sec. 3.2: a token's position is the vector of its tensor
 *      coordinates, and rotary embedding is applied with per-axis positions) -----------------
 * y = R x for a tensor in the Q layout with n_q_heads (which = 0) or in the key/value layout
 * with n_kv_heads (which = 1).  The paper gives no formula; this library rotates feature pair
 * (2p, 2p+1) of a block of width W by pos * base^(-2p/W), with
 *   axis in 0..m-1 : one block, W = head_dim, pos = the token's coordinate on that axis (the
 *                    encoding a hop along that axis would use);
 *   axis = -1      : m consecutive blocks of W = 2*floor(head_dim/(2m)), block i with pos = the
 *                    coordinate on axis i; left-over features are copied.
 * base = 0 means 10000.  inverse != 0 rotates by the negative angle (what a backward pass
 * applies to the gradient).  y may be x itself (in place); any other overlap is TA_ERR_ALIAS.
 * Needs N < 2^31. */
ta_status_t ta_rope_apply(const ta_plan_t* plan, int which, int axis, float base, int inverse,
                          const void* x, void* y, void* stream);

/* ---- measurement aid: a plain read-and-write copy of `bytes` bytes (multiple of 16)
 *      from src to dst on `stream`, used to measure the achievable HBM ceiling and to
 *      calibrate hardware counters against a transfer of known size. ------------------- */
ta_status_t ta_copy_bytes(const void* src, void* dst, size_t bytes, void* stream);
/* The same with a mix of reads and writes: per unit of 4,096 bytes the kernel reads `reads` consecutive units
 * of src and writes `writes` consecutive units of dst (src holds units * reads * 4096 bytes, dst units * writes
 * * 4096), i.e. what the memory gives a kernel that only moves that mix of bytes - the attainable rate that a
 * hop with the same read : write ratio is measured against.  Mixes 1:1, 3:2, 2:1, 9:4, 3:1, 4:3; any other
 * -> TA_ERR_UNSUPPORTED. */
ta_status_t ta_stream_mix(const void* src, void* dst, size_t units, int reads, int writes, void* stream);
/* The bytes of one pass of the fused pair (ta_axis_pair_attn_forward) in the pair's own access pattern and
 * nothing else: dense token-major tensors q, x, o [tokens, n_q_heads, 128] and k [tokens, n_kv_heads, 128] of
 * 2-byte elements (256-byte rows), tokens a multiple of 1,024.  One workgroup per (slab of 1,024 consecutive
 * tokens, query head), the heads of a key/value head on workgroups that run side by side, reads the slab's Q,
 * K (of its key/value head) and X rows and writes its O rows (o = x when q and k hold zeros), in pieces of
 *   granule = 1: one 128-byte line of a row at a time, every row of the slab, then the other line (what the
 *                pair does: its chunks of LDS hold half a row of every token);
 *   granule = 2: whole 256-byte rows;
 *   granule = 3: one workgroup per (slab, key/value head) moves the 1 KB of a token's whole head group at once.
 * It shows what the memory gives for that pattern: the rate the pair is measured against.  Other values of
 * granule, tokens not a multiple of 1,024, n_q_heads not a multiple of n_kv_heads -> TA_ERR_INVALID_ARG. */
ta_status_t ta_stream_slabs(const void* q, const void* k, const void* x, void* o, int64_t tokens, int n_q_heads,
                            int n_kv_heads, int granule, void* stream);

/* ---- errors and version ------------------------------------------------------------- */
const char* ta_status_string(ta_status_t status);
const char* ta_last_error_detail(void);          /* thread-local; "" when none */
void        ta_version(int* major, int* minor);  /* NULL-safe */

#ifdef __cplusplus
}
#endif
#endif /* TENSATTN_H */
