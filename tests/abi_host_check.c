/* Host-logic exerciser for the C ABI, meant to be built with -fsanitize=address,undefined and linked
 * against the library built the same way (tests/test_abi_sanitized.py does both).  It walks the plan
 * constructor, every query and every error path of the entry points with fabricated device addresses,
 * which are never dereferenced: each call returns before any launch, so no GPU is needed.  Any
 * out-of-bounds access, use after free, signed overflow or misaligned access in the host code aborts
 * the program; on success it prints "host checks passed" and the number of calls made. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "tensattn.h"

static int calls = 0;
#define EXPECT(expr, want)                                                                   \
    do {                                                                                     \
        ta_status_t got_ = (expr);                                                           \
        ++calls;                                                                             \
        if (got_ != (want)) {                                                                \
            fprintf(stderr, "%s:%d: %s returned %s (%s), expected %s\n", __FILE__, __LINE__, #expr, \
                    ta_status_string(got_), ta_last_error_detail(), ta_status_string(want)); \
            exit(1);                                                                         \
        }                                                                                    \
    } while (0)

static ta_desc_t desc(int order, const int* dims, int dtype, int hq, int hkv, int d) {
    ta_desc_t x;
    memset(&x, 0, sizeof(x));
    x.batch = 1; x.n_q_heads = hq; x.n_kv_heads = hkv; x.head_dim = d; x.order = order;
    for (int i = 0; i < TA_MAX_ORDER; ++i) { x.dims[i] = i < order ? dims[i] : 0; x.hop_order[i] = -1; }
    x.dtype = dtype; x.causal = 1;
    return x;
}

int main(void) {
    void* const Q = (void*)0x10000000, * const K = (void*)0x20000000, * const V = (void*)0x30000000;
    void* const O = (void*)0x40000000, * const W = (void*)0x50000000, * const G = (void*)0x60000000;
    void* const DQ = (void*)0x70000000, * const DK = (void*)0x80000000, * const DV = (void*)0x90000000, * const SC = (void*)0xa0000000;
    void* const S = (void*)0xdead0;
    ta_plan_t* p = NULL;

    /* every order, a few dtypes and head widths: create, query everything, destroy */
    for (int order = 1; order <= TA_MAX_ORDER; ++order)
        for (int dt = 0; dt < 2; ++dt)
            for (int d = 8; d <= 256; d += 60) {
                int dims[TA_MAX_ORDER];
                for (int i = 0; i < order; ++i) dims[i] = 1 + (i * 7 + order) % 5;
                ta_desc_t x = desc(order, dims, dt, 4, 2, d);
                x.window[order - 1] = 2;
                x.rope = order & 1;
                x.rope_base = 500.f;
                EXPECT(ta_plan_create(&x, &p), TA_OK);
                int64_t n = ta_plan_seq_len(p), prod = 1;
                for (int i = 0; i < order; ++i) prod *= dims[i];
                if (n != prod) { fprintf(stderr, "seq_len\n"); return 1; }
                for (int a = -1; a <= order; ++a) {
                    (void)ta_plan_axis_stride(p, a); (void)ta_plan_axis_fibres(p, a); (void)ta_plan_hop_axis(p, a);
                    for (int vin = -1; vin <= 2; ++vin) {
                        (void)ta_plan_hop_kernel(p, a, vin); (void)ta_plan_hop_backward_kernel(p, a, vin);
                        (void)ta_plan_pair_kernel(p, a, vin); (void)ta_plan_pair_bytes(p, a, vin);
                        (void)ta_plan_hop_bytes(p, a, vin, 1, 1); (void)ta_plan_hop_flops(p, a, 0);
                    }
                }
                (void)ta_plan_workspace_bytes(p, 0); (void)ta_plan_workspace_bytes(p, 1);
                (void)ta_plan_backward_scratch_bytes(p); (void)ta_plan_fused_position(p);
                ta_plan_destroy(p);
                calls += 8;
            }

    /* descriptors that must be refused */
    {
        int dims2[2] = {4, 3};
        ta_desc_t x = desc(2, dims2, TA_F32, 2, 2, 64);
        ta_desc_t y;
        y = x; y.order = 0;                      EXPECT(ta_plan_create(&y, &p), TA_ERR_SHAPE);
        y = x; y.order = TA_MAX_ORDER + 1;       EXPECT(ta_plan_create(&y, &p), TA_ERR_SHAPE);
        y = x; y.dims[1] = -3;                   EXPECT(ta_plan_create(&y, &p), TA_ERR_SHAPE);
        y = x; y.n_q_heads = 6; y.n_kv_heads = 4; EXPECT(ta_plan_create(&y, &p), TA_ERR_SHAPE);
        y = x; y.head_dim = 101;                 EXPECT(ta_plan_create(&y, &p), TA_ERR_UNSUPPORTED);
        y = x; y.dtype = 7;                      EXPECT(ta_plan_create(&y, &p), TA_ERR_INVALID_ARG);
        y = x; y.hop_order[0] = 0; y.hop_order[1] = 0; EXPECT(ta_plan_create(&y, &p), TA_ERR_INVALID_ARG);
        y = x; y.hop_order[0] = 5; y.hop_order[1] = 0; EXPECT(ta_plan_create(&y, &p), TA_ERR_INVALID_ARG);
        y = x; y.scale = -1.f;                   EXPECT(ta_plan_create(&y, &p), TA_ERR_INVALID_ARG);
        y = x; y.q_strides[0] = 64; y.q_strides[1] = 64; y.q_strides[2] = 64; EXPECT(ta_plan_create(&y, &p), TA_ERR_SHAPE);
        y = x; y.window[1] = -2;                 EXPECT(ta_plan_create(&y, &p), TA_ERR_INVALID_ARG);
        y = x; y.valid_len = 13;                 EXPECT(ta_plan_create(&y, &p), TA_ERR_SHAPE);
        y = x; y.valid_lens = (const int64_t*)0x1004; EXPECT(ta_plan_create(&y, &p), TA_ERR_INVALID_ARG);
        y = x; y.rope = 3;                       EXPECT(ta_plan_create(&y, &p), TA_ERR_INVALID_ARG);
        y = x; y.axis_mask[0] = (const void*)6;  EXPECT(ta_plan_create(&y, &p), TA_ERR_INVALID_ARG);
        y = x; y.dims[0] = 2147483647; y.dims[1] = 2147483647; EXPECT(ta_plan_create(&y, &p), TA_ERR_SHAPE);
        y = x; y.order = TA_MAX_ORDER; for (int i = 0; i < TA_MAX_ORDER; ++i) y.dims[i] = 2147483647;
        EXPECT(ta_plan_create(&y, &p), TA_ERR_SHAPE);
        EXPECT(ta_plan_create(NULL, &p), TA_ERR_NULL);
        EXPECT(ta_plan_create(&x, NULL), TA_ERR_NULL);
        ta_plan_destroy(NULL);
    }

    /* entry points: every error path returns before a launch */
    {
        int dims2[2] = {4, 3};
        ta_desc_t x = desc(2, dims2, TA_F32, 2, 1, 64);
        EXPECT(ta_plan_create(&x, &p), TA_OK);
        const size_t big = (size_t)1 << 20;
        EXPECT(ta_axis_attn_forward(p, 2, Q, K, V, 0, O, S), TA_ERR_INVALID_ARG);
        EXPECT(ta_axis_attn_forward(p, 0, Q, K, V, 3, O, S), TA_ERR_INVALID_ARG);
        EXPECT(ta_axis_attn_forward(p, 0, NULL, K, V, 0, O, S), TA_ERR_NULL);
        EXPECT(ta_axis_attn_forward(p, 0, (char*)Q + 4, K, V, 0, O, S), TA_ERR_INVALID_ARG);
        EXPECT(ta_axis_attn_forward(p, 0, Q, K, V, 0, V, S), TA_ERR_ALIAS);
        EXPECT(ta_axis_pair_attn_forward(p, 0, Q, K, V, 0, NULL, O, S), TA_ERR_UNSUPPORTED);
        EXPECT(ta_axis_pair_attn_forward(p, 1, Q, K, V, 0, NULL, O, S), TA_ERR_INVALID_ARG);
        EXPECT(ta_multihop_forward(p, Q, K, V, O, NULL, 0, 0, S), TA_ERR_NULL);
        EXPECT(ta_multihop_forward(p, Q, K, V, O, W, 16, 0, S), TA_ERR_WORKSPACE);
        EXPECT(ta_multihop_forward(p, Q, K, V, O, (char*)W + 16, big, 0, S), TA_ERR_INVALID_ARG);
        EXPECT(ta_multihop_forward(p, Q, K, V, O, O, big, 0, S), TA_ERR_ALIAS);
        EXPECT(ta_multihop_forward(p, Q, K, V, (char*)Q + 64, W, big, 0, S), TA_ERR_ALIAS);
        EXPECT(ta_axis_attn_backward(p, 0, Q, K, V, 0, O, Q, W, (char*)W + big, 0, S), TA_ERR_ALIAS);
        EXPECT(ta_axis_attn_backward(p, 0, Q, K, V, 0, NULL, W, W, W, 0, S), TA_ERR_NULL);
        EXPECT(ta_axis_attn_backward(p, 0, Q, K, V, 0, G, DV, DQ, DK, 2, S), TA_ERR_INVALID_ARG);
        EXPECT(ta_multihop_backward(p, Q, K, V, G, W, 16, DQ, DK, DV, SC, big, S), TA_ERR_WORKSPACE);
        EXPECT(ta_multihop_backward(p, Q, K, V, G, W, big, DQ, DK, DV, W, big, S), TA_ERR_ALIAS);
        EXPECT(ta_multihop_backward(p, Q, K, V, G, W, big, DQ, DK, DV, DQ, big, S), TA_ERR_ALIAS);
        EXPECT(ta_multihop_backward(p, Q, K, V, G, W, big, DQ, DQ, DV, SC, big, S), TA_ERR_ALIAS);
        EXPECT(ta_multihop_backward(p, Q, K, V, G, W, big, DQ, DK, DV, (char*)SC + 16, big, S), TA_ERR_INVALID_ARG);
        EXPECT(ta_rope_apply(p, 2, 0, 0.f, 0, Q, O, S), TA_ERR_INVALID_ARG);
        EXPECT(ta_rope_apply(p, 0, -1, 0.f, 0, Q, (char*)Q + 32, S), TA_ERR_ALIAS);
        EXPECT(ta_copy_bytes(Q, K, 24, S), TA_ERR_INVALID_ARG);
        EXPECT(ta_copy_bytes(NULL, K, 32, S), TA_ERR_NULL);
        ta_plan_destroy(p);
        /* an axis the fp32 backward cannot take: refused before the hop that could run is enqueued */
        int dims3[2] = {4096, 2};
        ta_desc_t z = desc(2, dims3, TA_F32, 8, 1, 64);
        EXPECT(ta_plan_create(&z, &p), TA_OK);
        const size_t huge = (size_t)1 << 28;
        EXPECT(ta_multihop_backward(p, (void*)(1ull << 32), (void*)(2ull << 32), (void*)(3ull << 32), (void*)(4ull << 32), (void*)(5ull << 32), huge,
                                    (void*)(6ull << 32), (void*)(7ull << 32), (void*)(8ull << 32), (void*)(9ull << 32), huge, S), TA_ERR_UNSUPPORTED);
        ta_plan_destroy(p);
    }
    int major = -1, minor = -1;
    ta_version(&major, &minor);
    ta_version(NULL, NULL);
    printf("host checks passed (%d calls, library version %d.%d)\n", calls, major, minor);
    return 0;
}
