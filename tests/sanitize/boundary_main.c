/*
 * Driver for a build of libmoepp.so whose host code is compiled with
 * -fsanitize=address,undefined: walks the host side of the C ABI (sizing,
 * context life cycle, Eq.8 arithmetic, every argument check that must come
 * before a launch) on a machine without a GPU.  Plain C, so it also shows
 * that include/moepp.h is a C header.  Prints "ok" and exits 0 when every
 * call returned what it must.
 */
#include "moepp.h"

#include <stdio.h>
#include <string.h>

static int failures;
#define EXPECT(cond)                                                          \
    do {                                                                      \
        if (!(cond)) {                                                        \
            printf("FAILED line %d: %s\n", __LINE__, #cond);                 \
            ++failures;                                                       \
        }                                                                     \
    } while (0)

int main(void)
{
    void *fake = (void *)0x10000;           /* aligned, non-null, never dereferenced */
    void *odd = (void *)0x10004;
    moepp_desc d = {128, 64, 96, 4, 1, 1, 2, 2, MOEPP_BF16};
    const size_t ws = moepp_workspace_bytes(&d);
    EXPECT(ws > 0 && ws % 256 == 0);
    EXPECT(moepp_packed_bytes(&d) == (size_t)4 * 3 * 96 * 64 * 2);
    EXPECT(moepp_workspace_bytes(NULL) == 0);

    moepp_desc bad = d;
    bad.D = 60;
    EXPECT(moepp_workspace_bytes(&bad) == 0);
    moepp_ctx *ctx = NULL;
    EXPECT(moepp_create(&bad, fake, (size_t)1 << 40, &ctx) == MOEPP_EUNSUPPORTED && !ctx);
    bad = d;
    bad.n_ffn = 61;
    EXPECT(moepp_create(&bad, fake, (size_t)1 << 40, &ctx) == MOEPP_EUNSUPPORTED);
    bad = d;
    bad.k = 0;
    EXPECT(moepp_create(&bad, fake, (size_t)1 << 40, &ctx) == MOEPP_EINVAL);
    EXPECT(moepp_create(&d, fake, ws - 1, &ctx) == MOEPP_ENOMEM);
    EXPECT(moepp_create(&d, odd, ws, &ctx) == MOEPP_EINVAL);
    EXPECT(moepp_create(&d, fake, ws, &ctx) == MOEPP_OK && ctx);

    /* the largest descriptor: N = 64 experts, 8 constant experts, K = 8 */
    moepp_desc wide = {4096, 4096, 5632, 52, 2, 2, 8, 8, MOEPP_BF16};
    moepp_ctx *cw = NULL;
    const size_t wsw = moepp_workspace_bytes(&wide);
    EXPECT(wsw > 0 && moepp_create(&wide, fake, wsw, &cw) == MOEPP_OK);
    int32_t cap[64];
    EXPECT(moepp_capacity(&wide, 4096, 8, 1.1, 0.75, 1, cap) == MOEPP_OK && cap[0] > 0 && cap[63] >= cap[0]);
    EXPECT(moepp_set_capacity(cw, cap) == MOEPP_OK);
    cap[63] = -1;
    EXPECT(moepp_set_capacity(cw, cap) == MOEPP_EINVAL);
    EXPECT(moepp_set_capacity(cw, NULL) == MOEPP_OK);
    EXPECT(moepp_destroy(cw) == MOEPP_OK);

    /* Eq.8 at the paper's defaults, both readings of S */
    moepp_desc paper = {32768, 4096, 5632, 16, 1, 1, 2, 2, MOEPP_BF16};
    EXPECT(moepp_capacity(&paper, 32768, 2, 1.1, 0.75, 1, cap) == MOEPP_OK && cap[0] == 3380 && cap[19] == 4506);
    EXPECT(moepp_capacity(&paper, 32768, 2, 1.1, 0.75, 0, cap) == MOEPP_OK && cap[0] == 1690 && cap[19] == 2253);
    EXPECT(moepp_capacity(&paper, 32769, 2, 1.1, 0.75, 1, cap) == MOEPP_EINVAL);
    EXPECT(moepp_capacity(&paper, 16, 2, 0.0, 0.75, 1, cap) == MOEPP_EINVAL);

    /* calls that must be refused before anything is launched */
    EXPECT(moepp_layer_forward(ctx, NULL, 129, fake, fake, fake, fake, fake, fake, fake, 2, fake, fake) == MOEPP_EINVAL);
    EXPECT(moepp_layer_forward(ctx, NULL, 16, NULL, fake, fake, fake, fake, fake, fake, 2, fake, fake) == MOEPP_EINVAL);
    EXPECT(moepp_layer_forward(ctx, NULL, 16, fake, NULL, fake, fake, fake, fake, fake, 2, fake, fake) == MOEPP_EINVAL);
    EXPECT(moepp_layer_forward(ctx, NULL, 16, fake, fake, fake, fake, fake, fake, fake, 3, fake, fake) == MOEPP_EINVAL);
    EXPECT(moepp_layer_forward(ctx, NULL, 16, fake, fake, fake, fake, fake, fake, fake, 2, odd, fake) == MOEPP_EINVAL);
    EXPECT(moepp_layer_forward(ctx, NULL, 0, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 2, NULL, NULL) == MOEPP_OK);
    EXPECT(moepp_route(ctx, NULL, 16, fake, fake, fake, NULL, fake, 2, fake) == MOEPP_EINVAL);
    EXPECT(moepp_permute(ctx, NULL, 1000, 2) == MOEPP_EINVAL);
    EXPECT(moepp_expert_ffn(ctx, NULL, 16, fake, NULL, 2) == MOEPP_EINVAL);
    EXPECT(moepp_combine(ctx, NULL, 16, fake, fake, 2, NULL) == MOEPP_EINVAL);
    EXPECT(moepp_set_variant(ctx, 4) == MOEPP_EINVAL && moepp_set_variant(ctx, 2) == MOEPP_OK);
    EXPECT(moepp_set_router_bias(ctx, (const float *)odd) == MOEPP_EINVAL);
    EXPECT(moepp_set_balance(ctx, 0.75) == MOEPP_OK);
    EXPECT(moepp_permute(ctx, NULL, 16, 2) == MOEPP_EINVAL);     /* statistics on, no routed call */
    EXPECT(moepp_set_balance(ctx, 0.0) == MOEPP_OK);
    moepp_experts ex = {fake, NULL, fake};
    EXPECT(moepp_pack_experts(ctx, NULL, &ex, fake, moepp_packed_bytes(&d)) == MOEPP_EINVAL);
    EXPECT(moepp_pack_experts(ctx, NULL, &ex, fake, 16) == MOEPP_ENOMEM);

    const int32_t *p_idx = NULL, *p_cnt = NULL, *p_off = NULL, *p_row = NULL, *p_src = NULL, *p_kept = NULL;
    const float *p_w = NULL, *p_f = NULL, *p_P = NULL, *p_loss = NULL, *p_a = NULL;
    const void *p_h = NULL, *p_y = NULL;
    EXPECT(moepp_get_routing(ctx, &p_idx, &p_w, &p_cnt, &p_off, &p_row, &p_src) == MOEPP_OK && p_idx && p_src);
    EXPECT(moepp_get_intermediates(ctx, &p_a, &p_h, &p_y) == MOEPP_OK && p_h && p_y);
    EXPECT(moepp_get_kept(ctx, &p_kept) == MOEPP_OK && p_kept);
    EXPECT(moepp_get_balance(ctx, &p_f, &p_P, &p_loss) == MOEPP_OK && p_loss);
    float ms[MOEPP_NUM_KERNELS];
    EXPECT(moepp_get_timing(ctx, NULL) == MOEPP_EINVAL);
    EXPECT(moepp_get_timing(ctx, ms) == MOEPP_OK && ms[0] == 0.f);

    /* the entry point on the library's static scratch */
    EXPECT(moepp_layer_forward_static(&d, NULL, 16, NULL, fake, fake, fake, fake, fake, fake, 2, fake, fake) == MOEPP_EINVAL);
    moepp_desc huge = {1 << 16, 4096, 5632, 16, 1, 1, 2, 2, MOEPP_BF16};
    EXPECT(moepp_workspace_bytes(&huge) > MOEPP_STATIC_SCRATCH_BYTES);
    EXPECT(moepp_layer_forward_static(&huge, NULL, 16, fake, fake, fake, fake, fake, fake, fake, 2, fake, fake) == MOEPP_ENOMEM);
    EXPECT(moepp_layer_forward_static(&d, NULL, 0, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 2, NULL, NULL) == MOEPP_OK);

    EXPECT(strcmp(moepp_status_str(MOEPP_ENOMEM), "buffer too small") == 0);
    EXPECT(strcmp(moepp_status_str(-99), "unknown status") == 0);
    EXPECT(moepp_destroy(ctx) == MOEPP_OK);
    EXPECT(moepp_destroy(NULL) == MOEPP_EINVAL);
    if (failures == 0) printf("ok\n");
    return failures != 0;
}
