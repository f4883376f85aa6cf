// Walks the host-side layer of liblory (argument validation, shape checks, workspace and
// merged-save sizing with its block planning, tuning knobs, the profiler's bookkeeping) for a
// build with -fsanitize=address,undefined on the host pass.  No call below reaches a kernel
// launch: every one returns from validation, or only computes sizes.
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "lory.h"

static int failures = 0;
#define EXPECT(cond)                                                  \
    do {                                                              \
        if (!(cond)) {                                                \
            printf("FAILED line %d: %s\n", __LINE__, #cond);          \
            ++failures;                                               \
        }                                                             \
    } while (0)

static lory_shape shape(int B, int L, int T, int d, int dff, int E, int dtype)
{
    lory_shape s;
    s.B = B; s.L = L; s.T = T; s.d = d; s.d_ff = dff; s.E = E; s.dtype = dtype;
    return s;
}

int main()
{
    void *fake = (void *)(uintptr_t)0x7F0000001000ull;   // aligned, never dereferenced on these paths
    void *odd = (void *)(uintptr_t)0x7F0000001004ull;
    for (int i = -1; i < 9; ++i) EXPECT(lory_status_string(i) != NULL && strlen(lory_status_string(i)) > 0);
    EXPECT(strlen(lory_version()) >= 3);

    const int shapes[][7] = {
        {2, 512, 128, 64, 256, 4, LORY_F32},      {8, 4096, 256, 1024, 2816, 8, LORY_BF16},
        {8, 4096, 256, 1024, 2816, 32, LORY_BF16}, {4, 4096, 256, 2048, 5632, 32, LORY_BF16},
        {4, 4096, 64, 2048, 5632, 16, LORY_BF16},  {4, 4096, 1024, 2048, 5632, 16, LORY_BF16},
        {5, 3840, 64, 64, 128, 64, LORY_BF16},     {3, 60, 20, 50, 70, 5, LORY_F32},
        {4, 4096, 256, 4096, 11008, 4, LORY_BF16}, {1, 65536 * 64, 64, 64, 64, 1, LORY_BF16},
    };
    const size_t budgets[] = {(size_t)64 << 10, (size_t)1 << 20, (size_t)128 << 20, (size_t)6144 << 20};
    for (size_t b = 0; b < sizeof(budgets) / sizeof(budgets[0]); ++b) {
        EXPECT(lory_set_slab_budget(budgets[b]) == LORY_OK);
        for (int fused = 0; fused <= 2; ++fused) {
            EXPECT(lory_set_fused_merge(fused) == LORY_OK);
            for (size_t i = 0; i < sizeof(shapes) / sizeof(shapes[0]); ++i) {
                const int *q = shapes[i];
                const lory_shape s = shape(q[0], q[1], q[2], q[3], q[4], q[5], q[6]);
                size_t f = 0, w = 0, m = 0;
                const int rf = lory_workspace_bytes(&s, LORY_PASS_FWD, &f);
                const int rb = lory_workspace_bytes(&s, LORY_PASS_BWD, &w);
                const int rm = lory_merged_save_bytes(&s, &m);
                EXPECT(rf == rb && rb == rm);
                if (rf == LORY_OK) EXPECT(f > 0 && w >= f / 2 && f % 256 == 0 && w % 256 == 0);
            }
        }
    }
    EXPECT(lory_set_slab_budget(1024) == LORY_ERR_SHAPE);
    EXPECT(lory_set_fused_merge(4) == LORY_ERR_SHAPE && lory_set_fused_merge(-1) == LORY_ERR_SHAPE);
    EXPECT(lory_set_slab_budget((size_t)6144 << 20) == LORY_OK && lory_set_fused_merge(1) == LORY_OK);

    size_t out = 0;
    lory_shape ok = shape(2, 512, 128, 64, 256, 4, LORY_F32);
    lory_shape ragged = shape(2, 500, 128, 64, 256, 4, LORY_F32);
    lory_shape manyE = shape(2, 512, 128, 64, 256, 65, LORY_F32);
    lory_shape baddt = shape(2, 512, 128, 64, 256, 4, 7);
    lory_shape gran = shape(2, 512, 32, 64, 256, 4, LORY_BF16);
    EXPECT(lory_workspace_bytes(NULL, 0, &out) == LORY_ERR_NULL);
    EXPECT(lory_workspace_bytes(&ok, 0, NULL) == LORY_ERR_NULL);
    EXPECT(lory_workspace_bytes(&ok, 9, &out) == LORY_ERR_SHAPE);
    EXPECT(lory_workspace_bytes(&ragged, 0, &out) == LORY_ERR_SHAPE);
    EXPECT(lory_workspace_bytes(&manyE, 0, &out) == LORY_ERR_SHAPE);
    EXPECT(lory_workspace_bytes(&baddt, 0, &out) == LORY_ERR_DTYPE);
    EXPECT(lory_workspace_bytes(&gran, 0, &out) == LORY_ERR_SHAPE);
    lory_shape dense = shape(4, 1, 1, 2048, 5632, 1, LORY_BF16);
    EXPECT(lory_workspace_bytes(&dense, LORY_PASS_DENSE, &out) == LORY_OK && out > 0);

    // entry points: NULL, misaligned, small workspace -> status before any launch
    EXPECT(lory_route(&ok, NULL, fake, (float *)fake, NULL, NULL) == LORY_ERR_NULL);
    EXPECT(lory_route(&ok, odd, fake, (float *)fake, NULL, NULL) == LORY_ERR_ALIGN);
    EXPECT(lory_route(&ragged, fake, fake, (float *)fake, NULL, NULL) == LORY_ERR_SHAPE);
    EXPECT(lory_route_bwd(&ok, fake, (float *)fake, (float *)fake, (float *)fake, fake, NULL, 0, NULL) == LORY_ERR_NULL);
    EXPECT(lory_route_bwd(&ok, fake, (float *)fake, (float *)fake, (float *)fake, fake, (float *)fake, 2, NULL) ==
           LORY_ERR_SHAPE);
    EXPECT(lory_merged_ffn_fwd(&ok, fake, (float *)fake, fake, fake, fake, fake, NULL, NULL, NULL, fake, 16, NULL) ==
           LORY_ERR_WORKSPACE);
    EXPECT(lory_merged_ffn_fwd(&ok, fake, (float *)fake, fake, fake, fake, fake, fake, NULL, NULL, fake, 1 << 30,
                               NULL) == LORY_ERR_NULL);   // G without U
    EXPECT(lory_merged_ffn_fwd(&ok, fake, (float *)fake, fake, fake, fake, fake, NULL, NULL, fake, fake, 1 << 30,
                               NULL) == LORY_ERR_SHAPE);  // Wbar_save for fp32
    EXPECT(lory_merged_ffn_bwd(&ok, fake, (float *)fake, fake, fake, fake, fake, NULL, NULL, NULL, fake, fake, fake,
                               fake, LORY_BF16, 0, (float *)fake, fake, 1 << 30, NULL) == LORY_ERR_DTYPE);
    EXPECT(lory_merged_ffn_bwd(&ok, fake, (float *)fake, fake, fake, fake, fake, NULL, NULL, NULL, fake, fake, fake,
                               fake, LORY_F32, 3, (float *)fake, fake, 1 << 30, NULL) == LORY_ERR_SHAPE);
    EXPECT(lory_merged_ffn_bwd(&ok, fake, (float *)fake, fake, fake, fake, fake, NULL, NULL, NULL, fake, fake, fake,
                               fake, LORY_F32, 0, (float *)fake, fake, 16, NULL) == LORY_ERR_WORKSPACE);
    lory_shape inf = shape(2, 40, 40, 64, 128, 4, LORY_F32);
    lory_shape inf_bad = shape(2, 40, 20, 64, 128, 4, LORY_F32);
    EXPECT(lory_prompt_merge(&inf_bad, fake, NULL, fake, fake, fake, fake, (float *)fake, fake, NULL) == LORY_ERR_SHAPE);
    EXPECT(lory_prompt_merge(&inf, fake, NULL, fake, fake, fake, NULL, (float *)fake, fake, NULL) == LORY_ERR_NULL);
    EXPECT(lory_prompt_merge(&inf, fake, (const int32_t *)((char *)fake + 2), fake, fake, fake, fake, (float *)fake,
                             fake, NULL) == LORY_ERR_ALIGN);
    EXPECT(lory_dense_ffn_fwd(&inf, fake, fake, fake, fake, 16, NULL) == LORY_ERR_WORKSPACE);
    EXPECT(lory_dense_ffn_fwd_static(&inf, fake, NULL, fake, NULL) == LORY_ERR_NULL);
    lory_shape big = shape(2, 8, 8, 2048, 5632, 1, LORY_BF16);
    EXPECT(lory_dense_ffn_fwd_static(&big, fake, fake, fake, NULL) == LORY_ERR_WORKSPACE);

    // profiler bookkeeping without launches
    lory_kernel_stat st[8];
    int n = -1;
    EXPECT(lory_profile_read(NULL, 8, &n) == LORY_ERR_NULL);
    EXPECT(lory_profile_read(st, 0, &n) == LORY_ERR_SHAPE);
    EXPECT(lory_profile_read(st, 8, &n) == LORY_OK && n == 0);

    printf("abi sanitizer run: %s (%d failures)\n", failures ? "FAILED" : "ok", failures);
    return failures ? 1 : 0;
}
