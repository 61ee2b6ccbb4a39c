/* Host-sanitizer driver for libilre's host code (test infrastructure).  tests/test_sanitizers.py builds the
 * library with the host pass under -fsanitize=address,undefined and links this program against it.  Everything
 * here is answered on the host: workspace sizing over a sweep of shapes (the scoring plan and the selection
 * layout) and calls whose arguments are refused before anything is enqueued.  Pointers named `fake` are never
 * dereferenced by a correct library; a library that did would trip the sanitizer. */
#include <stdio.h>
#include <string.h>

#include "ilre.h"

static int failures = 0;
#define EXPECT(call, want)                                                                  \
    do {                                                                                    \
        const int got_ = (call);                                                            \
        if (got_ != (want)) {                                                               \
            printf("line %d: %s -> %d (%s), wanted %d\n", __LINE__, #call, got_, ilre_last_error(), (want)); \
            ++failures;                                                                     \
        }                                                                                   \
    } while (0)

static ilre_opts base_opts(void)
{
    ilre_opts o;
    memset(&o, 0, sizeof o);
    o.struct_size = (int32_t)sizeof o;
    o.dtype = ILRE_BF16;
    o.n_pool_kernels = 2;
    return o;
}

int main(void)
{
    void *fake = (void *)(size_t)4096;
    const int32_t kern[2] = {3, 7}, even[2] = {3, 4}, huge[2] = {3, 4095};
    const int32_t mk[3] = {2, 4, 8}, ak[16] = {1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16};
    size_t bytes = 0, prev = 0;

    /* sizing sweep: monotone in L, finite, both element types, the paper's head counts */
    const int64_t Ls[] = {1, 2, 127, 128, 129, 4096, 32768, 131072, 1 << 20, (1ll << 31) - 1};
    const int shapes[][3] = {{32, 8, 256}, {28, 4, 256}, {64, 8, 128}, {8, 8, 1}, {5, 1, 33}};
    for (unsigned s = 0; s < sizeof shapes / sizeof shapes[0]; ++s) {
        for (int dt = 0; dt < 2; ++dt) {
            prev = 0;
            for (unsigned i = 0; i < sizeof Ls / sizeof Ls[0]; ++i) {
                EXPECT(ilre_workspace_bytes(Ls[i], shapes[s][2], shapes[s][0], shapes[s][1], 128, 5, dt, &bytes), ILRE_OK);
                if (bytes < prev || bytes == 0) {
                    printf("workspace not monotone at L=%lld\n", (long long)Ls[i]);
                    ++failures;
                }
                prev = bytes;
                EXPECT(ilre_workspace_bytes_max_avg(Ls[i], shapes[s][2], shapes[s][0], shapes[s][1], 128, Ls[i] > 4 ? 4 : 0, mk, 3, 16,
                                                    dt, &bytes), ILRE_OK);
            }
        }
    }
    EXPECT(ilre_workspace_bytes(0, 32, 32, 8, 128, 3, 0, &bytes), ILRE_EINVAL);
    EXPECT(ilre_workspace_bytes(4096, 32, 30, 8, 128, 3, 0, &bytes), ILRE_EINVAL);
    EXPECT(ilre_workspace_bytes(4096, 32, 32, 8, 64, 3, 0, &bytes), ILRE_EUNSUPPORTED);
    EXPECT(ilre_workspace_bytes(4096, 32, 32, 8, 128, 3, 0, NULL), ILRE_EINVAL);

    ilre_opts o = base_opts();
    /* refused before any device call */
    EXPECT(ilre_recall(NULL, fake, 1000, 8, 8, 2, 128, 64, kern, fake, fake, &o), ILRE_ENOMEM); /* workspace is checked first */
    EXPECT(ilre_recall(fake, fake, 1000, 8, 8, 2, 128, 64, kern, NULL, fake, &o), ILRE_EINVAL);
    EXPECT(ilre_recall(fake, fake, 1000, 8, 8, 2, 128, 64, kern, fake, fake, NULL), ILRE_EINVAL);
    EXPECT(ilre_recall(fake, fake, 1000, 8, 8, 2, 128, 64, even, fake, fake, &o), ILRE_EINVAL);
    EXPECT(ilre_recall(fake, fake, 1000, 8, 8, 2, 128, 64, huge, fake, fake, &o), ILRE_EUNSUPPORTED);
    EXPECT(ilre_recall(fake, fake, 1000, 8, 8, 2, 128, 0, kern, fake, fake, &o), ILRE_EINVAL);
    EXPECT(ilre_recall(fake, fake, 100000, 8, 8, 2, 128, 9000, kern, fake, fake, &o), ILRE_EUNSUPPORTED);
    o.sink = 2000;
    EXPECT(ilre_recall(fake, fake, 1000, 8, 8, 2, 128, 64, kern, fake, fake, &o), ILRE_EINVAL);
    o.sink = -1;
    EXPECT(ilre_select(fake, 1000, 64, kern, fake, &o), ILRE_EINVAL);
    o = base_opts();
    o.struct_size = 8;
    EXPECT(ilre_select(fake, 1000, 64, kern, fake, &o), ILRE_EINVAL);
    o = base_opts();
    o.score_mode = 9;
    EXPECT(ilre_col_scores(fake, fake, 1000, 8, 8, 2, 128, fake, fake, fake, &o), ILRE_EUNSUPPORTED);
    o = base_opts();
    EXPECT(ilre_select(fake, 1000, 64, kern, fake, &o), ILRE_ENOMEM);
    EXPECT(ilre_select(NULL, 1000, 64, kern, fake, &o), ILRE_EINVAL);
    EXPECT(ilre_select_max_avg(fake, 1000, 4, 64, mk, 3, ak, 16, fake, NULL, &o), ILRE_ENOMEM);
    EXPECT(ilre_select_max_avg(fake, 1000, 1001, 64, mk, 3, ak, 16, fake, NULL, &o), ILRE_EINVAL);
    EXPECT(ilre_select_max_avg(fake, 1000, 4, 64, mk, 0, ak, 16, fake, NULL, &o), ILRE_EINVAL);
    EXPECT(ilre_row_stats(fake, fake, 1000, 8, 8, 2, 128, NULL, fake, &o), ILRE_EINVAL);
    EXPECT(ilre_row_stats(fake, fake, 1000, 8, 8, 2, 128, fake, fake, &o), ILRE_ENOMEM);
    EXPECT(ilre_row_stats_static(fake, fake, 1 << 20, 16384, 64, 64, 128, fake, fake, &o), ILRE_EUNSUPPORTED);
    EXPECT(ilre_gather_ids(fake, 0, fake, 4, fake, &o), ILRE_EINVAL);
    EXPECT(ilre_gather_ids(fake, 100, fake, 0, fake, &o), ILRE_OK); /* nothing to do, nothing enqueued */
    EXPECT(ilre_rerope_keys(fake, fake, 1000, 2, 128, 0, 0, 10000.0, NULL, ILRE_ROPE_HALF, &o), ILRE_EINVAL);
    EXPECT(ilre_rerope_keys(fake, fake, 1000, 2, 128, 64, 0, -1.0, NULL, ILRE_ROPE_HALF, &o), ILRE_EINVAL);
    EXPECT(ilre_probe_mfma_ceiling(99, 10, fake, fake, (double *)fake, &o), ILRE_EINVAL);
    /* strides: rows may not overlap, 16-byte multiples; and the 32-bit tile offsets of the key stream */
    o.workspace = fake;
    o.workspace_bytes = (size_t)1 << 40;
    o.workspace = (void *)(size_t)(1 << 20);
    o.k_stride_token = 64;
    EXPECT(ilre_row_stats(fake, fake, 1000, 8, 8, 2, 128, fake, fake, &o), ILRE_EINVAL);
    o.k_stride_token = (int64_t)1 << 26;
    o.k_stride_head = 128;
    EXPECT(ilre_row_stats(fake, fake, 1000, 8, 8, 2, 128, fake, fake, &o), ILRE_EUNSUPPORTED);
    if (ilre_probe_describe(0) == NULL || ilre_probe_describe(1000) != NULL) ++failures;
    printf("%d failures\n", failures);
    return failures ? 1 : 0;
}
