/* Plain C11 client of the C-ABI: shows that include/cmn.h is valid C, that the
 * library links without any C++ or Python, and exercises the host-only calls
 * (no kernel is launched, so it runs without a GPU).  Built and run by
 * tests/test_host_api.py. */
#include <stdio.h>
#include <stdlib.h>

#include "cmn.h"

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            fprintf(stderr, "abi_check failed at line %d: %s\n", __LINE__, #cond); \
            return 1;                                                      \
        }                                                                  \
    } while (0)

int main(void)
{
    const int64_t numel[4] = {5000, 0, 37, 100000};
    cmn_plan *plan = NULL;
    CHECK(cmn_plan_create(&plan, 4, numel, 3, 6, 256, CMN_F32, 1) == CMN_OK);
    CHECK(plan != NULL);
    CHECK(cmn_plan_total_elems(plan) == 105037);
    /* ceil(105037 / 6) = 17507 -> next multiple of 64 = 17536 */
    CHECK(cmn_plan_chunk_elems(plan) == 17536);
    CHECK(cmn_plan_padded_elems(plan) == 6 * 17536);
    CHECK(cmn_plan_workspace_bytes(plan) % 256 == 0);

    int64_t n = cmn_plan_tile_count(plan);
    CHECK(n > 0);
    cmn_tile *tiles = (cmn_tile *)malloc((size_t)n * sizeof(cmn_tile));
    CHECK(tiles != NULL);
    CHECK(sizeof(cmn_tile) == 32);
    CHECK(cmn_plan_describe_tiles(plan, NULL, NULL, NULL, NULL, NULL, tiles) == CMN_OK);
    int64_t covered[4] = {0, 0, 0, 0};
    for (int64_t i = 0; i < n; ++i) {
        CHECK(tiles[i].tensor >= 0 && tiles[i].tensor < 4);
        CHECK(tiles[i].e0 == covered[tiles[i].tensor]);   /* in order, no gaps */
        CHECK(tiles[i].len > 0 && tiles[i].start_rank >= 0 && tiles[i].start_rank < 3);
        CHECK(tiles[i].head[CMN_HEAD_STEP] == -1);        /* nothing bound */
        covered[tiles[i].tensor] += tiles[i].len;
    }
    for (int t = 0; t < 4; ++t) CHECK(covered[t] == numel[t]);
    free(tiles);

    CHECK(cmn_allreduce_step(plan, 0.1f, 0.9f, 0.0f, CMN_MEAN_NONE, NULL) == CMN_EUNBOUND);
    CHECK(cmn_adam(plan, 1e-3f, 0.9f, 0.999f, 1e-8f, 0.0f, 1, NULL) == CMN_EUNBOUND);
    CHECK(cmn_plan_destroy(plan) == CMN_OK);
    CHECK(cmn_plan_create(&plan, 4, numel, 0, 6, 256, CMN_F32, 1) == CMN_EINVAL && plan == NULL);
    CHECK(cmn_strerror(CMN_EALIGN)[0] != '\0');
    CHECK(cmn_plan_destroy(NULL) == CMN_OK);
    puts("abi_check ok");
    return 0;
}
