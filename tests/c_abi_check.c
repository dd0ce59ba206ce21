/* A plain C99 caller of the boundary: includes the header as C, builds a
 * layout, reads it back, and exercises the error paths that need no GPU.
 * Compiled and run by tests/test_c_abi.py. */
#include <stdio.h>
#include <string.h>

#include "fcdp.h"

#define CHECK(cond)                                                   \
    do {                                                              \
        if (!(cond)) {                                                \
            printf("FAILED line %d: %s\n", __LINE__, #cond);          \
            return 1;                                                 \
        }                                                             \
    } while (0)

int main(void)
{
    const int64_t numel[4] = {1000, 24, 0, 3000};
    const uint8_t trainable[4] = {0, 1, 1, 0};
    fcdp_layout *L = NULL;
    int64_t rows[5 * 16];
    int64_t n;
    fcdp_cache_state *st = NULL;
    fcdp_source src;
    int32_t store, keep;

    CHECK(fcdp_layout_build(numel, trainable, 4, 4, 2, 64, &L) == FCDP_OK);
    CHECK(fcdp_layout_numel(L) == 4024);
    CHECK(fcdp_layout_padded_numel(L) == 4096);
    CHECK(fcdp_layout_shard_numel(L) == 1024);
    CHECK(fcdp_layout_trainable_numel(L) == 24);
    CHECK(fcdp_layout_packed_numel(L) == 256);
    CHECK(fcdp_layout_offsets(L)[4] == 4024);
    n = fcdp_layout_segments(L, rows, 16);
    CHECK(n == 5); /* 1000 | 24 | 3000 split over shards 1, 2, 3 */
    CHECK(rows[0] == 0 && rows[1] == 0 && rows[4] == 1000);
    CHECK(fcdp_layout_copy_plan(L, 2, rows, 16) >= 1); /* pack plan */
    {
        /* a failing build leaves NULL in its own output and the good layout alone */
        fcdp_layout *bad = (fcdp_layout *)rows;
        CHECK(fcdp_layout_build(numel, trainable, 4, 0, 2, 64, &bad) == FCDP_EINVAL);
        CHECK(bad == NULL);
        CHECK(strstr(fcdp_last_error(), "G must be") != NULL);
        CHECK(fcdp_layout_numel(L) == 4024);
    }
    CHECK(fcdp_reduce_grad_shard(NULL, 2, 0, 8, FCDP_F32, FCDP_F32, NULL, NULL) == FCDP_EINVAL);
    CHECK(fcdp_reduce_grad_shard_scaled(NULL, 2, 0, 8, FCDP_F32, FCDP_F32, 0.5f, NULL, NULL) == FCDP_EINVAL);
    CHECK(strcmp(fcdp_status_string(FCDP_OK), "FCDP_OK") == 0);

    CHECK(fcdp_cache_state_create(2, &st) == FCDP_OK);
    CHECK(fcdp_cache_state_forward_source(st, 0, 1, FCDP_SRC_HOST_DMA, &src, &store) == FCDP_OK);
    CHECK(src == FCDP_SRC_DEVICE_SHARDS && store == 1);
    CHECK(fcdp_cache_state_set_tau(st, 0.5) == FCDP_OK);
    CHECK(fcdp_cache_state_place(st, 0, 10, 100, &keep) == FCDP_OK && keep == 1);
    CHECK(fcdp_cache_state_backward_source(st, 0, 1, FCDP_SRC_HOST_DMA, &src) == FCDP_OK);
    CHECK(src == FCDP_SRC_DEVICE_RESIDENT);
    CHECK(fcdp_cache_state_backward_source(st, 1, 1, FCDP_SRC_HOST_DMA, &src) == FCDP_ESTATE);
    /* a store that failed after forward_source handed the class out: dirty again */
    CHECK(fcdp_cache_state_forward_source(st, 1, 0, FCDP_SRC_HOST_DMA, &src, &store) == FCDP_OK && store == 1);
    CHECK(fcdp_cache_state_is_dirty(st, 1, 0) == 0);
    CHECK(fcdp_cache_state_mark_dirty(st, 1, 0) == FCDP_OK);
    CHECK(fcdp_cache_state_is_dirty(st, 1, 0) == 1);
    CHECK(fcdp_cache_state_mark_dirty(st, 2, 0) == FCDP_EINVAL);
    fcdp_cache_state_destroy(st);
    fcdp_layout_destroy(L);
    printf("c abi ok\n");
    return 0;
}
