/*
 * The C ABI used from plain C99: the header compiles as C, every entry point links with the prototype the
 * header gives it, and the argument errors that are found before any device work come back as codes with a
 * reason.  Needs no GPU.  Built and run by tests/test_abi.py.
 */
#include <stdio.h>
#include <string.h>

#include "gmpgr_ann.h"

#define CHECK(cond)                                                          \
    do {                                                                     \
        if (!(cond)) {                                                       \
            printf("FAILED line %d: %s (last error: %s)\n", __LINE__, #cond, ann_last_error()); \
            return 1;                                                        \
        }                                                                    \
    } while (0)

int main(void) {
    /* one pointer per entry point, typed by the header: a changed signature fails to compile here */
    int (*p_graph_load)(const int32_t *, const void *, int64_t, int32_t, int32_t, int32_t, uint32_t, void *,
                        ann_graph **) = ann_graph_load;
    int (*p_search)(const ann_graph *, const ann_mlp *, const void *, int32_t, const int32_t *, int32_t, int32_t,
                    int32_t, int32_t, int32_t, void *, size_t, int32_t *, float *, void *) = ann_search;
    int (*p_brute)(const ann_graph *, const ann_mlp *, const void *, int32_t, int32_t, int32_t *, float *, void *,
                   size_t, void *) = ann_brute_force;
    int (*p_pairs)(const ann_graph *, const ann_mlp *, const void *, int32_t, int64_t, const int32_t *,
                   const int32_t *, float *, int32_t, void *) = ann_score_pairs;
    size_t (*p_ws)(const ann_graph *, const ann_mlp *, int32_t, int32_t, int32_t, int32_t, int32_t, int32_t) =
        ann_search_workspace_bytes;
    void *others[] = {(void *)ann_graph_free, (void *)ann_graph_set_locality,
                      (void *)ann_search_visited_set_is_bitmap, (void *)ann_mlp_load, (void *)ann_mlp_free, (void *)ann_mlp_uses_mfma,
                      (void *)ann_search_ragged, (void *)ann_search_layers_workspace_bytes, (void *)ann_search_layers,
                      (void *)ann_search_walkers_workspace_bytes, (void *)ann_search_walkers,
                      (void *)ann_search_stream_workspace_bytes, (void *)ann_search_stream, (void *)ann_stream_open,
                      (void *)ann_stream_submit, (void *)ann_stream_step, (void *)ann_stream_drain,
                      (void *)ann_stream_close, (void *)ann_users_add_noise, (void *)ann_quantize_e4m3,
                      (void *)ann_score_pairs_noalloc, (void *)ann_rerank, (void *)ann_rerank_workspace_bytes,
                      (void *)ann_brute_force_workspace_bytes, (void *)ann_set_progress_timeout, (void *)ann_search_stats,
                      (void *)ann_profile_enable, (void *)ann_profile_read, (void *)ann_profile_copy,
                      (void *)ann_last_error};
    size_t i;
    for (i = 0; i < sizeof(others) / sizeof(others[0]); ++i) CHECK(others[i] != NULL);

    /* argument errors, found before anything touches a device */
    {
        ann_graph *g = NULL;
        char fake[512];
        int32_t ids[4];
        float sc[4];
        memset(fake, 0, sizeof fake);
        CHECK(p_graph_load(NULL, fake, 10, 4, 8, ANN_F32, 0, NULL, &g) == ANN_EINVAL && g == NULL);
        CHECK(strlen(ann_last_error()) > 0);
        CHECK(p_graph_load((const int32_t *)fake, fake, 0, 4, 8, ANN_F32, 0, NULL, &g) == ANN_EINVAL);
        CHECK(p_graph_load((const int32_t *)fake, fake, 10, 4, 8, 17, 0, NULL, &g) == ANN_EINVAL);
        /* without ANN_VALIDATE a graph handle is host bookkeeping only */
        CHECK(p_graph_load((const int32_t *)fake, fake, 10, 4, 8, ANN_F32, 0, NULL, &g) == ANN_OK && g != NULL);
        CHECK(p_ws(g, NULL, 4, 1, 1, 8, 4, 0) == 0);
        CHECK(p_search(g, NULL, fake, 1, (const int32_t *)fake, 1, 1, 8, 4, 0, fake, sizeof fake, ids, sc, NULL) ==
              ANN_EINVAL);
        CHECK(p_brute(g, NULL, fake, 1, 4, ids, sc, NULL, 0, NULL) == ANN_EINVAL);
        CHECK(ann_brute_force_workspace_bytes(g, NULL, 1, 4) == 0 && ann_rerank_workspace_bytes(g, NULL, 1, 8, 4) == 0);
        CHECK(p_pairs(NULL, NULL, fake, 1, 1, ids, ids, sc, 0, NULL) == ANN_EINVAL);
        CHECK(ann_set_progress_timeout(-1.0) == ANN_EINVAL && ann_set_progress_timeout(600.0) == ANN_OK);
        CHECK(ann_stream_close(NULL) == ANN_OK && ann_stream_submit(NULL, 1) == ANN_EINVAL);
        CHECK(ann_graph_set_locality(NULL, NULL, NULL) == ANN_EINVAL && ann_graph_set_locality(g, NULL, NULL) == ANN_OK);
        ann_graph_free(g);
        ann_graph_free(NULL);
        ann_mlp_free(NULL);
    }
    printf("c abi ok\n");
    return 0;
}
