/* Compiled as plain C by tests/test_abi.py: the header must be valid C99 and
 * the host-only entry points callable without a GPU. */
#include <stdio.h>
#include <string.h>

#include "gids.h"

int main(void) {
    gids_store* store = NULL;
    gids_cache* cache = NULL;
    gids_stats st;
    memset(&st, 0, sizeof st);
    /* Eq. 2-3 of Section 3.2 with the numbers of Section 4.2 */
    double n = gids_accum_threshold(1.5e6, 25e-6, 5e-6, 0.95, 1);
    if (n < 854.9 || n > 855.1) { printf("threshold %f\n", n); return 1; }
    if (gids_store_create(0, 64, 8, NULL, &store) != GIDS_E_INVAL || store) return 2;
    if (gids_cache_create(NULL, 8, 2, 64, 0, 0, &cache) != GIDS_E_INVAL || cache) return 3;
    if (!strlen(gids_last_error())) return 4;
    if (gids_sample_capacity(NULL, 0, 7) != 7) return 5;
    {
        const uint32_t f[3] = {10, 10, 10};
        if (gids_sample_capacity(f, 3, 4096) != 4096ull * 1111) return 6;
    }
    if (gids_graph_reverse_pagerank(NULL, 55705, 10, NULL, NULL) != GIDS_E_INVAL) return 7;
    if (gids_cache_set_rows_per_line(NULL, 8) != GIDS_E_INVAL) return 8;
    printf("abi ok %zu\n", sizeof(gids_stats));
    return 0;
}
