/* Drives the oracle (compiled into this program) through the Tiny configuration under AddressSanitizer
 * and UndefinedBehaviorSanitizer: generator, sampler, hot nodes, rankings, the simulator with a window, a CPU
 * buffer, both policies and several rows per line, data plane on.  Built and run by tests/test_oracle_pins.py;
 * any sanitizer report ends the program with a non-zero status. */
#include "../oracle/gids_oracle.c"

#include <stdio.h>

#define CHECK(x) do { if (!(x)) { printf("check failed at line %d: %s\n", __LINE__, #x); return 1; } } while (0)

int main(void) {
    const uint64_t seed = 0x6A1D50001ull;
    const int64_t n = 10000;
    const int32_t fanouts[2] = {10, 5};
    go_graph* g = go_graph_create(seed, n, 1.0360073614865544, 4, 9999);
    CHECK(g && go_graph_edges(g) > 0);
    int64_t hot[500];
    CHECK(go_hot_nodes(g, 500, hot) == GO_OK);
    uint64_t* scores = (uint64_t*)malloc((size_t)n * sizeof(uint64_t));
    CHECK(go_visit_scores(g, fanouts, 2, 256, scores) == GO_OK);
    CHECK(go_reverse_pagerank(g, 55705, 5, scores) == GO_OK);
    free(scores);

    const int32_t dim = 128;
    float table[65536];
    for (int i = 0; i < 65536; i++) table[i] = (float)i;
    char* store = (char*)malloc((size_t)n * dim * sizeof(float));
    for (int64_t v = 0; v < n; v++) go_feat_row(seed, v, dim, 4, table, store + (size_t)v * dim * 4);

    for (int variant = 0; variant < 3; variant++) {
        const int64_t rows_per_line = variant == 2 ? 4 : 1;
        go_sim* s = go_sim_create(n, 1024, 4, 4, dim * 4, rows_per_line * dim * 4, store);
        CHECK(s);
        CHECK(go_sim_set_hot(s, hot, 500) == GO_OK);
        if (variant == 1) CHECK(go_sim_set_policy(s, 1, 99) == GO_OK);
        if (variant == 2) CHECK(go_sim_set_rows_per_line(s, rows_per_line) == GO_OK);
        CHECK(go_sim_set_accum(s, variant == 0 ? 9000 : 2000, variant == 1) == GO_OK);   /* the accumulator, both modes */
        enum { NB = 20, CAP = 256 * (1 + 10 + 50) };
        int64_t* raw[NB];
        int64_t len[NB];
        for (int b = 0; b < NB; b++) {
            raw[b] = (int64_t*)malloc(CAP * sizeof(int64_t));
            len[b] = go_sample(g, seed, b, fanouts, 2, 256, raw[b], CAP);
            CHECK(len[b] > 0 && len[b] <= CAP);
        }
        int64_t* uniq = (int64_t*)malloc(CAP * sizeof(int64_t));
        char* out = (char*)malloc((size_t)CAP * dim * 4);
        int32_t* cls = (int32_t*)malloc(CAP * sizeof(int32_t));
        int pushed = 0;
        for (int t = 0; t < NB; t++) {
            while (pushed < NB && pushed <= t + 4) { CHECK(go_sim_push(s, raw[pushed], len[pushed]) == GO_OK); pushed++; }
            int64_t stats[5];
            int64_t m = go_sim_gather(s, raw[t], len[t], uniq, out, stats, cls);
            CHECK(m > 0 && stats[1] + stats[2] + stats[3] == stats[0]);
            int64_t acc[3];
            go_sim_accum_last(s, acc);
            CHECK(acc[0] >= 0 && (acc[1] == 0 || acc[0] == 0) && acc[2] >= 2000);
            for (int64_t j = 0; j < m; j += 97)
                CHECK(memcmp(out + (size_t)j * dim * 4, store + (size_t)uniq[j] * dim * 4, (size_t)dim * 4) == 0);
        }
        CHECK(go_sim_flush(s) >= 0);
        CHECK(go_sim_push(s, raw[0], len[0]) == GO_OK);         /* a list left in the window is freed with it */
        for (int b = 0; b < NB; b++) free(raw[b]);
        free(uniq); free(out); free(cls);
        go_sim_free(s);
    }
    free(store);
    go_graph_free(g);
    printf("oracle sanitize ok\n");
    return 0;
}
