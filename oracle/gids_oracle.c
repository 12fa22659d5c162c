/* CPU oracle for the minibatch feature gather of the GIDS dataloader.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, single-threaded, deliberately slow C that
 * the tests, the smoke check and the benchmark's cpu_baseline leg compare the
 * HIP library against.  It shares no code with the HIP path and the HIP path
 * never calls it.
 *
 * What it covers, and the passage of the paper each part follows:
 *   - seeded power-law graph generator and feature closed form (synthetic
 *     stand-ins for the datasets of Section 4.1, Tables 2-3);
 *   - neighbourhood sampler: up to `fanout` neighbours per node per layer,
 *     uniformly at random (Section 2.2.2 and its two-layer worked example);
 *   - feature aggregation: out[j] = feature row of the j-th distinct node ID
 *     of the minibatch, ascending (Section 2.2.3);
 *   - constant CPU buffer: IDs pinned there are redirected to it and never
 *     enter the GPU cache (Section 3.3);
 *   - set-associative software cache with window buffering: a per-node count
 *     of the buffered future minibatches that reuse the node; lines whose
 *     count is positive are in the "USE" state and are not evicted, count 0 is
 *     "safe to evict" (Section 3.4, Fig. 6 steps 1-5);
 *   - the overlapped-access model N = r/(1-r) * IOPS * (Ti + Tt) (Section 3.2,
 *     Eq. 2-3), and the accumulator that merges minibatches until their node
 *     accesses reach a threshold, fixed or raised by the redirected share
 *     (Section 3.2);
 *   - the random base policy of the cache the paper builds on (Section 3.4),
 *     seeded; cache lines that hold several node rows (4 KB cache-lines,
 *     Section 3.3, under rows of 512 B and more, Section 2.1);
 *   - hot-node rankings: weighted reverse PageRank (the metric Section 3.3
 *     names) and the expected visits under this sampler.
 *
 * Parity pins (see tests/): brute-force row equality, count conservation,
 * cache >= store => only first-touch misses, depth 0 == textbook per-set LRU
 * by batch, pinned lines never evicted, CPU-buffer hits == |U ∩ P|, a
 * hand-traced fully-associative case, the sampler's worked example; the
 * random policy's uniformity and an independent model of its hash order;
 * several rows per line by reduction to the one-row simulator over line
 * numbers; PageRank against ring / chain / star closed forms and a linear
 * solve; visit scores against closed forms and the sampler's frequencies.  The
 * tie-breaks of the replacement policy (lowest way first, ascending ID first,
 * bypass when nothing is evictable) are fixed by this project, not the paper:
 * for those constants alone, parity unpinned.  The same holds for two
 * readings the paper leaves open: that a line of several rows stays while any
 * of its rows is needed again, and the exact weighting of the reverse
 * PageRank (the paper cites the metric without a formula).
 *
 * The replacement policy is batch-synchronous: every ID of a minibatch is
 * classified against the cache state at the start of the minibatch, then the
 * misses are installed set by set.  The paper's base policy is random
 * eviction; here it is least-recently-used by minibatch stamp so that two
 * implementations can agree bit for bit.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define GO_OK 0
#define GO_E_INVAL (-1)
#define GO_E_NOMEM (-2)
#define GO_E_RANGE (-3)
#define GO_E_ORDER (-4)
#define GO_E_FULL (-5)

/* ---------------------------------------------------------------- hashing */

static uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

enum { TAG_DEG = 1, TAG_EDGE = 2, TAG_FEAT = 3, TAG_SEED = 4, TAG_NBR = 5 };

static uint64_t key0(uint64_t seed, uint64_t tag) {
    return mix64(seed + tag * 0x9E3779B97F4A7C15ull);
}

uint64_t go_mix64(uint64_t z) { return mix64(z); }

/* ------------------------------------------------------------------ graph */

typedef struct {
    int64_t n, e;
    int64_t* indptr;   /* n + 1 */
    int64_t* indices;  /* e */
    uint64_t seed;
} go_graph;

static int64_t degree_of(uint64_t seed, int64_t v, double ell, int p4, int64_t d_max) {
    uint64_t h = mix64(key0(seed, TAG_DEG) ^ (uint64_t)v);
    double x = ((double)(h >> 32) + 1.0) / 4294967296.0;   /* (0, 1] */
    double q = sqrt(sqrt(x));
    double y = q;
    for (int i = 1; i < p4; i++) y = y * q;                /* x^(p4/4) */
    double d = floor(ell / y);
    if (d < 1.0) d = 1.0;
    if (d > (double)d_max) d = (double)d_max;
    return (int64_t)d;
}

/* the node u with indptr[u] <= slot < indptr[u+1] */
static int64_t owner_of(const int64_t* indptr, int64_t n, int64_t slot) {
    int64_t lo = 0, hi = n;            /* answer in [lo, hi) */
    while (hi - lo > 1) {
        int64_t mid = lo + (hi - lo) / 2;
        if (indptr[mid] <= slot) lo = mid; else hi = mid;
    }
    return lo;
}

go_graph* go_graph_create(uint64_t seed, int64_t n, double ell, int p4, int64_t d_max) {
    if (n < 2 || p4 < 1 || d_max < 1) return NULL;
    go_graph* g = (go_graph*)calloc(1, sizeof(go_graph));
    if (!g) return NULL;
    g->n = n; g->seed = seed;
    g->indptr = (int64_t*)malloc((size_t)(n + 1) * sizeof(int64_t));
    if (!g->indptr) { free(g); return NULL; }
    g->indptr[0] = 0;
    for (int64_t v = 0; v < n; v++) g->indptr[v + 1] = g->indptr[v] + degree_of(seed, v, ell, p4, d_max);
    g->e = g->indptr[n];
    g->indices = (int64_t*)malloc((size_t)g->e * sizeof(int64_t));
    if (!g->indices) { free(g->indptr); free(g); return NULL; }
    uint64_t k = key0(seed, TAG_EDGE);
    for (int64_t e = 0; e < g->e; e++) {
        int64_t slot = (int64_t)(mix64(k ^ (uint64_t)e) % (uint64_t)g->e);
        g->indices[e] = owner_of(g->indptr, n, slot);
    }
    return g;
}

/* a graph from caller-given CSR arrays (copied); for hand-built test cases */
go_graph* go_graph_from_csr(int64_t n, const int64_t* indptr, const int64_t* indices) {
    if (n < 1 || indptr[0] != 0) return NULL;
    go_graph* g = (go_graph*)calloc(1, sizeof(go_graph));
    if (!g) return NULL;
    g->n = n; g->e = indptr[n];
    g->indptr = (int64_t*)malloc((size_t)(n + 1) * sizeof(int64_t));
    g->indices = (int64_t*)malloc((size_t)(g->e > 0 ? g->e : 1) * sizeof(int64_t));
    if (!g->indptr || !g->indices) { free(g->indptr); free(g->indices); free(g); return NULL; }
    memcpy(g->indptr, indptr, (size_t)(n + 1) * sizeof(int64_t));
    memcpy(g->indices, indices, (size_t)g->e * sizeof(int64_t));
    return g;
}

void go_graph_free(go_graph* g) { if (g) { free(g->indptr); free(g->indices); free(g); } }
int64_t go_graph_edges(const go_graph* g) { return g->e; }
const int64_t* go_graph_indptr(const go_graph* g) { return g->indptr; }
const int64_t* go_graph_indices(const go_graph* g) { return g->indices; }

typedef struct { int64_t indeg, id; } hot_key;
static int cmp_hot(const void* a, const void* b) {
    const hot_key* x = (const hot_key*)a; const hot_key* y = (const hot_key*)b;
    if (x->indeg != y->indeg) return x->indeg > y->indeg ? -1 : 1;   /* larger in-degree first */
    return (x->id > y->id) - (x->id < y->id);                        /* then lower ID */
}

/* the k nodes of highest in-degree, ties to the lower ID (the configurations'
 * stand-in for the paper's reverse-PageRank hot-node ranking, Section 3.3) */
int go_hot_nodes(const go_graph* g, int64_t k, int64_t* out) {
    if (k < 0 || k > g->n) return GO_E_INVAL;
    hot_key* a = (hot_key*)malloc((size_t)g->n * sizeof(hot_key));
    if (!a) return GO_E_NOMEM;
    for (int64_t v = 0; v < g->n; v++) { a[v].indeg = 0; a[v].id = v; }
    for (int64_t e = 0; e < g->e; e++) a[g->indices[e]].indeg++;
    qsort(a, (size_t)g->n, sizeof(hot_key), cmp_hot);
    for (int64_t i = 0; i < k; i++) out[i] = a[i].id;
    free(a);
    return GO_OK;
}

/* ----------------------------------------------------------- sort-unique */

static int cmp_i64(const void* a, const void* b) {
    int64_t x = *(const int64_t*)a, y = *(const int64_t*)b;
    return (x > y) - (x < y);
}

/* ascending distinct values of raw[0..n); returns their count */
int64_t go_sort_unique(const int64_t* raw, int64_t n, int64_t* out) {
    if (n <= 0) return 0;
    memcpy(out, raw, (size_t)n * sizeof(int64_t));
    qsort(out, (size_t)n, sizeof(int64_t), cmp_i64);
    int64_t m = 1;
    for (int64_t i = 1; i < n; i++) if (out[i] != out[m - 1]) out[m++] = out[i];
    return m;
}

/* ---------------------------------------------------------------- sampler */

/* Raw node-ID list of minibatch `batch` (Section 2.2.2): the seed nodes, then
 * for each layer the sampled neighbours of every frontier node (frontier in
 * ascending ID order), duplicates kept.  A node of degree <= fanout gives all
 * of its neighbours; otherwise `fanout` distinct adjacency slots are drawn
 * without replacement (Floyd's subset sampling on hashed draws).  The next
 * frontier is the distinct set of nodes this hop sampled.
 * Returns the raw count, or a negative error when `cap` is too small. */
static int64_t sample_impl(const go_graph* g, uint64_t seed, int64_t batch, const int32_t* fanouts, int n_layers,
                           int64_t n_seeds, const uint64_t* rank_table, int64_t perm_mult, int64_t perm_add,
                           int64_t* out, int64_t cap) {
    if (n_seeds < 0 || n_seeds > cap) return GO_E_INVAL;
    uint64_t ks = mix64(key0(seed, TAG_SEED) ^ (uint64_t)batch);
    for (int64_t i = 0; i < n_seeds; i++) {
        uint64_t h = mix64(ks ^ (uint64_t)i);
        if (!rank_table) { out[i] = (int64_t)(h % (uint64_t)g->n); continue; }
        /* skewed seeds: rank r = number of cumulative thresholds <= (h >> 1), then the
         * seeded affine permutation (r * mult + add) mod n maps the rank to a node */
        uint64_t u = h >> 1;
        int64_t lo = 0, hi = g->n;                 /* first index with table[index] > u */
        while (lo < hi) {
            int64_t mid = lo + (hi - lo) / 2;
            if (rank_table[mid] <= u) lo = mid + 1; else hi = mid;
        }
        int64_t r = lo < g->n - 1 ? lo : g->n - 1;
        out[i] = (int64_t)(((unsigned __int128)(uint64_t)r * (uint64_t)perm_mult + (uint64_t)perm_add) % (uint64_t)g->n);
    }
    int64_t n_raw = n_seeds;
    int64_t* frontier = (int64_t*)malloc((size_t)(cap > 0 ? cap : 1) * sizeof(int64_t));
    if (!frontier) return GO_E_NOMEM;
    int64_t n_front = go_sort_unique(out, n_seeds, frontier);
    int64_t chosen[64];
    for (int layer = 0; layer < n_layers; layer++) {
        int64_t f = fanouts[layer];
        if (f < 1 || f > 64) { free(frontier); return GO_E_INVAL; }
        uint64_t kl = mix64(mix64(key0(seed, TAG_NBR) ^ (uint64_t)batch) ^ (uint64_t)layer);
        int64_t layer_begin = n_raw;
        for (int64_t i = 0; i < n_front; i++) {
            int64_t v = frontier[i];
            int64_t start = g->indptr[v], deg = g->indptr[v + 1] - start;
            int64_t take = deg <= f ? deg : f;
            if (n_raw + take > cap) { free(frontier); return GO_E_FULL; }
            if (deg <= f) {
                for (int64_t s = 0; s < deg; s++) out[n_raw++] = g->indices[start + s];
            } else {
                uint64_t kv = mix64(kl ^ (uint64_t)v);
                int64_t m = 0;
                for (int64_t j = deg - f; j < deg; j++) {
                    int64_t t = (int64_t)(mix64(kv ^ (uint64_t)j) % (uint64_t)(j + 1));
                    int seen = 0;
                    for (int64_t c = 0; c < m; c++) if (chosen[c] == t) seen = 1;
                    chosen[m++] = seen ? j : t;
                }
                for (int64_t c = 0; c < m; c++) out[n_raw++] = g->indices[start + chosen[c]];
            }
        }
        /* next frontier = the distinct nodes reached by this hop (the worked
         * example expands 1 -> 3 -> 6: only the previous hop's nodes) */
        n_front = go_sort_unique(out + layer_begin, n_raw - layer_begin, frontier);
    }
    free(frontier);
    return n_raw;
}

int64_t go_sample(const go_graph* g, uint64_t seed, int64_t batch, const int32_t* fanouts, int n_layers,
                  int64_t n_seeds, int64_t* out, int64_t cap) {
    return sample_impl(g, seed, batch, fanouts, n_layers, n_seeds, NULL, 0, 0, out, cap);
}

/* the same with seed nodes drawn Zipf-ranked: rank_table[r] = floor(2^63 * CDF(r + 1)) over g->n ranks */
int64_t go_sample_skewed(const go_graph* g, uint64_t seed, int64_t batch, const int32_t* fanouts, int n_layers,
                         int64_t n_seeds, const uint64_t* rank_table, int64_t perm_mult, int64_t perm_add,
                         int64_t* out, int64_t cap) {
    if (!rank_table) return GO_E_INVAL;
    return sample_impl(g, seed, batch, fanouts, n_layers, n_seeds, rank_table, perm_mult, perm_add, out, cap);
}

/* ------------------------------------------------------- hot-node scores */

/* Expected number of times each node appears in a minibatch's raw list under go_sample's law, in 32.32 fixed
 * point (a stand-in for the weighted reverse PageRank the paper ranks hot nodes with, Section 3.3: both
 * estimate how often neighbourhood sampling reaches a node; the paper gives no formula).
 *   lam_0(v) = n_seeds / n                       (uniform seeds)
 *   a node expected c = min(1, lam_l(v)) times in the frontier of hop l takes each of its deg(v) adjacency
 *   slots with probability min(deg, f_l) / deg, so every slot sends w = c * min(deg, f_l) / deg to its
 *   neighbour: lam_(l+1)(u) = sum of w over the slots that point to u
 *   score(u) = lam_0(u) + ... + lam_L(u)
 * Integer arithmetic throughout (floor divisions), so any implementation agrees bit for bit. */
int go_visit_scores(const go_graph* g, const int32_t* fanouts, int n_layers, int64_t n_seeds, uint64_t* scores) {
    const uint64_t ONE = 1ull << 32;
    if (n_seeds < 0 || n_seeds > (1ll << 30)) return GO_E_INVAL;
    uint64_t* cur = (uint64_t*)malloc((size_t)g->n * sizeof(uint64_t));
    uint64_t* nxt = (uint64_t*)malloc((size_t)g->n * sizeof(uint64_t));
    if (!cur || !nxt) { free(cur); free(nxt); return GO_E_NOMEM; }
    const uint64_t lam0 = ((uint64_t)n_seeds << 32) / (uint64_t)g->n;
    for (int64_t v = 0; v < g->n; v++) { cur[v] = lam0; scores[v] = lam0; }
    for (int l = 0; l < n_layers; l++) {
        const uint64_t f = (uint64_t)fanouts[l];
        memset(nxt, 0, (size_t)g->n * sizeof(uint64_t));
        for (int64_t v = 0; v < g->n; v++) {
            const uint64_t deg = (uint64_t)(g->indptr[v + 1] - g->indptr[v]);
            if (!deg || !cur[v]) continue;
            const uint64_t c = cur[v] < ONE ? cur[v] : ONE;
            const uint64_t take = deg < f ? deg : f;
            const uint64_t w = c * take / deg;
            for (int64_t e = g->indptr[v]; e < g->indptr[v + 1]; e++) nxt[g->indices[e]] += w;
        }
        for (int64_t v = 0; v < g->n; v++) scores[v] += nxt[v];
        uint64_t* tmp = cur; cur = nxt; nxt = tmp;
    }
    free(cur); free(nxt);
    return GO_OK;
}

/* Weighted reverse PageRank (the metric Section 3.3 names for choosing hot nodes).  Sampling walks from a
 * node to the nodes in its adjacency list, which is against the direction of the dataset's edges, hence
 * "reverse"; "weighted" because a node of degree deg passes 1/deg of its rank along each adjacency slot.
 * Textbook power iteration with damping d = damping_q16 / 65536 and uniform teleport, total mass 2^44:
 *   base = floor(2^44 / n);  r_0(v) = base;  teleport = floor(base * (65536 - damping_q16) / 65536)
 *   r_(k+1)(u) = teleport + sum over adjacency slots v -> u of floor(floor(r_k(v) * damping_q16 / 65536) / deg v)
 * scores = r_(n_iters).  A node without adjacency slots passes nothing on (its damped mass is dropped).
 * Integer arithmetic throughout, so any implementation agrees bit for bit. */
int go_reverse_pagerank(const go_graph* g, uint32_t damping_q16, int n_iters, uint64_t* scores) {
    if (damping_q16 > 65536u || n_iters < 0) return GO_E_INVAL;
    uint64_t* nxt = (uint64_t*)malloc((size_t)g->n * sizeof(uint64_t));
    if (!nxt) return GO_E_NOMEM;
    const uint64_t base = (1ull << 44) / (uint64_t)g->n;
    const uint64_t teleport = base * (65536u - damping_q16) >> 16;
    uint64_t* cur = scores;
    for (int64_t v = 0; v < g->n; v++) cur[v] = base;
    for (int k = 0; k < n_iters; k++) {
        for (int64_t v = 0; v < g->n; v++) nxt[v] = teleport;
        for (int64_t v = 0; v < g->n; v++) {
            const uint64_t deg = (uint64_t)(g->indptr[v + 1] - g->indptr[v]);
            if (!deg) continue;
            const uint64_t w = (cur[v] * damping_q16 >> 16) / deg;
            for (int64_t e = g->indptr[v]; e < g->indptr[v + 1]; e++) nxt[g->indices[e]] += w;
        }
        memcpy(cur, nxt, (size_t)g->n * sizeof(uint64_t));
    }
    free(nxt);
    return GO_OK;
}

/* --------------------------------------------------------------- features */

/* feat(v, c) for c = 0..dim-1 into out: four table indices per hashed word */
void go_feat_row(uint64_t seed, int64_t v, int32_t dim, int32_t itemsize, const void* table, void* out) {
    uint64_t kv = mix64(key0(seed, TAG_FEAT) ^ (uint64_t)v);
    for (int32_t c = 0; c < dim; c++) {
        uint64_t w = mix64(kv ^ (uint64_t)(c >> 2));
        uint32_t idx = (uint32_t)((w >> (16 * (c & 3))) & 0xFFFF);
        memcpy((char*)out + (size_t)c * itemsize, (const char*)table + (size_t)idx * itemsize, (size_t)itemsize);
    }
}

/* ----------------------------------------------- overlapped-access model */

/* Section 3.2, Eq. 2-3: N = IOPS_achieved * (Ti + Ts + Tt) * n_ssd with
 * Ts = N / (IOPS_peak * n_ssd) (per-SSD peak; all SSDs serve the N accesses
 * together).  Solved for N at IOPS_achieved = ratio * IOPS_peak. */
double go_accum_threshold(double iops_peak, double t_initial, double t_termination, double ratio, int n_ssd) {
    return ratio / (1.0 - ratio) * iops_peak * (double)n_ssd * (t_initial + t_termination);
}

/* -------------------------------------------------------------- simulator */

typedef struct {
    int64_t n_rows, lines, n_sets;
    int32_t ways, window;              /* window = number of future minibatches visible */
    int64_t row_bytes, line_bytes;
    int64_t t;                         /* index of the next minibatch to gather */
    int64_t* tag;                      /* lines, -1 = empty */
    int64_t* stamp;                    /* lines, -1 = never used */
    int32_t* reuse;                    /* n_rows: buffered future minibatches that contain the node */
    int64_t* hot_slot;                 /* n_rows: slot in the CPU buffer or -1 */
    int64_t n_hot;
    /* FIFO of buffered minibatch ID lists: the one to gather next + `window` later ones */
    int64_t** win_ids; int64_t* win_n; int32_t win_count;
    /* optional data plane */
    const char* store; char* cache_data; char* cpu_buf;
    /* base replacement policy: 0 = least recently used by minibatch, 1 = seeded random (BaM's policy, Section 3.4) */
    int32_t policy; uint64_t policy_seed;
    /* node rows per cache line (1 unless go_sim_set_rows_per_line): line `b` of the store = rows b*P .. b*P+P-1 */
    int64_t rows_per_line;
    /* storage access accumulator (Section 3.2): minibatches are merged until their node accesses reach a
     * threshold; acc_* describe the open group, hist_* every gather so far, last_* the latest gather */
    int64_t acc_threshold; int32_t acc_mode;
    int64_t acc_nodes, acc_rows; int32_t acc_batches;
    int64_t* hist_nodes; int64_t* hist_store; int64_t hist_cap;
    int64_t last_pending, last_flushed, last_limit;
} go_sim;

void go_sim_free(go_sim* s) {
    if (!s) return;
    for (int i = 0; i < s->win_count; i++) free(s->win_ids[i]);
    free(s->win_ids); free(s->win_n);
    free(s->tag); free(s->stamp); free(s->reuse); free(s->hot_slot); free(s->cache_data); free(s->cpu_buf);
    free(s->hist_nodes); free(s->hist_store);
    free(s);
}

/* store == NULL: counts only (no row is moved). */
go_sim* go_sim_create(int64_t n_rows, int64_t lines, int32_t ways, int32_t window, int64_t row_bytes,
                      int64_t line_bytes, const void* store) {
    if (n_rows < 1 || lines < 1 || ways < 1 || lines % ways || window < 0 || window > 254) return NULL;
    if (store && (line_bytes < row_bytes || row_bytes < 1)) return NULL;
    go_sim* s = (go_sim*)calloc(1, sizeof(go_sim));
    if (!s) return NULL;
    s->n_rows = n_rows; s->lines = lines; s->ways = ways; s->n_sets = lines / ways; s->window = window;
    s->row_bytes = row_bytes; s->line_bytes = line_bytes; s->store = (const char*)store;
    s->tag = (int64_t*)malloc((size_t)lines * sizeof(int64_t));
    s->stamp = (int64_t*)malloc((size_t)lines * sizeof(int64_t));
    s->reuse = (int32_t*)calloc((size_t)n_rows, sizeof(int32_t));
    s->hot_slot = (int64_t*)malloc((size_t)n_rows * sizeof(int64_t));
    s->win_ids = (int64_t**)calloc((size_t)window + 1, sizeof(int64_t*));
    s->win_n = (int64_t*)calloc((size_t)window + 1, sizeof(int64_t));
    if (store) s->cache_data = (char*)malloc((size_t)lines * (size_t)line_bytes);
    if (!s->tag || !s->stamp || !s->reuse || !s->hot_slot || !s->win_ids || !s->win_n || (store && !s->cache_data)) {
        go_sim_free(s); return NULL;
    }
    for (int64_t i = 0; i < lines; i++) { s->tag[i] = -1; s->stamp[i] = -1; }
    for (int64_t v = 0; v < n_rows; v++) s->hot_slot[v] = -1;
    s->rows_per_line = 1;
    return s;
}

/* Cache lines that hold several node rows: the cache the paper builds on keeps the storage's cache-lines
 * (4 KB in the example of Section 3.3) while a node's feature row is 512 B to 4 KB (Section 2.1), so with
 * small rows one line holds P consecutive rows and a miss brings all of them in.  The tag of a line is then
 * the store line number b = id div P, its set b mod n_sets; a line is pinned while any of its rows has a
 * buffered future use.  Before the first push or gather. */
int go_sim_set_rows_per_line(go_sim* s, int64_t rows) {
    if (s->t || s->win_count || rows < 1) return GO_E_INVAL;
    if (s->store && rows * s->row_bytes > s->line_bytes) return GO_E_INVAL;
    s->rows_per_line = rows;
    return GO_OK;
}

/* Section 3.3: pin the rows of `ids` in the constant CPU buffer (slot = position in the list) */
int go_sim_set_hot(go_sim* s, const int64_t* ids, int64_t k) {
    if (s->n_hot || s->t) return GO_E_INVAL;
    for (int64_t i = 0; i < k; i++) {
        if (ids[i] < 0 || ids[i] >= s->n_rows) return GO_E_RANGE;
        if (s->hot_slot[ids[i]] >= 0) return GO_E_INVAL;
        s->hot_slot[ids[i]] = i;
    }
    s->n_hot = k;
    if (s->store && k) {
        s->cpu_buf = (char*)malloc((size_t)k * (size_t)s->row_bytes);
        if (!s->cpu_buf) return GO_E_NOMEM;
        for (int64_t i = 0; i < k; i++)
            memcpy(s->cpu_buf + (size_t)i * s->row_bytes, s->store + (size_t)ids[i] * s->row_bytes, (size_t)s->row_bytes);
    }
    return GO_OK;
}

/* Choose the base policy that orders the evictable ways of a set (before the first gather).
 * Random: occupied evictable ways are ordered by the hash H(seed, 8, minibatch, set, way) instead of by
 * their last-use stamp; empty ways still go first, in way order.  Window pinning applies to both. */
int go_sim_set_policy(go_sim* s, int32_t policy, uint64_t seed) {
    if (s->t || (policy != 0 && policy != 1)) return GO_E_INVAL;
    s->policy = policy; s->policy_seed = seed;
    return GO_OK;
}

/* ------------------------------------------------------------ accumulator */

enum { GO_ACC_MAX_MERGE = 32, GO_ACC_LAG = 16, GO_ACC_MAX_RAISE = 8 };

/* Section 3.2.  The dataloader keeps merging the data preparation of consecutive iterations until the number
 * of node accesses passes a threshold; then the merged accesses are issued together.  The paper counts "node
 * accesses" per iteration (the sampler's output) and says that the threshold follows the number of accesses
 * that are redirected to CPU / GPU memory; it gives no formula for that.  Reading taken here:
 *   - a node access is one entry of a minibatch's raw ID list;
 *   - mode 0: the threshold is the given number N of node accesses;
 *   - mode 1: N is the number of accesses that should reach the store (Eq. 2-3's N_access), and the
 *     node-access threshold is N scaled by node accesses per store access, A / S, where A and S add up the
 *     raw list lengths and the misses of every gather at least GO_ACC_LAG gathers back (the redirected ones
 *     are the rest); bounded to [N, GO_ACC_MAX_RAISE * N]; N while nothing has been counted yet, the upper
 *     bound while no access has reached the store;
 *   - a group also closes after GO_ACC_MAX_MERGE minibatches (the paper: merging too many iterations costs
 *     buffer memory) and when go_sim_flush asks for it.
 * While a group is open the rows of its minibatches wait: pending = distinct IDs of the open group's
 * minibatches; the gather that closes the group reports flushed = 1 and pending = 0.  None of this touches
 * tags, counters or rows. */
int go_sim_set_accum(go_sim* s, int64_t threshold, int32_t mode) {
    if (s->t || threshold < 0 || (mode != 0 && mode != 1)) return GO_E_INVAL;
    s->acc_threshold = threshold; s->acc_mode = mode;
    return GO_OK;
}

static int64_t accum_limit(const go_sim* s, int64_t t) {
    const int64_t N = s->acc_threshold;
    if (s->acc_mode == 0) return N;
    int64_t A = 0, S = 0;
    for (int64_t i = 0; i + GO_ACC_LAG < t; i++) { A += s->hist_nodes[i]; S += s->hist_store[i]; }
    if (A == 0) return N;
    if (S == 0) return GO_ACC_MAX_RAISE * N;
    unsigned __int128 want = ((unsigned __int128)N * (uint64_t)A + (uint64_t)S - 1) / (uint64_t)S;   /* ceil(N * A / S) */
    if (want > (unsigned __int128)(GO_ACC_MAX_RAISE * N)) return GO_ACC_MAX_RAISE * N;
    return (int64_t)want < N ? N : (int64_t)want;
}

/* bookkeeping of gather t: n_raw node accesses, n_unique rows, n_miss store accesses */
static int accum_step(go_sim* s, int64_t t, int64_t n_raw, int64_t n_unique, int64_t n_miss) {
    if (t >= s->hist_cap) {
        int64_t cap = s->hist_cap ? 2 * s->hist_cap : 256;
        int64_t* a = (int64_t*)realloc(s->hist_nodes, (size_t)cap * sizeof(int64_t));
        if (!a) return GO_E_NOMEM;
        s->hist_nodes = a;
        int64_t* b = (int64_t*)realloc(s->hist_store, (size_t)cap * sizeof(int64_t));
        if (!b) return GO_E_NOMEM;
        s->hist_store = b; s->hist_cap = cap;
    }
    s->hist_nodes[t] = n_raw; s->hist_store[t] = n_miss;
    if (s->acc_threshold == 0) { s->last_pending = 0; s->last_flushed = 1; s->last_limit = 0; return GO_OK; }
    s->last_limit = accum_limit(s, t);
    s->acc_nodes += n_raw; s->acc_rows += n_unique; s->acc_batches++;
    if (s->acc_nodes >= s->last_limit || s->acc_batches >= GO_ACC_MAX_MERGE) {
        s->acc_nodes = s->acc_rows = 0; s->acc_batches = 0;
        s->last_flushed = 1;
    } else {
        s->last_flushed = 0;
    }
    s->last_pending = s->acc_rows;
    return GO_OK;
}

/* close the open group now; returns the rows that were waiting */
int64_t go_sim_flush(go_sim* s) {
    int64_t rows = s->acc_rows;
    s->acc_nodes = s->acc_rows = 0; s->acc_batches = 0;
    return rows;
}

/* {rows pending after the latest gather, 1 if it closed its group, the node-access threshold it was held to} */
void go_sim_accum_last(const go_sim* s, int64_t* out3) {
    out3[0] = s->last_pending; out3[1] = s->last_flushed; out3[2] = s->last_limit;
}

static int ids_in_range(const go_sim* s, const int64_t* raw, int64_t n) {
    for (int64_t i = 0; i < n; i++) if (raw[i] < 0 || raw[i] >= s->n_rows) return 0;
    return 1;
}

/* Fig. 6 steps 1-4: buffer the ID list of a future minibatch and count, per
 * node, one more future reuse.  The FIFO holds the minibatch to gather next
 * plus at most `window` later ones. */
int go_sim_push(go_sim* s, const int64_t* raw, int64_t n) {
    if (n < 0) return GO_E_INVAL;
    if (s->window == 0) return GO_E_INVAL;
    if (s->win_count == s->window + 1) return GO_E_FULL;
    if (!ids_in_range(s, raw, n)) return GO_E_RANGE;
    int64_t* u = (int64_t*)malloc((size_t)(n > 0 ? n : 1) * sizeof(int64_t));
    if (!u) return GO_E_NOMEM;
    int64_t m = go_sort_unique(raw, n, u);
    for (int64_t i = 0; i < m; i++) s->reuse[u[i]]++;
    s->win_ids[s->win_count] = u; s->win_n[s->win_count] = m; s->win_count++;
    return GO_OK;
}

typedef struct { int64_t set, id, j; } miss_rec;
static int cmp_miss(const void* a, const void* b) {
    const miss_rec* x = (const miss_rec*)a; const miss_rec* y = (const miss_rec*)b;
    if (x->set != y->set) return x->set < y->set ? -1 : 1;
    return (x->id > y->id) - (x->id < y->id);
}
typedef struct { int64_t stamp; int32_t way; } victim_rec;
static int cmp_victim(const void* a, const void* b) {
    const victim_rec* x = (const victim_rec*)a; const victim_rec* y = (const victim_rec*)b;
    if (x->stamp != y->stamp) return x->stamp < y->stamp ? -1 : 1;
    return (x->way > y->way) - (x->way < y->way);
}

enum { GO_CLS_HIT = 0, GO_CLS_CPU = 1, GO_CLS_MISS = 2, GO_CLS_BYPASS = 3 };

/* Gather minibatch t.
 *   unique_out  >= n entries; receives the ascending distinct IDs
 *   out_rows    NULL, or >= n * row_bytes: row j = feature row of unique_out[j]
 *   stats       {n_unique, hits, cpu_hits, misses (installed + bypass), bypasses}
 *   cls_out     NULL, or >= n entries: class of each distinct ID (GO_CLS_*)
 * Returns the distinct count or a negative error (state untouched on error). */
int64_t go_sim_gather(go_sim* s, const int64_t* raw, int64_t n, int64_t* unique_out, void* out_rows,
                      int64_t* stats, int32_t* cls_out) {
    if (n < 0) return GO_E_INVAL;
    if (!ids_in_range(s, raw, n)) return GO_E_RANGE;
    int64_t m = go_sort_unique(raw, n, unique_out);
    const int64_t t = s->t;
    const int64_t P = s->rows_per_line;

    /* window: the buffered head must be this minibatch; drop it and take back
     * its reuse counts (a reuse consumes one count) */
    if (s->window > 0) {
        if (s->win_count == 0) return GO_E_ORDER;
        if (s->win_n[0] != m || memcmp(s->win_ids[0], unique_out, (size_t)m * sizeof(int64_t))) return GO_E_ORDER;
        for (int64_t i = 0; i < m; i++) s->reuse[unique_out[i]]--;
        free(s->win_ids[0]);
        for (int i = 1; i < s->win_count; i++) { s->win_ids[i - 1] = s->win_ids[i]; s->win_n[i - 1] = s->win_n[i]; }
        s->win_count--; s->win_ids[s->win_count] = NULL;
    }

    int64_t hits = 0, cpu_hits = 0, misses = 0, bypasses = 0;
    miss_rec* miss = (miss_rec*)malloc((size_t)(m > 0 ? m : 1) * sizeof(miss_rec));
    int64_t* src_line = (int64_t*)malloc((size_t)(m > 0 ? m : 1) * sizeof(int64_t));   /* cache line serving j, or -1 */
    int32_t* cls = (int32_t*)malloc((size_t)(m > 0 ? m : 1) * sizeof(int32_t));
    victim_rec* vict = (victim_rec*)malloc((size_t)s->ways * sizeof(victim_rec));
    if (!miss || !src_line || !cls || !vict) { free(miss); free(src_line); free(cls); free(vict); return GO_E_NOMEM; }

    /* classify every ID against the state at the start of the minibatch */
    for (int64_t j = 0; j < m; j++) {
        int64_t v = unique_out[j];
        src_line[j] = -1;
        if (s->hot_slot[v] >= 0) { cls[j] = GO_CLS_CPU; cpu_hits++; continue; }
        int64_t blk = v / P;                                 /* the store line that holds the row */
        int64_t set = blk % s->n_sets;
        int32_t way = -1;
        for (int32_t w = 0; w < s->ways; w++) if (s->tag[set * s->ways + w] == blk) way = w;
        if (way >= 0) {
            cls[j] = GO_CLS_HIT; hits++;
            s->stamp[set * s->ways + way] = t;
            src_line[j] = set * s->ways + way;
        } else {
            cls[j] = GO_CLS_MISS;
            miss[misses].set = set; miss[misses].id = blk; miss[misses].j = j; misses++;
        }
    }

    /* install, set by set: the k-th missing line (ascending; with one row per line that is the k-th missing
     * ID) takes the k-th evictable way in (stamp, way) order; a way is evictable when it was not touched in
     * this minibatch and is empty or holds no row that a buffered future minibatch reuses; misses beyond that
     * bypass the cache.  Every requested row of a missing line counts as a miss of its own. */
    qsort(miss, (size_t)misses, sizeof(miss_rec), cmp_miss);
    for (int64_t a = 0; a < misses;) {
        int64_t b = a;
        while (b < misses && miss[b].set == miss[a].set) b++;
        int64_t set = miss[a].set;
        int32_t n_vict = 0;
        for (int32_t w = 0; w < s->ways; w++) {
            int64_t line = set * s->ways + w;
            if (s->stamp[line] == t) continue;
            if (s->tag[line] != -1) {
                int pinned = 0;
                for (int64_t r = s->tag[line] * P; r < (s->tag[line] + 1) * P && r < s->n_rows; r++)
                    if (s->reuse[r] != 0) pinned = 1;
                if (pinned) continue;
            }
            if (s->policy == 1 && s->tag[line] != -1) {
                /* random order among occupied ways: a 55-bit hash, never negative, sorts after every empty way (-1) */
                uint64_t k = mix64(mix64(mix64(key0(s->policy_seed, 8) ^ (uint64_t)t) ^ (uint64_t)set) ^ (uint64_t)w);
                vict[n_vict].stamp = (int64_t)(k >> 9);
            } else {
                vict[n_vict].stamp = s->policy == 1 ? -1 : s->stamp[line];
            }
            vict[n_vict].way = w; n_vict++;
        }
        qsort(vict, (size_t)n_vict, sizeof(victim_rec), cmp_victim);
        int64_t rank = -1, prev = -1;                        /* rank of the current line among the set's missing lines */
        for (int64_t k = a; k < b; k++) {
            if (miss[k].id != prev) { rank++; prev = miss[k].id; }
            if (rank < n_vict) {
                int64_t line = set * s->ways + vict[rank].way;
                s->tag[line] = miss[k].id; s->stamp[line] = t;
                src_line[miss[k].j] = line;
            } else {
                cls[miss[k].j] = GO_CLS_BYPASS; bypasses++;
            }
        }
        a = b;
    }

    /* data: fills first (store -> cache line; an installed miss always fills
     * its line, whether or not the caller wants the output rows), then every
     * row to the output */
    if (s->store) {
        for (int64_t j = 0; j < m; j++)
            if (cls[j] == GO_CLS_MISS) {                     /* the whole store line (clipped at the table's end) */
                int64_t first = unique_out[j] / P * P;
                int64_t rows = first + P <= s->n_rows ? P : s->n_rows - first;
                memcpy(s->cache_data + (size_t)src_line[j] * s->line_bytes,
                       s->store + (size_t)first * s->row_bytes, (size_t)(rows * s->row_bytes));
            }
    }
    if (s->store && out_rows) {
        for (int64_t j = 0; j < m; j++) {
            const char* src;
            if (cls[j] == GO_CLS_CPU) src = s->cpu_buf + (size_t)s->hot_slot[unique_out[j]] * s->row_bytes;
            else if (cls[j] == GO_CLS_BYPASS) src = s->store + (size_t)unique_out[j] * s->row_bytes;
            else src = s->cache_data + (size_t)src_line[j] * s->line_bytes + (size_t)(unique_out[j] % P) * s->row_bytes;
            memcpy((char*)out_rows + (size_t)j * s->row_bytes, src, (size_t)s->row_bytes);
        }
    }
    if (cls_out) memcpy(cls_out, cls, (size_t)m * sizeof(int32_t));
    if (stats) { stats[0] = m; stats[1] = hits; stats[2] = cpu_hits; stats[3] = misses; stats[4] = bypasses; }
    free(miss); free(src_line); free(cls); free(vict);
    if (accum_step(s, t, n, m, misses) != GO_OK) return GO_E_NOMEM;
    s->t = t + 1;
    return m;
}

const int64_t* go_sim_tags(const go_sim* s) { return s->tag; }
const int64_t* go_sim_stamps(const go_sim* s) { return s->stamp; }
const int32_t* go_sim_reuse(const go_sim* s) { return s->reuse; }
int64_t go_sim_batch(const go_sim* s) { return s->t; }
int32_t go_sim_window_count(const go_sim* s) { return s->win_count; }
