/* Multi-threaded writer of the synthetic feature table (an input generator, no
 * part of the gather).  Same closed form as workload/synth.py:
 *   feat(v, c) = T[(H(seed, FEAT, v, c >> 2) >> (16 * (c & 3))) & 0xFFFF]
 * with H the chained 64-bit mixer documented there. */
#include <stdint.h>
#include <string.h>
#include <omp.h>

static inline uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31; return z;
}

void wl_fill_store(uint64_t seed, uint64_t row_lo, uint64_t n_rows, uint32_t dim, uint32_t itemsize,
                   const void* table, void* out, int threads) {
    const uint64_t k0 = mix64(seed + 3ull * 0x9E3779B97F4A7C15ull);   /* tag FEAT = 3 */
    const uint32_t groups = dim / 4;
    if (threads < 1) threads = 1;
    #pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t r = 0; r < (int64_t)n_rows; r++) {
        const uint64_t kv = mix64(k0 ^ (row_lo + (uint64_t)r));
        if (itemsize == 2) {
            const uint16_t* T = (const uint16_t*)table;
            uint16_t* dst = (uint16_t*)out + (size_t)r * dim;
            for (uint32_t g = 0; g < groups; g++) {
                uint64_t w = mix64(kv ^ (uint64_t)g);
                dst[4 * g + 0] = T[w & 0xFFFF];
                dst[4 * g + 1] = T[(w >> 16) & 0xFFFF];
                dst[4 * g + 2] = T[(w >> 32) & 0xFFFF];
                dst[4 * g + 3] = T[(w >> 48) & 0xFFFF];
            }
        } else {
            const uint32_t* T = (const uint32_t*)table;
            uint32_t* dst = (uint32_t*)out + (size_t)r * dim;
            for (uint32_t g = 0; g < groups; g++) {
                uint64_t w = mix64(kv ^ (uint64_t)g);
                dst[4 * g + 0] = T[w & 0xFFFF];
                dst[4 * g + 1] = T[(w >> 16) & 0xFFFF];
                dst[4 * g + 2] = T[(w >> 32) & 0xFFFF];
                dst[4 * g + 3] = T[(w >> 48) & 0xFFFF];
            }
        }
    }
}

/* Destinations of edge slots lo..hi-1 (same definition as make_graph in
 * synth.py): the node that owns edge slot (H(seed, EDGE, e) mod E). */
void wl_make_edges(uint64_t seed, int64_t n, const int64_t* indptr, int64_t lo, int64_t hi, void* indices,
                   uint32_t itemsize, int threads) {
    const uint64_t k = mix64(seed + 2ull * 0x9E3779B97F4A7C15ull);   /* tag EDGE = 2 */
    const uint64_t e_total = (uint64_t)indptr[n];
    if (threads < 1) threads = 1;
    #pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t e = lo; e < hi; e++) {
        const int64_t slot = (int64_t)(mix64(k ^ (uint64_t)e) % e_total);
        int64_t a = 0, b = n;
        while (b - a > 1) {
            const int64_t mid = a + (b - a) / 2;
            if (indptr[mid] <= slot) a = mid; else b = mid;
        }
        if (itemsize == 4) ((int32_t*)indices)[e] = (int32_t)a;
        else ((int64_t*)indices)[e] = a;
    }
}

/* In-degree histogram of an int64 / int32 destination array. */
void wl_indegree(const void* indices, int64_t e_total, uint32_t itemsize, int64_t* indeg) {
    if (itemsize == 4) for (int64_t e = 0; e < e_total; e++) indeg[((const int32_t*)indices)[e]]++;
    else for (int64_t e = 0; e < e_total; e++) indeg[((const int64_t*)indices)[e]]++;
}
