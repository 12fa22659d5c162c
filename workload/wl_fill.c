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
