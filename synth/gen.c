/* Counter-based fill routines for synthetic weights and prompts.
 *
 * Every element is a pure function of (key, element index): a 32-bit integer
 * mixer produces a hash; weights take a value from a caller-supplied
 * 65536-entry table (Gaussian quantiles, already scaled and rounded to the
 * storage type) indexed by the hash's top 16 bits; token ids take the hash
 * modulo the vocabulary.  No state, so any slice of any tensor can be
 * regenerated independently.  synth/gen.py holds an identical NumPy version.
 */
#include <stdint.h>
#include <stddef.h>

static inline uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352dU;
    x ^= x >> 15; x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

/* out[i] = table[mix32(start + i + key) >> 16] for 2-byte elements */
void synth_fill_table_u16(uint16_t *out, uint64_t n, uint64_t start, uint32_t key,
                          const uint16_t *table) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i)
        out[i] = table[mix32((uint32_t)(start + (uint64_t)i) + key) >> 16];
}

/* same for 4-byte elements */
void synth_fill_table_u32(uint32_t *out, uint64_t n, uint64_t start, uint32_t key,
                          const uint32_t *table) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i)
        out[i] = table[mix32((uint32_t)(start + (uint64_t)i) + key) >> 16];
}

/* out[i] = mix32(start + i + key) % vocab */
void synth_fill_tokens(int32_t *out, uint64_t n, uint64_t start, uint32_t key, uint32_t vocab) {
    for (uint64_t i = 0; i < n; ++i)
        out[i] = (int32_t)(mix32((uint32_t)(start + i) + key) % vocab);
}
