/*
 * Seeded payload generators for the synthetic tiered-fetch workloads.
 *
 * This file only produces INPUT bytes (the contents of KV blocks and expert
 * weight matrices).  It contains nothing of the fetch method itself: no
 * directory, no tiers, no gather.  Both the CPU checker and the GPU library
 * are handed the buffers these functions fill.
 *
 * Every chunk (one object's slice in one plane and one layer) is generated
 * from a 64-bit key alone, so any single chunk can be regenerated later
 * without materialising the pool it lives in.
 *
 *   chunk key = mix(seed, class, plane, layer, object id)
 *   16-bit lane j of word w of the chunk = bits [16j, 16j+16) of
 *                                          splitmix64(key + w * GOLDEN)
 *
 * Normal fill: lane -> table[lane], where the 65536-entry table holds the
 * bf16 bit patterns of sigma * Phi^-1((u + 0.5) / 65536) (inverse-CDF sampling
 * of N(0, sigma) on a 16-bit uniform; the table is built by the Python side).
 *
 * Tag fill: every 16-byte word describes itself:
 *   { u32 (class << 28 | plane << 24 | layer), u32 object id,
 *     u32 word index inside the chunk, u32 salt(seed, object id) }
 * so a misrouted copy can never look like correct data.
 */
#include <stddef.h>
#include <stdint.h>

#define GOLDEN 0x9E3779B97F4A7C15ull

static inline uint64_t splitmix64(uint64_t x)
{
    x += GOLDEN;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

uint64_t wl_chunk_key(uint64_t seed, uint32_t cls, uint32_t plane, uint32_t layer, uint32_t object)
{
    uint64_t k = splitmix64(seed ^ 0x48415256455354ull); /* "HARVEST" */
    k = splitmix64(k ^ (((uint64_t)cls << 40) | ((uint64_t)plane << 32) | layer));
    k = splitmix64(k ^ ((uint64_t)object << 1 | 1));
    return k;
}

/* n_elems 16-bit elements, n_elems % 4 == 0 */
void wl_fill_chunk_normal(uint16_t *dst, size_t n_elems, uint64_t key, const uint16_t *table)
{
    size_t n_words = n_elems / 4;
    for (size_t w = 0; w < n_words; ++w) {
        uint64_t h = splitmix64(key + (uint64_t)w * GOLDEN);
        dst[4 * w + 0] = table[h & 0xFFFF];
        dst[4 * w + 1] = table[(h >> 16) & 0xFFFF];
        dst[4 * w + 2] = table[(h >> 32) & 0xFFFF];
        dst[4 * w + 3] = table[(h >> 48) & 0xFFFF];
    }
}

/* chunk_bytes % 16 == 0 */
void wl_fill_chunk_tag(uint32_t *dst, size_t chunk_bytes, uint64_t seed, uint32_t cls, uint32_t plane,
                       uint32_t layer, uint32_t object)
{
    size_t n_words = chunk_bytes / 16;
    uint32_t head = (cls << 28) | (plane << 24) | (layer & 0xFFFFFF);
    uint32_t salt = (uint32_t)splitmix64(seed ^ ((uint64_t)object * GOLDEN));
    for (size_t w = 0; w < n_words; ++w) {
        dst[4 * w + 0] = head;
        dst[4 * w + 1] = object;
        dst[4 * w + 2] = (uint32_t)w;
        dst[4 * w + 3] = salt;
    }
}

/*
 * Fill a whole pool plane laid out [layer][slot][chunk_bytes].
 * slot_object[s] = object id whose bytes go to slot s, or 0xFFFFFFFF to leave
 * the slot untouched.  mode 0 = normal (table required), 1 = tag.  The first
 * layer of the buffer is model layer layer_base (a buffer may hold a slice of
 * the layers).
 */
void wl_fill_pool(void *pool, uint32_t n_layers, uint32_t n_slots, size_t chunk_bytes,
                  const uint32_t *slot_object, uint64_t seed, uint32_t cls, uint32_t plane,
                  int mode, const uint16_t *table, uint32_t layer_base)
{
    long total = (long)n_layers * (long)n_slots;
#pragma omp parallel for schedule(static)
    for (long i = 0; i < total; ++i) {
        uint32_t layer = layer_base + (uint32_t)(i / n_slots);
        uint32_t slot = (uint32_t)(i % n_slots);
        uint32_t obj = slot_object[slot];
        if (obj == 0xFFFFFFFFu)
            continue;
        uint8_t *dst = (uint8_t *)pool + (size_t)i * chunk_bytes;
        if (mode == 0)
            wl_fill_chunk_normal((uint16_t *)dst, chunk_bytes / 2, wl_chunk_key(seed, cls, plane, layer, obj), table);
        else
            wl_fill_chunk_tag((uint32_t *)dst, chunk_bytes, seed, cls, plane, layer, obj);
    }
}
