/*
 * A position-dependent 64-bit checksum of a byte buffer, for the harness only.
 *
 * Long runs (hundreds of decode steps at full size) compare what the CPU
 * checker and the GPU library delivered in every step; keeping or copying
 * gigabytes per step for a byte-wise comparison would dominate the run, so
 * each side reduces its buffer to one word and the words are compared, with
 * byte-wise comparisons on sampled steps.  Nothing of the fetch method is
 * here: the function knows bytes and positions only.
 *
 * Definition.  The buffer is n little-endian 64-bit words x[0..n).  With
 * M = 65536, w[j] = splitmix64(j) | 1 and c[p] = splitmix64(2^32 + p) | 1:
 *
 *     digest = sum over p of c[p] * (sum over j < M, pM + j < n of x[pM + j] * w[j])    (mod 2^64)
 *
 * Every multiplier is odd, so changing one word always changes the digest,
 * and moving a run of words to another position changes it except by
 * coincidence (probability about 2^-64 for independent data).
 * The same definition is written with tensor operations in digest.py for
 * buffers that live in device memory.
 */
#include <stddef.h>
#include <stdint.h>

#define GOLDEN 0x9E3779B97F4A7C15ull
#define DIGEST_M 65536u

static inline uint64_t splitmix64(uint64_t x)
{
    x += GOLDEN;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

uint64_t wl_digest_weight(uint64_t j) { return splitmix64(j) | 1ull; }
uint64_t wl_digest_piece_factor(uint64_t p) { return splitmix64((1ull << 32) + p) | 1ull; }

uint64_t wl_digest(const uint64_t *x, size_t n_words)
{
    static uint64_t w[DIGEST_M];
    static int ready = 0;
#pragma omp critical(wl_digest_init)
    {
        if (!ready) {
            for (uint64_t j = 0; j < DIGEST_M; ++j) w[j] = wl_digest_weight(j);
            ready = 1;
        }
    }
    long n_pieces = (long)((n_words + DIGEST_M - 1) / DIGEST_M);
    uint64_t total = 0;
#pragma omp parallel for schedule(static) reduction(+ : total)
    for (long p = 0; p < n_pieces; ++p) {
        size_t first = (size_t)p * DIGEST_M;
        size_t len = n_words - first < DIGEST_M ? n_words - first : DIGEST_M;
        uint64_t s = 0;
        for (size_t j = 0; j < len; ++j) s += x[first + j] * w[j];
        total += wl_digest_piece_factor((uint64_t)p) * s;
    }
    return total;
}
