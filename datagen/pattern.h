/* Seeded synthetic payload generator: one word per (state kind, tensor, global linear index).
 *
 * This header holds no layout or routing arithmetic.  It only turns a
 * (seed, kind, tensor id, linear index) tuple into a pseudo-random word, so that a
 * buffer filled through it encodes "which logical element lives here" in its bits.
 * The mixing steps are the SplitMix64 output finaliser (Steele, Lea, Flood 2014),
 * applied to a key built from the tuple.
 */
#ifndef VPS_DATAGEN_PATTERN_H
#define VPS_DATAGEN_PATTERN_H

#include <stdint.h>

static inline uint64_t vps_pattern_mix64(uint64_t seed, uint32_t kind, uint32_t tensor,
                                         uint64_t linear)
{
    uint64_t z = seed ^ (0x9E3779B97F4A7C15ull * (linear + 1ull));
    z += ((((uint64_t)tensor) << 2) | (uint64_t)(kind & 3u)) * 0xD1B54A32D192ED03ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* Per-rank salt: lets a test give every replica of an element different bits, so that the
 * rank a value was copied from becomes visible in the destination. salt==0 disables it. */
static inline uint64_t vps_pattern_seed_for_rank(uint64_t seed, uint64_t rank_salt, uint32_t rank)
{
    return seed + rank_salt * (uint64_t)(rank + 1u);
}

/* kind 0 is a 16-bit word (bf16 payload), kinds 1..3 are 32-bit words (fp32 payload). */
static inline uint32_t vps_pattern_word(uint64_t seed, uint32_t kind, uint32_t tensor,
                                        uint64_t linear)
{
    uint64_t z = vps_pattern_mix64(seed, kind, tensor, linear);
    return kind == 0u ? (uint32_t)(z & 0xFFFFull) : (uint32_t)(z & 0xFFFFFFFFull);
}

#endif
