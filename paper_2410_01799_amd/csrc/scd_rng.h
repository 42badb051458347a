// The keyed random stream of the starts t_0 (Algorithm 4 line 2, Algorithm 12 line 1): the one device-side
// statement of it, included by every kernel file.  Word p of (seed, term, mode) is
// mix(mix(mix(seed ^ G (term+1)) + H (mode+1)) + K (p+1)) with mix the SplitMix64 finaliser.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace scd {

__device__ __forceinline__ uint64_t mix64(uint64_t z)
{
    // SplitMix64 finaliser
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

__device__ __forceinline__ uint64_t rng_word(uint64_t seed, uint64_t term, uint32_t mode, uint64_t word)
{
    uint64_t h = mix64(seed ^ (0x9E3779B97F4A7C15ull * (term + 1)));
    h = mix64(h + 0xD1B54A32D192ED03ull * ((uint64_t)mode + 1));
    h = mix64(h + 0x8CB92BA72F3D8DD7ull * (word + 1));
    return h;
}

// word `word` of a vector of n signs: bits past the end cleared
__device__ __forceinline__ uint64_t rng_word_masked(uint64_t seed, uint64_t term, uint32_t mode, int64_t word,
                                                    int64_t n)
{
    uint64_t v = rng_word(seed, term, mode, (uint64_t)word);
    int64_t rem = n - word * 64;
    if (rem < 64) v &= (rem <= 0) ? 0ull : ((~0ull) >> (64 - rem));
    return v;
}

}  // namespace scd
