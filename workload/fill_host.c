/*
 * Stateless SplitMix64 pool fill on the host, in C: word k of the buffer
 * (counted from start_word) receives mix64(state0 + (k+1)*GAMMA), the same
 * pattern as workload/splitmix.py (fill_words) and workload/fill_gpu.hip.
 * Input generation only; a faster twin of the NumPy version for pools of
 * gigabytes, tested against it.
 */
#include <stdint.h>

static inline uint64_t wl_mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

void wl_fill_words_host(uint64_t *dst, uint64_t start_word, uint64_t n_words, uint64_t state0)
{
    for (uint64_t i = 0; i < n_words; ++i)
        dst[i] = wl_mix64(state0 + (start_word + i + 1) * 0x9E3779B97F4A7C15ull);
}
