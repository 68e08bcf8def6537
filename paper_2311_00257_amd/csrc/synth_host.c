/* Host side of the seeded synthetic-input generator, in plain C for speed: the same bits as
 * synth.py's numpy formulas and as the device fill kernels.  Input production only.
 * Element i of a stream with key K: h = SplitMix64 output function of (K + i * GOLDEN);
 * value = table[h >> 48] * sigma in fp32 (fabs if asked); bf16 keeps the high 16 bits. */
#include <math.h>
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

void amsp_synth_host_f32(float *out, uint64_t n, uint64_t key, uint64_t index0, const float *table, float sigma,
                         int absolute) {
    for (uint64_t i = 0; i < n; ++i) {
        float x = table[mix64(key + (index0 + i) * 0x9E3779B97F4A7C15ull) >> 48] * sigma;
        out[i] = absolute ? fabsf(x) : x;
    }
}

void amsp_synth_host_bf16(uint16_t *out, uint64_t n, uint64_t key, uint64_t index0, const float *table, float sigma) {
    for (uint64_t i = 0; i < n; ++i) {
        float x = table[mix64(key + (index0 + i) * 0x9E3779B97F4A7C15ull) >> 48] * sigma;
        uint32_t u;
        memcpy(&u, &x, sizeof u);
        out[i] = (uint16_t)(u >> 16);
    }
}
