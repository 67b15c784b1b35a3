/* Host implementation of the counter-based synthetic tensor generator.
 *
 * Same definition as generator.py: SplitMix64 output function, three stream
 * outputs per element, sum of twelve 16-bit fields -> Irwin-Hall(12) variate,
 * one fp64 multiply by sigma, fp32 round-to-nearest, optional bf16 RNE.
 * Holds no MoE arithmetic: it only fills input tensors.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>

#define GOLDEN 0x9E3779B97F4A7C15ULL

static inline uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

static inline double variate(uint64_t key, uint64_t i) {
    int64_t s = 0;
    for (int m = 0; m < 3; ++m) {
        uint64_t h = mix64(key + (3ULL * i + (uint64_t)m + 1ULL) * GOLDEN);
        s += (int64_t)(h & 0xFFFF) + (int64_t)((h >> 16) & 0xFFFF) + (int64_t)((h >> 32) & 0xFFFF) +
             (int64_t)(h >> 48);
    }
    return (double)(2 * s - 12 * 65535) / 131072.0;
}

static inline uint16_t f32_to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

uint64_t lexi_synth_key(uint64_t seed, uint64_t tid) { return mix64(seed ^ mix64(tid + GOLDEN)); }

/* dtype: 0 = fp32 (float out[]), 1 = bf16 (uint16_t out[]).  Returns 0, or -1 on a bad dtype. */
int lexi_synth_fill_host(void* out, int dtype, uint64_t seed, uint64_t tid, uint64_t start, uint64_t count,
                         double sigma) {
    if (dtype != 0 && dtype != 1) return -1;
    const uint64_t key = lexi_synth_key(seed, tid);
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < (int64_t)count; ++n) {
        float v = (float)(sigma * variate(key, start + (uint64_t)n));
        if (dtype == 0) ((float*)out)[n] = v;
        else ((uint16_t*)out)[n] = f32_to_bf16(v);
    }
    return 0;
}
