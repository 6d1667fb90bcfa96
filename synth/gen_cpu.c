/* Fast host fill for the synthetic-tensor recipe defined in gen.py (same integer steps, OpenMP).
 * Holds no arithmetic of the decode method: hash -> byte sum -> one float multiply -> storage rounding. */
#include <stdint.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

static inline float synth_value(uint64_t seed, uint64_t tid, uint64_t idx, float scale) {
    uint64_t z = mix64(seed + 0x9E3779B97F4A7C15ULL * ((tid << 40) + idx));
    int s = 0;
    for (int b = 0; b < 8; ++b) s += (int)((z >> (8 * b)) & 0xFF);
    return (float)(s - 1020) * scale;
}

static inline uint16_t f32_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

/* dtype: 0 = float32 out, 1 = bf16 bit patterns (uint16) out */
void synth_fill_host(void *out, int dtype, uint64_t seed, uint64_t tid, uint64_t start, uint64_t n, float scale) {
    if (dtype == 0) {
        float *o = (float *)out;
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < (int64_t)n; ++i) o[i] = synth_value(seed, tid, start + (uint64_t)i, scale);
    } else {
        uint16_t *o = (uint16_t *)out;
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < (int64_t)n; ++i)
            o[i] = f32_to_bf16_rne(synth_value(seed, tid, start + (uint64_t)i, scale));
    }
}
