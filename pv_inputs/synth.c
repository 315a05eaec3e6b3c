/*
 * Seeded synthetic-input generator (weights, prompt tokens, draft perturbation).
 *
 * This module only draws numbers.  It holds none of the decoder's or the
 * verification rule's arithmetic; both the GPU library's callers and the CPU
 * oracle's callers take their inputs from here so that they see identical bits.
 *
 * Generator: counter based.  value(seed, tensor, i) = table[ h >> 48 ] where
 * h = mix64( mix64(seed ^ mix64(tensor + G)) + i * G ), mix64 is the
 * splitmix64 finaliser and G the 64-bit golden-ratio constant.  `table` holds
 * 65536 quantiles of N(0, sigma^2) already rounded to the storage type (2 or 4
 * bytes per element); the caller computes it once (see synth.py).
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>

#define PVS_GOLDEN 0x9E3779B97F4A7C15ull

static inline uint64_t pvs_mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

uint64_t pvs_stream_key(uint64_t seed, uint64_t stream)
{
    return pvs_mix64(seed ^ pvs_mix64(stream + PVS_GOLDEN));
}

uint64_t pvs_draw(uint64_t key, uint64_t i)
{
    return pvs_mix64(key + i * PVS_GOLDEN);
}

/* out[j] = table[draw(key, start + j) >> 48], elem_bytes in {2, 4}. */
int pvs_fill_table(uint64_t seed, uint64_t tensor, uint64_t start, uint64_t count,
                   const void *table, int elem_bytes, void *out)
{
    const uint64_t key = pvs_stream_key(seed, tensor);
    if (elem_bytes == 2) {
        const uint16_t *t = (const uint16_t *)table;
        uint16_t *o = (uint16_t *)out;
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < (int64_t)count; ++j)
            o[j] = t[pvs_draw(key, start + (uint64_t)j) >> 48];
    } else if (elem_bytes == 4) {
        const uint32_t *t = (const uint32_t *)table;
        uint32_t *o = (uint32_t *)out;
#pragma omp parallel for schedule(static)
        for (int64_t j = 0; j < (int64_t)count; ++j)
            o[j] = t[pvs_draw(key, start + (uint64_t)j) >> 48];
    } else {
        return -1;
    }
    return 0;
}

/* out[j] = draw(key, start + j) mod modulus (uniform token ids). */
int pvs_fill_uniform_ids(uint64_t seed, uint64_t stream, uint64_t start, uint64_t count,
                         uint32_t modulus, int32_t *out)
{
    const uint64_t key = pvs_stream_key(seed, stream);
    if (modulus == 0) return -1;
    for (uint64_t j = 0; j < count; ++j)
        out[j] = (int32_t)(pvs_draw(key, start + j) % modulus);
    return 0;
}

/* out[j] = top 53 bits of draw(key, start + j) scaled to [0, 1). */
int pvs_fill_unit(uint64_t seed, uint64_t stream, uint64_t start, uint64_t count, double *out)
{
    const uint64_t key = pvs_stream_key(seed, stream);
    for (uint64_t j = 0; j < count; ++j)
        out[j] = (double)(pvs_draw(key, start + j) >> 11) * (1.0 / 9007199254740992.0);
    return 0;
}
