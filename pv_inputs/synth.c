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

/* ---- 4-bit weight format (input preparation: the stand-in for a 4-bit checkpoint) ----
 *
 * A matrix row is cut into groups of 32 consecutive input features.  Each group carries one
 * bf16 scale s = bf16(max|w| / 7) (s = bf16(2^-126-ish floor) replaced by 1.0 for an all-zero
 * group) and 32 codes c = clamp(rint(w / s) + 8, 0, 15); the weight the model uses is
 * (c - 8) * s.  Codes are packed two per byte, the even feature in the low nibble.
 * w: bf16 bit patterns [rows][cols], cols % 32 == 0.  Arithmetic in float, round-half-even.
 */
#include <math.h>

static inline float pvs_bf16_to_f32(uint16_t b) { uint32_t u = (uint32_t)b << 16; float f; memcpy(&f, &u, 4); return f; }
static inline uint16_t pvs_f32_to_bf16(float f)
{
    uint32_t u; memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

int pvs_quantize_q4(const uint16_t *w, int64_t rows, int64_t cols, uint8_t *codes, uint16_t *scales)
{
    if (cols % 32) return -1;
    const int64_t groups = cols / 32;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t g = 0; g < groups; ++g) {
            const uint16_t *src = w + r * cols + g * 32;
            float v[32], m = 0.f;
            for (int k = 0; k < 32; ++k) { v[k] = pvs_bf16_to_f32(src[k]); const float a = fabsf(v[k]); if (a > m) m = a; }
            uint16_t sb = pvs_f32_to_bf16(m / 7.0f);
            float s = pvs_bf16_to_f32(sb);
            if (!(s > 0.f)) { sb = 0x3F80; s = 1.0f; }
            scales[r * groups + g] = sb;
            uint8_t *dst = codes + r * (cols / 2) + g * 16;
            for (int k = 0; k < 32; k += 2) {
                int c0 = (int)rintf(v[k] / s) + 8, c1 = (int)rintf(v[k + 1] / s) + 8;
                c0 = c0 < 0 ? 0 : c0 > 15 ? 15 : c0; c1 = c1 < 0 ? 0 : c1 > 15 ? 15 : c1;
                dst[k / 2] = (uint8_t)(c0 | (c1 << 4));
            }
        }
    }
    return 0;
}
