// Device helpers and launcher declarations shared by the kernel files.
#pragma once
#include "pv_internal.h"

// storage-type access: float, or bfloat16 kept as raw uint16_t bit patterns
__device__ inline float pv_bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ inline uint16_t pv_f32_to_bf16(float f)      // round to nearest, ties to even
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ inline float pv_ld(const float *p, size_t i) { return p[i]; }
__device__ inline float pv_ld(const uint16_t *p, size_t i) { return pv_bf16_to_f32(p[i]); }
__device__ inline void pv_st(float *p, size_t i, float v) { p[i] = v; }
__device__ inline void pv_st(uint16_t *p, size_t i, float v) { p[i] = pv_f32_to_bf16(v); }

pv_kv_geom pv_geom(const pv_cache *c);
int pv_k_begin(pv_cache *c, int rows_pad, hipStream_t s);
int pv_k_rope_append(pv_cache *c, int layer, int rows, hipStream_t s);
int pv_k_argmax(pv_cache *c, int rows, hipStream_t s);
int pv_k_finish(pv_cache *c, int rows, const float *pmax_val, const int32_t *pmax_idx, int strips, hipStream_t s);
int pv_k_tree_compact(pv_cache *c, hipStream_t s);
int pv_k_set_state(pv_cache *c, int len, int pending, hipStream_t s);
int pv_k_export(pv_cache *c, size_t e0, size_t n, void *d_out, hipStream_t s);
