// Pieces shared by the matrix-core kernel files: MFMA wrapper, split-bf16 operand writers.
#pragma once
#include "pv_kernels_common.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// D(16x16, fp32) += A(16x32, bf16) * B(32x16, bf16).  Lane l holds A[l%16][8*(l/16)..+7],
// B[8*(l/16)..+7][l%16] and D[4*(l/16)+r][l%16], r = 0..3.
__device__ inline f32x4 mfma16(uint4 a, uint4 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Loads of data that a kernel reads once (the weight stream): marked non-temporal, so that these lines do not
// push the activation tiles, which every workgroup reads again, out of the L2.  Measured on whole steps: 8B shape
// 3.49 -> 3.30 ms, 70B shape 24.3 -> 22.2 ms.
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
__device__ inline uint4 load_once(const uint4 *p)
{
    const u32x4 v = __builtin_nontemporal_load((const u32x4 *)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ inline uint2 load_once(const uint2 *p)
{
    const u32x2 v = __builtin_nontemporal_load((const u32x2 *)p);
    return make_uint2(v.x, v.y);
}

// ------------------------------------------------------------------------------------------
// Operand writers.  Element (row j, K-index k) of an activation lives at
//   arr[(k/32)*512 + (col + 16*((k%32)/8))*8 + k%8],  col = j (hi) / j + lo_off (lo) when NB == 1
//   (at most 8 rows; lo_off = 8, or 4 for blocks of at most 4 rows: columns 0..7 are then all a
//   reader needs, half the 128-byte lines of a tile).  When NB == 2 the rows come in column tiles of 16: tile j/16 owns a hi
//   array followed by a lo array ((K/32)*512 elements each), col = j%16 in both.
// ------------------------------------------------------------------------------------------
__device__ inline uint16_t bf16_rne(float f) { return pv_f32_to_bf16(f); }

// four consecutive k (k0 % 4 == 0) of row j
// lo column offset of a packed-row block of `rows` rows
__host__ __device__ inline int pv_lo_off(int rows) { return rows <= 4 ? 4 : 8; }

template <int NB>
__device__ inline void store_operand4(uint16_t *xop, int K, int j, int k0, const float y[4], int lo_off)
{
    uint16_t hi[4], lo[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) { hi[r] = bf16_rne(y[r]); lo[r] = bf16_rne(y[r] - pv_bf16_to_f32(hi[r])); }
    const size_t tile = (size_t)(k0 >> 5) * 512, in = (size_t)(((k0 & 31) >> 3) * 16) * 8 + (k0 & 7);
    const uint2 vh = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
    const uint2 vl = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
    if (NB == 1) {
        *(uint2 *)(xop + tile + in + (size_t)j * 8) = vh;
        *(uint2 *)(xop + tile + in + (size_t)(j + lo_off) * 8) = vl;
    } else {
        const size_t arr = (size_t)(K / 32) * 512;
        uint16_t *base = xop + (size_t)(j >> 4) * 2 * arr + tile + in + (size_t)(j & 15) * 8;
        *(uint2 *)base = vh;
        *(uint2 *)(base + arr) = vl;
    }
}

