// Per-block building blocks shared by the dense control kernel, the value pass and the metadata kernel:
// how one wave reads a 4 KiB (page, KV head) slice and what each lane holds, and the 16x16x16 matrix
// product with 16-bit operands that both attention kernels accumulate values with.
//
// Lane layout of a wave over one K or V slice [16 tokens][128 channels] of 2-byte elements:
//   rg = lane / 16  (row group 0..3),  cl = lane % 16  (channel slot: channels 8*cl .. 8*cl+7)
//   load i (0..3) fetches token row 4*i + rg, 16 bytes per lane, so one load instruction of the
//   wave covers rows 4*i .. 4*i+3 = 1 KiB of contiguous memory.
#pragma once

#include "psa_device.h"

namespace psa {

struct Slice {
    uint4 r[4];
};

__device__ __forceinline__ Slice load_slice(const uint8_t *slice_base, int lane) {
    Slice s;
    const uint8_t *p = slice_base + lane * 16;
#pragma unroll
    for (int i = 0; i < 4; ++i) s.r[i] = ld16_stream(p + i * 1024);
    return s;
}

// Rows of a partly filled block beyond `valid` may hold anything (NaN included): make them zero.
__device__ __forceinline__ void zero_invalid_rows(Slice &v, int rg, int valid) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (4 * i + rg >= valid) v.r[i] = make_uint4(0, 0, 0, 0);
}

// D(16x16, fp32) += A(16x16) * B(16x16) on the matrix cores, 16-bit inputs.  Lane l supplies row l%16 of A
// and column l%16 of B, k values 4*(l/16) .. +3 of each; it receives column l%16 of D, rows 4*(l/16) .. +3.
typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
template <int DT>
__device__ __forceinline__ f32x4_t mfma_16x16x16(const uint2 &a, const uint2 &b, f32x4_t c) {
    if constexpr (DT == 0) {
        return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4_t, a), __builtin_bit_cast(f16x4_t, b), c, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, a), __builtin_bit_cast(s16x4_t, b), c, 0, 0, 0);
    }
}

// p = hi + lo with both halves in the 16-bit type of the cache (round to nearest each): the bits of the two.
template <int DT>
__device__ __forceinline__ void split16(float p, uint32_t &hi, uint32_t &lo) {
    if constexpr (DT == 0) {
        const _Float16 h = (_Float16)p;
        const _Float16 l = (_Float16)(p - (float)h);
        hi = __builtin_bit_cast(uint16_t, h);
        lo = __builtin_bit_cast(uint16_t, l);
    } else {
        const uint32_t u = __float_as_uint(p);
        hi = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
        const uint32_t w = __float_as_uint(p - __uint_as_float(hi << 16));
        lo = (w + 0x7fffu + ((w >> 16) & 1u)) >> 16;
    }
}

__device__ __forceinline__ uint32_t pick_word(const uint4 &v, int w) {
    return w == 0 ? v.x : (w == 1 ? v.y : (w == 2 ? v.z : v.w));
}

}  // namespace psa
