// Per-block building blocks shared by the dense control kernel and the progressive kernel:
// how one wave reads a 4 KiB (page, KV head) slice and what each lane holds.
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
    for (int i = 0; i < 4; ++i) s.r[i] = ld16(p + i * 1024);
    return s;
}

// Query of head g as this lane sees it: the 8 channels of its channel slot, packed in pairs.
template <int G>
struct QueryRegs {
    uint32_t w[G][4];
};

template <int G>
__device__ __forceinline__ QueryRegs<G> load_query(const uint8_t *q, int r, int h, int num_q_heads,
                                                   int cl) {
    QueryRegs<G> out;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        uint4 t = ld16(q + ((size_t)(r * num_q_heads + h * G + g) * kHeadDim + cl * 8) * 2);
        out.w[g][0] = t.x; out.w[g][1] = t.y; out.w[g][2] = t.z; out.w[g][3] = t.w;
    }
    return out;
}

// Scaled logits (log2 units) of token rows 4*i + rg for i = 0..3 and every head of the group.
// Rows at or beyond `valid` get -inf.  Every lane of a row group ends up with the same values.
template <int DT, int G>
__device__ __forceinline__ void slice_logits(const Slice &k, const QueryRegs<G> &q, int rg, int valid,
                                             float (&s)[4][G]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const bool ok = (4 * i + rg) < valid;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float p = dot2<DT>(k.r[i].x, q.w[g][0], 0.0f);
            p = dot2<DT>(k.r[i].y, q.w[g][1], p);
            p = dot2<DT>(k.r[i].z, q.w[g][2], p);
            p = dot2<DT>(k.r[i].w, q.w[g][3], p);
            p = row_sum16(p);
            s[i][g] = ok ? p * kScaleLog2 : -INFINITY;
        }
    }
}

// acc[c] += p * v[c] for the lane's 8 channels of one token row.
template <int DT>
__device__ __forceinline__ void axpy_row(const uint4 &v, float p, float (&acc)[8]) {
    acc[0] = fmaf(p, cvt_lo<DT>(v.x), acc[0]);
    acc[1] = fmaf(p, cvt_hi<DT>(v.x), acc[1]);
    acc[2] = fmaf(p, cvt_lo<DT>(v.y), acc[2]);
    acc[3] = fmaf(p, cvt_hi<DT>(v.y), acc[3]);
    acc[4] = fmaf(p, cvt_lo<DT>(v.z), acc[4]);
    acc[5] = fmaf(p, cvt_hi<DT>(v.z), acc[5]);
    acc[6] = fmaf(p, cvt_lo<DT>(v.w), acc[6]);
    acc[7] = fmaf(p, cvt_hi<DT>(v.w), acc[7]);
}

// Rows of a partly filled block beyond `valid` may hold anything (NaN included): make them zero.
__device__ __forceinline__ void zero_invalid_rows(Slice &v, int rg, int valid) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (4 * i + rg >= valid) v.r[i] = make_uint4(0, 0, 0, 0);
}

}  // namespace psa
