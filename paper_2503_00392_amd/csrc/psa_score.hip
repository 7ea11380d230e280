// Block scoring (Algorithm 1, line 5): the criticality score of every block of every stream from
// its per-channel min/max key metadata.
#include "psa_host.h"

namespace psa {

constexpr int kScoreBlocks = 64;   // blocks per workgroup: 16 per wave

// =================================================================================================
// Scoring.  Upper bound (CENTER = 0):
//   UB[g][b] = (1/sqrt d) sum_c max(q_c kmin_c, q_c kmax_c) = (1/sqrt d) (q+ . kmax + q- . kmin)
//   with q+ = max(q,0), q- = min(q,0).
// Cuboid centre (CENTER = 1): (1/sqrt d) q . (kmin + kmax)/2 = (1/(2 sqrt d)) (q . kmax + q . kmin).
// Either way CS[b] = max over the heads g of the group.
// grid (ceil(max_blocks/64), S), 256 threads.  A 16-lane row handles one block: lanes 0-7 take
// 32 bytes each of the min row (against q-, or q), lanes 8-15 of the max row (against q+, or q).
// =================================================================================================
template <int DT, int G, int CENTER>
__global__ __launch_bounds__(256) void score_kernel(KvView kv, const uint8_t *__restrict__ q,
                                                    const uint8_t *__restrict__ meta,
                                                    float *__restrict__ scores,
                                                    float *__restrict__ scores_out, int32_t *header) {
    const int s = blockIdx.y, r = s / kv.num_kv_heads, h = s % kv.num_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, row = lane >> 4, cl = lane & 15;
    const int is_max = cl >> 3, slot = cl & 7;
    // first kernel of a decode call: it clears the sticky error word and clamps silently; the
    // ranking kernel, which sees the same table entries and contexts, reports them
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < 2) header[threadIdx.x] = 0;
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 2) header[kValueCount] = 0;   // value work list
    const int ctx = ctx_clamped_quiet(kv, r);
    const int N = (ctx + kPage - 1) / kPage;
    const int base = blockIdx.x * kScoreBlocks + wave * 16;
    if (base >= N) return;

    // the lane's 16 channels of every query head, with the entries of the wrong sign zeroed
    uint32_t qs[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const uint8_t *qp = q + ((size_t)(r * kv.num_q_heads + h * G + g) * kHeadDim + slot * 16) * 2;
        const uint4 a = ld16(qp), b = ld16(qp + 16);
        const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t neg = ((w[j] >> 15) & 0x00010001u) * 0xFFFFu;
            qs[g][j] = CENTER ? w[j] : (w[j] & (is_max ? ~neg : neg));
        }
    }

    const int32_t *table = kv.block_table + (size_t)r * kv.max_blocks;
    uint4 ma[4], mb[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int b = base + it * 4 + row;
        if (b < N) {
            const int page = clamp_page_quiet(table[b], kv.num_pages);
            const uint8_t *mp = meta + ((size_t)page * kv.num_kv_heads + h) * kMetaBytes + is_max * 256 + slot * 32;
            ma[it] = ld16(mp);
            mb[it] = ld16(mp + 16);
        } else {
            ma[it] = make_uint4(0, 0, 0, 0);
            mb[it] = make_uint4(0, 0, 0, 0);
        }
    }
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int b = base + it * 4 + row;
        const uint32_t w[8] = {ma[it].x, ma[it].y, ma[it].z, ma[it].w, mb[it].x, mb[it].y, mb[it].z, mb[it].w};
        float cs = -INFINITY;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float p = 0.0f;
#pragma unroll
            for (int j = 0; j < 8; ++j) p = dot2<DT>(w[j], qs[g][j], p);
            p = row_sum16(p);
            cs = fmaxf(cs, p * (CENTER ? 0.5f * kScale : kScale));
        }
        if (cl == 0 && b < N) {
            scores[(size_t)s * kv.max_blocks + b] = cs;
            if (scores_out) scores_out[(size_t)s * kv.max_blocks + b] = cs;
        }
    }
}

// =================================================================================================
// Scoring on the matrix cores (used at G = 8, where the version above is bound by its arithmetic; at G <= 4
// it is the faster one, its loads being fully coalesced).  Upper bound (CENTER = 0):
//   UB[g][b] = (1/sqrt d) sum_c max(q_c kmin_c, q_c kmax_c) = (1/sqrt d) (q- . kmin + q+ . kmax)
//   with q+ = max(q,0), q- = min(q,0).
// Cuboid centre (CENTER = 1): (1/sqrt d) q . (kmin + kmax)/2 = (1/(2 sqrt d)) (q . kmin + q . kmax).
// Either way CS[b] = max over the heads g of the group.
// Both are one matrix product over the 256 numbers of a block's record [min(128) | max(128)]:
//   D[block][head] = sum_e record[block][e] * qq[e][head],  qq = (q- | q+) or (q | q),
// done as eight 16x16x32 steps on the matrix cores: 16 blocks per wave, row = block, the record's 512
// contiguous bytes are the k dimension; columns beyond G are zero and left out of the maximum.
// grid (ceil(max_blocks/64), S), 256 threads: wave w takes blocks 64*blockIdx.x + 16*w .. +15.
// =================================================================================================
template <int DT, int G, int CENTER>
__global__ __launch_bounds__(256) void score_mfma_kernel(KvView kv, const uint8_t *__restrict__ q,
                                                    const uint8_t *__restrict__ meta,
                                                    float *__restrict__ scores,
                                                    float *__restrict__ scores_out, int32_t *header) {
    const int s = blockIdx.y, r = s / kv.num_kv_heads, h = s % kv.num_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, kq = lane >> 4, n = lane & 15;
    // first kernel of a decode call: it clears the sticky error word and clamps silently; the
    // ranking kernel, which sees the same table entries and contexts, reports them
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < 2) header[threadIdx.x] = 0;
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 2) header[kValueCount] = 0;   // value work list
    const int ctx = ctx_clamped_quiet(kv, r);
    const int N = (ctx + kPage - 1) / kPage;
    const int base = blockIdx.x * kScoreBlocks + wave * 16;
    if (base >= N) return;

    // A operand: row n = block base + n; step kk holds bytes 64*kk + 16*kq .. +15 of its record
    const int32_t *table = kv.block_table + (size_t)r * kv.max_blocks;
    const int page = clamp_page_quiet(table[min(base + n, N - 1)], kv.num_pages);
    const uint8_t *mp = meta + ((size_t)page * kv.num_kv_heads + h) * kMetaBytes + kq * 16;
    uint4 a[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) a[kk] = ld16(mp + kk * 64);
    // B operand: column n = head n; the same 8 numbers of the record's index range, taken from q with the
    // entries of the wrong sign zeroed (steps 0-3 meet the minima, 4-7 the maxima)
    f32x4_t d = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        uint4 b = make_uint4(0, 0, 0, 0);
        if (n < G) {
            const int ch = (32 * kk + 8 * kq) & 127;
            b = ld16(q + ((size_t)(r * kv.num_q_heads + h * G + n) * kHeadDim + ch) * 2);
            if (!CENTER) {
                uint32_t w[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t neg = ((w[j] >> 15) & 0x00010001u) * 0xFFFFu;
                    w[j] &= (kk >= 4) ? ~neg : neg;
                }
                b = make_uint4(w[0], w[1], w[2], w[3]);
            }
        }
        d = mfma_16x16x32<DT>(a[kk], b, d);
    }
    // lane (kq, n): head n of blocks base + 4kq .. + 4kq+3; the maximum over the heads of the group
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float v = n < G ? d[j] : -INFINITY;
        v = row_max16(v) * (CENTER ? 0.5f * kScale : kScale);
        const int b2 = base + 4 * kq + j;
        if (n == 0 && b2 < N) {
            scores[(size_t)s * kv.max_blocks + b2] = v;
            if (scores_out) scores_out[(size_t)s * kv.max_blocks + b2] = v;
        }
    }
}

template <int DT, int G>
static hipError_t launch_score_t(const KvView &kv, int scorer, const void *q, const void *meta, const DecodeWs &ws,
                                 float *scores_out, hipStream_t st) {
    const int S = kv.batch * kv.num_kv_heads;
    const dim3 grid((kv.max_blocks + kScoreBlocks - 1) / kScoreBlocks, S);
    if constexpr (G >= 8) {
        if (scorer == 1)
            score_mfma_kernel<DT, G, 1><<<grid, 256, 0, st>>>(kv, (const uint8_t *)q, (const uint8_t *)meta, ws.scores,
                                                              scores_out, ws.header);
        else
            score_mfma_kernel<DT, G, 0><<<grid, 256, 0, st>>>(kv, (const uint8_t *)q, (const uint8_t *)meta, ws.scores,
                                                              scores_out, ws.header);
    } else {
        if (scorer == 1)
            score_kernel<DT, G, 1><<<grid, 256, 0, st>>>(kv, (const uint8_t *)q, (const uint8_t *)meta, ws.scores,
                                                         scores_out, ws.header);
        else
            score_kernel<DT, G, 0><<<grid, 256, 0, st>>>(kv, (const uint8_t *)q, (const uint8_t *)meta, ws.scores,
                                                         scores_out, ws.header);
    }
    return hipGetLastError();
}

hipError_t launch_score(const KvView &kv, int dtype, int G, int scorer, const void *q, const void *meta,
                        const DecodeWs &ws, float *scores_out, hipStream_t st) {
#define PSA_CASE(DT, GG) \
    if (dtype == DT && G == GG) return launch_score_t<DT, GG>(kv, scorer, q, meta, ws, scores_out, st);
    PSA_CASE(0, 1) PSA_CASE(0, 2) PSA_CASE(0, 4) PSA_CASE(0, 8)
    PSA_CASE(1, 1) PSA_CASE(1, 2) PSA_CASE(1, 4) PSA_CASE(1, 8)
#undef PSA_CASE
    return hipErrorInvalidValue;
}

}  // namespace psa
