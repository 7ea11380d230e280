// Block scoring (Algorithm 1, line 5): the criticality score of every block of every stream from
// its per-channel min/max key metadata.
#include "psa_host.h"

namespace psa {

constexpr int kScoreIts = 4;                  // blocks per 16-lane row of a wave (2 and 8 measured: no faster)
constexpr int kScoreBlocks = 16 * kScoreIts;  // blocks per workgroup

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
    const int base = blockIdx.x * kScoreBlocks + wave * (4 * kScoreIts);
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
    uint4 ma[kScoreIts], mb[kScoreIts];
#pragma unroll
    for (int it = 0; it < kScoreIts; ++it) {
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
    for (int it = 0; it < kScoreIts; ++it) {
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

template <int DT, int G>
static hipError_t launch_score_t(const KvView &kv, int scorer, const void *q, const void *meta, const DecodeWs &ws,
                                 float *scores_out, hipStream_t st) {
    const int S = kv.batch * kv.num_kv_heads;
    const dim3 grid((kv.max_blocks + kScoreBlocks - 1) / kScoreBlocks, S);
    if (scorer == 1)
        score_kernel<DT, G, 1><<<grid, 256, 0, st>>>(kv, (const uint8_t *)q, (const uint8_t *)meta, ws.scores,
                                                     scores_out, ws.header);
    else
        score_kernel<DT, G, 0><<<grid, 256, 0, st>>>(kv, (const uint8_t *)q, (const uint8_t *)meta, ws.scores,
                                                     scores_out, ws.header);
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
