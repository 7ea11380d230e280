// Block scoring (Algorithm 1, line 5): the criticality score of every block of every stream from
// its per-channel min/max key metadata.
#include "psa_host.h"

namespace psa {

constexpr int kScoreBlocks = 64;   // blocks per workgroup and round: 16 per wave (the matrix version: per workgroup)
constexpr int kMaxRounds = 4;      // rounds a workgroup of score_kernel makes at most

// =================================================================================================
// Scoring.  Upper bound (CENTER = 0):
//   UB[g][b] = (1/sqrt d) sum_c max(q_c kmin_c, q_c kmax_c) = (1/sqrt d) (q+ . kmax + q- . kmin)
//   with q+ = max(q,0), q- = min(q,0).
// Cuboid centre (CENTER = 1): (1/sqrt d) q . (kmin + kmax)/2 = (1/(2 sqrt d)) (q . kmax + q . kmin).
// Mean key (CENTER = 2, this kernel only): `meta` holds one vector per (page, KV head), 256 bytes, the mean of the
// block's keys; the score is (1/sqrt d) q . mean.
// Either way CS[b] = max over the heads g of the group.
// grid (ceil(max_blocks / (64 rounds)), S), 256 threads; a workgroup covers 64*rounds consecutive blocks, wave w
// the 16*rounds blocks from 16*rounds*w.  A 16-lane row handles one block per step: lane cl takes channels
// 8cl..8cl+7 of the min row (against q-, or q) and of the max row (against q+, or q), so each row's two loads
// are 256 contiguous bytes.  The wave fetches the pages of all its blocks with one load (lane = block) and
// keeps the records of one round (16 blocks, 8 KiB) in flight while it computes the round before.
// =================================================================================================
template <int DT, int G, int CENTER>
__global__ __launch_bounds__(256) void score_kernel(KvView kv, const uint8_t *__restrict__ q,
                                                    const uint8_t *__restrict__ meta,
                                                    float *__restrict__ scores,
                                                    float *__restrict__ scores_out, int32_t *header, int rounds) {
    const int s = blockIdx.y, r = s / kv.num_kv_heads, h = s % kv.num_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, row = lane >> 4, cl = lane & 15;
    // first kernel of a decode call: it clears the sticky error word and clamps silently; the
    // ranking kernel, which sees the same table entries and contexts, reports them
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < 2) header[threadIdx.x] = 0;
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 2) header[kValueCount] = 0;   // value work list
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 3) header[kClosedStreams] = 0;
    const int ctx = ctx_clamped_quiet(kv, r);
    const int N = (ctx + kPage - 1) / kPage;
    const int base = (blockIdx.x * 4 + wave) * 16 * rounds;      // the wave's first block
    if (base >= N) return;
    const int mine = min(16 * rounds, N - base);                 // blocks of this wave

    // pages of the wave's blocks: lane = block
    const int32_t *table = kv.block_table + (size_t)r * kv.max_blocks;
    const int page_of_lane = clamp_page_quiet(table[base + min(lane, mine - 1)], kv.num_pages);

    // the lane's 8 channels of every query head: the negative parts (for the minima) and the positive parts (for
    // the maxima), or the whole of it twice for the centre
    uint32_t qn[G][4], qp[G][4];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const uint4 a = ld16(q + ((size_t)(r * kv.num_q_heads + h * G + g) * kHeadDim + cl * 8) * 2);
        const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t neg = ((w[j] >> 15) & 0x00010001u) * 0xFFFFu;   // 0xFFFF in each negative half
            qn[g][j] = CENTER ? w[j] : (w[j] & neg);
            qp[g][j] = CENTER == 2 ? 0u : (CENTER ? w[j] : (w[j] & ~neg));
        }
    }

    // round rd: blocks base + 16 rd + 4 it + row, it = 0..3
    uint4 mn[2][4], mx[2][4];
    auto fetch = [&](int rd, uint4 (&lo)[4], uint4 (&hi)[4]) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int j = min(16 * rd + 4 * it + row, mine - 1);     // (clamped: the loads need no branch)
            const int page = __shfl(page_of_lane, j);
            const uint8_t *mp = meta + ((size_t)page * kv.num_kv_heads + h) * (CENTER == 2 ? 256 : kMetaBytes) + cl * 16;
            lo[it] = ld16_stream(mp);
            if constexpr (CENTER == 2) hi[it] = make_uint4(0, 0, 0, 0);
            else hi[it] = ld16_stream(mp + 256);
        }
    };
    auto reduce = [&](int rd, const uint4 (&lo)[4], const uint4 (&hi)[4]) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int j = 16 * rd + 4 * it + row;
            const uint32_t a[4] = {lo[it].x, lo[it].y, lo[it].z, lo[it].w};
            const uint32_t b[4] = {hi[it].x, hi[it].y, hi[it].z, hi[it].w};
            float cs = -INFINITY;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float p = 0.0f;
#pragma unroll
                for (int x = 0; x < 4; ++x) p = dot2<DT>(a[x], qn[g][x], p);
#pragma unroll
                for (int x = 0; x < 4; ++x) p = dot2<DT>(b[x], qp[g][x], p);
                p = row_sum16(p);
                cs = fmaxf(cs, p * (CENTER == 1 ? 0.5f * kScale : kScale));
            }
            if (cl == 0 && j < mine) {
                scores[(size_t)s * kv.max_blocks + base + j] = cs;
                if (scores_out) scores_out[(size_t)s * kv.max_blocks + base + j] = cs;
            }
        }
    };
    const int nr = (mine + 15) / 16;
    fetch(0, mn[0], mx[0]);
#pragma unroll
    for (int rd = 0; rd < kMaxRounds; ++rd) {
        if (rd < nr) {
            if (rd + 1 < nr) fetch(rd + 1, mn[(rd + 1) & 1], mx[(rd + 1) & 1]);
            reduce(rd, mn[rd & 1], mx[rd & 1]);
        }
    }
}

// =================================================================================================
// The same scoring, page by page instead of stream by stream, for KV-head counts that divide 16.  The metadata of
// a page is [KV head][min | max], 512 bytes per head, so the KV heads of one page are contiguous (4 KiB with eight):
// a workgroup that scores ALL heads of its blocks reads whole pages' metadata at a time, where the stream-by-stream
// kernel picks one isolated 512-byte record out of every page.
// grid (ceil(max_blocks / nb), batch), 256 threads; a workgroup covers nb consecutive blocks (nb <= 64, a multiple
// of 64/H) of one request.  The 16 rows of the workgroup (4 waves x 4 rows of 16 lanes) form a (16/H blocks) x
// (H heads) tile per step: row rho takes head rho % H of block step * 16/H + rho / H; four steps are a round, and
// a round's records stay in flight while the round before is computed.
// =================================================================================================
template <int DT, int G, int CENTER>
__global__ __launch_bounds__(256) void score_pages_kernel(KvView kv, const uint8_t *__restrict__ q,
                                                          const uint8_t *__restrict__ meta,
                                                          float *__restrict__ scores,
                                                          float *__restrict__ scores_out, int32_t *header, int nb) {
    const int r = blockIdx.y, H = kv.num_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, row = lane >> 4, cl = lane & 15;
    const int rho = wave * 4 + row, h = rho % H, sub = rho / H, BS = 16 / H;
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < 2) header[threadIdx.x] = 0;
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 2) header[kValueCount] = 0;   // value work list
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 3) header[kClosedStreams] = 0;
    const int ctx = ctx_clamped_quiet(kv, r);
    const int N = (ctx + kPage - 1) / kPage;
    const int base = blockIdx.x * nb;
    if (base >= N) return;
    const int mine = min(nb, N - base);                 // blocks of this workgroup
    const int32_t *table = kv.block_table + (size_t)r * kv.max_blocks;
    const int page_of_lane = clamp_page_quiet(table[base + min(lane, mine - 1)], kv.num_pages);   // lane = block
    const int s = r * H + h;

    uint32_t qn[G][4], qp[G][4];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const uint4 a = ld16(q + ((size_t)(r * kv.num_q_heads + h * G + g) * kHeadDim + cl * 8) * 2);
        const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t neg = ((w[j] >> 15) & 0x00010001u) * 0xFFFFu;   // 0xFFFF in each negative half
            qn[g][j] = CENTER ? w[j] : (w[j] & neg);
            qp[g][j] = CENTER ? w[j] : (w[j] & ~neg);
        }
    }

    uint4 mn[2][4], mx[2][4];
    auto fetch = [&](int rd, uint4 (&lo)[4], uint4 (&hi)[4]) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int j = min((4 * rd + it) * BS + sub, mine - 1);     // (clamped: the loads need no branch)
            const int page = __shfl(page_of_lane, j);
            const uint8_t *mp = meta + ((size_t)page * H + h) * kMetaBytes + cl * 16;
            lo[it] = ld16_stream(mp);
            hi[it] = ld16_stream(mp + 256);
        }
    };
    auto reduce = [&](int rd, const uint4 (&lo)[4], const uint4 (&hi)[4]) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int j = (4 * rd + it) * BS + sub;
            const uint32_t a[4] = {lo[it].x, lo[it].y, lo[it].z, lo[it].w};
            const uint32_t b[4] = {hi[it].x, hi[it].y, hi[it].z, hi[it].w};
            float cs = -INFINITY;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float p = 0.0f;
#pragma unroll
                for (int x = 0; x < 4; ++x) p = dot2<DT>(a[x], qn[g][x], p);
#pragma unroll
                for (int x = 0; x < 4; ++x) p = dot2<DT>(b[x], qp[g][x], p);
                p = row_sum16(p);
                cs = fmaxf(cs, p * (CENTER ? 0.5f * kScale : kScale));
            }
            if (cl == 0 && j < mine) {
                scores[(size_t)s * kv.max_blocks + base + j] = cs;
                if (scores_out) scores_out[(size_t)s * kv.max_blocks + base + j] = cs;
            }
        }
    };
    const int nr = (mine + 4 * BS - 1) / (4 * BS);       // rounds: at most 64 / (4 BS) = 16
    fetch(0, mn[0], mx[0]);
#pragma nounroll
    for (int rd = 0; rd < nr; rd += 2) {
        if (rd + 1 < nr) fetch(rd + 1, mn[1], mx[1]);
        reduce(rd, mn[0], mx[0]);
        if (rd + 1 < nr) {
            if (rd + 2 < nr) fetch(rd + 2, mn[0], mx[0]);
            reduce(rd + 1, mn[1], mx[1]);
        }
    }
}

// =================================================================================================
// Scoring on the matrix cores (used at G = 8 when the KV-head count does not allow the page-by-page kernel above:
// the stream-by-stream packed-dot kernel is bound by its arithmetic there).  Upper bound (CENTER = 0):
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
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 3) header[kClosedStreams] = 0;
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
    for (int kk = 0; kk < 8; ++kk) a[kk] = ld16(mp + kk * 64);      // (half a cache line per record and load: the other half is the next load's, so not marked read-once)
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
    // rounds per workgroup of score_kernel: as many (up to kMaxRounds) as still leave four workgroups per compute unit
    long long per = ((long long)S * kv.max_blocks) / (4ll * compute_units() * kScoreBlocks);
    const int rounds = per < 1 ? 1 : (per > kMaxRounds ? kMaxRounds : (int)per);
    const dim3 grid_r((kv.max_blocks + kScoreBlocks * rounds - 1) / (kScoreBlocks * rounds), S);
    if (scorer == 2) {
        score_kernel<DT, G, 2><<<grid_r, 256, 0, st>>>(kv, (const uint8_t *)q, (const uint8_t *)meta, ws.scores,
                                                       scores_out, ws.header, rounds);
        return hipGetLastError();
    }
    if (kv.num_kv_heads > 1 && 16 % kv.num_kv_heads == 0) {
        // all KV heads of a page together; blocks per workgroup: as many (up to 64) as still leave four
        // workgroups per compute unit, in whole rounds of four steps
        const int round_blocks = 4 * (16 / kv.num_kv_heads);
        long long want = ((long long)kv.batch * kv.max_blocks) / (4ll * compute_units());
        int nb = (int)(want / round_blocks) * round_blocks;
        nb = nb < round_blocks ? round_blocks : (nb > 64 ? 64 : nb);
        const dim3 grid_p((kv.max_blocks + nb - 1) / nb, kv.batch);
        if (scorer == 1)
            score_pages_kernel<DT, G, 1><<<grid_p, 256, 0, st>>>(kv, (const uint8_t *)q, (const uint8_t *)meta, ws.scores,
                                                                 scores_out, ws.header, nb);
        else
            score_pages_kernel<DT, G, 0><<<grid_p, 256, 0, st>>>(kv, (const uint8_t *)q, (const uint8_t *)meta, ws.scores,
                                                                 scores_out, ws.header, nb);
    } else if constexpr (G >= 8) {
        if (scorer == 1)
            score_mfma_kernel<DT, G, 1><<<grid, 256, 0, st>>>(kv, (const uint8_t *)q, (const uint8_t *)meta, ws.scores,
                                                              scores_out, ws.header);
        else
            score_mfma_kernel<DT, G, 0><<<grid, 256, 0, st>>>(kv, (const uint8_t *)q, (const uint8_t *)meta, ws.scores,
                                                              scores_out, ws.header);
    } else {
        if (scorer == 1)
            score_kernel<DT, G, 1><<<grid_r, 256, 0, st>>>(kv, (const uint8_t *)q, (const uint8_t *)meta, ws.scores,
                                                           scores_out, ws.header, rounds);
        else
            score_kernel<DT, G, 0><<<grid_r, 256, 0, st>>>(kv, (const uint8_t *)q, (const uint8_t *)meta, ws.scores,
                                                           scores_out, ws.header, rounds);
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
