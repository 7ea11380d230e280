// Dense control: exact paged decode attention (softmax(q K^T / sqrt d) V over every block),
// split over the context, with fp32 online softmax; a second kernel merges the splits.
#include "psa_attend.h"
#include "psa_host.h"

namespace psa {

constexpr int kDenseStride = 132;  // M, l, pad, pad, acc[128]

// grid (nsplit, S); 256 threads.  Wave w of the workgroup takes blocks b0+w, b0+w+4, ... and carries its own
// online softmax over them, both products on the matrix cores:
//   logits  D[token][head] = K[token][channel] Q[channel][head]: four 16x16x32 steps.  Row r of the A operand
//           stands for token 4*(r%4) + r/4, so that lane (kq, n) = (lane/16, lane%16) ends up with the logits
//           of head n for tokens kq, 4+kq, 8+kq, 12+kq -- the token rows its value loads fetch;
//   values  D[head][channel] += P[head][token] V[token][channel]: eight 16x16x16 products per block (one per
//           channel of the lane's eight), the weights split into two 16-bit halves; lane (kq, cl) accumulates
//           heads 4kq..4kq+3 of channels 8cl..8cl+7.
// The running maximum of a head is shared by the wave (two exchanges per block); the four waves are merged
// once at the end.
template <int DT, int G>
__global__ __launch_bounds__(256) void dense_split_kernel(KvView kv, const uint8_t *__restrict__ q,
                                                          float *__restrict__ partial,
                                                          int blocks_per_split, int32_t *header) {
    const int s = blockIdx.y, split = blockIdx.x, nsplit = gridDim.x;
    const int r = s / kv.num_kv_heads, h = s % kv.num_kv_heads;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, rg = lane >> 4, cl = lane & 15;
    const int ctx = ctx_clamped(kv, r, header);
    const int N = (ctx + kPage - 1) / kPage;
    // every request is cut into the same number of splits, each over its own length: ragged batches stay balanced
    const int bps = min(blocks_per_split, (N + nsplit - 1) / nsplit);
    const int b0 = split * bps;
    const int b1 = min(N, b0 + bps);

    // B operand of the logits: column cl = head cl (zero beyond the group), channels 8*(4kk + rg) .. +7 in step kk
    uint4 qb[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        qb[kk] = make_uint4(0, 0, 0, 0);
        if (cl < G) qb[kk] = ld16(q + ((size_t)(r * kv.num_q_heads + h * G + cl) * kHeadDim + (4 * kk + rg) * 8) * 2);
    }
    const int row_token = 4 * (cl & 3) + (cl >> 2);      // the token this lane's row of the A operand stands for
    float m = -INFINITY, l = 0.0f;                       // head cl: running maximum (whole wave), exp-sum (this row group)
    f32x4_t acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};

    const int32_t *table = kv.block_table + (size_t)r * kv.max_blocks;
    for (int b = b0 + wave; b < b1; b += 4) {
        const int page = clamp_page(table[b], kv.num_pages, header);
        const size_t off = ((size_t)page * kv.num_kv_heads + h) * kSliceBytes;
        const uint8_t *kp = kv.k_pool + off + row_token * kRowBytes + rg * 16;
        uint4 ka[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) ka[kk] = ld16(kp + kk * 64);     // (operand layout: half a cache line per row and load, the
                                                                         // next load takes the other half -- not marked read-once)
        Slice v = load_slice(kv.v_pool + off, lane);
        const int valid = min(kPage, ctx - b * kPage);
        f32x4_t s4 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) s4 = mfma_16x16x32<DT>(ka[kk], qb[kk], s4);
        float sc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) sc[j] = (4 * j + rg < valid) ? s4[j] * kScaleLog2 : -INFINITY;
        if (valid < kPage) zero_invalid_rows(v, rg, valid);
        float bm = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
        bm = fmaxf(bm, __shfl_xor(bm, 16));
        bm = fmaxf(bm, __shfl_xor(bm, 32));
        const float mn = fmaxf(m, bm);                   // finite: every block below N has a valid token
        const float alpha = exp2_fast(m - mn);
        float p[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) p[j] = exp2_fast(sc[j] - mn);
        l = l * alpha + ((p[0] + p[1]) + (p[2] + p[3]));
        m = mn;
        // the accumulators hold heads 4rg .. 4rg+3: rescale each by its head's factor (held by lane = head)
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const float ax = __shfl(alpha, 4 * rg + x);
#pragma unroll
            for (int t = 0; t < 8; ++t) acc[t][x] *= ax;
        }
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) split16<DT>(p[j], hi[j], lo[j]);
        const uint2 a_hi = make_uint2(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16));
        const uint2 a_lo = make_uint2(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16));
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const uint32_t w0 = pick_word(v.r[0], t >> 1), w1 = pick_word(v.r[1], t >> 1);
            const uint32_t w2 = pick_word(v.r[2], t >> 1), w3 = pick_word(v.r[3], t >> 1);
            const uint2 bv = (t & 1) ? make_uint2((w0 >> 16) | (w1 & 0xffff0000u), (w2 >> 16) | (w3 & 0xffff0000u))
                                     : make_uint2((w0 & 0xffffu) | (w1 << 16), (w2 & 0xffffu) | (w3 << 16));
            acc[t] = mfma_16x16x16<DT>(a_hi, bv, acc[t]);
            acc[t] = mfma_16x16x16<DT>(a_lo, bv, acc[t]);
        }
    }
    // the exp-sum over the four row groups
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);

    // merge the 4 waves through LDS
    __shared__ float st_acc[4][G][kHeadDim];
    __shared__ float st_m[4][G], st_l[4][G];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int g = 4 * rg + x;
        if (g < G) {
#pragma unroll
            for (int t = 0; t < 8; ++t) st_acc[wave][g][cl * 8 + t] = acc[t][x];
        }
    }
    if (rg == 0 && cl < G) { st_m[wave][cl] = m; st_l[wave][cl] = l; }
    __syncthreads();
    float *dst = partial + ((size_t)s * nsplit + split) * G * kDenseStride;
    for (int idx = tid; idx < G * kHeadDim; idx += 256) {
        const int g = idx / kHeadDim, ch = idx % kHeadDim;
        float M = fmaxf(fmaxf(st_m[0][g], st_m[1][g]), fmaxf(st_m[2][g], st_m[3][g]));
        float lsum = 0.0f, a = 0.0f;
        if (M != -INFINITY) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float sc = exp2_fast(st_m[w][g] - M);
                lsum += st_l[w][g] * sc;
                a += st_acc[w][g][ch] * sc;
            }
        }
        dst[g * kDenseStride + 4 + ch] = a;
        if (ch == 0) { dst[g * kDenseStride] = M; dst[g * kDenseStride + 1] = lsum; }
    }
}

// grid (S*G); 512 threads = 4 split lanes x 128 channels.  Split lane j takes splits j, j+4, ... in
// ascending order (loads issued four deep, no branches); the 4 lanes are then added in a fixed order.
__global__ __launch_bounds__(512) void dense_combine_kernel(const float *__restrict__ partial, int nsplit,
                                                            int G, int num_kv_heads, int num_q_heads,
                                                            float *__restrict__ out,
                                                            float *__restrict__ lse) {
    __shared__ float red[8];
    __shared__ float wgt[1024];                 // rescale factor of every split (nsplit <= 1024)
    __shared__ float num_part[4][kHeadDim];
    __shared__ float den_part[4];
    const int s = blockIdx.x / G, g = blockIdx.x % G, tid = threadIdx.x;
    const int ch = tid & 127, sl = tid >> 7;
    const int r = s / num_kv_heads, h = s % num_kv_heads;
    const float *src = partial + ((size_t)s * nsplit * G + g) * kDenseStride;
    const size_t stride = (size_t)G * kDenseStride;
    float M = -INFINITY;
    for (int i = tid; i < nsplit; i += 512) { const float mi = src[i * stride]; wgt[i] = mi; M = fmaxf(M, mi); }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) M = fmaxf(M, __shfl_xor(M, d));
    if ((tid & 63) == 0) red[tid >> 6] = M;
    __syncthreads();
    M = fmaxf(fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])), fmaxf(fmaxf(red[4], red[5]), fmaxf(red[6], red[7])));
    for (int i = tid; i < nsplit; i += 512) {
        const float mi = wgt[i];
        wgt[i] = (mi == -INFINITY || M == -INFINITY) ? 0.0f : exp2_fast(mi - M);
    }
    __syncthreads();
    float num = 0.0f, den = 0.0f;
    for (int i0 = sl; i0 < nsplit; i0 += 16) {
        float a[4], l[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int i = min(i0 + 4 * k, nsplit - 1);          // clamped: the loads need no branch
            a[k] = src[i * stride + 4 + ch];
            l[k] = src[i * stride + 1];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float w = (i0 + 4 * k < nsplit) ? wgt[i0 + 4 * k] : 0.0f;
            num = fmaf(a[k], w, num);
            den = fmaf(l[k], w, den);
        }
    }
    num_part[sl][ch] = num;
    if (ch == 0) den_part[sl] = den;
    __syncthreads();
    if (tid < kHeadDim) {
        const float n = (num_part[0][tid] + num_part[1][tid]) + (num_part[2][tid] + num_part[3][tid]);
        const float dsum = (den_part[0] + den_part[1]) + (den_part[2] + den_part[3]);
        const size_t qi = (size_t)r * num_q_heads + h * G + g;
        out[qi * kHeadDim + tid] = dsum > 0.0f ? n / dsum : 0.0f;
        if (lse && tid == 0) lse[qi] = dsum > 0.0f ? (M + log2_fast(dsum)) * kLn2 : -INFINITY;
    }
}

// ---- host side ----------------------------------------------------------------------------------
int dense_num_splits(const psa_kv_desc *d) {
    const int S = d->batch * d->num_kv_heads;
    // aim at ~8 workgroups per CU over the whole grid, at least 8 blocks (64 KiB of K+V) per split
    int want = (2048 + S - 1) / S;
    int max_by_len = (d->max_blocks_per_seq + 7) / 8;
    int n = want < max_by_len ? want : max_by_len;
    return n < 1 ? 1 : n;
}

size_t dense_workspace_bytes(const psa_kv_desc *d) {
    const size_t S = (size_t)d->batch * d->num_kv_heads;
    const int G = d->num_q_heads / d->num_kv_heads;
    return 256 + S * dense_num_splits(d) * G * kDenseStride * sizeof(float);
}

template <int DT, int G>
static hipError_t launch_dense_t(const KvView &kv, const void *q, float *out, float *lse, void *ws,
                                 int nsplit, hipStream_t st) {
    int32_t *header = reinterpret_cast<int32_t *>(ws);
    float *partial = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(ws) + 256);
    const int S = kv.batch * kv.num_kv_heads;
    const int bps = (kv.max_blocks + nsplit - 1) / nsplit;
    clear_words_kernel<<<1, 64, 0, st>>>(header, 64);
    dense_split_kernel<DT, G><<<dim3(nsplit, S), 256, 0, st>>>(kv, (const uint8_t *)q, partial, bps, header);
    dense_combine_kernel<<<S * G, 512, 0, st>>>(partial, nsplit, G, kv.num_kv_heads, kv.num_q_heads, out, lse);
    return hipGetLastError();
}

hipError_t launch_dense(const psa_kv_desc *d, const void *q, float *out, float *lse, void *ws,
                        hipStream_t st) {
    const KvView kv = make_view(d);
    const int G = d->num_q_heads / d->num_kv_heads;
    const int nsplit = dense_num_splits(d);
#define PSA_CASE(DT, GG) \
    if (d->dtype == DT && G == GG) return launch_dense_t<DT, GG>(kv, q, out, lse, ws, nsplit, st);
    PSA_CASE(0, 1) PSA_CASE(0, 2) PSA_CASE(0, 4) PSA_CASE(0, 8)
    PSA_CASE(1, 1) PSA_CASE(1, 2) PSA_CASE(1, 4) PSA_CASE(1, 8)
#undef PSA_CASE
    return hipErrorInvalidValue;
}

}  // namespace psa
