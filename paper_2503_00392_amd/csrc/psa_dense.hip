// Dense control: exact paged decode attention (softmax(q K^T / sqrt d) V over every block),
// split over the context, with fp32 online softmax; a second kernel merges the splits.
#include "psa_attend.h"
#include "psa_host.h"

namespace psa {

constexpr int kDenseStride = 132;  // M, l, pad, pad, acc[128]

template <int DT>
__device__ __forceinline__ void row_to_float(const uint4 &v, float (&f)[8]) {
    f[0] = cvt_lo<DT>(v.x); f[1] = cvt_hi<DT>(v.x);
    f[2] = cvt_lo<DT>(v.y); f[3] = cvt_hi<DT>(v.y);
    f[4] = cvt_lo<DT>(v.z); f[5] = cvt_hi<DT>(v.z);
    f[6] = cvt_lo<DT>(v.w); f[7] = cvt_hi<DT>(v.w);
}

// grid (nsplit, S); 256 threads.  Wave w of the workgroup takes blocks b0+w, b0+w+4, ...; every
// 16-lane row group keeps its own running (m, l, acc) over the token rows it sees, so the loop has
// no cross-row-group traffic; the 16 states of a workgroup are merged once at the end.
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

    const QueryRegs<G> qr = load_query<G>(q, r, h, kv.num_q_heads, cl);
    float m[G], l[G], acc[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = -INFINITY; l[g] = 0.0f;
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[g][c] = 0.0f;
    }

    const int32_t *table = kv.block_table + (size_t)r * kv.max_blocks;
    for (int b = b0 + wave; b < b1; b += 4) {
        const int page = clamp_page(table[b], kv.num_pages, header);
        const size_t off = ((size_t)page * kv.num_kv_heads + h) * kSliceBytes;
        Slice k = load_slice(kv.k_pool + off, lane);
        Slice v = load_slice(kv.v_pool + off, lane);
        const int valid = min(kPage, ctx - b * kPage);
        float sc[4][G];
        slice_logits<DT, G>(k, qr, rg, valid, sc);
        if (valid < kPage) zero_invalid_rows(v, rg, valid);
        float vf[4][8];
#pragma unroll
        for (int i = 0; i < 4; ++i) row_to_float<DT>(v.r[i], vf[i]);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float mn = fmaxf(fmaxf(fmaxf(sc[0][g], sc[1][g]), fmaxf(sc[2][g], sc[3][g])), m[g]);
            if (mn == -INFINITY) continue;   // this row group has seen no valid token yet
            const float alpha = exp2_fast(m[g] - mn);
            float p[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) p[i] = exp2_fast(sc[i][g] - mn);
            l[g] = l[g] * alpha + ((p[0] + p[1]) + (p[2] + p[3]));
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                float a = acc[g][c] * alpha;
                a = fmaf(p[0], vf[0][c], a);
                a = fmaf(p[1], vf[1][c], a);
                a = fmaf(p[2], vf[2][c], a);
                a = fmaf(p[3], vf[3][c], a);
                acc[g][c] = a;
            }
            m[g] = mn;
        }
    }

    // merge the 4 row groups of the wave (lanes l, l^16, l^32, l^48 hold the same channel slot)
#pragma unroll
    for (int step = 16; step <= 32; step <<= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float mo = __shfl_xor(m[g], step);
            const float lo = __shfl_xor(l[g], step);
            const float mn = fmaxf(m[g], mo);
            const float a = (mn == -INFINITY) ? 0.0f : exp2_fast(m[g] - mn);
            const float bsc = (mn == -INFINITY) ? 0.0f : exp2_fast(mo - mn);
            l[g] = l[g] * a + lo * bsc;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const float ao = __shfl_xor(acc[g][c], step);
                acc[g][c] = acc[g][c] * a + ao * bsc;
            }
            m[g] = mn;
        }
    }

    // merge the 4 waves through LDS
    __shared__ float st_acc[4][G][kHeadDim];
    __shared__ float st_m[4][G], st_l[4][G];
    if (rg == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int c = 0; c < 8; ++c) st_acc[wave][g][cl * 8 + c] = acc[g][c];
            if (cl == 0) { st_m[wave][g] = m[g]; st_l[wave][g] = l[g]; }
        }
    }
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
    __shared__ float red[512];
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
    red[tid] = M;
    __syncthreads();
    for (int d = 256; d >= 1; d >>= 1) {
        if (tid < d) red[tid] = fmaxf(red[tid], red[tid + d]);
        __syncthreads();
    }
    M = red[0];
    __syncthreads();
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
