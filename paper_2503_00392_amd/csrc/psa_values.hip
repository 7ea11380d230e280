// Value pass and final merge of one PSA decode step (Algorithm 1, lines 10-12 and 19).
//
// By the time these kernels run, the selection kernel has fixed every query head's stop n_g and
// left the exact scaled logits of the ranked blocks in the workspace.  What remains is plain
// attention over each head's own prefix: softmax numerators from the stored logits, times the value
// slices of the selected blocks -- every workgroup independent, no waiting, and only blocks
// actually selected are read.
//   attend_kernel    per value unit (chunk, stream) on the work list the selection kernel wrote:
//                    p = exp(logit - chunk max), partial numerator sum_t p_t v_t per head (on the matrix
//                    cores, the weights as a sum of two 16-bit halves), exp-sum and reference maximum
//   finalize_kernel  merges a head's chunks (the online-softmax merge of line 11, all at once):
//                    out_g = sum over the chunks of the head's own prefix of the partial numerators,
//                    over the sum of the partial exp-sums, both rescaled to one reference maximum
#include "psa_attend.h"
#include "psa_host.h"

namespace psa {

constexpr int kBatch = 4;   // slices a wave keeps in flight

// CBMAX: blocks per value unit at most (32 for the default chunk size and below, else 64): it sizes the LDS
// arrays, and with them how many workgroups fit a CU.
template <int G, int CBMAX>
struct AttendShared {
    float p[CBMAX][kPage][G];              // logits, then softmax numerators
    float st_acc[4][G][kHeadDim];          // per-wave partial numerators
    float red[256];
    int page[CBMAX];
    int valid[CBMAX];
    int cnt[G];
    float Mref[G];
    float lsum[G];
};

// Stop of head g of a stream: (n, P_acc) as the selection kernel left it, n = N when it never stopped.
__device__ __forceinline__ int head_stop(const StreamCtl *ctl, int g, int N) {
    const unsigned long long st = ctl->stop[g];
    return (st != ~0ull && (int)(st >> 32) <= N) ? (int)(st >> 32) : N;
}

// One value unit: chunk c of stream s.  Called by all 256 threads of a workgroup.
template <int DT, int G, int CBMAX>
__device__ void attend_unit(AttendShared<G, CBMAX> &sh, const KvView &kv, const DecodeWs &ws, int CB, int s, int c) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, rg = lane >> 4, cl = lane & 15;
    const int h = s % kv.num_kv_heads;
    int ctx = kv.ctx_lens[s / kv.num_kv_heads];
    ctx = ctx < 0 ? 0 : (ctx > kv.max_blocks * kPage ? kv.max_blocks * kPage : ctx);
    const int N = (ctx + kPage - 1) / kPage;
    const int start = c * CB;
    if (start >= N) return;
    const int nblk = min(CB, N - start);
    const StreamCtl *ctl = &ws.ctl[s];
    int cnt[G], maxcnt = 0;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        cnt[g] = min(nblk, max(0, head_stop(ctl, g, N) - start));
        maxcnt = max(maxcnt, cnt[g]);
    }
    if (maxcnt == 0) return;    // no head of the group reaches this chunk

    if (tid < maxcnt) {
        const size_t at = (size_t)s * kv.max_blocks + start + tid;
        sh.page[tid] = ws.ranked_page[at];
        sh.valid[tid] = min(kPage, ctx - ws.order[at] * kPage);
    }
    lds_barrier();
    // first batch of value slices, issued before the softmax bookkeeping so that they overlap it
    Slice v[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
        const int i = wave * kBatch + u;
        if (i < maxcnt) {
            v[u] = load_slice(value_slice(kv, sh.page[i], h), lane);
        }
    }
    // logits of the chunk (contiguous in the workspace as [block][head][token]) -> LDS as
    // [block][token][head], with each head's maximum over the blocks it uses
    const float *lg = ws.logits + ((size_t)s * kv.max_blocks + start) * (kPage * G);
    const int total = maxcnt * kPage * G;
    float mx = -INFINITY;                       // thread-local, for head g = (tid / 16) % G
    for (int idx = tid; idx < total; idx += 256) {
        const int t = idx % kPage, g = (idx / kPage) % G, i = idx / (kPage * G);
        const float x = lg[idx];
        sh.p[i][t][g] = x;
        if (i < cnt[g]) mx = fmaxf(mx, x);
    }
    // thread tid holds head (tid / 16) % G: reduce each 16-lane row, then the 16/G rows of a head
    mx = row_max16(mx);
    if (cl == 0) sh.red[tid >> 4] = mx;
    lds_barrier();
    if (tid < G) {
        float M = -INFINITY;
        for (int j = tid; j < 16; j += G) M = fmaxf(M, sh.red[j]);
        sh.Mref[tid] = M;
    }
    lds_barrier();
    float sum = 0.0f;
    for (int idx = tid; idx < total; idx += 256) {
        const int t = idx % kPage, g = (idx / kPage) % G, i = idx / (kPage * G);
        float *p = &sh.p[i][t][g];
        const float e = (i < cnt[g]) ? exp2_fast(*p - sh.Mref[g]) : 0.0f;   // masked tokens hold -inf
        *p = e;
        sum += e;
    }
    sum = row_sum16(sum);
    if (cl == 0) sh.red[16 + (tid >> 4)] = sum;
    lds_barrier();
    if (tid < G) {
        float l = 0.0f;
        for (int j = tid; j < 16; j += G) l += sh.red[16 + j];
        sh.lsum[tid] = l;
    }

    // Numerators on the matrix cores: per block D[head][channel] += P[head][token] V[token][channel] as eight
    // 16x16x16 products (one per channel of the lane's eight) with the softmax weights split into two
    // 16-bit halves (hi + lo keeps fp32 accuracy; the values are 16-bit already).  The k index of both
    // operands is the token: lane (rg, *) holds tokens rg, 4+rg, 8+rg, 12+rg -- exactly the rows its four
    // loads fetched -- so the B operand is four 16-bit picks from registers, no transposition.  A: row =
    // head lane%16 (zero beyond G).  D: lane (rg, cl) gets heads 4rg..4rg+3 of channel 8cl + tile.
    f32x4_t acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
    for (int i0 = wave * kBatch; i0 < maxcnt; i0 += 4 * kBatch) {
        if (i0 != wave * kBatch) {
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                if (i0 + u < maxcnt) {
                    v[u] = load_slice(value_slice(kv, sh.page[i0 + u], h), lane);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int i = i0 + u;
            if (i < maxcnt) {
                if (sh.valid[i] < kPage) zero_invalid_rows(v[u], rg, sh.valid[i]);
                uint32_t hi[4], lo[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float pj = cl < G ? sh.p[i][4 * j + rg][cl] : 0.0f;
                    split16<DT>(pj, hi[j], lo[j]);
                }
                const uint2 a_hi = make_uint2(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16));
                const uint2 a_lo = make_uint2(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16));
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const uint32_t w0 = pick_word(v[u].r[0], t >> 1), w1 = pick_word(v[u].r[1], t >> 1);
                    const uint32_t w2 = pick_word(v[u].r[2], t >> 1), w3 = pick_word(v[u].r[3], t >> 1);
                    const uint2 b = (t & 1) ? make_uint2((w0 >> 16) | (w1 & 0xffff0000u), (w2 >> 16) | (w3 & 0xffff0000u))
                                            : make_uint2((w0 & 0xffffu) | (w1 << 16), (w2 & 0xffffu) | (w3 << 16));
                    acc[t] = mfma_16x16x16<DT>(a_hi, b, acc[t]);
                    acc[t] = mfma_16x16x16<DT>(a_lo, b, acc[t]);
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int g = 4 * rg + r;
        if (g < G) {
#pragma unroll
            for (int t = 0; t < 8; ++t) sh.st_acc[wave][g][cl * 8 + t] = acc[t][r];
        }
    }
    lds_barrier();
    float *dst = ws.partial + ((size_t)s * ws.max_units + c) * G * kPartialStride;
    for (int idx = tid; idx < G * kHeadDim; idx += 256) {
        const int g = idx / kHeadDim, ch = idx % kHeadDim;
        dst[g * kPartialStride + 4 + ch] =
            (sh.st_acc[0][g][ch] + sh.st_acc[1][g][ch]) + (sh.st_acc[2][g][ch] + sh.st_acc[3][g][ch]);
        if (ch == 0) { dst[g * kPartialStride] = sh.Mref[g]; dst[g * kPartialStride + 1] = sh.lsum[g]; }
    }
}

// One workgroup per entry of the work list the selection kernel left; the grid is sized for the most
// there can be, and a workgroup beyond the list's end returns after one load.
template <int DT, int G, int CBMAX>
__global__ __launch_bounds__(256) void attend_kernel(KvView kv, DecodeWs ws, int CB) {
    __shared__ AttendShared<G, CBMAX> sh;
    if ((int)blockIdx.x >= ws.header[kValueCount]) return;
    const int item = ws.value_items[blockIdx.x];
    attend_unit<DT, G, CBMAX>(sh, kv, ws, CB, item / ws.max_chunks, item % ws.max_chunks);
}

constexpr int kUnitLanes = 16;   // value units merged side by side by one workgroup

// =================================================================================================
// grid (S*G), 512 threads = 16 unit lanes x 32 channel quads; unit lane j takes units j, j+16, ...
// in ascending order, and the 16 lanes are then added in a fixed order.
__global__ __launch_bounds__(512) void finalize_kernel(KvView kv, DecodeWs ws, int G, int VU,
                                                       float *__restrict__ out,
                                                       int32_t *__restrict__ n_selected,
                                                       float *__restrict__ mass_est,
                                                       int32_t *__restrict__ blocks_read,
                                                       float *__restrict__ lse_out,
                                                       int32_t *__restrict__ traffic_out) {
    __shared__ float red[512];
    __shared__ float wgt[kMaxBlocks / 4];        // per-unit rescale factor (value units are >= 4 blocks)
    __shared__ __attribute__((aligned(16))) float num_part[kUnitLanes][kHeadDim];
    const int s = blockIdx.x / G, g = blockIdx.x % G, tid = threadIdx.x;
    const int cq = tid & 31, uj = tid >> 5;
    const int r = s / kv.num_kv_heads, h = s % kv.num_kv_heads;
    int ctx = kv.ctx_lens[r];
    ctx = ctx < 0 ? 0 : (ctx > kv.max_blocks * kPage ? kv.max_blocks * kPage : ctx);
    const int N = (ctx + kPage - 1) / kPage;
    const StreamCtl *ctl = &ws.ctl[s];
    const unsigned long long st = ctl->stop[g];
    int n = N;
    float P = N > 0 ? 1.0f : 0.0f;
    if (st != ~0ull && (int)(st >> 32) <= N) { n = (int)(st >> 32); P = __uint_as_float((uint32_t)st); }
    const int nun = (n + VU - 1) / VU;
    const float *src = ws.partial + ((size_t)s * ws.max_units * G + g) * kPartialStride;
    const size_t stride = (size_t)G * kPartialStride;

    // reference maximum over the units
    float M = -INFINITY;
    for (int i = tid; i < nun; i += 512) { const float mi = src[i * stride]; wgt[i] = mi; M = fmaxf(M, mi); }
    red[tid] = M;
    __syncthreads();
    for (int d = 256; d >= 1; d >>= 1) {
        if (tid < d) red[tid] = fmaxf(red[tid], red[tid + d]);
        __syncthreads();
    }
    M = red[0];
    __syncthreads();
    // per-unit weights and the denominator
    float den = 0.0f;
    for (int i = tid; i < nun; i += 512) {
        const float mi = wgt[i];
        const float w = (mi == -INFINITY || M == -INFINITY) ? 0.0f : exp2_fast(mi - M);
        wgt[i] = w;
        den += src[i * stride + 1] * w;
    }
    red[tid] = den;
    __syncthreads();
    for (int d = 256; d >= 1; d >>= 1) {
        if (tid < d) red[tid] += red[tid + d];
        __syncthreads();
    }
    den = red[0];
    // numerator: channels 4*cq .. 4*cq+3, units uj, uj+16, ...; four loads in flight per thread
    float4 num = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (int i0 = uj; i0 < nun; i0 += 4 * kUnitLanes) {
        float4 a[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int i = i0 + k * kUnitLanes;
            a[k] = (i < nun) ? *reinterpret_cast<const float4 *>(src + i * stride + 4 + 4 * cq)
                             : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int i = i0 + k * kUnitLanes;
            const float w = (i < nun) ? wgt[i] : 0.0f;
            num.x = fmaf(a[k].x, w, num.x); num.y = fmaf(a[k].y, w, num.y);
            num.z = fmaf(a[k].z, w, num.z); num.w = fmaf(a[k].w, w, num.w);
        }
    }
    *reinterpret_cast<float4 *>(&num_part[uj][4 * cq]) = num;
    __syncthreads();
    if (tid < kHeadDim) {
        float t = 0.0f;
#pragma unroll
        for (int j = 0; j < kUnitLanes; ++j) t += num_part[j][tid];
        const size_t qi = (size_t)r * kv.num_q_heads + h * G + g;
        out[qi * kHeadDim + tid] = den > 0.0f ? t / den : 0.0f;
        if (tid == 0) {
            n_selected[qi] = n;
            mass_est[qi] = P;
            if (lse_out) lse_out[qi] = den > 0.0f ? (M + log2_fast(den)) * kLn2 : -INFINITY;
            if (g == 0) {
                int mx = 0;
                for (int x = 0; x < G; ++x) {
                    const unsigned long long sx = ctl->stop[x];
                    const int nx = (sx != ~0ull && (int)(sx >> 32) <= N) ? (int)(sx >> 32) : N;
                    mx = max(mx, nx);
                }
                if (blocks_read) blocks_read[s] = mx;
                if (traffic_out) { traffic_out[2 * s] = ctl->k_blocks; traffic_out[2 * s + 1] = mx; }
            }
        }
    }
}

template <int DT, int G>
static hipError_t launch_attend_t(const KvView &kv, const DecodeWs &ws, const DecodePlan &plan, hipStream_t st) {
    const unsigned grid = (unsigned)(kv.batch * kv.num_kv_heads) * (unsigned)plan.max_chunks;
    if (plan.chunk_blocks <= 32)
        attend_kernel<DT, G, 32><<<grid, 256, 0, st>>>(kv, ws, plan.chunk_blocks);
    else
        attend_kernel<DT, G, kMaxChunkBlocks><<<grid, 256, 0, st>>>(kv, ws, plan.chunk_blocks);
    return hipGetLastError();
}

hipError_t launch_attend(const KvView &kv, int dtype, int G, const DecodeWs &ws, const DecodePlan &plan,
                         hipStream_t st) {
#define PSA_CASE(DT, GG) \
    if (dtype == DT && G == GG) return launch_attend_t<DT, GG>(kv, ws, plan, st);
    PSA_CASE(0, 1) PSA_CASE(0, 2) PSA_CASE(0, 4) PSA_CASE(0, 8)
    PSA_CASE(1, 1) PSA_CASE(1, 2) PSA_CASE(1, 4) PSA_CASE(1, 8)
#undef PSA_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_finalize(const KvView &kv, const DecodeWs &ws, int G, int VU, float *out,
                           int32_t *n_selected, float *mass_est, int32_t *blocks_read, float *lse_out,
                           int32_t *traffic_out, hipStream_t st) {
    finalize_kernel<<<kv.batch * kv.num_kv_heads * G, 512, 0, st>>>(kv, ws, G, VU, out, n_selected, mass_est,
                                                                    blocks_read, lse_out, traffic_out);
    return hipGetLastError();
}

}  // namespace psa
