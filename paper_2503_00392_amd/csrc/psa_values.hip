// Value pass and final merge of one PSA decode step (Algorithm 1, lines 10-12 and 19).
//
// By the time these kernels run, the selection kernel has fixed every query head's stop n_g and
// left the exact scaled logits of the ranked blocks in the workspace.  What remains is plain
// attention over each head's own prefix: softmax numerators from the stored logits, times the value
// slices of the selected blocks -- every workgroup independent, no waiting, and only blocks
// actually selected are read.
//   attend_kernel    per value unit (chunk, stream) on the work list the selection kernel wrote:
//                    p = exp(logit - reference), partial numerator sum_t p_t v_t per head (on the
//                    matrix cores, the weights as a sum of two 16-bit halves) and exp-sum
//   finalize_kernel  merges a head's chunks (the online-softmax merge of line 11, all at once):
//                    out_g = sum over the chunks of the head's own prefix of the partial numerators,
//                    over the sum of the partial exp-sums, both rescaled to one reference maximum
#include "psa_attend.h"
#include "psa_host.h"

namespace psa {

// Stop of head g of a stream: (n, P_acc) as the selection kernel left it, n = N when it never stopped.
__device__ __forceinline__ int head_stop(const StreamCtl *ctl, int g, int N) {
    const unsigned long long st = ctl->stop[g];
    return (st != ~0ull && (int)(st >> 32) <= N) ? (int)(st >> 32) : N;
}

// =================================================================================================
// One workgroup per entry of the work list the selection kernel left (value unit = chunk c of stream s);
// the grid is sized for the most there can be, and a workgroup beyond the list's end returns after one
// load.  256 threads.  The four waves stream independently: wave w takes blocks w, w+4, ... of the unit,
// two value slices (8 KiB) in flight at a time, and nothing is shared until the final merge.
//   weights   p = exp(logit - L), L = per head the largest log-sum-exp of a block the head uses (the selection
//             kernel left one per block): a reference every wave knows beforehand, so nothing is rescaled
//             on the way and the four waves' sums simply add up.  (p <= 1, and the largest weight is at least
//             1/16: the weights keep their precision as 16-bit halves.)
//   numerator D[head][channel] += P[head][token] V[token][channel]: eight 16x16x16 products per block (one
//             per channel of the lane's eight) with the weights split into hi + lo 16-bit halves.  The k
//             index of both operands is the token: lane (rg, *) holds the value rows rg, 4+rg, 8+rg, 12+rg
//             -- the rows its four loads fetched -- and the selection kernel stored the logits so that the
//             16 bytes at [block][head][4 rg] are those same four tokens: one load, no transposition.
//             A: row = head lane%16 (zero beyond G).  D: lane (rg, cl) gets heads 4rg..4rg+3 of channels
//             8cl..8cl+7.
// Output per unit and head: (L, sum of p, numerator[128]) for the final merge.
// =================================================================================================
constexpr int kValueDepth = 2;      // value slices a wave keeps in flight
template <int DT, int G>
__global__ __launch_bounds__(256, 4) void attend_kernel(KvView kv, DecodeWs ws, int CB) {
    __shared__ float st_acc[4][G][kHeadDim];
    __shared__ float st_l[4][G];
    __shared__ float st_ref[G];
    if ((int)blockIdx.x >= ws.header[kValueCount]) return;
    const int item = ws.value_items[blockIdx.x];
    const int s = item / ws.max_chunks, c = item % ws.max_chunks;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, rg = lane >> 4, cl = lane & 15;
    const int h = s % kv.num_kv_heads;
    int ctx = kv.ctx_lens[s / kv.num_kv_heads];
    ctx = ctx < 0 ? 0 : (ctx > kv.max_blocks * kPage ? kv.max_blocks * kPage : ctx);
    const int N = (ctx + kPage - 1) / kPage;
    const int start = c * CB;
    if (start >= N) return;
    const int nblk = min(CB, N - start);
    const StreamCtl *ctl = &ws.ctl[s];
    // blocks of this chunk each head uses: those before its stop
    int maxcnt = 0, mycnt = 0;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int cg = min(nblk, max(0, head_stop(ctl, g, N) - start));
        maxcnt = max(maxcnt, cg);
        if (g == cl) mycnt = cg;
    }
    if (maxcnt == 0) return;    // no head of the group reaches this chunk
    const size_t row0 = (size_t)s * kv.max_blocks + start;
    // the wave's blocks are wave, wave + 4, ...: lane j fetches the page and the logical index of the j-th
    const int jmax = (maxcnt - wave + 3) / 4;           // how many of them there are (may be <= 0)
    int pg = 0, od = 0;
    if (lane < jmax) {
        pg = ws.ranked_page[row0 + wave + 4 * lane];
        if (!(kv.slot_pool != nullptr && pg < 0)) pg = clamp_page_quiet(pg, kv.num_pages);   // (a page of the pool, or ~slot)
        od = ws.order[row0 + wave + 4 * lane];
    }
    // Reference exponent per head: the largest block log-sum-exp among the blocks the head uses (log2 units; the
    // selection kernel left one per block and head).  Lane = (block, head) pairs, 64 / G blocks per load, then a
    // butterfly over the lanes of a head: every lane l ends with the reference of head l % G, so lane (rg, cl < G)
    // holds head cl's.  Every wave computes the same bits.
    float Lc = -INFINITY;
    {
        const float *bl = ws.block_lse + row0 * G;
        const int g = lane % G;
        int cg = 0;
#pragma unroll
        for (int x = 0; x < G; ++x) cg = (x == g) ? min(nblk, max(0, head_stop(ctl, x, N) - start)) : cg;
        for (int i = lane / G; i < maxcnt; i += 64 / G) {
            const float v = bl[(size_t)i * G + g];
            if (i < cg) Lc = fmaxf(Lc, v);
        }
#pragma unroll
        for (int d = G; d < 64; d <<= 1) Lc = fmaxf(Lc, __shfl_xor(Lc, d));
    }
    const float *lg = ws.logits + row0 * (kPage * G) + (size_t)(cl < G ? cl : 0) * kPage + 4 * rg;

    f32x4_t acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
    float l = 0.0f;
    for (int j0 = 0; j0 < jmax; j0 += kValueDepth) {
        Slice v[kValueDepth];
        f32x4_t x[kValueDepth];
        int valid[kValueDepth], blk[kValueDepth];
#pragma unroll
        for (int u = 0; u < kValueDepth; ++u) {    // (index clamped, loads made anyway: no branch around a load)
            const int j = min(j0 + u, jmax - 1);
            blk[u] = wave + 4 * j;
            v[u] = load_slice(value_slice(kv, __shfl(pg, j), h), lane);
            x[u] = load_stream(lg + (size_t)blk[u] * (kPage * G));
            valid[u] = min(kPage, ctx - __shfl(od, j) * kPage);
        }
#pragma unroll
        for (int u = 0; u < kValueDepth; ++u) {
            if (j0 + u < jmax) {
                if (kv.staging != nullptr) {               // (second tier: see stage_key_slice)
                    const int loc = __shfl(pg, j0 + u);
                    if (loc >= 0) stage_value_slice(kv, loc, h, v[u].r, lane);
                }
                if (valid[u] < kPage) zero_invalid_rows(v[u], rg, valid[u]);
                // tokens beyond `valid` hold -inf logits; blocks beyond the head's stop, and heads beyond the
                // group, weigh nothing
                const bool on = cl < G && blk[u] < mycnt;
                float pw[4] = {x[u][0], x[u][1], x[u][2], x[u][3]};
                uint32_t hi[4], lo[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    pw[j] = on ? exp2_fast(pw[j] - Lc) : 0.0f;      // (a head that uses no block of the unit is never `on`)
                    split16<DT>(pw[j], hi[j], lo[j]);
                }
                l += (pw[0] + pw[1]) + (pw[2] + pw[3]);
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
    // the exp-sum over the four row groups, then the four waves through LDS (one reference: plain sums)
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int g = 4 * rg + r;
        if (g < G) {
#pragma unroll
            for (int t = 0; t < 8; ++t) st_acc[wave][g][cl * 8 + t] = acc[t][r];
        }
    }
    if (rg == 0 && cl < G) st_l[wave][cl] = l;
    if (wave == 0 && rg == 0 && cl < G) st_ref[cl] = Lc;
    __syncthreads();
    float *dst = ws.partial + ((size_t)s * ws.max_units + c) * G * kPartialStride;
    for (int idx = tid; idx < G * kHeadDim; idx += 256) {
        const int g = idx / kHeadDim, ch = idx % kHeadDim;
        dst[g * kPartialStride + 4 + ch] =
            (st_acc[0][g][ch] + st_acc[1][g][ch]) + (st_acc[2][g][ch] + st_acc[3][g][ch]);
        if (ch == 0) {
            dst[g * kPartialStride] = st_ref[g];
            dst[g * kPartialStride + 1] = (st_l[0][g] + st_l[1][g]) + (st_l[2][g] + st_l[3][g]);
        }
    }
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
    __shared__ float red[8];
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
    // (over the wave with lane exchanges, over the eight waves through LDS: two barriers instead of ten)
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) M = fmaxf(M, __shfl_xor(M, d));
    if ((tid & 63) == 0) red[tid >> 6] = M;
    __syncthreads();
    M = fmaxf(fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])), fmaxf(fmaxf(red[4], red[5]), fmaxf(red[6], red[7])));
    __syncthreads();
    // per-unit weights and the denominator
    float den = 0.0f;
    for (int i = tid; i < nun; i += 512) {
        const float mi = wgt[i];
        const float w = (mi == -INFINITY || M == -INFINITY) ? 0.0f : exp2_fast(mi - M);
        wgt[i] = w;
        den += src[i * stride + 1] * w;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) den += __shfl_xor(den, d);          // (a fixed tree: reproducible)
    if ((tid & 63) == 0) red[tid >> 6] = den;
    __syncthreads();
    den = ((red[0] + red[1]) + (red[2] + red[3])) + ((red[4] + red[5]) + (red[6] + red[7]));
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
    attend_kernel<DT, G><<<grid, 256, 0, st>>>(kv, ws, plan.chunk_blocks);
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
