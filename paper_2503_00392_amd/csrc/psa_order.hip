// Ranking of a stream's blocks (Algorithm 1, line 6): criticality score descending, ties to the
// smaller logical block.  One workgroup per stream, everything in LDS and registers.
//
// Main path: a monotone bucket map + exact in-bucket ranking.
//   1. every thread holds 8 keys (order-preserving 32-bit images of the scores, inverted so that a
//      smaller key is a larger score) and the workgroup reduces their minimum and maximum;
//   2. bucket(key) = floor((key - min) * scale) is monotone in the key, so bucket order is key
//      order; an LDS counter per bucket and a workgroup scan give each bucket its output range;
//   3. an element's final rank is its bucket's base plus the number of elements of the same bucket
//      that precede it under (key, index) -- counted exactly, so the result does not depend on the
//      order in which the LDS atomics arrived.
// Buckets hold 8 elements on average.  If one bucket holds more than kBucketLimit elements
// (near-identical scores) the quadratic in-bucket count would be slow, and the workgroup falls back
// to a bitonic network over 64-bit (key, index) words: compare distances below 8 stay in registers,
// below 512 go through wave shuffles, the rest through LDS.  Both paths give the same total order.
//
// The kernel also resets the stream's control block and chunk words for the progressive kernel and
// reports out-of-range contexts and block-table entries.
// grid (S), Np/8 threads, Np*8 bytes of dynamic LDS; Np = power of two >= max(512, max_blocks).
#include <limits.h>

#include "psa_host.h"

namespace psa {

constexpr int kBucketLimit = 192;

__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long v, int mask) {
    const int lo = __shfl_xor((int)(v & 0xffffffffull), mask);
    const int hi = __shfl_xor((int)(v >> 32), mask);
    return ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo;
}

// Smaller key = larger score; -0 ranks as +0.
__device__ __forceinline__ uint32_t descending_key(float score) {
    uint32_t u = __float_as_uint(score);
    if (u == 0x80000000u) u = 0u;
    const uint32_t asc = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ~asc;
}

__device__ void bitonic_sort(unsigned long long (&e)[8], unsigned long long *lds_keys, int Np, int tid,
                             int nthreads) {
    for (int k = 2; k <= Np; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            if (j >= 8) {
                const int tj = j >> 3;   // partner thread distance
                unsigned long long o[8];
                if (tj >= 64) {
#pragma unroll
                    for (int x = 0; x < 8; ++x) lds_keys[x * nthreads + tid] = e[x];
                    __syncthreads();
#pragma unroll
                    for (int x = 0; x < 8; ++x) o[x] = lds_keys[x * nthreads + (tid ^ tj)];
                    __syncthreads();
                } else {
#pragma unroll
                    for (int x = 0; x < 8; ++x) o[x] = shfl_xor_u64(e[x], tj);
                }
                const bool up = ((tid * 8) & k) == 0;        // ascending region of this merge
                const bool lower = (tid & tj) == 0;
                const bool keep_min = (lower == up);
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    const unsigned long long lo = e[x] < o[x] ? e[x] : o[x];
                    const unsigned long long hi = e[x] < o[x] ? o[x] : e[x];
                    e[x] = keep_min ? lo : hi;
                }
            } else {
                // partner inside the thread's own 8 keys
#define PSA_CE(A, B)                                                              \
    {                                                                             \
        const bool up = ((tid * 8 + (A)) & k) == 0;                               \
        const bool sw = (e[A] > e[B]) == up;                                      \
        const unsigned long long t0 = sw ? e[B] : e[A], t1 = sw ? e[A] : e[B];    \
        e[A] = t0;                                                                \
        e[B] = t1;                                                                \
    }
                if (j == 4) {
                    PSA_CE(0, 4) PSA_CE(1, 5) PSA_CE(2, 6) PSA_CE(3, 7)
                } else if (j == 2) {
                    PSA_CE(0, 2) PSA_CE(1, 3) PSA_CE(4, 6) PSA_CE(5, 7)
                } else {
                    PSA_CE(0, 1) PSA_CE(2, 3) PSA_CE(4, 5) PSA_CE(6, 7)
                }
#undef PSA_CE
            }
        }
    }
}

__global__ __launch_bounds__(1024) void order_kernel(KvView kv, DecodeWs ws, int G, int KU, int Np,
                                                      int force_bitonic,
                                                      int32_t *__restrict__ order_out) {
    extern __shared__ unsigned long long lds_raw[];
    const int s = blockIdx.x, r = s / kv.num_kv_heads;
    const int tid = threadIdx.x, nthreads = blockDim.x, lane = tid & 63, wave = tid >> 6;
    const int nwaves = nthreads >> 6;
    // the scoring kernel clamps silently (it clears the error word); out-of-range inputs are reported here
    const int ctx = (tid == 0) ? ctx_clamped(kv, r, ws.header) : ctx_clamped_quiet(kv, r);
    const int N = (ctx + kPage - 1) / kPage;

    // ---- reset of the progressive kernel's per-stream state ------------------------------------
    if (tid == 0) {
        StreamCtl *c = &ws.ctl[s];
        const unsigned nch = (unsigned)((N + KU - 1) / KU);
        c->k_next = 0; c->v_next = 0; c->k_blocks = 0; c->attached = 0;
        c->key_progress = (unsigned long long)nch << 32;                                  // frontier 0
        c->value_progress = (unsigned long long)(N == 0 ? 0u : (unsigned)kUnknownTotal) << 32;   // nothing released
        for (int g = 0; g < 8; ++g) { c->Lacc[g] = -INFINITY; c->Lmin[g] = INFINITY; c->stop[g] = ~0ull; }
    }
    {
        unsigned long long *a = ws.agg + (size_t)s * ws.max_chunks * G;
        // chunk 0 starts out as the place where the fold waits: its publisher starts folding
        for (int i = tid; i < ws.max_chunks * G; i += nthreads) a[i] = (i == 0) ? kAggArmed : kAggSentinel;
    }

    // LDS carve-up of the bucket path (7*Np bytes + scratch in the last Np bytes)
    uint32_t *key_of = reinterpret_cast<uint32_t *>(lds_raw);                 // [Np] key by logical block
    uint16_t *slot = reinterpret_cast<uint16_t *>(key_of + Np);               // [Np] logical block by slot
    uint32_t *cnt = reinterpret_cast<uint32_t *>(slot + Np);                  // [NB]
    uint32_t *base = cnt + nthreads;                                          // [NB]
    uint32_t *scratch = base + nthreads;                                      // >= 64 words
    const int NB = nthreads;                                                  // one bucket per thread

    const float *sc = ws.scores + (size_t)s * kv.max_blocks;
    uint32_t key[8];
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int p = tid * 8 + j;
        key[j] = 0xFFFFFFFFu;
        if (p < N) {
            key[j] = descending_key(sc[p]);
            kmin = min(kmin, key[j]);
            kmax = max(kmax, key[j]);
        }
        key_of[p] = key[j];
    }
    cnt[tid] = 0;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, d));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, d));
    }
    if (lane == 0) { scratch[wave] = kmin; scratch[16 + wave] = kmax; }
    __syncthreads();
    kmin = 0xFFFFFFFFu; kmax = 0u;
    for (int w = 0; w < nwaves; ++w) { kmin = min(kmin, scratch[w]); kmax = max(kmax, scratch[16 + w]); }
    const float scale = (float)NB / ((float)(kmax - kmin) + 1.0f);

    int bkt[8], arrival[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        bkt[j] = 0; arrival[j] = 0;
        if (tid * 8 + j < N) {
            int b = (int)((float)(key[j] - kmin) * scale);
            b = b < 0 ? 0 : (b > NB - 1 ? NB - 1 : b);
            bkt[j] = b;
            arrival[j] = (int)atomicAdd(&cnt[b], 1u);
        }
    }
    __syncthreads();

    // exclusive scan of the bucket counts (bucket = thread) and the largest bucket
    const uint32_t mine = cnt[tid];
    uint32_t incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = (uint32_t)__shfl_up((int)incl, d);
        if (lane >= d) incl += o;
    }
    uint32_t biggest = mine;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) biggest = max(biggest, (uint32_t)__shfl_xor((int)biggest, d));
    if (lane == 63) scratch[32 + wave] = incl;
    if (lane == 0) scratch[48 + wave] = biggest;
    __syncthreads();
    uint32_t wave_off = 0, max_bucket = 0;
    for (int w = 0; w < nwaves; ++w) {
        if (w < wave) wave_off += scratch[32 + w];
        max_bucket = max(max_bucket, scratch[48 + w]);
    }
    base[tid] = wave_off + incl - mine;
    __syncthreads();

    const int32_t *table = kv.block_table + (size_t)r * kv.max_blocks;
    int32_t *ord = ws.order + (size_t)s * kv.max_blocks;
    int32_t *rpage = ws.ranked_page + (size_t)s * kv.max_blocks;
    int32_t *oout = order_out ? order_out + (size_t)s * kv.max_blocks : nullptr;

    if (max_bucket <= (uint32_t)kBucketLimit && !force_bitonic) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (tid * 8 + j < N) slot[base[bkt[j]] + arrival[j]] = (uint16_t)(tid * 8 + j);
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int p = tid * 8 + j;
            if (p < N) {
                const uint32_t b0 = base[bkt[j]], c = cnt[bkt[j]];
                uint32_t before = 0;
                for (uint32_t i = 0; i < c; ++i) {
                    const uint32_t other = slot[b0 + i];
                    const uint32_t ko = key_of[other];
                    before += (ko < key[j] || (ko == key[j] && other < (uint32_t)p)) ? 1u : 0u;
                }
                const uint32_t rank = b0 + before;
                ord[rank] = p;
                rpage[rank] = clamp_page(table[p], kv.num_pages, ws.header);
                if (oout) oout[rank] = p;
            }
        }
    } else {
        __syncthreads();   // everyone is done with the bucket arrays before LDS is reused
        unsigned long long e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int p = tid * 8 + j;
            e[j] = p < N ? (((unsigned long long)key[j] << 32) | (unsigned)p) : ~0ull;
        }
        bitonic_sort(e, lds_raw, Np, tid, nthreads);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int p = tid * 8 + j;
            if (p < N) {
                const int b = (int)(e[j] & 0xffffffffull);
                ord[p] = b;
                rpage[p] = clamp_page(table[b], kv.num_pages, ws.header);
                if (oout) oout[p] = b;
            }
        }
    }
    if (oout)
        for (int p = N + tid; p < kv.max_blocks; p += nthreads) oout[p] = -1;
}

hipError_t launch_order(const KvView &kv, const DecodeWs &ws, int G, int KU, int force_bitonic,
                        int32_t *order_out, hipStream_t st) {
    const int S = kv.batch * kv.num_kv_heads;
    int Np = 512;
    while (Np < kv.max_blocks) Np <<= 1;
    order_kernel<<<S, Np / 8, (size_t)Np * 8, st>>>(kv, ws, G, KU, Np, force_bitonic, order_out);
    return hipGetLastError();
}

}  // namespace psa
