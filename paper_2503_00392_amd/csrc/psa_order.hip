// Ranking of a stream's blocks (Algorithm 1, line 6): criticality score descending, ties to the
// smaller logical block.  One workgroup per stream, everything in LDS and registers.
//
// Main path: a monotone bucket map + exact in-bucket ranking.
//   1. every thread holds 8 keys (order-preserving 32-bit images of the scores, inverted so that a
//      smaller key is a larger score) and the workgroup reduces their minimum and maximum;
//   2. bucket = floor((largest score - score) * scale) is monotone in the score, so bucket order is
//      rank order; an LDS counter per bucket and a workgroup scan give each bucket its output range;
//   3. the elements are laid out bucket by bucket ("slots"); an element's final rank is its bucket's base
//      plus the number of elements of the same bucket that precede it under (key, index) -- counted
//      exactly, so the result does not depend on the order in which the LDS atomics arrived.  The
//      counting goes slot by slot, every thread of the workgroup taking its share, so that neighbouring
//      lanes look at the same bucket.
// There are as many buckets as element slots, so a bucket holds about one element.  If one bucket
// holds more than kBucketLimit elements
// (near-identical scores) the quadratic in-bucket count would be slow, and the workgroup falls back
// to a bitonic network over 64-bit (key, index) words: compare distances below 8 stay in registers,
// below 512 go through wave shuffles, the rest through LDS.  Both paths give the same total order.
//
// With few streams several workgroups share one stream: each builds the bucket table (cheap) and
// ranks its share of the elements (the expensive part, bound by LDS traffic).
//
// The kernel also resets the stream's control block and chunk words for the progressive kernel and
// reports out-of-range contexts and block-table entries.
// grid (S), Np/8 threads, 10*Np + 512 bytes of dynamic LDS; Np = power of two >= max(512, max_blocks).
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

// The score a key stands for (with -0 read as +0).
__device__ __forceinline__ float score_of_key(uint32_t key) {
    const uint32_t asc = ~key;
    return __uint_as_float((asc & 0x80000000u) ? (asc & 0x7FFFFFFFu) : ~asc);
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

__global__ __launch_bounds__(1024) void order_kernel(KvView kv, DecodeWs ws, int G, int KU, int budget_blocks, int Np,
                                                      int force_bitonic,
                                                      int32_t *__restrict__ order_out) {
    extern __shared__ unsigned long long lds_raw[];
    const int s = blockIdx.y, r = s / kv.num_kv_heads;
    const int part = blockIdx.x, nparts = gridDim.x;
    const int tid = threadIdx.x, nthreads = blockDim.x, lane = tid & 63, wave = tid >> 6;
    const int nwaves = nthreads >> 6;
    // what this thread needs from memory, requested before anything else: its 8 scores (two 16-byte loads
    // where the row's length allows)
    const float *sc = ws.scores + (size_t)s * kv.max_blocks;
    const int32_t *table = kv.block_table + (size_t)r * kv.max_blocks;
    float scv[8];
    if ((kv.max_blocks & 7) == 0 && kv.max_blocks >= 8) {
        const float4 *v4 = reinterpret_cast<const float4 *>(sc + min(tid * 8, kv.max_blocks - 8));   // (clamped: no branch)
        const float4 a = v4[0], b = v4[1];
        scv[0] = a.x; scv[1] = a.y; scv[2] = a.z; scv[3] = a.w; scv[4] = b.x; scv[5] = b.y; scv[6] = b.z; scv[7] = b.w;
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) scv[j] = sc[min(tid * 8 + j, max(kv.max_blocks - 1, 0))];
    }
    // the scoring kernel clamps silently (it clears the error word); out-of-range inputs are reported here
    const int ctx = (tid == 0 && blockIdx.x == 0) ? ctx_clamped(kv, r, ws.header) : ctx_clamped_quiet(kv, r);
    const int N = (ctx + kPage - 1) / kPage;
    // ---- reset of the progressive kernel's per-stream state ------------------------------------
    if (tid == 0 && part == 0) {
        StreamCtl *c = &ws.ctl[s];
        // key chunks that may ever be handed out: all of them, or those a fixed budget of blocks covers
        const int nlim = budget_blocks > 0 ? min(N, budget_blocks) : N;
        const unsigned nch = (unsigned)((nlim + KU - 1) / KU);
        c->k_blocks = 0;
        c->key_progress = (unsigned long long)nch << 32;                                  // frontier 0
        for (int g = 0; g < 8; ++g) c->stop[g] = ~0ull;
    }
    if (part == 0) {
        unsigned long long *a = ws.agg + (size_t)s * ws.max_chunks * G;
        for (int i = tid; i < ws.max_chunks * G; i += nthreads) a[i] = kAggSentinel;      // nothing published yet
    }

    // LDS carve-up of the bucket path: 10*Np bytes + scratch
    uint32_t *skey = reinterpret_cast<uint32_t *>(lds_raw);                   // [Np] key by slot
    uint32_t *cnt = skey + Np;                                                // [Np + 4] bucket counts, then bases
    uint16_t *slot = reinterpret_cast<uint16_t *>(cnt + Np + 4);              // [Np] logical block by slot
    uint32_t *scratch = reinterpret_cast<uint32_t *>(slot + Np);              // 64 words
    const int NB = Np;                                                        // one bucket per element slot

    uint32_t key[8];
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int p = tid * 8 + j;
        key[j] = 0xFFFFFFFFu;
        if (p < N) {
            key[j] = descending_key(scv[j]);
            kmin = min(kmin, key[j]);
            kmax = max(kmax, key[j]);
        }
    }
    *reinterpret_cast<uint4 *>(cnt + tid * 8) = make_uint4(0, 0, 0, 0);
    *reinterpret_cast<uint4 *>(cnt + tid * 8 + 4) = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, d));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, d));
    }
    if (lane == 0) { scratch[wave] = kmin; scratch[16 + wave] = kmax; }
    lds_barrier();
    kmin = 0xFFFFFFFFu; kmax = 0u;
    for (int w = 0; w < nwaves; ++w) { kmin = min(kmin, scratch[w]); kmax = max(kmax, scratch[16 + w]); }
    // Buckets are equal steps of the SCORE between the largest and the smallest one (not of its bit
    // pattern, which would crowd scores of small magnitude or mixed sign into a few buckets).  Every
    // operation below is monotone in the score, so a block that ranks before another never lands in a
    // later bucket; the exact order inside a bucket is settled by counting.
    const float smax = score_of_key(kmin), span = smax - score_of_key(kmax);
    const bool span_ok = span > 0.0f && span < INFINITY;       // false also for NaN: the fallback ranks then
    const float scale = span_ok ? (float)NB / span : 0.0f;
    int bkt[8], arrival[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        bkt[j] = 0; arrival[j] = 0;
        if (tid * 8 + j < N) {
            const float fb = (smax - score_of_key(key[j])) * scale;
            int b = fb >= (float)(NB - 1) ? NB - 1 : (int)fb;     // (a NaN compares false and converts to 0)
            b = b < 0 ? 0 : b;
            bkt[j] = b;
            arrival[j] = (int)atomicAdd(&cnt[b], 1u);
        }
    }
    lds_barrier();
    // exclusive scan of the bucket counts (8 buckets per thread) and the largest bucket
    uint32_t c8[8];
    {
        const uint4 a = *reinterpret_cast<const uint4 *>(cnt + tid * 8), b4 = *reinterpret_cast<const uint4 *>(cnt + tid * 8 + 4);
        c8[0] = a.x; c8[1] = a.y; c8[2] = a.z; c8[3] = a.w; c8[4] = b4.x; c8[5] = b4.y; c8[6] = b4.z; c8[7] = b4.w;
    }
    uint32_t mine = 0, biggest = 0, e8[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { e8[j] = mine; mine += c8[j]; biggest = max(biggest, c8[j]); }
    uint32_t incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = (uint32_t)__shfl_up((int)incl, d);
        if (lane >= d) incl += o;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) biggest = max(biggest, (uint32_t)__shfl_xor((int)biggest, d));
    if (lane == 63) scratch[32 + wave] = incl;
    if (lane == 0) scratch[48 + wave] = biggest;
    lds_barrier();
    uint32_t wave_off = 0, max_bucket = 0;
    for (int w = 0; w < nwaves; ++w) {
        if (w < wave) wave_off += scratch[32 + w];
        max_bucket = max(max_bucket, scratch[48 + w]);
    }
    // A workgroup's share of the ranking work is a run of whole buckets (the workgroups of a stream agree on the
    // buckets' ranges, not on the arrangement inside a bucket): share p starts with the first bucket that begins at
    // or after slot p * N / nparts.  Whoever holds the bucket that slot falls into notes where the next one begins.
    const int share = (N + nparts - 1) / nparts;
    if (tid < 8) scratch[64 + tid] = 0u;               // (share 0 starts at slot 0; nparts <= 4)
    {
        const uint32_t t0 = wave_off + incl - mine;
        *reinterpret_cast<uint4 *>(cnt + tid * 8) = make_uint4(t0 + e8[0], t0 + e8[1], t0 + e8[2], t0 + e8[3]);
        *reinterpret_cast<uint4 *>(cnt + tid * 8 + 4) = make_uint4(t0 + e8[4], t0 + e8[5], t0 + e8[6], t0 + e8[7]);
        if (tid == 0) cnt[NB] = (uint32_t)N;
    }
    lds_barrier();
    {
        const uint32_t t0 = wave_off + incl - mine;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t lo = t0 + e8[j], hi = lo + c8[j];          // bucket's slots [lo, hi)
            for (int p = 1; p < nparts; ++p) {
                const uint32_t target = (uint32_t)min(p * share, N);
                if (lo < target && target <= hi) scratch[64 + p] = hi;
            }
        }
    }
    lds_barrier();
    const uint32_t *base = cnt;                                               // base[b] .. base[b+1]: bucket b's slots

    int32_t *ord = ws.order + (size_t)s * kv.max_blocks;
    int32_t *rpage = ws.ranked_page + (size_t)s * kv.max_blocks;
    int32_t *oout = order_out ? order_out + (size_t)s * kv.max_blocks : nullptr;

    if (max_bucket <= (uint32_t)kBucketLimit && !force_bitonic) {
        // every workgroup of the stream builds the whole slot table: the elements of a bucket side by side, in
        // arrival order (which may differ between the workgroups; the exact count below does not depend on it) ...
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (tid * 8 + j < N) {
                const uint32_t at = base[bkt[j]] + arrival[j];
                slot[at] = (uint16_t)(tid * 8 + j);
                skey[at] = key[j];
            }
        }
        lds_barrier();
        // ... and ranks its own share of the SLOTS, all threads taking part: thread t takes slots first + t,
        // first + t + nthreads, ...  Neighbouring lanes hold neighbouring slots, that is the same bucket or the
        // next, so a wave's reads of the bucket's members are mostly the same addresses.  The final rank of a
        // slot's element is its bucket's base plus the number of the bucket's members that precede it under
        // (key, block index).
        const int first = (int)scratch[64 + part];
        const int last = part == nparts - 1 ? N : (int)scratch[64 + part + 1];
        const int mine = last - first;
        for (int q0 = 0; q0 < mine; q0 += 2 * nthreads) {         // two slots per thread and turn
            uint32_t mk[2], me[2], b0[2], cn[2], before[2], cmax = 0;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int q = q0 + tid + j * nthreads;
                mk[j] = 0; me[j] = 0; b0[j] = 0; cn[j] = 0; before[j] = 0;
                if (q < mine) {
                    mk[j] = skey[first + q];
                    me[j] = slot[first + q];
                    const float fb = (smax - score_of_key(mk[j])) * scale;     // the bucket, exactly as it was computed above
                    int b = fb >= (float)(NB - 1) ? NB - 1 : (int)fb;
                    b = b < 0 ? 0 : b;
                    b0[j] = base[b];
                    cn[j] = base[b + 1] - b0[j];
                    cmax = max(cmax, cn[j]);
                }
            }
            for (uint32_t i = 0; i < cmax; ++i) {
                uint32_t ko[2], so[2];
#pragma unroll
                for (int j = 0; j < 2; ++j) {              // reads past a bucket's end stay inside the table
                    const uint32_t at = min(b0[j] + i, (uint32_t)(Np - 1));
                    ko[j] = skey[at];
                    so[j] = slot[at];
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const bool precedes = ko[j] < mk[j] || (ko[j] == mk[j] && so[j] < me[j]);
                    before[j] += (i < cn[j] && precedes) ? 1u : 0u;
                }
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if (q0 + tid + j * nthreads < mine) {
                    const uint32_t rank = b0[j] + before[j];
                    ord[rank] = (int)me[j];
                    rpage[rank] = clamp_page(table[me[j]], kv.num_pages, ws.header);
                    if (oout) oout[rank] = (int)me[j];
                }
            }
        }
    } else if (part == 0) {     // (uniform over the workgroup) the fallback is one workgroup's work
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
    if (oout && part == 0)
        for (int p = N + tid; p < kv.max_blocks; p += nthreads) oout[p] = -1;
}

hipError_t launch_order(const KvView &kv, const DecodeWs &ws, int G, const DecodePlan &plan, int budget_blocks,
                        int32_t *order_out, hipStream_t st) {
    const int S = kv.batch * kv.num_kv_heads;
    int Np = 512;
    while (Np < kv.max_blocks) Np <<= 1;
    const size_t lds = (size_t)Np * 10 + 512;
    static bool raised = false;       // more than 64 KiB of dynamic LDS has to be asked for once
    if (!raised) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(order_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kMaxBlocks * 10 + 512) != hipSuccess)
            return hipErrorInvalidValue;
        raised = true;
    }
    // with few streams, up to 4 workgroups share a stream's ranking
    int parts = 256 / (S > 0 ? S : 1);
    parts = parts < 1 ? 1 : (parts > 4 ? 4 : parts);
    if (Np < 2048) parts = 1;
    order_kernel<<<dim3(parts, S), Np / 8, lds, st>>>(kv, ws, G, plan.chunk_blocks, budget_blocks, Np, plan.force_bitonic,
                                                      order_out);
    return hipGetLastError();
}

}  // namespace psa
