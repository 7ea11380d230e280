// One decode step of Progressive Sparse Attention (Algorithm 1 of the paper) as four kernels on one
// stream, with no host involvement between them:
//   score_kernel        criticality score of every block from its min/max metadata      (line 5)
//   order_kernel        per (request, KV head) ranking, a bitonic sort in registers/LDS  (line 6)
//   progressive_kernel  exact attention over the ranked blocks with the stop rule decided on the
//                       GPU                                                              (lines 7-18)
//   finalize_kernel     merges the per-chunk partial results of each head's own prefix   (line 19)
//
// A "stream" below is one (request, KV head) pair: one ranking, G query heads.
// A "chunk" is `CB` consecutive ranked blocks of a stream, the unit of work of a workgroup.
#include <limits.h>

#include "psa_attend.h"
#include "psa_host.h"

namespace psa {

__device__ __forceinline__ int ld_relaxed(const int32_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_relaxed(const unsigned long long *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_relaxed(unsigned long long *p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long pack2(float a, float b) {
    return ((unsigned long long)__float_as_uint(b) << 32) | __float_as_uint(a);
}

// =================================================================================================
// Scoring.  UB[g][b] = (1/sqrt d) sum_c max(q_c kmin_c, q_c kmax_c) = (1/sqrt d) (q+ . kmax + q- . kmin)
// with q+ = max(q,0), q- = min(q,0); CS[b] = max_g UB[g][b].
// grid (ceil(max_blocks/64), S), 256 threads.  A 16-lane row handles one block: lanes 0-7 take
// 32 bytes each of the min row against q-, lanes 8-15 of the max row against q+.
// =================================================================================================
template <int DT, int G>
__global__ __launch_bounds__(256) void score_kernel(KvView kv, const uint8_t *__restrict__ q,
                                                    const uint8_t *__restrict__ meta,
                                                    float *__restrict__ scores,
                                                    float *__restrict__ scores_out, int32_t *header) {
    const int s = blockIdx.y, r = s / kv.num_kv_heads, h = s % kv.num_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, row = lane >> 4, cl = lane & 15;
    const int is_max = cl >> 3, slot = cl & 7;
    const int ctx = ctx_clamped(kv, r, header);
    const int N = (ctx + kPage - 1) / kPage;
    const int base = blockIdx.x * 64 + wave * 16;
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
            qs[g][j] = w[j] & (is_max ? ~neg : neg);
        }
    }

    const int32_t *table = kv.block_table + (size_t)r * kv.max_blocks;
    uint4 ma[4], mb[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int b = base + it * 4 + row;
        if (b < N) {
            const int page = clamp_page(table[b], kv.num_pages, header);
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
            cs = fmaxf(cs, p * kScale);
        }
        if (cl == 0 && b < N) {
            scores[(size_t)s * kv.max_blocks + b] = cs;
            if (scores_out) scores_out[(size_t)s * kv.max_blocks + b] = cs;
        }
    }
}

// =================================================================================================
// Ranking.  One workgroup per stream sorts (score descending, logical block ascending) with a
// bitonic network over 64-bit keys: 8 keys per thread in registers; compare distances below 8 stay
// in registers, below 512 go through wave shuffles, the rest through LDS.  It also resets the
// stream's control block and the chunk aggregates for the progressive kernel.
// grid (S), Np/8 threads, Np*8 bytes of dynamic LDS; Np = power of two >= max(512, max_blocks).
// =================================================================================================
__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long v, int mask) {
    const int lo = __shfl_xor((int)(v & 0xffffffffull), mask);
    const int hi = __shfl_xor((int)(v >> 32), mask);
    return ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo;
}

__global__ __launch_bounds__(1024) void order_kernel(KvView kv, DecodeWs ws, int G, int Np,
                                                      int32_t *__restrict__ order_out) {
    extern __shared__ unsigned long long lds_keys[];
    const int s = blockIdx.x, r = s / kv.num_kv_heads;
    const int tid = threadIdx.x, nthreads = blockDim.x;
    int ctx = kv.ctx_lens[r];
    ctx = ctx < 0 ? 0 : (ctx > kv.max_blocks * kPage ? kv.max_blocks * kPage : ctx);
    const int N = (ctx + kPage - 1) / kPage;

    if (tid == 0) {
        StreamCtl *c = &ws.ctl[s];
        c->done_chunk = INT_MAX; c->resolved = 0; c->k_blocks = 0; c->v_blocks = 0;
        for (int g = 0; g < 8; ++g) c->stop[g] = ~0ull;
        if (s == 0) ws.header[0] = 0;
    }
    {
        unsigned long long *a = ws.agg + (size_t)s * ws.max_chunks * G;
        for (int i = tid; i < ws.max_chunks * G; i += nthreads) a[i] = kAggSentinel;
    }

    const float *sc = ws.scores + (size_t)s * kv.max_blocks;
    unsigned long long e[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int p = tid * 8 + j;
        if (p < N) {
            uint32_t u = __float_as_uint(sc[p]);
            if (u == 0x80000000u) u = 0u;                                     // -0 ranks as +0
            const uint32_t asc = (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // numeric order as unsigned
            e[j] = ((unsigned long long)(~asc) << 32) | (unsigned)p;          // descending score, then index
        } else {
            e[j] = ~0ull;
        }
    }

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

    const int32_t *table = kv.block_table + (size_t)r * kv.max_blocks;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int p = tid * 8 + j;
        if (p < N) {
            const int b = (int)(e[j] & 0xffffffffull);
            ws.order[(size_t)s * kv.max_blocks + p] = b;
            ws.ranked_page[(size_t)s * kv.max_blocks + p] = clamp_page(table[b], kv.num_pages, ws.header);
            if (order_out) order_out[(size_t)s * kv.max_blocks + p] = b;
        } else if (p < kv.max_blocks && order_out) {
            order_out[(size_t)s * kv.max_blocks + p] = -1;
        }
    }
}

// =================================================================================================
// Progressive attention.
//
// Work items are (chunk c, stream s) pairs handed out in chunk-major order by an atomic ticket, so
// that whenever a workgroup holds an item, every earlier chunk of the same stream is held by a
// workgroup that is already running or has finished: waiting on earlier chunks cannot deadlock.
//
// A workgroup (4 waves)
//   1. waits until chunk c is within `window` chunks of the stream's resolved chunks (bounds how
//      far K is read ahead of the stop), or leaves if the stream is known to be finished;
//   2. K phase: reads its blocks' key slices, computes the scaled logits of all G heads into LDS,
//      and each block's log-sum-exp L_b (= log AS of line 10) and maximum;
//   3. publishes the chunk's aggregate (log-sum-exp and minimum of its L_b) as one 64-bit word per
//      head, then reads the aggregates of all earlier chunks and folds them in a fixed order into
//      the exclusive prefix (AS_acc, AS_min of lines 12-13 at the chunk's first block);
//   4. scans its own blocks to get P_acc (lines 15-16) at every position it owns, finds the first
//      admissible position with P_acc > eps (line 17) per head and records it with a 64-bit
//      atomic minimum; the global minimum over chunks is the head's stop;
//   5. V phase: reads the value slices of the blocks before the stop only, and writes the chunk's
//      partial numerator, reference maximum and exp-sum per head.
// Every wait is bounded by `spin_limit` polls; running out marks the stream finished, sets the
// sticky error bit and lets every workgroup leave.
// =================================================================================================
template <int G>
struct ProgShared {
    float lg[kMaxChunkBlocks][kPage][G];   // logits, later softmax numerators p
    float Lb[kMaxChunkBlocks][G];          // per-block log2-sum-exp2
    float mb[kMaxChunkBlocks][G];          // per-block maximum logit
    float st_acc[4][G][kHeadDim];          // per-wave partial numerators
    int page[kMaxChunkBlocks];
    int valid[kMaxChunkBlocks];
    int cnt[G];
    int stopped[G];
    float Mref[G];
    float lsum[G];
    int ticket;
    int go;
    int abort_flag;
};

template <int DT, int G>
__global__ __launch_bounds__(256) void progressive_kernel(KvView kv, const uint8_t *__restrict__ q,
                                                          DecodeWs ws, float eps, int m, int CB,
                                                          int window, int spin_limit) {
    __shared__ ProgShared<G> sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, rg = lane >> 4, cl = lane & 15;
    if (tid == 0) { sh.ticket = atomicAdd(&ws.header[0], 1); sh.abort_flag = 0; }
    __syncthreads();
    const int S = kv.batch * kv.num_kv_heads;
    const int c = sh.ticket / S, s = sh.ticket % S;
    const int r = s / kv.num_kv_heads, h = s % kv.num_kv_heads;
    int ctx = kv.ctx_lens[r];
    ctx = ctx < 0 ? 0 : (ctx > kv.max_blocks * kPage ? kv.max_blocks * kPage : ctx);
    const int N = (ctx + kPage - 1) / kPage;
    const int start = c * CB;
    if (start >= N) return;
    const int nblk = min(CB, N - start);
    StreamCtl *ctl = &ws.ctl[s];

    // ---- 1. window wait --------------------------------------------------------------------------
    if (tid == 0) {
        int go = 1, spins = 0;
        while (true) {
            if (ld_relaxed(&ctl->done_chunk) < c) { go = 0; break; }
            if (c < ld_relaxed(&ctl->resolved) + window) break;
            if (++spins > spin_limit) {
                set_error(ws.header, PSA_DEVERR_WAIT_EXPIRED);
                atomicMin(&ctl->done_chunk, -1);
                go = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(16);
        }
        sh.go = go;
    }
    if (tid < kMaxChunkBlocks) {
        if (tid < nblk) {
            const size_t at = (size_t)s * kv.max_blocks + start + tid;
            const int lb = ws.order[at];
            sh.page[tid] = ws.ranked_page[at];
            sh.valid[tid] = min(kPage, ctx - lb * kPage);
        }
    }
    const QueryRegs<G> qr = load_query<G>(q, r, h, kv.num_q_heads, cl);
    __syncthreads();
    if (!sh.go) return;

    // ---- 2. K phase ------------------------------------------------------------------------------
    for (int i = wave; i < nblk; i += 4) {
        const size_t off = ((size_t)sh.page[i] * kv.num_kv_heads + h) * kSliceBytes;
        const Slice k = load_slice(kv.k_pool + off, lane);
        float sc[4][G];
        slice_logits<DT, G>(k, qr, rg, sh.valid[i], sc);
        if (cl == 0) {
#pragma unroll
            for (int x = 0; x < 4; ++x)
#pragma unroll
                for (int g = 0; g < G; ++g) sh.lg[i][4 * x + rg][g] = sc[x][g];
        }
    }
    __syncthreads();
    for (int idx = tid; idx < kMaxChunkBlocks * G; idx += 256) {
        const int i = idx / G, g = idx % G;
        float mx = -INFINITY, L = -INFINITY;
        if (i < nblk) {
#pragma unroll
            for (int t = 0; t < kPage; ++t) mx = fmaxf(mx, sh.lg[i][t][g]);
            float sum = 0.0f;
#pragma unroll
            for (int t = 0; t < kPage; ++t) sum += exp2_fast(sh.lg[i][t][g] - mx);
            L = mx + log2_fast(sum);
        }
        sh.Lb[i][g] = L;
        sh.mb[i][g] = mx;
    }
    __syncthreads();

    // ---- 3 + 4. aggregate, prefix, stop rule: wave w serves heads w, w+4 ------------------------------
    for (int g = wave; g < G; g += 4) {
        const float L = sh.Lb[lane][g];                       // -inf beyond nblk
        float accL = L, mn = (lane < nblk) ? L : INFINITY;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const float oL = __shfl_up(accL, d), om = __shfl_up(mn, d);
            if (lane >= d) { accL = lse2(accL, oL); mn = fminf(mn, om); }
        }
        const float Lagg = __shfl(accL, 63), Mnagg = __shfl(mn, 63);
        unsigned long long *agg = ws.agg + (size_t)s * ws.max_chunks * G;
        if (lane == 0) st_relaxed(&agg[(size_t)c * G + g], pack2(Lagg, Mnagg));

        // exclusive prefix over chunks 0..c-1, folded in a fixed order
        float pL = -INFINITY, pMin = INFINITY;
        int bad = 0;
        for (int j = lane; j < c; j += 64) {
            unsigned long long v;
            int spins = 0;
            while (true) {
                v = ld_relaxed(&agg[(size_t)j * G + g]);
                if (v != kAggSentinel) break;
                ++spins;
                if ((spins & 7) == 0 && ld_relaxed(&ctl->done_chunk) < c) { bad = 1; break; }
                if (spins > spin_limit) { bad = 2; break; }
                __builtin_amdgcn_s_sleep(4);
            }
            if (bad) break;
            pL = lse2(pL, __uint_as_float((uint32_t)(v & 0xffffffffull)));
            pMin = fminf(pMin, __uint_as_float((uint32_t)(v >> 32)));
        }
        const int any_bad = __any(bad != 0);
        if (__any(bad == 2)) {
            if (lane == 0) { set_error(ws.header, PSA_DEVERR_WAIT_EXPIRED); atomicMin(&ctl->done_chunk, -1); }
        }
        if (any_bad) { if (lane == 0) sh.abort_flag = 1; break; }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            pL = lse2(pL, __shfl_xor(pL, d));
            pMin = fminf(pMin, __shfl_xor(pMin, d));
        }

        // P_acc at position n = start + lane + 1 (after this lane's block)
        const float Lacc_n = lse2(pL, accL), Lmin_n = fminf(pMin, mn);
        const int n = start + lane + 1;
        const float P = 1.0f / (1.0f + (float)(N - n) * exp2_fast(Lmin_n - Lacc_n));
        const bool adm = (lane < nblk) && ((n % m) == 0 || n == N);
        const unsigned long long hits = __ballot(adm && (P > eps));
        // position n = start is also this chunk's to test when it is admissible
        int ls = -1;
        float Ps = 0.0f;
        if (c > 0 && (start % m) == 0) {
            const float P0 = 1.0f / (1.0f + (float)(N - start) * exp2_fast(pMin - pL));
            if (P0 > eps) { ls = start; Ps = P0; }
        }
        if (ls < 0 && hits) {
            const int f = __ffsll((long long)hits) - 1;
            ls = start + f + 1;
            Ps = __shfl(P, f);
        }
        int cnt = nblk, stopped = 0;
        if (ls >= 0) {
            cnt = ls - start;
            stopped = 1;
            if (lane == 0) atomicMin(&ctl->stop[g], ((unsigned long long)ls << 32) | __float_as_uint(Ps));
        }
        const unsigned long long cur = ld_relaxed(&ctl->stop[g]);
        if ((cur >> 32) <= (unsigned long long)start) { cnt = 0; stopped = 1; }
        if (lane == 0) { sh.cnt[g] = cnt; sh.stopped[g] = stopped; }
    }
    __syncthreads();
    if (sh.abort_flag) return;
    int maxcnt = 0;
    {
        int all = 1;
#pragma unroll
        for (int g = 0; g < G; ++g) { maxcnt = max(maxcnt, sh.cnt[g]); all &= sh.stopped[g]; }
        if (tid == 0) {
            if (all) atomicMin(&ctl->done_chunk, c);
            atomicAdd(&ctl->resolved, 1);
            atomicAdd(&ctl->k_blocks, nblk);
            if (maxcnt > 0) atomicAdd(&ctl->v_blocks, maxcnt);
        }
    }
    if (maxcnt == 0) return;

    // ---- 5. V phase ------------------------------------------------------------------------------
    if (tid < G) {
        const int g = tid, cg = sh.cnt[g];
        float M = -INFINITY;
        for (int i = 0; i < cg; ++i) M = fmaxf(M, sh.mb[i][g]);
        float lsum = 0.0f;
        for (int i = 0; i < cg; ++i) lsum += exp2_fast(sh.Lb[i][g] - M);
        sh.Mref[g] = M;
        sh.lsum[g] = lsum;
    }
    __syncthreads();
    for (int idx = tid; idx < maxcnt * kPage * G; idx += 256) {
        const int g = idx % G, i = idx / (kPage * G);
        float *p = &sh.lg[0][0][0] + idx;
        *p = (i < sh.cnt[g]) ? exp2_fast(*p - sh.Mref[g]) : 0.0f;
    }
    __syncthreads();

    float acc[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int x = 0; x < 8; ++x) acc[g][x] = 0.0f;
    for (int i = wave; i < maxcnt; i += 4) {
        const size_t off = ((size_t)sh.page[i] * kv.num_kv_heads + h) * kSliceBytes;
        Slice v = load_slice(kv.v_pool + off, lane);
        if (sh.valid[i] < kPage) zero_invalid_rows(v, rg, sh.valid[i]);
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            float vf[8];
            vf[0] = cvt_lo<DT>(v.r[x].x); vf[1] = cvt_hi<DT>(v.r[x].x);
            vf[2] = cvt_lo<DT>(v.r[x].y); vf[3] = cvt_hi<DT>(v.r[x].y);
            vf[4] = cvt_lo<DT>(v.r[x].z); vf[5] = cvt_hi<DT>(v.r[x].z);
            vf[6] = cvt_lo<DT>(v.r[x].w); vf[7] = cvt_hi<DT>(v.r[x].w);
            const float *pp = sh.lg[i][4 * x + rg];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float p = pp[g];
#pragma unroll
                for (int y = 0; y < 8; ++y) acc[g][y] = fmaf(p, vf[y], acc[g][y]);
            }
        }
    }
    // sum the 4 row groups of the wave, then the 4 waves
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            float a = acc[g][x];
            a += __shfl_xor(a, 16);
            a += __shfl_xor(a, 32);
            acc[g][x] = a;
        }
    if (rg == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int x = 0; x < 8; ++x) sh.st_acc[wave][g][cl * 8 + x] = acc[g][x];
    }
    __syncthreads();
    float *dst = ws.partial + ((size_t)s * ws.max_chunks + c) * G * kPartialStride;
    for (int idx = tid; idx < G * kHeadDim; idx += 256) {
        const int g = idx / kHeadDim, ch = idx % kHeadDim;
        dst[g * kPartialStride + 4 + ch] =
            (sh.st_acc[0][g][ch] + sh.st_acc[1][g][ch]) + (sh.st_acc[2][g][ch] + sh.st_acc[3][g][ch]);
        if (ch == 0) { dst[g * kPartialStride] = sh.Mref[g]; dst[g * kPartialStride + 1] = sh.lsum[g]; }
    }
}

// =================================================================================================
// Finalize: out_g = sum over the chunks of the head's own prefix of the partial numerators, over
// the sum of the partial exp-sums, both rescaled to one reference.  grid (S*G), 128 threads.
// =================================================================================================
__global__ __launch_bounds__(128) void finalize_kernel(KvView kv, DecodeWs ws, int G, int CB,
                                                       float *__restrict__ out,
                                                       int32_t *__restrict__ n_selected,
                                                       float *__restrict__ mass_est,
                                                       int32_t *__restrict__ blocks_read,
                                                       int32_t *__restrict__ traffic_out) {
    __shared__ float red[128];
    const int s = blockIdx.x / G, g = blockIdx.x % G, ch = threadIdx.x;
    const int r = s / kv.num_kv_heads, h = s % kv.num_kv_heads;
    int ctx = kv.ctx_lens[r];
    ctx = ctx < 0 ? 0 : (ctx > kv.max_blocks * kPage ? kv.max_blocks * kPage : ctx);
    const int N = (ctx + kPage - 1) / kPage;
    const StreamCtl *ctl = &ws.ctl[s];
    const unsigned long long st = ctl->stop[g];
    int n = N;
    float P = N > 0 ? 1.0f : 0.0f;
    if (st != ~0ull && (int)(st >> 32) <= N) { n = (int)(st >> 32); P = __uint_as_float((uint32_t)st); }
    const int nch = (n + CB - 1) / CB;
    const float *src = ws.partial + ((size_t)s * ws.max_chunks * G + g) * kPartialStride;
    const size_t stride = (size_t)G * kPartialStride;

    float M = -INFINITY;
    for (int i = ch; i < nch; i += 128) M = fmaxf(M, src[i * stride]);
    red[ch] = M;
    __syncthreads();
    for (int d = 64; d >= 1; d >>= 1) {
        if (ch < d) red[ch] = fmaxf(red[ch], red[ch + d]);
        __syncthreads();
    }
    M = red[0];
    float num = 0.0f, den = 0.0f;
    if (M != -INFINITY) {
        for (int i = 0; i < nch; ++i) {
            const float mi = src[i * stride];
            if (mi == -INFINITY) continue;
            const float w = exp2_fast(mi - M);
            den += src[i * stride + 1] * w;
            num += src[i * stride + 4 + ch] * w;
        }
    }
    const size_t qi = (size_t)r * kv.num_q_heads + h * G + g;
    out[qi * kHeadDim + ch] = den > 0.0f ? num / den : 0.0f;
    if (ch == 0) {
        n_selected[qi] = n;
        mass_est[qi] = P;
        if (g == 0) {
            int mx = 0;
            for (int x = 0; x < G; ++x) {
                const unsigned long long sx = ctl->stop[x];
                const int nx = (sx != ~0ull && (int)(sx >> 32) <= N) ? (int)(sx >> 32) : N;
                mx = max(mx, nx);
            }
            if (blocks_read) blocks_read[s] = mx;
            if (traffic_out) { traffic_out[2 * s] = ctl->k_blocks; traffic_out[2 * s + 1] = ctl->v_blocks; }
        }
    }
}

// ---- host side -------------------------------------------------------------------------------------
static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

DecodePlan make_plan(const psa_kv_desc *d, const psa_tuning *t) {
    DecodePlan p;
    const int S = d->batch * d->num_kv_heads;
    p.chunk_blocks = (t && t->chunk_blocks) ? t->chunk_blocks : 32;
    if (p.chunk_blocks < 8) p.chunk_blocks = 8;
    if (p.chunk_blocks > kMaxChunkBlocks) p.chunk_blocks = kMaxChunkBlocks;
    if (t && t->window_chunks > 0) {
        p.window_chunks = t->window_chunks;
    } else {
        // enough chunks in flight over all streams to cover the chip (~1024 workgroups), per stream
        int w = (1024 + S - 1) / (S > 0 ? S : 1);
        p.window_chunks = w < 2 ? 2 : (w > 16 ? 16 : w);
    }
    p.spin_limit = (t && t->spin_limit > 0) ? t->spin_limit : (1 << 22);
    p.max_chunks = (d->max_blocks_per_seq + p.chunk_blocks - 1) / p.chunk_blocks;
    if (p.max_chunks < 1) p.max_chunks = 1;
    return p;
}

struct WsLayout {
    size_t header, ctl, scores, order, ranked_page, agg, partial, total;
};

static WsLayout layout(const psa_kv_desc *d, const DecodePlan &p) {
    const size_t S = (size_t)d->batch * d->num_kv_heads;
    const size_t G = (size_t)(d->num_q_heads / d->num_kv_heads);
    const size_t MB = (size_t)d->max_blocks_per_seq;
    WsLayout L;
    size_t at = 0;
    L.header = at;      at = align_up(at + 256, 256);
    L.ctl = at;         at = align_up(at + S * sizeof(StreamCtl), 256);
    L.scores = at;      at = align_up(at + S * MB * 4, 256);
    L.order = at;       at = align_up(at + S * MB * 4, 256);
    L.ranked_page = at; at = align_up(at + S * MB * 4, 256);
    L.agg = at;         at = align_up(at + S * p.max_chunks * G * 8, 256);
    L.partial = at;     at = align_up(at + S * p.max_chunks * G * kPartialStride * 4, 256);
    L.total = at;
    return L;
}

size_t decode_workspace_bytes_plan(const psa_kv_desc *d, const DecodePlan &p) { return layout(d, p).total; }

template <int DT, int G>
static hipError_t launch_decode_t(const psa_kv_desc *d, const KvView &kv, const DecodeArgs &a,
                                  const DecodePlan &plan, const DecodeWs &ws, hipStream_t st) {
    const int S = kv.batch * kv.num_kv_heads;
    clear_words_kernel<<<1, 64, 0, st>>>(ws.header, 64);
    score_kernel<DT, G><<<dim3((kv.max_blocks + 63) / 64, S), 256, 0, st>>>(
        kv, (const uint8_t *)a.q, (const uint8_t *)a.meta, ws.scores, a.scores_out, ws.header);
    int Np = 512;
    while (Np < kv.max_blocks) Np <<= 1;
    order_kernel<<<S, Np / 8, (size_t)Np * 8, st>>>(kv, ws, G, Np, a.order_out);
    const unsigned items = (unsigned)S * (unsigned)plan.max_chunks;
    progressive_kernel<DT, G><<<items, 256, 0, st>>>(kv, (const uint8_t *)a.q, ws, a.threshold,
                                                     a.check_granularity, plan.chunk_blocks,
                                                     plan.window_chunks, plan.spin_limit);
    finalize_kernel<<<S * G, 128, 0, st>>>(kv, ws, G, plan.chunk_blocks, a.out, a.n_selected, a.mass_est,
                                           a.blocks_read, a.traffic_out);
    return hipGetLastError();
}

hipError_t launch_decode(const psa_kv_desc *d, const DecodeArgs &a, const DecodePlan &plan, void *wsp,
                         hipStream_t st) {
    const KvView kv = make_view(d);
    const WsLayout L = layout(d, plan);
    uint8_t *base = static_cast<uint8_t *>(wsp);
    DecodeWs ws;
    ws.header = reinterpret_cast<int32_t *>(base + L.header);
    ws.ctl = reinterpret_cast<StreamCtl *>(base + L.ctl);
    ws.scores = reinterpret_cast<float *>(base + L.scores);
    ws.order = reinterpret_cast<int32_t *>(base + L.order);
    ws.ranked_page = reinterpret_cast<int32_t *>(base + L.ranked_page);
    ws.agg = reinterpret_cast<unsigned long long *>(base + L.agg);
    ws.partial = reinterpret_cast<float *>(base + L.partial);
    ws.max_chunks = plan.max_chunks;
    const int G = d->num_q_heads / d->num_kv_heads;
    if (kv.batch == 0) return hipSuccess;
#define PSA_CASE(DT, GG) \
    if (d->dtype == DT && G == GG) return launch_decode_t<DT, GG>(d, kv, a, plan, ws, st);
    PSA_CASE(0, 1) PSA_CASE(0, 2) PSA_CASE(0, 4) PSA_CASE(0, 8)
    PSA_CASE(1, 1) PSA_CASE(1, 2) PSA_CASE(1, 4) PSA_CASE(1, 8)
#undef PSA_CASE
    return hipErrorInvalidValue;
}

}  // namespace psa
