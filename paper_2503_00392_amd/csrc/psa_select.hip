// Progressive selection (Algorithm 1, lines 7-18 without the value side): walks every stream's ranked
// blocks, computes the exact scaled logits q.k/sqrt(d) of each block from its key slice, keeps them
// for the value pass, and decides on the GPU where every query head stops.
//
// A "stream" is one (request, KV head) pair: one ranking, G query heads.  A "chunk" is `CB`
// consecutive ranked blocks of a stream, the unit of work of a workgroup.
//
// Work distribution: a persistent grid of workgroups.  Each stream hands out its chunks in order
// through an atomic ticket of its own, so whoever holds chunk c knows that every earlier chunk of
// that stream is held by a workgroup that is running or has finished: waiting on earlier chunks
// cannot deadlock, whatever the number of resident workgroups.  A workgroup stays with a stream
// while that stream has chunks to hand out inside its read-ahead window, and otherwise moves on,
// round-robin, to the next stream that has; it leaves when no stream has anything left.
// The window -- chunks handed out beyond the resolved ones -- is max(window_chunks, resolved/2),
// at most 64: it bounds the keys read beyond the stop to a fixed amount for streams that stop early
// and to a fraction of what was needed for streams that go deep.
//
// For one chunk, a workgroup (8 waves)
//   1. reads its blocks' key slices (each wave keeps 4 slices = 16 KiB in flight), computes the
//      scaled logits of all G heads as a 16-token x 16-head x 128-channel product on the matrix
//      cores (heads beyond G are zero columns), writes them to the workspace, and reduces each
//      block's log-sum-exp L_b (= log AS of line 10);
//   2. publishes the chunk's aggregate (log-sum-exp and minimum of its L_b) as one 64-bit word per
//      head, then reads the aggregates of all earlier chunks and folds them in a fixed order into
//      the exclusive prefix (AS_acc, AS_min of lines 12-13 at the chunk's first block);
//   3. scans its own blocks to get P_acc (lines 15-16) at every position it owns, finds the first
//      admissible position with P_acc > eps (line 17) per head and records it with a 64-bit
//      atomic minimum; the global minimum over chunks is the head's stop.
// Every wait is bounded by `spin_limit` polls; running out marks the stream finished, sets the
// sticky error bit and lets every workgroup leave.
//
// Every reduction has a fixed order, so results are bitwise reproducible although the scheduling
// is dynamic.
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

constexpr int kBatch = 4;            // key slices a wave keeps in flight
constexpr int kSelectThreads = 512;  // 8 waves: a 32-block chunk is one batch per wave


#ifdef PSA_ENABLE_TRACE
// One record per processed chunk: ids, then 100 MHz timestamps of begin / K done / resolved.
#define PSA_TRACE_EMIT(CNT)                                                                  \
    if (threadIdx.x == 0) {                                                                  \
        const unsigned long long slot_ = atomicAdd(ws.trace, 1ull);                          \
        if (slot_ < (unsigned long long)kTraceRecords) {                                     \
            unsigned long long *rec_ = ws.trace + 8 + slot_ * 8;                             \
            rec_[0] = ((unsigned long long)s << 32) | (unsigned)c;                           \
            rec_[1] = ((unsigned long long)blockIdx.x << 32) | (unsigned)(CNT);              \
            rec_[2] = t_begin; rec_[3] = t_kdone; rec_[4] = wall_clock64(); rec_[5] = rec_[4]; \
        }                                                                                    \
    }
#else
#define PSA_TRACE_EMIT(CNT)
#endif

template <int G>
struct SelectShared {
    float Lb[kMaxChunkBlocks][G];          // per-block log2-sum-exp2
    int page[kMaxChunkBlocks];
    int valid[kMaxChunkBlocks];
    int cnt[G];
    int stopped[G];
    int w_first[8];
    int w_busy[8];
    int chunk;
    int state;
    int abort_flag;
};

// Blocks of stream s's request, clamped like everywhere else.
__device__ __forceinline__ int stream_ctx(const KvView &kv, int s) {
    int ctx = kv.ctx_lens[s / kv.num_kv_heads];
    return ctx < 0 ? 0 : (ctx > kv.max_blocks * kPage ? kv.max_blocks * kPage : ctx);
}

// 0: stream s can hand out a chunk now; 1: it is at its read-ahead window; 2: nothing left to do.
// The window grows with the stream's progress: max(window, resolved/2), at most 64 chunks.
__device__ __forceinline__ int classify_stream(const KvView &kv, const DecodeWs &ws, int s, int CB,
                                               int window) {
    const int N = (stream_ctx(kv, s) + kPage - 1) / kPage;
    const int nch = (N + CB - 1) / CB;
    const StreamCtl *ctl = &ws.ctl[s];
    const int nx = ld_relaxed(&ctl->next_chunk);
    if (nx >= nch || nx > ld_relaxed(&ctl->done_chunk)) return 2;
    const int res = ld_relaxed(&ctl->resolved);
    int w = max(window, res >> 1);
    w = w > 64 ? 64 : w;
    if (nx >= res + w) return 1;
    return 0;
}

template <int DT, int G>
__device__ void process_chunk(SelectShared<G> &sh, const KvView &kv, const uint8_t *__restrict__ q,
                              const DecodeWs &ws, float eps, int m, int CB, int spin_limit, int s, int c) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = s / kv.num_kv_heads, h = s % kv.num_kv_heads;
    const int ctx = stream_ctx(kv, s);
    const int N = (ctx + kPage - 1) / kPage;
    const int start = c * CB;
    const int nblk = min(CB, N - start);
    StreamCtl *ctl = &ws.ctl[s];

    PSA_TRACE_STAMP(t_begin);
    if (tid == 0) sh.abort_flag = 0;
    for (int idx = tid; idx < kMaxChunkBlocks * G; idx += kSelectThreads) {   // blocks beyond nblk take no part
        const int i = idx / G, g = idx % G;
        if (i >= nblk) sh.Lb[i][g] = -INFINITY;
    }
    float *lg_out = ws.logits + ((size_t)s * kv.max_blocks + start) * (kPage * G);
    lds_barrier();
    // B operand of the QK^T product: column n = lane%16 is query head n (zero beyond the group),
    // k block kq = lane/16; for step kk the lane holds channels 8*(4*kk + kq) .. +7.
    const int n = lane & 15, kq = lane >> 4;
    uint4 qb[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        qb[kk] = make_uint4(0, 0, 0, 0);
        if (n < G)
            qb[kk] = ld16(q + ((size_t)(r * kv.num_q_heads + h * G + n) * kHeadDim + (4 * kk + kq) * 8) * 2);
    }

    // ---- 1. keys: wave w takes blocks [32*it + 4*w, +4).  A operand: row n = token n of the block,
    //         same channel assignment as the queries; 64 contiguous bytes per token and step. --------
    for (int i0 = wave * kBatch; i0 < nblk; i0 += (kSelectThreads / 64) * kBatch) {
        uint4 ka[kBatch][4];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            if (i0 + u < nblk) {
                const uint8_t *kp = kv.k_pool + ((size_t)sh.page[i0 + u] * kv.num_kv_heads + h) * kSliceBytes +
                                    n * kRowBytes + kq * 16;
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) ka[u][kk] = ld16(kp + kk * 64);
            }
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int i = i0 + u;
            if (i < nblk) {
                f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) acc = mfma_16x16x32<DT>(ka[u][kk], qb[kk], acc);
                // the lane now holds head n's logits of tokens 4*kq .. 4*kq+3
                const int valid = sh.valid[i];
                float sc[4];
#pragma unroll
                for (int x = 0; x < 4; ++x) sc[x] = (4 * kq + x < valid) ? acc[x] * kScaleLog2 : -INFINITY;
                if (n < G)
                    *reinterpret_cast<float4 *>(lg_out + ((size_t)i * G + n) * kPage + 4 * kq) =
                        make_float4(sc[0], sc[1], sc[2], sc[3]);
                // the block's log-sum-exp for head n, across the 4 token groups
                float mx = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                float sum = (exp2_fast(sc[0] - mx) + exp2_fast(sc[1] - mx)) +
                            (exp2_fast(sc[2] - mx) + exp2_fast(sc[3] - mx));
                sum += __shfl_xor(sum, 16);
                sum += __shfl_xor(sum, 32);
                if (lane < G) sh.Lb[i][lane] = mx + log2_fast(sum);
            }
        }
    }
    lds_barrier();
    PSA_TRACE_STAMP(t_kdone);

    // ---- 2 + 3. aggregate, prefix, stop rule: wave w serves head w ------------------------------
    for (int g = wave; g < G; g += kSelectThreads / 64) {
        // the head's best known stop so far; only a hint (it may be stale), requested early
        const unsigned long long known = ld_relaxed(&ctl->stop[g]);
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

        // exclusive prefix over chunks 0..c-1, folded in a fixed order: lane l folds chunks l, l+64, ...
        // in ascending order, then the lanes are combined by a butterfly.  Four aggregates per lane
        // are requested at once; one still missing is polled.
        float pL = -INFINITY, pMin = INFINITY;
        int bad = 0;
        for (int j0 = lane; j0 < c && !bad; j0 += 256) {
            unsigned long long v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                v[u] = (j0 + 64 * u < c) ? ld_relaxed(&agg[(size_t)(j0 + 64 * u) * G + g]) : 0ull;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = j0 + 64 * u;
                if (j < c && !bad) {
                    int spins = 0;
                    while (v[u] == kAggSentinel) {
                        ++spins;
                        if ((spins & 7) == 0 && ld_relaxed(&ctl->done_chunk) < c) { bad = 1; break; }
                        if (spins > spin_limit) { bad = 2; break; }
                        __builtin_amdgcn_s_sleep(16);
                        v[u] = ld_relaxed(&agg[(size_t)j * G + g]);
                    }
                    if (!bad) {
                        pL = lse2(pL, __uint_as_float((uint32_t)(v[u] & 0xffffffffull)));
                        pMin = fminf(pMin, __uint_as_float((uint32_t)(v[u] >> 32)));
                    }
                }
            }
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
        if ((known >> 32) <= (unsigned long long)start) { cnt = 0; stopped = 1; }
        if (lane == 0) { sh.cnt[g] = cnt; sh.stopped[g] = stopped; }
    }
    lds_barrier();
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
        }
    }
    PSA_TRACE_EMIT(maxcnt);
}

// Holder of ticket c waits here until the chunk is inside the stream's read-ahead window
// (1), or learns that the stream finished before it (0).  One thread polls, with a sleep.
__device__ int wait_for_window(const DecodeWs &ws, StreamCtl *ctl, int c, int window, int spin_limit) {
    int spins = 0;
    while (true) {
        if (ld_relaxed(&ctl->done_chunk) < c) return 0;
        const int res = ld_relaxed(&ctl->resolved);
        int w = max(window, res >> 1);
        w = w > 64 ? 64 : w;
        if (c < res + w) return 1;
        if (++spins > spin_limit) {
            set_error(ws.header, PSA_DEVERR_WAIT_EXPIRED);
            atomicMin(&ctl->done_chunk, -1);
            return 0;
        }
        __builtin_amdgcn_s_sleep(32);
    }
}

// Physical page and valid-token count of each ranked block of chunk c of stream s -> LDS.
template <int G>
__device__ __forceinline__ void stage_chunk_pages(SelectShared<G> &sh, const KvView &kv, const DecodeWs &ws,
                                                  int s, int c, int CB, int lane_in_group) {
    const int ctx = stream_ctx(kv, s);
    const int N = (ctx + kPage - 1) / kPage;
    const int start = c * CB, nblk = min(CB, N - start);
    const int i = lane_in_group;
    if (i < kMaxChunkBlocks) {
        int page = 0, valid = 0;
        if (i < nblk) {
            const size_t at = (size_t)s * kv.max_blocks + start + i;
            page = ws.ranked_page[at];
            valid = min(kPage, ctx - ws.order[at] * kPage);
        }
        sh.page[i] = page;
        sh.valid[i] = valid;
    }
}

// The persistent scheduler.  grid = two workgroups per CU; 512 threads.  A workgroup starts at its
// home stream (blockIdx % S) and keeps taking that stream's next chunk ticket; when a ticket shows
// that the stream has nothing left (past its last block, or past a chunk in which every head had
// stopped) it looks, round-robin, for the next stream that has work, preferring one whose window
// is open, and leaves when there is none.  The holder of a ticket beyond the stream's window waits
// for the window before it reads any key; the chunk's page numbers are fetched during that wait.
template <int DT, int G>
__global__ __launch_bounds__(kSelectThreads) void select_kernel(KvView kv, const uint8_t *__restrict__ q,
                                                                DecodeWs ws, float eps, int m, int CB,
                                                                int window, int spin_limit) {
    __shared__ SelectShared<G> sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int S = kv.batch * kv.num_kv_heads;
    int home = blockIdx.x % S;
    while (true) {
        // ---- next ticket of the home stream; wave 1 stages its pages while thread 0 waits --------
        StreamCtl *ctl = &ws.ctl[home];
        const int N = (stream_ctx(kv, home) + kPage - 1) / kPage;
        if (tid == 0) sh.chunk = atomicAdd(&ctl->next_chunk, 1);
        lds_barrier();
        const int c = sh.chunk;
        int go = 0;
        if (c * CB < N) {
            if (tid == 0) sh.state = wait_for_window(ws, ctl, c, window, spin_limit);
            if (wave == 1) stage_chunk_pages<G>(sh, kv, ws, home, c, CB, lane);
            lds_barrier();
            go = sh.state;
        }
        if (go) {
            process_chunk<DT, G>(sh, kv, q, ws, eps, m, CB, spin_limit, home, c);
            lds_barrier();
            continue;
        }
        lds_barrier();
        // ---- the home stream is finished: first stream in rotation order that has work -----------------
        int first_open = INT_MAX, first_busy = INT_MAX;
        for (int b0 = 0; b0 < S && first_open == INT_MAX; b0 += kSelectThreads) {
            int st = 2;
            if (b0 + tid < S) st = classify_stream(kv, ws, (home + b0 + tid) % S, CB, window);
            const unsigned long long open = __ballot(st == 0), busy = __ballot(st == 1);
            if (lane == 0) {
                sh.w_first[wave] = open ? b0 + wave * 64 + (__ffsll((long long)open) - 1) : INT_MAX;
                sh.w_busy[wave] = busy ? b0 + wave * 64 + (__ffsll((long long)busy) - 1) : INT_MAX;
            }
            lds_barrier();
#pragma unroll
            for (int w = 0; w < kSelectThreads / 64; ++w) {
                first_open = min(first_open, sh.w_first[w]);
                first_busy = min(first_busy, sh.w_busy[w]);
            }
            lds_barrier();
        }
        const int first = first_open != INT_MAX ? first_open : first_busy;
        if (first == INT_MAX) break;               // every stream is finished
        home = (home + first) % S;
    }
}

template <int DT, int G>
static hipError_t launch_select_t(const KvView &kv, const void *q, const DecodeWs &ws, float eps, int m,
                                  const DecodePlan &plan, hipStream_t st) {
    const unsigned items = (unsigned)(kv.batch * kv.num_kv_heads) * (unsigned)plan.max_chunks;
    const unsigned grid = items < (unsigned)plan.persistent_wgs ? items : (unsigned)plan.persistent_wgs;
    select_kernel<DT, G><<<grid, kSelectThreads, 0, st>>>(kv, (const uint8_t *)q, ws, eps, m, plan.chunk_blocks,
                                               plan.window_chunks, plan.spin_limit);
    return hipGetLastError();
}

hipError_t launch_select(const KvView &kv, int dtype, int G, const void *q, const DecodeWs &ws, float eps,
                         int m, const DecodePlan &plan, hipStream_t st) {
#define PSA_CASE(DT, GG) \
    if (dtype == DT && G == GG) return launch_select_t<DT, GG>(kv, q, ws, eps, m, plan, st);
    PSA_CASE(0, 1) PSA_CASE(0, 2) PSA_CASE(0, 4) PSA_CASE(0, 8)
    PSA_CASE(1, 1) PSA_CASE(1, 2) PSA_CASE(1, 4) PSA_CASE(1, 8)
#undef PSA_CASE
    return hipErrorInvalidValue;
}

}  // namespace psa
