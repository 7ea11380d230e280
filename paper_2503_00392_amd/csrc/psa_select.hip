// Progressive selection (Algorithm 1, lines 7-18 without the value side): walks every stream's ranked
// blocks, computes the exact scaled logits q.k/sqrt(d) of each block from its key slice, keeps them
// for the value pass, and decides on the GPU where every query head stops.
//
// Terms.  "Stream": one (request, KV head) pair -- one ranking, G query heads.  "Chunk": CB
// consecutive ranked blocks, the unit of work of a workgroup.
//
// One workgroup (4 waves) per (chunk, stream), in a one-dimensional grid with the streams varying
// fastest: the hardware hands workgroups out in that order, so each stream's chunks start in rank
// order, interleaved over the streams, and a compute unit takes the next one the moment a slot is free
// (four fit).  A workgroup
//   1. returns at once if its chunk lies beyond the stream's blocks or beyond the limit the fold has set
//      (the stream is closed, or cannot go that far any more);
//   2. fetches the chunk's page numbers and waits (napping about a microsecond between looks at one
//      progress word, a bounded number of times) until the chunk is inside the read-ahead window --
//      chunks read beyond the fold's frontier are at most max(window, frontier/4), 256 at most, which
//      bounds the keys read beyond the stop -- or the limit falls below it (with a second tier, a
//      chunk that has slices in host memory waits until the fold is one chunk away, unless it lies
//      inside the depth hint: the host link is too slow to read ahead over it);
//   3. reads the chunk's key slices (each wave keeps 4 slices = 16 KiB in flight, loaded as coalesced
//      1 KiB rows and turned into the matrix-operand layout through a patch of LDS), computes the
//      scaled logits of all G heads as a 16-token x 16-head x 128-channel product on the matrix
//      cores (heads beyond G are zero columns), stores them for the value pass, and reduces each
//      block's log-sum-exp L_b (= log AS of line 10);
//   4. publishes the chunk's (log-sum-exp, minimum) of L_b per head as one 64-bit word per head.
// The wait of step 2 is a courtesy, not a dependency: no chunk workgroup needs anything to proceed
// (when the looks run out it simply reads its chunk), so the grid drains whatever order it runs in.
// THE FOLD applies lines 12-17 strictly in rank order: AS_acc, AS_min, N_left and P_acc at the end
// of each published chunk after the frontier and, in the first chunk where P_acc exceeds the
// threshold, with a prefix scan over the chunk's blocks to find the head's exact stop.  One wave per
// stream does it, in workgroups of its own at the head of the grid (so they start first): it looks at the
// words of the next chunks, folds what is published, moves the frontier, tells the readers how far the
// stream can still go (stop_bound), and looks again.  Once every head has stopped (or the blocks ran
// out) it closes the stream -- the chunks beyond what it used are never read -- and puts the stream's
// value units on the work list of the value pass.
//
// Communication between workgroups: every shared word is read and written with relaxed agent-scope
// atomics (coherent accesses); a writer waits for its data stores to complete before it stores the
// word that announces them (the chunk words, the progress word), and a reader looks at the announcing
// word before it issues the loads that depend on it.  Accesses to one cache line are served one at a
// time (tens of nanoseconds each), which is why one thread per workgroup touches the stream's control
// block.  The logits are plain stores: their reader is the next kernel.
//
// The fold is one scan in rank order and every reduction has a fixed shape, so results are bitwise
// reproducible although the scheduling is dynamic.
#include <limits.h>

#include "psa_host.h"

namespace psa {

// ---- agent-scope atomics ---------------------------------------------------------------------
__device__ __forceinline__ int ld_relaxed(const int32_t *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_relaxed(const unsigned long long *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_relaxed(const float *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_relaxed(int32_t *p, int v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_relaxed(unsigned long long *p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_relaxed(float *p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Every word one wave writes and another reads inside this kernel travels through the relaxed
// agent-scope atomics above (cache-coherent accesses), never through plain loads and stores, so no
// cache write-back or invalidation is ever needed.  What remains is ORDER: a wave's earlier
// stores must have completed before the store that announces them is issued.
__device__ __forceinline__ void stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ unsigned long long pack2(float a, float b) {
    return ((unsigned long long)__float_as_uint(b) << 32) | __float_as_uint(a);
}
__device__ __forceinline__ unsigned long long shfl_u64(unsigned long long v, int src) {
    const int lo = __shfl((int)(v & 0xffffffffull), src);
    const int hi = __shfl((int)(v >> 32), src);
    return ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo;
}
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }


constexpr int kBatch = 4;            // key slices a wave keeps in flight
constexpr int kSelectThreads = 256;  // 4 waves; four such workgroups fit a CU (register budget)

// Tokens of stream s's request, clamped like everywhere else.
__device__ __forceinline__ int stream_ctx(const KvView &kv, int s) {
    const int ctx = kv.ctx_lens[s / kv.num_kv_heads];
    return ctx < 0 ? 0 : (ctx > kv.max_blocks * kPage ? kv.max_blocks * kPage : ctx);
}

__device__ __forceinline__ int window_of(int window, int frontier) {
    const int w = max(window, frontier >> 2);
    return w > kMaxWindowChunks ? kMaxWindowChunks : w;
}

// P_acc of Algorithm 1 lines 15-16 in the log2 domain: AS_acc / (AS_acc + AS_min * N_left).
__device__ __forceinline__ float p_acc(float Lacc, float Lmin, int n_left) {
    return 1.0f / (1.0f + (float)n_left * exp2_fast(Lmin - Lacc));
}

__device__ __forceinline__ void nap(int tries) {
    // about half a microsecond, then about one: long enough that the pollers of one stream stay below
    // what one cache line serves, short enough that an opening window is noticed at once
    __builtin_amdgcn_s_sleep(20);
    if (tries > 1) __builtin_amdgcn_s_sleep(20);
}

constexpr int kStagedBlocks = 32;     // chunks of up to this many blocks keep their logits in LDS until they are done

template <int G, bool STAGE>
struct SelectShared {
    uint4 qb[4][64];                       // B operand of the QK^T product of the workgroup's stream, by lane
    float Lb[kMaxChunkBlocks][G];          // per-block log2-sum-exp2
    int page[kMaxChunkBlocks];
    int valid[kMaxChunkBlocks];
    int go;                                // after the wait for the window: 1 = read the chunk, 0 = the stream closed
    unsigned long long kp0;                // the stream's progress word as the workgroup first saw it
    uint4 stage[kSelectThreads / 64][16 * 17];   // per wave: one key slice, rows padded to 272 bytes
    // the chunk's logits in the layout of the workspace, written out as one piece (STAGE only)
    __attribute__((aligned(16))) float lg[STAGE ? kStagedBlocks : 1][G][kPage];
};

// How far a stream can still go, in chunks, given what the fold knows after n blocks.  AS_acc only grows and
// AS_min only shrinks as more blocks are folded, so for any n* >= n
//     P_acc(n*) >= AS_acc(n) / (AS_acc(n) + AS_min(n) (N - n*)),
// and the right-hand side exceeds eps as soon as N - n* < (AS_acc(n) / AS_min(n)) (1 - eps) / eps: the head stops at
// the first tested position from there on, whatever the blocks in between hold.  Lane g < G carries head g
// (a stopped head needs its stop, lanes >= G nothing); the result, the largest need of the group plus one chunk
// to spare against rounding, is the same in every lane.  Keys beyond it are never worth reading.
template <int G>
__device__ __forceinline__ int stop_bound(float Lacc, float Lmin, unsigned long long stop, int n, int N, int m, int KU,
                                          float odds) {
    const int lane = threadIdx.x & 63;
    int need = 0;
    if (lane < G) {
        if (stop != ~0ull) {
            need = (int)(stop >> 32);
        } else {
            // blocks that may be left over when the test first passes: fewer than ratio * odds (taken a little
            // low, and one lower still: the bound must hold in binary32)
            const float room = exp2_fast(Lacc - Lmin) * odds * 0.999f - 1.0f;
            int nstar = room >= (float)N ? 0 : N - (int)fmaxf(room, 0.0f);     // (NaN compares false: N, no bound)
            nstar = max(nstar, n + 1);
            nstar = (int)min((long long)N, ((long long)nstar + m - 1) / m * m);   // the next tested position
            need = nstar;
        }
    }
#pragma unroll
    for (int d = 1; d < 8; d <<= 1) need = max(need, __shfl_xor(need, d));
    need = uniform(__shfl(need, 0));
    return (need + KU - 1) / KU + 1;
}

// The progress word of a stream that is still open (see StreamCtl).
__device__ __forceinline__ unsigned long long progress_word(int lim, int grant, int walked) {
    return ((unsigned long long)(unsigned)lim << 32) | ((unsigned)grant << 16) | (unsigned)walked;
}
// The read-ahead window of a stream when `closed` of the S streams have finished: the launch's total of chunks in
// flight (window per stream x S) shared by the streams still open.
__device__ __forceinline__ int granted(int window, int S, int closed) {
    return min(kMaxWindowChunks, (int)(((long long)window * S) / max(1, S - closed)));
}

// =================================================================================================
// The fold (Algorithm 1 lines 12-18 in rank order): one wave per stream, from the kernel's first moment until
// the stream closes.
//
// Chunks are folded a GROUP at a time: 64 / G consecutive chunks, aligned, lane = (chunk of the group, head).  One
// load fetches the group's words; a prefix scan over the chunks (steps of G lanes) gives every head's AS_acc and
// AS_min after every chunk of the group at once -- combined with the state carried into the group -- hence P_acc at
// every chunk's end.  The chunks in which an open head passes the threshold are then visited in order (there are at
// most G stops per stream) for the head's exact stop, with a second prefix scan over that chunk's blocks.  A
// sequential walk, chunk by chunk on G lanes, cost a deep stream 0.3 us per chunk -- more than reading the chunk
// costs the rest of the machine.
// The expression that gives the state after a chunk is fixed by the chunk's place in its group (the scan's tree over
// the group's earlier chunks, then the carry), whatever part of the group was published when the wave looked: the
// fold is reproducible bit for bit although its timing is not.
//
// The wave waits for nothing but chunks whose workgroups are in this kernel's grid and never wait for anything
// themselves beyond a bounded number of looks, so it always ends; a count of looks bounds it all the same
// (kFoldPatience: about half a second), after which the stream is closed as it stands and PSA_DEVERR_STALLED is
// raised.  With more streams than folding waves (4 * kMaxFoldGroups) a wave folds several streams, one after
// the other.
// =================================================================================================
constexpr int kFoldPatience = 1 << 19;
constexpr int kMaxFoldGroups = 128;            // workgroups of four folding waves at most: they must leave the
                                               // compute units room for the chunks they wait for

template <int G>
__device__ void fold_stream(const KvView &kv, const DecodeWs &ws, int s, float eps, int m, int KU, int budget,
                            int window) {
    constexpr int CPG = 64 / G;                // chunks per group
    const int lane = threadIdx.x & 63, g = lane % G, jl = lane / G;     // my head, my chunk of the group
    StreamCtl *ctl = &ws.ctl[s];
    const int ctx = stream_ctx(kv, s);
    const int N = (ctx + kPage - 1) / kPage;
    const unsigned long long *agg = ws.agg + (size_t)s * ws.max_chunks * G;
    // chunks that may ever be folded: all of them, or those a fixed budget of blocks covers (the limit in the
    // progress word is for the readers of keys and may be tighter: see stop_bound)
    const int nch = ((budget > 0 ? min(N, budget) : N) + KU - 1) / KU;
    if (nch == 0) {                            // an empty request: the ranking kernel left it closed
        if (lane == 0) atomicAdd(&ws.header[kClosedStreams], 1);
        return;
    }
    const int S = kv.batch * kv.num_kv_heads;
    const float odds = eps > 0.0f ? (1.0f - eps) / eps : INFINITY;      // (1 - eps) / eps of the stop test
    const unsigned long long head_lanes = (~0ull / ((1ull << G) - 1ull)) << g;   // the lanes of my head
    float Cacc = -INFINITY, Cmin = INFINITY;   // my head's (L_acc, L_min) at the start of the group
    unsigned long long stop = ~0ull;           // my head's stop (n << 32 | P_acc bits), ~0 = still open
    int base = 0, walked = 0;                  // the group's first chunk; chunks folded so far
    int closed = 0, lim_now = nch;             // streams seen closed at the last look; the limit last published
    int looks = 0;
    bool finished = false;
    while (!finished) {
        // the group's words, and (in flight at the same time) how many streams have closed
        const int ci = base + jl;
        const unsigned long long v = (ci < nch) ? ld_relaxed(&agg[(size_t)ci * G + g]) : kAggSentinel;
        const int closed_now = uniform(ld_relaxed(&ws.header[kClosedStreams]));
        const unsigned long long pub = __ballot(v != kAggSentinel);
        const int k = ((pub == ~0ull) ? 64 : (__ffsll((long long)~pub) - 1)) / G;     // leading published chunks
        if (base + k <= walked) {
            // Nothing new.  While the wait lasts, tell the readers if other streams have closed meanwhile, which
            // widens this one's window.
            if (++looks > kFoldPatience) {
                if (lane == 0) set_error(ws.header, PSA_DEVERR_STALLED);
                break;
            }
            if (closed_now != closed && walked > 0) {
                closed = closed_now;
                if (lane == 0) st_relaxed(&ctl->key_progress, progress_word(lim_now, granted(window, S, closed), walked));
            }
            __builtin_amdgcn_s_sleep(8);
            continue;
        }
        closed = closed_now;
        // (L_acc, L_min) of my head after my chunk: scan over the group's chunks, then the carry
        float L = __uint_as_float((uint32_t)(v & 0xffffffffull)), M = __uint_as_float((uint32_t)(v >> 32));
#pragma unroll
        for (int d = G; d < 64; d <<= 1) {
            const float ol = __shfl_up(L, d), om = __shfl_up(M, d);
            if (lane >= d) { L = lse2(ol, L); M = fminf(om, M); }
        }
        L = lse2(Cacc, L);
        M = fminf(Cmin, M);
        const int b0 = ci * KU, n_end = min(b0 + KU, N);
        // a stop inside a chunk needs a position where the rule is tested (line 17 is reached every m blocks and
        // at the last block) and, P_acc being non-decreasing, a pass at the chunk's end
        const bool passes = ((n_end / m) * m > b0 || n_end == N) && p_acc(L, M, N - n_end) > eps;
        int j = walked - base;                 // the next chunk of the group to fold
        while (j < k) {
            const unsigned long long cand = __ballot(jl >= j && jl < k && stop == ~0ull && passes);
            if (cand == 0ull) { j = k; break; }
            const int js = (__ffsll((long long)cand) - 1) / G;          // the first chunk in which an open head passes
            const bool scan = (cand >> (js * G + g)) & 1ull;            // does mine?
            {
                // That chunk's blocks' L_b are fetched 64 at a time, lane = (block, head); a prefix scan over the
                // blocks of each head (steps of G lanes), on top of the state after the chunk before, gives AS_acc
                // and AS_min after every block, hence P_acc at every position; the first tested position that
                // passes is the stop.
                const int cb0 = (base + js) * KU, cn_end = min(cb0 + KU, N);
                const float *lb = ws.block_lse + ((size_t)s * kv.max_blocks + cb0) * G;
                const int cnt = (cn_end - cb0) * G;
                float cl = js == 0 ? Cacc : __shfl(L, (js - 1) * G + g);
                float cm = js == 0 ? Cmin : __shfl(M, (js - 1) * G + g);
                bool found = false;
#pragma nounroll
                for (int x0 = 0; x0 < cnt; x0 += 64) {
                    const bool valid = x0 + lane < cnt;
                    float pl = ld_relaxed(&lb[min(x0 + lane, cnt - 1)]);
                    float pm = pl;
#pragma nounroll
                    for (int d = G; d < 64; d <<= 1) {
                        const float ol = __shfl_up(pl, d), om = __shfl_up(pm, d);
                        if (lane >= d) { pl = lse2(ol, pl); pm = fminf(om, pm); }
                    }
                    const float fl = lse2(cl, pl), fm = fminf(cm, pm);
                    const int nn = cb0 + (x0 + lane) / G + 1;
                    const float P = p_acc(fl, fm, N - nn);
                    const unsigned long long hits = __ballot(valid && (nn % m == 0 || nn == N) && P > eps) & head_lanes;
                    const int src = hits ? (__ffsll((long long)hits) - 1) : 0;
                    const float Pf = __shfl(P, src);
                    if (scan && !found && hits) {
                        stop = ((unsigned long long)(cb0 + (x0 + src) / G + 1) << 32) | __float_as_uint(Pf);
                        found = true;
                    }
                    const int last = (min(64, cnt - x0) / G - 1) * G + g;   // my head's last block of this batch
                    cl = __shfl(fl, last);
                    cm = __shfl(fm, last);
                }
            }
            j = js + 1;
            if (__ballot(stop == ~0ull) == 0ull) { finished = true; break; }
        }
        walked = base + j;
        if (walked >= nch) finished = true;
        if (finished) break;
        // my head's state at the frontier (for stop_bound), and the carry once the whole group is folded
        const float Lw = j == 0 ? Cacc : __shfl(L, (j - 1) * G + g), Mw = j == 0 ? Cmin : __shfl(M, (j - 1) * G + g);
        if (j == CPG) { Cacc = Lw; Cmin = Mw; base += CPG; }
        // The frontier opens the window for waiting workgroups; the limit tells them how far the stream can still go.
        // The window: the launch's total of chunks in flight is shared by the streams still open, so the last,
        // deepest streams are read as wide as the whole batch was (a window sized for all streams leaves the
        // machine idle once most of them have closed).
        const int lim = min(nch, stop_bound<G>(Lw, Mw, stop, walked * KU, N, m, KU, odds));
        lim_now = lim;
        if (lane == 0) st_relaxed(&ctl->key_progress, progress_word(lim, granted(window, S, closed), walked));
    }
    // every head has stopped, or the blocks ran out: close the key side (limit = frontier)
    if (lane < G) st_relaxed(&ctl->stop[lane], stop);
    if (lane == 0) {
        st_relaxed(&ctl->key_progress, ((unsigned long long)(unsigned)walked << 32) | (unsigned)walked);
        atomicAdd(&ws.header[kClosedStreams], 1);
    }
    // the stream's value units (the chunks up to its slowest head's stop) go onto the work list of the
    // value pass, which therefore starts no workgroup for a chunk nobody selected
    int nmax = (lane < G) ? ((stop == ~0ull) ? N : (int)(stop >> 32)) : 0;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) nmax = max(nmax, __shfl_xor(nmax, d));
    const int units = (nmax + KU - 1) / KU;
    int base_item = 0;
    if (lane == 0) base_item = atomicAdd(&ws.header[kValueCount], units);
    base_item = uniform(base_item);
    for (int i = lane; i < units; i += 64) ws.value_items[base_item + i] = s * ws.max_chunks + i;
}

// Physical page and valid-token count of each ranked block of chunk c of stream s -> LDS.  Issued before
// the workgroup looks at the window, so that the loads overlap its wait.
template <int G, bool STAGE>
__device__ __forceinline__ void stage_pages(SelectShared<G, STAGE> &sh, const KvView &kv, const DecodeWs &ws, int CB,
                                            int s, int c) {
    const int tid = threadIdx.x;
    const int ctx = stream_ctx(kv, s);
    const int N = (ctx + kPage - 1) / kPage;
    const int nblk = min(CB, N - c * CB);
    const size_t row0 = (size_t)s * kv.max_blocks + c * CB;
    if (tid < nblk) {
        const int page = ws.ranked_page[row0 + tid];
        // (the ranking kernel wrote a page of the pool, or with a second tier possibly ~slot; anything else
        // is taken for page 0 rather than for an address)
        sh.page[tid] = (kv.slot_pool != nullptr && page < 0) ? page : clamp_page_quiet(page, kv.num_pages);
        sh.valid[tid] = min(kPage, ctx - ws.order[row0 + tid] * kPage);
    }
}

// B operand of the QK^T product of stream s -> LDS (every wave of the workgroup reads it from there): column
// n = lane%16 is query head n (zero beyond the group), k block kq = lane/16; for step kk the lane holds
// channels 8*(4*kk + kq) .. +7.  (The caller's next barrier makes it visible.)
template <int G, bool STAGE>
__device__ __forceinline__ void load_queries(SelectShared<G, STAGE> &sh, const KvView &kv, const uint8_t *__restrict__ q,
                                             int s) {
    const int tid = threadIdx.x;
    if (tid < 256) {
        const int kk = tid >> 6, ln = tid & 63, n = ln & 15, kq = ln >> 4;
        const int r = s / kv.num_kv_heads, h = s % kv.num_kv_heads;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (n < G) v = ld16(q + ((size_t)(r * kv.num_q_heads + h * G + n) * kHeadDim + (4 * kk + kq) * 8) * 2);
        sh.qb[kk][ln] = v;
    }
}

// =================================================================================================
// Key work of one workgroup: chunk c of stream s.  Ends with the chunk published (wave 0 stores the chunk's
// words, which the stream's folding wave is looking at).
// =================================================================================================
template <int DT, int G, bool STAGE>
__device__ void process_chunk(SelectShared<G, STAGE> &sh, const KvView &kv, const uint8_t *__restrict__ q,
                              const DecodeWs &ws, float eps, int m, int CB, int budget, int s, int c) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = s % kv.num_kv_heads;
    const int ctx = stream_ctx(kv, s);
    const int N = (ctx + kPage - 1) / kPage;
    const int start = c * CB;
    const int nblk = min(CB, N - start);
    const size_t row0 = (size_t)s * kv.max_blocks + start;
    // (the chunk's pages and valid-token counts are in LDS already: stage_pages)
    // B operand of the QK^T product (see load_queries): the same for every chunk of the stream
    const int n = lane & 15, kq = lane >> 4;
    // Row r of the A operand stands for token 4*(r%4) + r/4, so that lane (kq, n) ends up with head n's logits of
    // tokens kq, 4+kq, 8+kq, 12+kq: the value pass wants the four tokens whose value rows ITS lane (kq, *) loads,
    // and finds them as the 16 bytes at [block][head][4 kq] of the stored logits.
    const int arow = 4 * (n & 3) + (n >> 2);
    uint4 qb[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) qb[kk] = sh.qb[kk][lane];
    float *lg_out = ws.logits + row0 * (kPage * G);
    lds_barrier();
    // ---- keys: wave w takes blocks [16*it + 4*w, +4), each a 4 KiB slice read as four coalesced 1 KiB
    //      loads.  A operand of the product: row n = token n of the block, same channel assignment as
    //      the queries. ----------------------------------------------------------------------------
    auto issue = [&](int i, uint4 (&dst)[4]) {
        const uint8_t *kp = key_slice(kv, sh.page[i], h) + lane * 16;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) dst[kk] = ld16_stream(kp + kk * 1024);
    };
    auto consume = [&](int i, const uint4 (&k)[4]) {
        // (second tier with a staging buffer: a slice that came over the host link is kept for the update)
        if (kv.staging != nullptr && sh.page[i] >= 0) stage_key_slice(kv, sh.page[i], h, k, lane);
        f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
        // the slice arrived as four coalesced 1 KiB rows of lanes (loading it in the operand's layout
        // would touch sixteen 64-byte segments per instruction); the wave turns it into that layout
        // through its own LDS patch (row = token, 17 16-byte words apart: no bank conflicts)
        uint4 *stg = sh.stage[wave];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) stg[(kk * 4 + (lane >> 4)) * 17 + (lane & 15)] = k[kk];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
        uint4 a[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) a[kk] = stg[arow * 17 + kk * 4 + kq];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) acc = mfma_16x16x32<DT>(a[kk], qb[kk], acc);
        // the lane now holds head n's logits of tokens kq, 4+kq, 8+kq, 12+kq
        const int valid = sh.valid[i];
        float sc[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) sc[x] = (4 * x + kq < valid) ? acc[x] * kScaleLog2 : -INFINITY;
        if (n < G) {
            if constexpr (STAGE) *reinterpret_cast<f32x4_t *>(&sh.lg[i][n][4 * kq]) = f32x4_t{sc[0], sc[1], sc[2], sc[3]};
            else store_stream(lg_out + ((size_t)i * G + n) * kPage + 4 * kq, f32x4_t{sc[0], sc[1], sc[2], sc[3]});
        }
        // the block's log-sum-exp for head n, across the 4 token groups
        float mx = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        float sum = (exp2_fast(sc[0] - mx) + exp2_fast(sc[1] - mx)) +
                    (exp2_fast(sc[2] - mx) + exp2_fast(sc[3] - mx));
        sum += __shfl_xor(sum, 16);
        sum += __shfl_xor(sum, 32);
        if (lane < G) sh.Lb[i][lane] = mx + log2_fast(sum);
    };
    constexpr int kWaves = kSelectThreads / 64;
    if (nblk == 2 * kWaves * kBatch) {
        // A whole chunk of 32 blocks, eight per wave: a rolling window.  Four slices are in flight; the oldest is
        // worked on and its registers go to the next load at once, so the wave never stands with nothing in
        // flight between rounds (a quarter of a round is arithmetic, LDS and stores).
        uint4 ka[kBatch][4];
        auto block_of = [&](int k) { return (k / kBatch) * (kWaves * kBatch) + wave * kBatch + (k % kBatch); };
#pragma unroll
        for (int u = 0; u < kBatch; ++u) issue(block_of(u), ka[u]);
#pragma unroll
        for (int k = 0; k < 2 * kBatch; ++k) {
            consume(block_of(k), ka[k % kBatch]);
            if (k + kBatch < 2 * kBatch) issue(block_of(k + kBatch), ka[k % kBatch]);
        }
    } else {
        for (int i0 = wave * kBatch; i0 < nblk; i0 += kWaves * kBatch) {
            uint4 ka[kBatch][4];
#pragma unroll
            for (int u = 0; u < kBatch; ++u)
                if (i0 + u < nblk) issue(i0 + u, ka[u]);
#pragma unroll
            for (int u = 0; u < kBatch; ++u)
                if (i0 + u < nblk) consume(i0 + u, ka[u]);
        }
    }
    lds_barrier();
    // The chunk's logits leave as one contiguous piece (8 KiB at G = 4), every thread 16 bytes at a time.  Writes
    // are what this kernel pays most for per byte (the stored logits are 6 % of what it moves and a tenth of its
    // time); in whole, neighbouring cache lines they cost a third less than as 256 bytes per block in between
    // the loads.
    if constexpr (STAGE) {
        const float *staged = &sh.lg[0][0][0];
        for (int idx = tid * 4; idx < nblk * G * kPage; idx += kSelectThreads * 4)
            store_stream(lg_out + idx, *reinterpret_cast<const f32x4_t *>(staged + idx));
    }
    // the blocks' L_b, for the fold's block-by-block pass; complete before the chunk is published
    for (int idx = tid; idx < nblk * G; idx += kSelectThreads)
        st_relaxed(&ws.block_lse[row0 * G + idx], sh.Lb[idx / G][idx % G]);
    stores_done();
    lds_barrier();
    if (wave != 0) return;

    // ---- publish: the chunk's (log-sum-exp, minimum) of its blocks' L_b per head.  Lane = (slot, head):
    //      64/G slots each fold every (64/G)-th block, then a butterfly over the slots -- a fixed tree, so
    //      the word is reproducible; lse2 is symmetric, so every lane of a head ends with the same bits. -------
    float aggL = -INFINITY, aggMin = INFINITY;
    {
        constexpr int kSlots = 64 / G;
        const int g = lane % G;
        for (int i = lane / G; i < nblk; i += kSlots) {
            const float Lb = sh.Lb[i][g];
            aggL = lse2(aggL, Lb);
            aggMin = fminf(aggMin, Lb);
        }
#pragma unroll
        for (int d = G; d < 64; d <<= 1) {
            aggL = lse2(aggL, __shfl_xor(aggL, d));
            aggMin = fminf(aggMin, __shfl_xor(aggMin, d));
        }
    }
    unsigned long long w = pack2(aggL, aggMin);
    if (w == kAggSentinel) w = kAggSentinel - 1;     // a NaN pair that happens to look like "not published"
    // The G words need no order among themselves: the fold takes a chunk only when it sees all of them.
    if (lane < G) st_relaxed(&ws.agg[((size_t)s * ws.max_chunks + c) * G + lane], w);
}

// =================================================================================================
// grid = folders + S * max_chunks workgroups of 256 threads.  The first `folders` = min(ceil(S / 4), kMaxFoldGroups)
// workgroups are the folds, one wave per stream (they start first and stay until their streams close); then one
// workgroup per (chunk, stream), streams fastest.
// =================================================================================================
template <int DT, int G, bool STAGE>
__global__ __launch_bounds__(kSelectThreads, 4) void select_kernel(KvView kv, const uint8_t *__restrict__ q,
                                                                DecodeWs ws, float eps, int m, int CB, int budget,
                                                                int window, int spin_limit,
                                                                const int32_t *depth_hint) {
    __shared__ SelectShared<G, STAGE> sh;
    const int S = kv.batch * kv.num_kv_heads;
    const int folders = min((S + 3) / 4, kMaxFoldGroups);
    if ((int)blockIdx.x < folders) {
        for (int fs = (int)blockIdx.x * 4 + (int)(threadIdx.x >> 6); fs < S; fs += 4 * folders)
            fold_stream<G>(kv, ws, fs, eps, m, CB, budget, window > 0 ? window : 1);
        return;
    }
    // Workgroups go to the chip's eight partitions by index, round robin.  With the streams in the same order in
    // every batch of S workgroups, and S a multiple of eight, all chunks of a stream would land on one partition:
    // the last, deepest streams would then be read by an eighth of the machine.  So the streams' order rotates by
    // one from chunk to chunk (when S is even; an odd S rotates by itself).
    const int c = ((int)blockIdx.x - folders) / S;
    const int s = (((int)blockIdx.x - folders) % S + ((S & 1) ? 0 : c)) % S;
    // One round trip for everything a workgroup needs to know first: the stream's progress word (asked for before
    // anything else), its length, its queries, its chunk's pages.  Most workgroups of a launch belong to chunks
    // beyond their stream's stop and leave right here; the faster they do, the sooner the slots they hold go to
    // chunks that matter.
    unsigned long long kp_first = 0;
    if (threadIdx.x == 0) kp_first = ld_relaxed(&ws.ctl[s].key_progress);
    const int N = (stream_ctx(kv, s) + kPage - 1) / kPage;
    if (c * CB >= N) return;
    load_queries<G, STAGE>(sh, kv, q, s);
    stage_pages<G, STAGE>(sh, kv, ws, CB, s, c);
    if (threadIdx.x == 0) sh.kp0 = kp_first;
    lds_barrier();
    if (c >= (int)(sh.kp0 >> 32)) return;          // closed, out of reach, or beyond a block budget
    // Second tier: a chunk with slices that are not cached is read over the host link, where reading ahead
    // of the stop costs far more than waiting does: such a chunk is read when it is expected to be needed
    // (inside the hint) or when the fold is about to reach it.
    const bool tiered = kv.slot_pool != nullptr;
    if (threadIdx.x == 0) {
        bool from_host = false;
        if (tiered)
            for (int i = 0; i < min(CB, N - c * CB); ++i) from_host |= sh.page[i] >= 0;
        // chunks read beyond the fold's frontier are at most the window: wait until this one is inside
        // it, or the stream closes before it
        const int hinted = hinted_chunks(depth_hint, s, N, CB);
        int go = 1;
        for (int tries = 0;; ++tries) {
            const unsigned long long kp = tries == 0 ? sh.kp0 : ld_relaxed(&ws.ctl[s].key_progress);
            const int fr = (int)(kp & 0xffffull), grant = (int)((kp >> 16) & 0xffffull), lim = (int)(kp >> 32);
            const int win = max(window_of(window, fr), grant);      // (the fold grants more once streams have closed)
            if (c >= lim) { go = 0; break; }       // closed, or a block budget ends before this chunk
            // with a hint: everything up to it plus a margin (a sixteenth and two chunks: the depth of a
            // decode step differs a little from the previous step's) at once; past that, a window that
            // starts at 8 chunks and doubles with the distance the hint fell short by
            const int padded = hinted + (hinted >> 4) + 2;
            int reach = hinted > 0 ? max(padded, fr + min(max(8, 2 * (fr - hinted)), win)) : fr + win;
            if (from_host) reach = min(reach, max(hinted, fr + 2));
            if (c < reach || tries >= spin_limit) break;
            nap(tries);
        }
        sh.go = go;
    }
    lds_barrier();
    if (!sh.go) return;
    if (threadIdx.x == 0) atomicAdd(&ws.ctl[s].k_blocks, min(CB, N - c * CB));     // traffic accounting
    process_chunk<DT, G, STAGE>(sh, kv, q, ws, eps, m, CB, budget, s, c);
}

template <int DT, int G>
static hipError_t launch_select_t(const KvView &kv, const void *q, const DecodeWs &ws, float eps, int m,
                                  int budget, const DecodePlan &plan, hipStream_t st) {
    const unsigned S = (unsigned)(kv.batch * kv.num_kv_heads);
    const unsigned folders = (S + 3) / 4 < (unsigned)kMaxFoldGroups ? (S + 3) / 4 : (unsigned)kMaxFoldGroups;
    const unsigned grid = folders + S * (unsigned)plan.max_chunks;
    if (plan.chunk_blocks <= kStagedBlocks)
        select_kernel<DT, G, true><<<grid, kSelectThreads, 0, st>>>(kv, (const uint8_t *)q, ws, eps, m, plan.chunk_blocks,
                                                         budget, plan.window_chunks, plan.spin_limit, plan.depth_hint);
    else
        select_kernel<DT, G, false><<<grid, kSelectThreads, 0, st>>>(kv, (const uint8_t *)q, ws, eps, m, plan.chunk_blocks,
                                                          budget, plan.window_chunks, plan.spin_limit, plan.depth_hint);
    return hipGetLastError();
}

hipError_t launch_select(const KvView &kv, int dtype, int G, const void *q, const DecodeWs &ws, float eps,
                         int m, int budget, const DecodePlan &plan, hipStream_t st) {
#define PSA_CASE(DT, GG) \
    if (dtype == DT && G == GG) return launch_select_t<DT, GG>(kv, q, ws, eps, m, budget, plan, st);
    PSA_CASE(0, 1) PSA_CASE(0, 2) PSA_CASE(0, 4) PSA_CASE(0, 8)
    PSA_CASE(1, 1) PSA_CASE(1, 2) PSA_CASE(1, 4) PSA_CASE(1, 8)
#undef PSA_CASE
    return hipErrorInvalidValue;
}

}  // namespace psa
