// Two-tier block store (Sec. 3.1 KV cache manager, Sec. 3.4 unified memory management), GPU side.
// The pools of a tiered descriptor live in GPU-addressable host memory; one pool of 8 KiB slots, shared by
// all layers, caches (page, KV head) slices.  Everything here runs on the GPU: which slices have slots,
// which slot is the least recently used, and the copies from host memory into slots (the kernels read
// host memory directly; no host thread and no copy engine is involved, so an update is just more work on
// a stream and overlaps the next layer's attention when put on a second one).
//
// Replacement is least-recently-used at the granularity of one update (Sec. 3.4): every update has a time
// stamp; the slices an attention call used get it; the misses, ordered by (stream, rank), take the
// candidate slots ordered by (age, slot index), oldest first.  The first order comes from prefix sums, the
// second from a stable counting sort of the slots by their 17-bit age key, done here in two passes (8 and 9
// bits): per-tile digit counts, one scan over the (digit, tile) table, a scatter that keeps slot order inside
// a digit.
#include "psa_host.h"

namespace psa {

constexpr int kTierThreads = 256;
constexpr unsigned long long kNoKey = ~0ull;
constexpr uint32_t kMaxAge = 65535;      // updates after which a slot is as old as it gets
// words of the state header
constexpr int kClock = 0, kMisses = 1, kHits = 3, kEvicted = 4, kFromStaging = 5;

size_t tier_state_bytes(long long total_slices, long long num_slots) {
    return tier_staged_at_offset(total_slices, num_slots) + tier_align((size_t)total_slices * 4);
}

size_t tier_staging_bytes(long long staging_slices) {
    return staging_entries_offset((int)staging_slices) + (size_t)staging_slices * (2 * kSliceBytes);
}

TierView make_tier_view(const psa_tier *t) {
    TierView v;
    uint8_t *base = static_cast<uint8_t *>(t->state);
    v.header = reinterpret_cast<uint32_t *>(base);
    v.slot_of = reinterpret_cast<int32_t *>(base + 256);
    v.owner = reinterpret_cast<int32_t *>(base + 256 + tier_align((size_t)t->total_slices * 4));
    v.stamp = reinterpret_cast<uint32_t *>(base + 256 + tier_align((size_t)t->total_slices * 4) +
                                           tier_align((size_t)t->num_slots * 4));
    v.slot_pool = static_cast<uint8_t *>(t->slot_pool);
    v.slice_base = t->slice_base;
    v.total_slices = t->total_slices;
    v.num_slots = (int)t->num_slots;
    v.staged_at = reinterpret_cast<int32_t *>(base + tier_staged_at_offset(t->total_slices, t->num_slots));
    v.staging = static_cast<uint8_t *>(t->staging);
    v.staging_cap = t->staging ? (int)t->staging_slices : 0;
    return v;
}

__global__ __launch_bounds__(kTierThreads) void tier_init_kernel(TierView t) {
    const long long i = (long long)blockIdx.x * kTierThreads + threadIdx.x;
    const long long stride = (long long)gridDim.x * kTierThreads;
    if (i < 64) t.header[i] = 0;
    for (long long j = i; j < t.total_slices; j += stride) { t.slot_of[j] = -1; t.staged_at[j] = -1; }
    if (i == 0 && t.staging) *staging_count(t.staging) = 0;
    for (long long j = i; j < t.num_slots; j += stride) { t.owner[j] = -1; t.stamp[j] = 0; }
}

// Decode side: a ranked block whose slice has a slot is read from the slot.  ranked_page keeps the page
// (>= 0) for slices in host memory and holds ~slot (< 0) for cached ones.
// grid (ceil(max_blocks / 256), S)
__global__ __launch_bounds__(kTierThreads) void tier_resolve_kernel(KvView kv, TierView t, int32_t *ranked_page) {
    const int s = blockIdx.y, r = s / kv.num_kv_heads, h = s % kv.num_kv_heads;
    const int i = blockIdx.x * kTierThreads + threadIdx.x;
    const int N = (ctx_clamped_quiet(kv, r) + kPage - 1) / kPage;
    if (i >= N) return;
    int32_t *p = ranked_page + (size_t)s * kv.max_blocks + i;
    const int page = *p;                                         // clamped into the pool by the ranking kernel
    const int slot = t.slot_of[t.slice_base + (long long)page * kv.num_kv_heads + h];
    if (slot >= 0) *p = ~slot;
}

// The slices the call used: stamp the cached ones, list the others -- per stream, in rank order, packed at
// the front of the stream's row of `miss_ids` (a block-wide prefix sum per tile of 1024 ranks keeps the
// order).  grid (S), 256 threads, 4 ranks per thread and tile.
constexpr int kTouchPerThread = 4;
__global__ __launch_bounds__(kTierThreads) void tier_touch_kernel(KvView kv, TierView t,
                                                                  const int32_t *__restrict__ order,
                                                                  const int32_t *__restrict__ blocks_read,
                                                                  int32_t *__restrict__ miss_ids,
                                                                  uint32_t *__restrict__ miss_count) {
    __shared__ int wave_sum[kTierThreads / 64];
    const int s = blockIdx.x, r = s / kv.num_kv_heads, h = s % kv.num_kv_heads;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = (ctx_clamped_quiet(kv, r) + kPage - 1) / kPage;
    const int used = min(max(blocks_read[s], 0), N);
    const uint32_t now = t.header[kClock] + 1;
    int32_t *row = miss_ids + (size_t)s * kv.max_blocks;
    int placed = 0, hits = 0;
    for (int base = 0; base < used; base += kTierThreads * kTouchPerThread) {
        // the thread's 4 consecutive ranks: block, page, slot, loaded side by side
        int b[kTouchPerThread], page[kTouchPerThread], slot[kTouchPerThread];
        long long id[kTouchPerThread];
        bool live[kTouchPerThread];
#pragma unroll
        for (int u = 0; u < kTouchPerThread; ++u) {
            const int i = base + tid * kTouchPerThread + u;
            live[u] = i < used;
            b[u] = order[(size_t)s * kv.max_blocks + min(i, kv.max_blocks - 1)];
        }
#pragma unroll
        for (int u = 0; u < kTouchPerThread; ++u) {
            live[u] = live[u] && b[u] >= 0 && b[u] < kv.max_blocks;
            page[u] = kv.block_table[(size_t)r * kv.max_blocks + (live[u] ? b[u] : 0)];
        }
#pragma unroll
        for (int u = 0; u < kTouchPerThread; ++u) {
            live[u] = live[u] && (unsigned)page[u] < (unsigned)kv.num_pages;
            id[u] = t.slice_base + (live[u] ? (long long)page[u] * kv.num_kv_heads + h : 0);
            slot[u] = live[u] ? t.slot_of[id[u]] : -1;
        }
        int mine = 0;
#pragma unroll
        for (int u = 0; u < kTouchPerThread; ++u) {
            if (live[u] && slot[u] >= 0) { t.stamp[slot[u]] = now; ++hits; }
            if (live[u] && slot[u] < 0) ++mine;
        }
        // exclusive prefix of `mine` over the workgroup
        int incl = mine;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_up(incl, d);
            if (lane >= d) incl += o;
        }
        __syncthreads();                                   // (the previous tile's sums have been read)
        if (lane == 63) wave_sum[wave] = incl;
        __syncthreads();
        int before = incl - mine, total = 0;
        for (int w = 0; w < kTierThreads / 64; ++w) {
            if (w < wave) before += wave_sum[w];
            total += wave_sum[w];
        }
        int at = placed + before;
#pragma unroll
        for (int u = 0; u < kTouchPerThread; ++u)
            if (live[u] && slot[u] < 0) row[at++] = (int32_t)id[u];
        placed += total;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) hits += __shfl_xor(hits, d);
    if (lane == 0 && hits) atomicAdd(&t.header[kHits], (uint32_t)hits);
    if (tid == 0) miss_count[s] = (uint32_t)placed;
}

// Exclusive prefix sum of the streams' miss counts (one workgroup; S is small) and their total.
__global__ __launch_bounds__(kTierThreads) void tier_offsets_kernel(TierView t, const uint32_t *__restrict__ miss_count,
                                                                    uint32_t *__restrict__ miss_offset, int S) {
    __shared__ uint32_t wave_sum[kTierThreads / 64];
    __shared__ uint32_t carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < S; base += kTierThreads) {
        const int i = base + tid;
        const uint32_t v = i < S ? miss_count[i] : 0u;
        uint32_t incl = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t o = (uint32_t)__shfl_up((int)incl, d);
            if (lane >= d) incl += o;
        }
        if (lane == 63) wave_sum[wave] = incl;
        __syncthreads();
        uint32_t before = carry + incl - v, total = 0;
        for (int w = 0; w < kTierThreads / 64; ++w) {
            if (w < wave) before += wave_sum[w];
            total += wave_sum[w];
        }
        if (i < S) miss_offset[i] = before;
        __syncthreads();
        if (tid == 0) carry += total;
        __syncthreads();
    }
    if (tid == 0) { miss_offset[S] = carry; t.header[kMisses] = carry; }
}

// Slots that may be given away, as keys that sort oldest first: (65535 - age) in bits 32..48, where age = updates
// since the slot's last use, saturating at 65535 (a slot never used counts as that old); the slot index below
// it, so that the stable sort's ties go to the lower slot.  Slots that may not be taken get the key that sorts last.
__global__ __launch_bounds__(kTierThreads) void tier_candidates_kernel(TierView t, long long busy_first,
                                                                       long long busy_count,
                                                                       unsigned long long *cand_keys) {
    const uint32_t now = t.header[kClock] + 1;
    for (int slot = blockIdx.x * kTierThreads + threadIdx.x; slot < t.num_slots; slot += gridDim.x * kTierThreads) {
        const uint32_t st = t.stamp[slot];
        const long long o = t.owner[slot];
        const bool ok = st < now && !(o >= 0 && o >= busy_first && o < busy_first + busy_count);
        const uint32_t age = st == 0 ? kMaxAge : min(now - st, kMaxAge);
        cand_keys[slot] = ok ? (((unsigned long long)(kMaxAge - age) << 32) | (uint32_t)slot) : kNoKey;
    }
}

// ---- stable sort of the candidate keys by bits [SHIFT, SHIFT + BITS) -------------------------------------------
// One pass of a least-significant-digit radix sort: tiles of 256 consecutive keys (one per thread); within a
// tile a key's rank among the keys with its digit comes from ballots (the lanes of a wave that share the digit)
// plus the counts of the waves before; `counts` is laid out [digit][tile], so that one exclusive scan over the
// whole table gives every (digit, tile) its first output position and equal digits keep their input order.
constexpr int kSortTile = kTierThreads;

template <int SHIFT, int BITS>
__device__ __forceinline__ void tile_ranks(const unsigned long long *__restrict__ keys, int n, uint16_t (*wave_hist)[1 << BITS],
                                           unsigned long long &key, int &digit, int &rank, bool &live) {
    constexpr int BINS = 1 << BITS;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i = blockIdx.x * kSortTile + tid;
    live = i < n;
    key = live ? keys[i] : 0ull;
    digit = (int)((key >> SHIFT) & (unsigned long long)(BINS - 1));
    for (int b = tid; b < (kTierThreads / 64) * BINS; b += kTierThreads) (&wave_hist[0][0])[b] = 0;
    __syncthreads();
    unsigned long long peers = __ballot(live);
#pragma unroll
    for (int b = 0; b < BITS; ++b) {
        const bool bit = (digit >> b) & 1;
        const unsigned long long bal = __ballot(bit);
        peers &= bit ? bal : ~bal;
    }
    const int in_wave = __popcll(peers & ((1ull << lane) - 1ull));
    if (live && in_wave == 0) wave_hist[wave][digit] = (uint16_t)__popcll(peers);
    __syncthreads();
    rank = in_wave;
    for (int w = 0; w < wave; ++w) rank += wave_hist[w][digit];
}

template <int SHIFT, int BITS>
__global__ __launch_bounds__(kTierThreads) void sort_count_kernel(const unsigned long long *__restrict__ keys, int n,
                                                                  uint32_t *__restrict__ counts, int tiles) {
    constexpr int BINS = 1 << BITS;
    __shared__ uint16_t wave_hist[kTierThreads / 64][BINS];
    unsigned long long key; int digit, rank; bool live;
    tile_ranks<SHIFT, BITS>(keys, n, wave_hist, key, digit, rank, live);
    for (int b = threadIdx.x; b < BINS; b += kTierThreads) {
        uint32_t c = 0;
#pragma unroll
        for (int w = 0; w < kTierThreads / 64; ++w) c += wave_hist[w][b];
        counts[(size_t)b * tiles + blockIdx.x] = c;
    }
}

// Exclusive prefix sum over `total` counters in place, in two launches: every workgroup owns a span of
// kScanSpan consecutive counters (16 per thread).  First the spans' sums; then every workgroup adds up the sums of
// the spans before its own (a few hundred numbers at most per million slots) and rewrites its span.  (One
// workgroup walking the whole table -- 512 counters per tile of 256 slots -- took a millisecond per pass.)
constexpr int kScanPerThread = 16;
constexpr int kScanSpan = kTierThreads * kScanPerThread;

// Sum of v over the workgroup, the same in every thread.  `part` holds one word per wave.
__device__ __forceinline__ uint32_t group_sum(uint32_t v, uint32_t *part) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += (uint32_t)__shfl_xor((int)v, d);
    __syncthreads();                       // (the previous use of `part` is over)
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
    __syncthreads();
    uint32_t all = 0;
#pragma unroll
    for (int w = 0; w < kTierThreads / 64; ++w) all += part[w];
    return all;
}

__global__ __launch_bounds__(kTierThreads) void sort_scan_sums_kernel(const uint32_t *__restrict__ counts, int total,
                                                                      uint32_t *__restrict__ span_sums) {
    __shared__ uint32_t part[kTierThreads / 64];
    const int base = blockIdx.x * kScanSpan;
    uint32_t mine = 0;
#pragma unroll
    for (int k = 0; k < kScanPerThread; ++k) {
        const int i = base + k * kTierThreads + (int)threadIdx.x;
        mine += i < total ? counts[i] : 0u;
    }
    const uint32_t all = group_sum(mine, part);
    if (threadIdx.x == 0) span_sums[blockIdx.x] = all;
}

__global__ __launch_bounds__(kTierThreads) void sort_scan_apply_kernel(uint32_t *__restrict__ counts, int total,
                                                                       const uint32_t *__restrict__ span_sums) {
    __shared__ uint32_t part[kTierThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t before = 0;
    for (int i = tid; i < (int)blockIdx.x; i += kTierThreads) before += span_sums[i];
    before = group_sum(before, part);
    // thread t owns counters first .. first + 15 of the span
    const int first = blockIdx.x * kScanSpan + tid * kScanPerThread;
    uint32_t c[kScanPerThread], mine = 0;
#pragma unroll
    for (int k = 0; k < kScanPerThread; ++k) {
        c[k] = first + k < total ? counts[first + k] : 0u;
        mine += c[k];
    }
    uint32_t incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = (uint32_t)__shfl_up((int)incl, d);
        if (lane >= d) incl += o;
    }
    __syncthreads();
    if (lane == 63) part[wave] = incl;
    __syncthreads();
    uint32_t run = before + incl - mine;
    for (int w = 0; w < wave; ++w) run += part[w];
#pragma unroll
    for (int k = 0; k < kScanPerThread; ++k) {
        if (first + k < total) counts[first + k] = run;
        run += c[k];
    }
}

template <int SHIFT, int BITS>
__global__ __launch_bounds__(kTierThreads) void sort_scatter_kernel(const unsigned long long *__restrict__ keys, int n,
                                                                    const uint32_t *__restrict__ counts, int tiles,
                                                                    unsigned long long *__restrict__ out) {
    constexpr int BINS = 1 << BITS;
    __shared__ uint16_t wave_hist[kTierThreads / 64][BINS];
    unsigned long long key; int digit, rank; bool live;
    tile_ranks<SHIFT, BITS>(keys, n, wave_hist, key, digit, rank, live);
    if (live) out[counts[(size_t)digit * tiles + blockIdx.x] + rank] = key;
}

// The j-th miss takes the j-th candidate slot: the slice is copied into it (two 4 KiB slices, one 16-byte load
// per thread each) -- from the staging buffer if the attention kernels left it there, from host memory if not --
// and the tables are brought up to date.  Workgroups stride over the pairs.
__global__ __launch_bounds__(kTierThreads) void tier_promote_kernel(KvView kv, TierView t,
                                                                    const int32_t *__restrict__ miss_ids,
                                                                    const uint32_t *__restrict__ miss_offset, int S,
                                                                    const unsigned long long *__restrict__ cands) {
    const uint32_t misses_n = t.header[kMisses];
    const uint32_t now = t.header[kClock] + 1;
    for (uint32_t j = blockIdx.x; j < misses_n && j < (uint32_t)t.num_slots; j += gridDim.x) {
        const unsigned long long cand = cands[j];
        if (cand == kNoKey) break;                         // sorted: no slot left to give, here or further on
        int lo = 0, hi = S;                                // the stream whose misses include the j-th of all
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (miss_offset[mid] <= j) lo = mid; else hi = mid;
        }
        const long long id = miss_ids[(size_t)lo * kv.max_blocks + (j - miss_offset[lo])];
        const int slot = (int)(uint32_t)cand;
        const size_t src = (size_t)(id - t.slice_base) * kSliceBytes + threadIdx.x * 16;
        const int entry = t.staging ? t.staged_at[id] : -1;
        uint4 k, v;
        if (entry >= 0 && entry < t.staging_cap) {
            const uint8_t *e = staging_entry(t.staging, t.staging_cap, entry) + threadIdx.x * 16;
            k = ld16(e);
            v = ld16(e + kSliceBytes);
        } else {
            k = ld16(kv.k_pool + src);
            v = ld16(kv.v_pool + src);
        }
        uint8_t *dst = t.slot_pool + (size_t)slot * (2 * kSliceBytes) + threadIdx.x * 16;
        *reinterpret_cast<uint4 *>(dst) = k;
        *reinterpret_cast<uint4 *>(dst + kSliceBytes) = v;
        if (threadIdx.x == 0) {
            const int old = t.owner[slot];
            if (old >= 0 && t.slot_of[old] == slot) {      // (a slot that lost its slice to a twin keeps no claim)
                t.slot_of[old] = -1;
                atomicAdd(&t.header[kEvicted], 1u);
            }
            t.owner[slot] = (int)id;
            t.slot_of[id] = slot;
            t.stamp[slot] = now;
            if (entry >= 0 && entry < t.staging_cap) atomicAdd(&t.header[kFromStaging], 1u);
        }
    }
}

// Empties the staging buffer: every entry's slice forgets it.  (The counter itself is cleared by the finishing kernel.)
__global__ __launch_bounds__(kTierThreads) void tier_unstage_kernel(TierView t) {
    const uint32_t n = min(*staging_count(t.staging), (uint32_t)t.staging_cap);
    for (uint32_t i = blockIdx.x * kTierThreads + threadIdx.x; i < n; i += gridDim.x * kTierThreads) {
        const int id = staging_ids(t.staging)[i];
        if (id >= 0 && id < t.total_slices) t.staged_at[id] = -1;
    }
}

__global__ void tier_finish_kernel(TierView t, const unsigned long long *__restrict__ cands, int32_t *stats_out) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    if (stats_out) {
        int lo = 0, hi = t.num_slots;                      // first position of the sorted keys that is no candidate
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (cands[mid] == kNoKey) hi = mid; else lo = mid + 1;
        }
        stats_out[0] = (int32_t)t.header[kHits];
        stats_out[1] = (int32_t)t.header[kMisses];
        stats_out[2] = (int32_t)min(t.header[kMisses], (uint32_t)lo);
        stats_out[3] = (int32_t)t.header[kEvicted];
        stats_out[4] = (int32_t)t.header[kFromStaging];
    }
    if (t.staging) *staging_count(t.staging) = 0;
    t.header[kFromStaging] = 0;
    t.header[kClock] += 1;
    t.header[kMisses] = 0;
    t.header[kHits] = 0;
    t.header[kEvicted] = 0;
}

hipError_t launch_tier_init(const psa_tier *tier, hipStream_t st) {
    const TierView t = make_tier_view(tier);
    tier_init_kernel<<<1024, kTierThreads, 0, st>>>(t);
    return hipGetLastError();
}

hipError_t launch_tier_resolve(const KvView &kv, const psa_tier *tier, int32_t *ranked_page, hipStream_t st) {
    const TierView t = make_tier_view(tier);
    const dim3 grid((kv.max_blocks + kTierThreads - 1) / kTierThreads, kv.batch * kv.num_kv_heads);
    tier_resolve_kernel<<<grid, kTierThreads, 0, st>>>(kv, t, ranked_page);
    return hipGetLastError();
}

struct TierScratch {
    size_t miss_ids, miss_count, miss_offset, cand_in, cand_out, counts, span_sums, total;
    int tiles;
};
constexpr int kSortBitsLow = 8, kSortBitsHigh = 9;       // the 17 bits of the age key, low digit first

static TierScratch tier_scratch(const psa_kv_desc *d) {
    const size_t S = (size_t)d->batch * d->num_kv_heads;
    const size_t cap = S * d->max_blocks_per_seq;
    const size_t slots = (size_t)d->tier->num_slots;
    TierScratch L;
    L.tiles = (int)((slots + kSortTile - 1) / kSortTile);
    size_t at = 0;
    L.miss_ids = at;    at = tier_align(at + cap * 4);
    L.miss_count = at;  at = tier_align(at + S * 4);
    L.miss_offset = at; at = tier_align(at + (S + 1) * 4);
    L.cand_in = at;     at = tier_align(at + slots * 8);
    L.cand_out = at;    at = tier_align(at + slots * 8);
    const size_t counters = ((size_t)1 << kSortBitsHigh) * L.tiles;
    L.counts = at;      at = tier_align(at + counters * 4);
    L.span_sums = at;   at = tier_align(at + (counters + kScanSpan - 1) / kScanSpan * 4);
    L.total = at;
    return L;
}

size_t tier_update_workspace_bytes(const psa_kv_desc *d) { return tier_scratch(d).total; }

hipError_t launch_tier_update(const psa_kv_desc *d, const int32_t *order, const int32_t *blocks_read,
                              long long busy_first, long long busy_count, int32_t *stats_out, void *workspace,
                              hipStream_t st) {
    const KvView kv = make_view(d);
    const TierView t = make_tier_view(d->tier);
    const TierScratch L = tier_scratch(d);
    uint8_t *base = static_cast<uint8_t *>(workspace);
    auto *miss_ids = reinterpret_cast<int32_t *>(base + L.miss_ids);
    auto *miss_count = reinterpret_cast<uint32_t *>(base + L.miss_count);
    auto *miss_offset = reinterpret_cast<uint32_t *>(base + L.miss_offset);
    auto *cand_in = reinterpret_cast<unsigned long long *>(base + L.cand_in);
    auto *cand_out = reinterpret_cast<unsigned long long *>(base + L.cand_out);
    const int S = kv.batch * kv.num_kv_heads;
    hipError_t e;
    tier_touch_kernel<<<S, kTierThreads, 0, st>>>(kv, t, order, blocks_read, miss_ids, miss_count);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    tier_offsets_kernel<<<1, kTierThreads, 0, st>>>(t, miss_count, miss_offset, S);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int cgrid = (t.num_slots + kTierThreads - 1) / kTierThreads;
    tier_candidates_kernel<<<cgrid < 2048 ? cgrid : 2048, kTierThreads, 0, st>>>(t, busy_first, busy_count, cand_in);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // candidates by bits 32..48, low digit first (each pass is stable: equal ages stay in slot order)
    auto *counts = reinterpret_cast<uint32_t *>(base + L.counts);
    const int n = t.num_slots, tiles = L.tiles;
    auto *span_sums = reinterpret_cast<uint32_t *>(base + L.span_sums);
    const int total_low = (1 << kSortBitsLow) * tiles, total_high = (1 << kSortBitsHigh) * tiles;
    const int spans_low = (total_low + kScanSpan - 1) / kScanSpan, spans_high = (total_high + kScanSpan - 1) / kScanSpan;
    sort_count_kernel<32, kSortBitsLow><<<tiles, kTierThreads, 0, st>>>(cand_in, n, counts, tiles);
    sort_scan_sums_kernel<<<spans_low, kTierThreads, 0, st>>>(counts, total_low, span_sums);
    sort_scan_apply_kernel<<<spans_low, kTierThreads, 0, st>>>(counts, total_low, span_sums);
    sort_scatter_kernel<32, kSortBitsLow><<<tiles, kTierThreads, 0, st>>>(cand_in, n, counts, tiles, cand_out);
    sort_count_kernel<32 + kSortBitsLow, kSortBitsHigh><<<tiles, kTierThreads, 0, st>>>(cand_out, n, counts, tiles);
    sort_scan_sums_kernel<<<spans_high, kTierThreads, 0, st>>>(counts, total_high, span_sums);
    sort_scan_apply_kernel<<<spans_high, kTierThreads, 0, st>>>(counts, total_high, span_sums);
    sort_scatter_kernel<32 + kSortBitsLow, kSortBitsHigh><<<tiles, kTierThreads, 0, st>>>(cand_out, n, counts, tiles, cand_in);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    tier_promote_kernel<<<2048, kTierThreads, 0, st>>>(kv, t, miss_ids, miss_offset, S, cand_in);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (t.staging) {
        const int ugrid = (t.staging_cap + kTierThreads - 1) / kTierThreads;
        tier_unstage_kernel<<<ugrid < 1024 ? ugrid : 1024, kTierThreads, 0, st>>>(t);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    tier_finish_kernel<<<1, 64, 0, st>>>(t, cand_in, stats_out);
    return hipGetLastError();
}

}  // namespace psa
