// Two-tier block store (Sec. 3.1 KV cache manager, Sec. 3.4 unified memory management), GPU side.
// The pools of a tiered descriptor live in GPU-addressable host memory; one pool of 8 KiB slots, shared by
// all layers, caches (page, KV head) slices.  Everything here runs on the GPU: which slices have slots,
// which slot is the least recently used, and the copies from host memory into slots (the kernels read
// host memory directly; no host thread and no copy engine is involved, so an update is just more work on
// a stream and overlaps the next layer's attention when put on a second one).
//
// Replacement is least-recently-used at the granularity of one update (Sec. 3.4): every update has a time
// stamp; the slices an attention call used get it; the misses, ordered by (stream, rank), take the
// candidate slots ordered by (stamp, slot index).  Both orders are made by sorting 64-bit keys with the
// device radix sort of rocPRIM -- the one library routine in this file; bookkeeping, not attention.
#include <rocprim/device/device_radix_sort.hpp>

#include "psa_host.h"

namespace psa {

constexpr int kTierThreads = 256;
constexpr unsigned long long kNoKey = ~0ull;
// words of the state header
constexpr int kClock = 0, kMisses = 1, kCandidates = 2, kHits = 3, kEvicted = 4;

static size_t tier_align(size_t v) { return (v + 255) / 256 * 256; }

size_t tier_state_bytes(long long total_slices, long long num_slots) {
    return 256 + tier_align((size_t)total_slices * 4) + 2 * tier_align((size_t)num_slots * 4);
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
    return v;
}

__global__ __launch_bounds__(kTierThreads) void tier_init_kernel(TierView t) {
    const long long i = (long long)blockIdx.x * kTierThreads + threadIdx.x;
    const long long stride = (long long)gridDim.x * kTierThreads;
    if (i < 64) t.header[i] = 0;
    for (long long j = i; j < t.total_slices; j += stride) t.slot_of[j] = -1;
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

__global__ __launch_bounds__(kTierThreads) void tier_begin_kernel(TierView t, unsigned long long *miss_keys, int cap) {
    const int i = blockIdx.x * kTierThreads + threadIdx.x;
    if (i >= 1 && i <= 4) t.header[i] = 0;
    for (int j = i; j < cap; j += gridDim.x * kTierThreads) miss_keys[j] = kNoKey;
}

// The slices the call used: stamp the cached ones, list the others.  grid (ceil(max_blocks / 256), S)
__global__ __launch_bounds__(kTierThreads) void tier_touch_kernel(KvView kv, TierView t,
                                                                  const int32_t *__restrict__ order,
                                                                  const int32_t *__restrict__ blocks_read,
                                                                  unsigned long long *miss_keys) {
    const int s = blockIdx.y, r = s / kv.num_kv_heads, h = s % kv.num_kv_heads;
    const int i = blockIdx.x * kTierThreads + threadIdx.x;
    const int N = (ctx_clamped_quiet(kv, r) + kPage - 1) / kPage;
    const int used = min(max(blocks_read[s], 0), N);
    const uint32_t now = t.header[kClock] + 1;
    bool hit = false;
    if (i < used) {
        const int b = order[(size_t)s * kv.max_blocks + i];
        if (b >= 0 && b < kv.max_blocks) {
            const int page = kv.block_table[(size_t)r * kv.max_blocks + b];
            if ((unsigned)page < (unsigned)kv.num_pages) {
                const long long id = t.slice_base + (long long)page * kv.num_kv_heads + h;
                const int slot = t.slot_of[id];
                if (slot >= 0) {
                    t.stamp[slot] = now;
                    hit = true;
                } else {
                    const uint32_t at = atomicAdd(&t.header[kMisses], 1u);
                    miss_keys[at] = ((unsigned long long)((size_t)s * kv.max_blocks + i) << 32) | (uint32_t)id;
                }
            }
        }
    }
    const int nh = __popcll(__ballot(hit));
    if ((threadIdx.x & 63) == 0 && nh) atomicAdd(&t.header[kHits], (uint32_t)nh);
}

// Slots that may be given away, as keys (stamp, slot); the others get the key that sorts last.
__global__ __launch_bounds__(kTierThreads) void tier_candidates_kernel(TierView t, long long busy_first,
                                                                       long long busy_count,
                                                                       unsigned long long *cand_keys) {
    const int slot = blockIdx.x * kTierThreads + threadIdx.x;
    const uint32_t now = t.header[kClock] + 1;
    bool ok = false;
    if (slot < t.num_slots) {
        const uint32_t st = t.stamp[slot];
        const long long o = t.owner[slot];
        ok = st < now && !(o >= 0 && o >= busy_first && o < busy_first + busy_count);
        cand_keys[slot] = ok ? (((unsigned long long)st << 32) | (uint32_t)slot) : kNoKey;
    }
    const int n = __popcll(__ballot(ok));
    if ((threadIdx.x & 63) == 0 && n) atomicAdd(&t.header[kCandidates], (uint32_t)n);
}

// The j-th miss takes the j-th candidate slot: the slice is copied from host memory (two 4 KiB slices, one
// 16-byte load per thread each) and the tables are brought up to date.  Workgroups stride over the pairs.
__global__ __launch_bounds__(kTierThreads) void tier_promote_kernel(KvView kv, TierView t,
                                                                    const unsigned long long *__restrict__ misses,
                                                                    const unsigned long long *__restrict__ cands) {
    const uint32_t take = min(t.header[kMisses], t.header[kCandidates]);
    const uint32_t now = t.header[kClock] + 1;
    for (uint32_t j = blockIdx.x; j < take; j += gridDim.x) {
        const long long id = (long long)(uint32_t)misses[j];
        const int slot = (int)(uint32_t)cands[j];
        const size_t src = (size_t)(id - t.slice_base) * kSliceBytes + threadIdx.x * 16;
        const uint4 k = ld16(kv.k_pool + src), v = ld16(kv.v_pool + src);
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
        }
    }
}

__global__ void tier_finish_kernel(TierView t, int32_t *stats_out) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    if (stats_out) {
        stats_out[0] = (int32_t)t.header[kHits];
        stats_out[1] = (int32_t)t.header[kMisses];
        stats_out[2] = (int32_t)min(t.header[kMisses], t.header[kCandidates]);
        stats_out[3] = (int32_t)t.header[kEvicted];
    }
    t.header[kClock] += 1;
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
    size_t miss_in, miss_out, cand_in, cand_out, temp, temp_bytes, total;
};

static TierScratch tier_scratch(const psa_kv_desc *d) {
    const size_t cap = (size_t)d->batch * d->num_kv_heads * d->max_blocks_per_seq;
    const size_t slots = (size_t)d->tier->num_slots;
    size_t t1 = 0, t2 = 0;
    unsigned long long *none = nullptr;
    (void)rocprim::radix_sort_keys(nullptr, t1, none, none, cap, 0, 64, (hipStream_t)0);
    (void)rocprim::radix_sort_keys(nullptr, t2, none, none, slots, 0, 64, (hipStream_t)0);
    TierScratch L;
    size_t at = 0;
    L.miss_in = at;  at = tier_align(at + cap * 8);
    L.miss_out = at; at = tier_align(at + cap * 8);
    L.cand_in = at;  at = tier_align(at + slots * 8);
    L.cand_out = at; at = tier_align(at + slots * 8);
    L.temp = at;     L.temp_bytes = t1 > t2 ? t1 : t2;
    at = tier_align(at + L.temp_bytes);
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
    auto *miss_in = reinterpret_cast<unsigned long long *>(base + L.miss_in);
    auto *miss_out = reinterpret_cast<unsigned long long *>(base + L.miss_out);
    auto *cand_in = reinterpret_cast<unsigned long long *>(base + L.cand_in);
    auto *cand_out = reinterpret_cast<unsigned long long *>(base + L.cand_out);
    const int S = kv.batch * kv.num_kv_heads;
    const size_t cap = (size_t)S * kv.max_blocks;
    hipError_t e;
    tier_begin_kernel<<<(unsigned)((cap + kTierThreads - 1) / kTierThreads < 2048 ? (cap + kTierThreads - 1) / kTierThreads : 2048),
                        kTierThreads, 0, st>>>(t, miss_in, (int)cap);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const dim3 grid((kv.max_blocks + kTierThreads - 1) / kTierThreads, S);
    tier_touch_kernel<<<grid, kTierThreads, 0, st>>>(kv, t, order, blocks_read, miss_in);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    tier_candidates_kernel<<<(t.num_slots + kTierThreads - 1) / kTierThreads, kTierThreads, 0, st>>>(t, busy_first, busy_count,
                                                                                              cand_in);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    size_t tb = L.temp_bytes;
    if ((e = rocprim::radix_sort_keys(base + L.temp, tb, miss_in, miss_out, cap, 0, 64, st)) != hipSuccess) return e;
    tb = L.temp_bytes;
    if ((e = rocprim::radix_sort_keys(base + L.temp, tb, cand_in, cand_out, (size_t)t.num_slots, 0, 64, st)) != hipSuccess)
        return e;
    tier_promote_kernel<<<2048, kTierThreads, 0, st>>>(kv, t, miss_out, cand_out);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    tier_finish_kernel<<<1, 64, 0, st>>>(t, stats_out);
    return hipGetLastError();
}

}  // namespace psa
