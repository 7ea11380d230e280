// Incremental decode: one new token per request goes into the paged cache and the metadata of the
// block it lands in is brought up to date (Sec. 3.1: block metadata is created on the GPU as the
// block fills and stays there).  The metadata of a partly filled block covers its valid tokens, so it
// is maintained per token: the first token of a block sets min = max = key, later ones fold in with
// the same order-preserving 16-bit min/max the bulk build uses -- the result is bit for bit what the
// bulk build gives on the new cache.  With a second tier the token is written to host memory and, if the
// slice has a slot, to the slot as well.
#include "psa_host.h"

namespace psa {

// grid (batch), 256 threads: wave w takes KV heads w, w+4, ...; a lane owns two channels (one 32-bit
// word).  Every wave reads the request's length before the barrier; thread 0 bumps it after.
__global__ __launch_bounds__(256) void append_kernel(uint8_t *__restrict__ k_pool, uint8_t *__restrict__ v_pool,
                                                     const int32_t *__restrict__ block_table,
                                                     int32_t *__restrict__ ctx_lens,
                                                     const uint8_t *__restrict__ k_new,
                                                     const uint8_t *__restrict__ v_new,
                                                     uint8_t *__restrict__ meta, int32_t *__restrict__ status,
                                                     int num_kv_heads, int num_pages, int max_blocks,
                                                     const int32_t *__restrict__ slot_of, uint8_t *__restrict__ slot_pool,
                                                     long long slice_base) {
    const int r = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ctx = ctx_lens[r];
    int err = 0, page = 0;
    if (ctx < 0 || ctx >= max_blocks * kPage) {
        err = PSA_DEVERR_CTX_RANGE;                 // no room in the request's row of the block table
    } else {
        page = block_table[(size_t)r * max_blocks + ctx / kPage];
        if ((unsigned)page >= (unsigned)num_pages) err = PSA_DEVERR_PAGE_RANGE;
    }
    if (!err) {
        const int slot = ctx % kPage;
        for (int h = wave; h < num_kv_heads; h += 4) {
            const size_t src = ((size_t)r * num_kv_heads + h) * kRowBytes + lane * 4;
            const uint32_t kw = *reinterpret_cast<const uint32_t *>(k_new + src);
            const uint32_t vw = *reinterpret_cast<const uint32_t *>(v_new + src);
            const size_t unit = (size_t)page * num_kv_heads + h;
            const size_t dst = unit * kSliceBytes + (size_t)slot * kRowBytes + lane * 4;
            *reinterpret_cast<uint32_t *>(k_pool + dst) = kw;
            *reinterpret_cast<uint32_t *>(v_pool + dst) = vw;
            if (slot_of) {      // second tier: the pools are host memory; a cached copy of the slice gets the token too
                const int cached = slot_of[slice_base + (long long)unit];
                if (cached >= 0) {
                    uint8_t *c = slot_pool + (size_t)cached * (2 * kSliceBytes) + (size_t)slot * kRowBytes + lane * 4;
                    *reinterpret_cast<uint32_t *>(c) = kw;
                    *reinterpret_cast<uint32_t *>(c + kSliceBytes) = vw;
                }
            }
            uint32_t *mn = reinterpret_cast<uint32_t *>(meta + unit * kMetaBytes + lane * 4);
            uint32_t *mx = reinterpret_cast<uint32_t *>(meta + unit * kMetaBytes + 256 + lane * 4);
            if (slot == 0) {
                *mn = kw;
                *mx = kw;
            } else {
                const uint32_t key = to_ordered(kw);
                *mn = from_ordered(pk_min(to_ordered(*mn), key));
                *mx = from_ordered(pk_max(to_ordered(*mx), key));
            }
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (!err) ctx_lens[r] = ctx + 1;
        if (status) status[r] = err;
    }
}

hipError_t launch_append(const psa_kv_desc *d, const void *k_new, const void *v_new, void *meta,
                         int32_t *status, hipStream_t st) {
    if (d->batch == 0) return hipSuccess;
    TierView t{};
    if (d->tier) t = make_tier_view(d->tier);
    append_kernel<<<d->batch, 256, 0, st>>>((uint8_t *)d->k_pool, (uint8_t *)d->v_pool, d->block_table,
                                            (int32_t *)d->ctx_lens, (const uint8_t *)k_new,
                                            (const uint8_t *)v_new, (uint8_t *)meta, status, d->num_kv_heads,
                                            d->num_pages, d->max_blocks_per_seq, d->tier ? t.slot_of : nullptr,
                                            t.slot_pool, t.slice_base);
    return hipGetLastError();
}

}  // namespace psa
