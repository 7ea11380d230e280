// Host-side glue shared by the translation units of libpsa: launcher prototypes and small helpers.
#pragma once

#include <hip/hip_runtime.h>

#include "psa_device.h"

namespace psa {

// Layout of a psa_tier's state: header, slice -> slot, slot -> slice, slot -> stamp, slice -> staging entry.
inline size_t tier_align(size_t v) { return (v + 255) / 256 * 256; }
inline size_t tier_staged_at_offset(long long total_slices, long long num_slots) {
    return 256 + tier_align((size_t)total_slices * 4) + 2 * tier_align((size_t)num_slots * 4);
}

inline KvView make_view(const psa_kv_desc *d) {
    KvView kv;
    kv.k_pool = static_cast<const uint8_t *>(d->k_pool);
    kv.v_pool = static_cast<const uint8_t *>(d->v_pool);
    kv.block_table = d->block_table;
    kv.ctx_lens = d->ctx_lens;
    kv.batch = d->batch;
    kv.num_q_heads = d->num_q_heads;
    kv.num_kv_heads = d->num_kv_heads;
    kv.num_pages = d->num_pages;
    kv.max_blocks = d->max_blocks_per_seq;
    kv.slot_pool = d->tier ? static_cast<const uint8_t *>(d->tier->slot_pool) : nullptr;
    const bool staged = d->tier && d->tier->staging;
    kv.staging = staged ? static_cast<uint8_t *>(d->tier->staging) : nullptr;
    kv.staged_at = staged ? reinterpret_cast<int32_t *>(static_cast<uint8_t *>(d->tier->state) +
                                                        tier_staged_at_offset(d->tier->total_slices, d->tier->num_slots))
                          : nullptr;
    kv.slice_base = d->tier ? d->tier->slice_base : 0;
    kv.staging_cap = staged ? (int32_t)d->tier->staging_slices : 0;
    return kv;
}

// Zero-fill by kernel (kept out of hipMemsetAsync so that callers may capture the calls in a graph).
static __global__ void clear_words_kernel(int32_t *p, int n) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0;
}

// psa_dense.hip
int dense_num_splits(const psa_kv_desc *d);
size_t dense_workspace_bytes(const psa_kv_desc *d);
hipError_t launch_dense(const psa_kv_desc *d, const void *q, float *out, float *lse, void *ws,
                        hipStream_t st);

// psa_meta.hip
hipError_t launch_metadata(const psa_kv_desc *d, void *meta, const int32_t *page_fill,
                           const int32_t *page_list, int num_listed, hipStream_t st);

hipError_t launch_means(const psa_kv_desc *d, void *means, const int32_t *page_fill, const int32_t *page_list,
                        int num_listed, hipStream_t st);

// psa_append.hip
hipError_t launch_append(const psa_kv_desc *d, const void *k_new, const void *v_new, void *meta,
                         int32_t *status, hipStream_t st);

// psa_decode.hip
struct DecodePlan {
    int chunk_blocks;     // CB: ranked blocks per chunk (keys and values alike)
    int window_chunks;
    int spin_limit;
    int max_chunks;
    int force_bitonic;
    const int32_t *depth_hint;   // NULL or [S] expected blocks per stream (device)
    hipEvent_t *events;   // NULL or 6 events recorded between the kernels
};
DecodePlan make_plan(const psa_kv_desc *d, const psa_tuning *t);
int compute_units();      // of the current device (256 on MI355X); read once
size_t decode_workspace_bytes_plan(const psa_kv_desc *d, const DecodePlan &p);
struct DecodeArgs {
    const void *q, *meta;
    float threshold;
    int check_granularity;
    int scorer;           // psa_scorer
    int budget_blocks;    // > 0: keys are handed out no further than this many ranked blocks
    float *out;
    int32_t *n_selected;
    float *mass_est;
    int32_t *blocks_read, *order_out;
    float *lse_out;
    float *scores_out;
    int32_t *traffic_out;
};
// psa_tier.hip
size_t tier_state_bytes(long long total_slices, long long num_slots);
size_t tier_staging_bytes(long long staging_slices);
TierView make_tier_view(const psa_tier *t);
size_t tier_update_workspace_bytes(const psa_kv_desc *d);
hipError_t launch_tier_init(const psa_tier *tier, hipStream_t st);
hipError_t launch_tier_resolve(const KvView &kv, const psa_tier *tier, int32_t *ranked_page, hipStream_t st);
hipError_t launch_tier_update(const psa_kv_desc *d, const int32_t *order, const int32_t *blocks_read,
                              long long busy_first, long long busy_count, int32_t *stats_out, void *workspace,
                              hipStream_t st);

hipError_t launch_decode(const psa_kv_desc *d, const DecodeArgs &a, const DecodePlan &plan, void *ws,
                         hipStream_t st);

// psa_score.hip, psa_order.hip, psa_select.hip, psa_values.hip: the kernels of one decode call
hipError_t launch_score(const KvView &kv, int dtype, int G, int scorer, const void *q, const void *meta,
                        const DecodeWs &ws, float *scores_out, hipStream_t st);
hipError_t launch_order(const KvView &kv, const DecodeWs &ws, int G, const DecodePlan &plan, int budget_blocks,
                        int32_t *order_out, hipStream_t st);
hipError_t launch_select(const KvView &kv, int dtype, int G, const void *q, const DecodeWs &ws, float eps,
                         int m, int budget_blocks, const DecodePlan &plan, hipStream_t st);
hipError_t launch_attend(const KvView &kv, int dtype, int G, const DecodeWs &ws, const DecodePlan &plan,
                         hipStream_t st);
hipError_t launch_finalize(const KvView &kv, const DecodeWs &ws, int G, int VU, float *out,
                           int32_t *n_selected, float *mass_est, int32_t *blocks_read, float *lse_out,
                           int32_t *traffic_out, hipStream_t st);

}  // namespace psa
