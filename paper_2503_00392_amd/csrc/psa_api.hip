// The C ABI of libpsa: argument validation on the host, then kernel launches.  See include/psa.h
// for the contract of every entry point.
#include <math.h>
#include <stdint.h>

#include <mutex>

#include "psa_host.h"

namespace {

bool supported_group(int g) { return g == 1 || g == 2 || g == 4 || g == 8; }

// Shape checks common to all entry points.  `need_tables`: the call reads block_table / ctx_lens.
psa_status check_desc(const psa_kv_desc *d, bool need_tables, bool need_v) {
    if (!d) return PSA_ERR_INVALID_ARG;
    if (d->batch < 0 || d->num_q_heads <= 0 || d->num_kv_heads <= 0 || d->num_pages < 0 ||
        d->max_blocks_per_seq < 0)
        return PSA_ERR_INVALID_ARG;
    if (d->num_q_heads % d->num_kv_heads != 0) return PSA_ERR_INVALID_ARG;
    if (d->dtype != PSA_F16 && d->dtype != PSA_BF16) return PSA_ERR_UNSUPPORTED;
    if (d->head_dim != psa::kHeadDim || d->page_size != psa::kPage) return PSA_ERR_UNSUPPORTED;
    if (!supported_group(d->num_q_heads / d->num_kv_heads)) return PSA_ERR_UNSUPPORTED;
    if ((long long)d->batch * d->num_kv_heads > (1 << 24)) return PSA_ERR_UNSUPPORTED;
    if (d->num_pages > 0 && !d->k_pool) return PSA_ERR_INVALID_ARG;
    if (need_v && d->num_pages > 0 && !d->v_pool) return PSA_ERR_INVALID_ARG;
    if (need_tables && d->batch > 0) {
        // a block table with at least one column, even if every request is empty
        if (!d->ctx_lens || !d->block_table || d->max_blocks_per_seq < 1) return PSA_ERR_INVALID_ARG;
    }
    return PSA_OK;
}

// A descriptor with a second tier: the tier's own fields, the id range, and the pools -- they must be
// memory the GPU can address (device memory, or pinned host memory); `out` gets the descriptor with the
// pools' device-side addresses.
psa_status check_tier(const psa_kv_desc *d, psa_kv_desc *out) {
    const psa_tier *t = d->tier;
    if (!t || !t->state || !t->slot_pool) return PSA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(t->state) & 255u) || (reinterpret_cast<uintptr_t>(t->slot_pool) & 15u))
        return PSA_ERR_INVALID_ARG;
    if (t->total_slices < 1 || t->total_slices > INT32_MAX || t->num_slots < 1 || t->num_slots > PSA_TIER_MAX_SLOTS)
        return PSA_ERR_INVALID_ARG;
    if (t->staging && ((reinterpret_cast<uintptr_t>(t->staging) & 255u) || t->staging_slices < 1 ||
                       t->staging_slices > (1 << 24)))
        return PSA_ERR_INVALID_ARG;
    if (d->num_pages < 1) return PSA_ERR_INVALID_ARG;
    if (t->slice_base < 0 || t->slice_base + (long long)d->num_pages * d->num_kv_heads > t->total_slices)
        return PSA_ERR_INVALID_ARG;
    *out = *d;
    const void *pools[2] = {d->k_pool, d->v_pool};
    const void *resolved[2] = {nullptr, nullptr};
    for (int i = 0; i < 2; ++i) {
        if (!pools[i]) continue;                       // (num_pages == 0)
        hipPointerAttribute_t attr;
        if (hipPointerGetAttributes(&attr, pools[i]) != hipSuccess) {
            (void)hipGetLastError();
            return PSA_ERR_INVALID_ARG;
        }
        if (attr.type != hipMemoryTypeHost && attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged)
            return PSA_ERR_INVALID_ARG;
        if (!attr.devicePointer) return PSA_ERR_INVALID_ARG;
        resolved[i] = attr.devicePointer;
    }
    out->k_pool = resolved[0];
    out->v_pool = resolved[1];
    return PSA_OK;
}

}  // namespace

extern "C" {

const char *psa_status_string(psa_status s) {
    switch (s) {
        case PSA_OK: return "PSA_OK";
        case PSA_ERR_INVALID_ARG: return "PSA_ERR_INVALID_ARG";
        case PSA_ERR_UNSUPPORTED: return "PSA_ERR_UNSUPPORTED";
        case PSA_ERR_WORKSPACE_TOO_SMALL: return "PSA_ERR_WORKSPACE_TOO_SMALL";
        case PSA_ERR_LAUNCH: return "PSA_ERR_LAUNCH";
    }
    return "PSA_ERR_UNKNOWN";
}

size_t psa_decode_workspace_bytes(const psa_kv_desc *d, const psa_tuning *tuning) {
    if (check_desc(d, false, false) != PSA_OK) return 0;
    if (d->max_blocks_per_seq > psa::kMaxBlocks) return 0;
    return psa::decode_workspace_bytes_plan(d, psa::make_plan(d, tuning));
}

size_t psa_dense_workspace_bytes(const psa_kv_desc *d) {
    if (check_desc(d, false, false) != PSA_OK) return 0;
    return psa::dense_workspace_bytes(d);
}

psa_status psa_build_block_metadata(const psa_kv_desc *d, void *meta, const int32_t *page_fill,
                                    const int32_t *page_list, int32_t num_listed, void *stream) {
    psa_status st = check_desc(d, false, false);
    if (st != PSA_OK) return st;
    psa_kv_desc tiered;
    if (d->tier) {      // pools in host memory: the kernels read them over the host link
        if ((st = check_tier(d, &tiered)) != PSA_OK) return st;
        d = &tiered;
    }
    if (!meta && d->num_pages > 0) return PSA_ERR_INVALID_ARG;
    if (num_listed < 0 || (num_listed > 0 && !page_list)) return PSA_ERR_INVALID_ARG;
    if ((long long)d->num_pages * d->num_kv_heads > INT32_MAX) return PSA_ERR_UNSUPPORTED;
    if (page_list && num_listed == 0) return PSA_OK;
    hipError_t e = psa::launch_metadata(d, meta, page_fill, page_list, num_listed, (hipStream_t)stream);
    return e == hipSuccess ? PSA_OK : PSA_ERR_LAUNCH;
}

psa_status psa_build_block_means(const psa_kv_desc *d, void *means, const int32_t *page_fill,
                                 const int32_t *page_list, int32_t num_listed, void *stream) {
    psa_status st = check_desc(d, false, false);
    if (st != PSA_OK) return st;
    psa_kv_desc tiered;
    if (d->tier) {      // pools in host memory: the kernel reads them over the host link
        if ((st = check_tier(d, &tiered)) != PSA_OK) return st;
        d = &tiered;
    }
    if (!means && d->num_pages > 0) return PSA_ERR_INVALID_ARG;
    if (num_listed < 0 || (num_listed > 0 && !page_list)) return PSA_ERR_INVALID_ARG;
    if ((long long)d->num_pages * d->num_kv_heads > INT32_MAX) return PSA_ERR_UNSUPPORTED;
    if (page_list && num_listed == 0) return PSA_OK;
    hipError_t e = psa::launch_means(d, means, page_fill, page_list, num_listed, (hipStream_t)stream);
    return e == hipSuccess ? PSA_OK : PSA_ERR_LAUNCH;
}

psa_status psa_append_kv(const psa_kv_desc *d, const void *k_new, const void *v_new, void *meta,
                         int32_t *status, void *stream) {
    psa_status st = check_desc(d, true, true);
    if (st != PSA_OK) return st;
    psa_kv_desc tiered;
    if (d->tier) {
        if ((st = check_tier(d, &tiered)) != PSA_OK) return st;
        d = &tiered;
    }
    if (d->batch == 0) return PSA_OK;
    if (!k_new || !v_new || !meta) return PSA_ERR_INVALID_ARG;
    hipError_t e = psa::launch_append(d, k_new, v_new, meta, status, (hipStream_t)stream);
    return e == hipSuccess ? PSA_OK : PSA_ERR_LAUNCH;
}

static psa_status decode_common(const psa_kv_desc *d, const void *q, const void *meta, float threshold,
                                int32_t check_granularity, int32_t budget_blocks, int32_t scorer, float *out, int32_t *n_selected,
                                float *mass_est, int32_t *blocks_read, float *lse_out, int32_t *order_out,
                                float *scores_out, int32_t *traffic_out, const psa_tuning *tuning,
                                void *workspace, size_t workspace_bytes, void *stream) {
    psa_status st = check_desc(d, true, true);
    if (st != PSA_OK) return st;
    if (!(threshold >= 0.0f && threshold <= 1.0f)) return PSA_ERR_INVALID_ARG;   // also rejects NaN
    if (check_granularity < 1) return PSA_ERR_INVALID_ARG;
    if (scorer != PSA_SCORE_UPPER_BOUND && scorer != PSA_SCORE_CUBOID_CENTER && scorer != PSA_SCORE_MEAN_KEY)
        return PSA_ERR_INVALID_ARG;
    if (d->max_blocks_per_seq > psa::kMaxBlocks) return PSA_ERR_UNSUPPORTED;
    if (tuning) {
        const int cb = tuning->chunk_blocks;
        if (cb != 0 && (cb < 8 || cb > psa::kMaxChunkBlocks || cb % 4 != 0)) return PSA_ERR_INVALID_ARG;
        if (tuning->window_chunks < 0 || tuning->spin_limit < 0) return PSA_ERR_INVALID_ARG;
        if (tuning->force_bitonic < 0 || tuning->force_bitonic > 1) return PSA_ERR_INVALID_ARG;
    }
    psa_kv_desc tiered;
    if (d->tier) {
        if ((st = check_tier(d, &tiered)) != PSA_OK) return st;
        d = &tiered;
    }
    if (d->batch == 0) return PSA_OK;
    if (!q || !out || !n_selected || !mass_est || !workspace) return PSA_ERR_INVALID_ARG;
    if (d->num_pages > 0 && !meta) return PSA_ERR_INVALID_ARG;
    const psa::DecodePlan plan = psa::make_plan(d, tuning);
    if (workspace_bytes < psa::decode_workspace_bytes_plan(d, plan)) return PSA_ERR_WORKSPACE_TOO_SMALL;
    psa::DecodeArgs a;
    a.q = q; a.meta = meta; a.threshold = threshold; a.check_granularity = check_granularity;
    a.out = out; a.n_selected = n_selected; a.mass_est = mass_est; a.blocks_read = blocks_read; a.lse_out = lse_out;
    a.order_out = order_out; a.scores_out = scores_out; a.traffic_out = traffic_out;
    a.budget_blocks = budget_blocks; a.scorer = scorer;
    hipError_t e = psa::launch_decode(d, a, plan, workspace, (hipStream_t)stream);
    return e == hipSuccess ? PSA_OK : PSA_ERR_LAUNCH;
}

psa_status psa_decode_attention(const psa_kv_desc *d, const void *q, const void *meta, float threshold,
                                int32_t check_granularity, int32_t scorer, float *out, int32_t *n_selected,
                                float *mass_est, int32_t *blocks_read, float *lse_out, int32_t *order_out,
                                float *scores_out, int32_t *traffic_out, const psa_tuning *tuning,
                                void *workspace, size_t workspace_bytes, void *stream) {
    return decode_common(d, q, meta, threshold, check_granularity, 0, scorer, out, n_selected, mass_est, blocks_read,
                         lse_out, order_out, scores_out, traffic_out, tuning, workspace, workspace_bytes, stream);
}

// A fixed budget of k blocks is Algorithm 1 with threshold 0 tested once every k blocks: P_acc > 0
// holds at the first test, so every head stops at min(k, N); the key read-ahead ends there too.
psa_status psa_topk_attention(const psa_kv_desc *d, const void *q, const void *meta, int32_t k_blocks,
                              int32_t scorer, float *out, int32_t *n_selected, float *mass_est, int32_t *blocks_read,
                              float *lse_out, int32_t *order_out, float *scores_out, int32_t *traffic_out,
                              const psa_tuning *tuning, void *workspace, size_t workspace_bytes, void *stream) {
    if (k_blocks < 1) return PSA_ERR_INVALID_ARG;
    return decode_common(d, q, meta, 0.0f, k_blocks, k_blocks, scorer, out, n_selected, mass_est, blocks_read,
                         lse_out, order_out, scores_out, traffic_out, tuning, workspace, workspace_bytes, stream);
}

// ---- the entry point that allocates nothing ------------------------------------------------------------
// Its workspace is this array: device memory that belongs to the loaded library, one copy per GPU, there
// until the process ends.  In host code the array's NAME is only a handle for the runtime's symbol table,
// not a device address: the address on the current GPU comes from hipGetSymbolAddress (once per device),
// and only that pointer is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[PSA_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];      // per device: where `scratch` lives there; NULL = not asked yet
std::mutex g_scratch_mutex;

// The current device's copy of `scratch`.
psa_status static_scratch(void **ptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PSA_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return PSA_ERR_LAUNCH;
        }
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return PSA_OK;
}

__global__ void copy_error_word_kernel(const int32_t *header, int32_t *dst) { *dst = header[1]; }
}  // namespace

psa_status psa_decode_attention_static(const psa_kv_desc *d, const void *q, const void *meta, float threshold,
                                       int32_t check_granularity, int32_t scorer, float *out, int32_t *n_selected,
                                       float *mass_est, int32_t *blocks_read, float *lse_out, int32_t *order_out,
                                       int32_t *device_error_out, const psa_tuning *tuning, void *stream) {
    // the size first: a shape that does not fit is refused before anything touches the GPU
    psa_status st = check_desc(d, true, true);
    if (st != PSA_OK) return st;
    if (d->tier) return PSA_ERR_UNSUPPORTED;
    if (d->max_blocks_per_seq > psa::kMaxBlocks) return PSA_ERR_UNSUPPORTED;
    if (tuning) {
        const int cb = tuning->chunk_blocks;
        if (cb != 0 && (cb < 8 || cb > psa::kMaxChunkBlocks || cb % 4 != 0)) return PSA_ERR_INVALID_ARG;
    }
    if (psa::decode_workspace_bytes_plan(d, psa::make_plan(d, tuning)) > (size_t)PSA_STATIC_SCRATCH_BYTES)
        return PSA_ERR_WORKSPACE_TOO_SMALL;
    if (d->batch == 0) return PSA_OK;
    void *ws = nullptr;
    if ((st = static_scratch(&ws)) != PSA_OK) return st;
    st = decode_common(d, q, meta, threshold, check_granularity, 0, scorer, out, n_selected, mass_est, blocks_read,
                       lse_out, order_out, nullptr, nullptr, tuning, ws, (size_t)PSA_STATIC_SCRATCH_BYTES, stream);
    if (st == PSA_OK && device_error_out) {
        copy_error_word_kernel<<<1, 1, 0, (hipStream_t)stream>>>(static_cast<const int32_t *>(ws), device_error_out);
        if (hipGetLastError() != hipSuccess) return PSA_ERR_LAUNCH;
    }
    return st;
}

psa_status psa_dense_attention(const psa_kv_desc *d, const void *q, float *out, float *lse,
                               void *workspace, size_t workspace_bytes, void *stream) {
    psa_status st = check_desc(d, true, true);
    if (st != PSA_OK) return st;
    psa_kv_desc tiered;
    if (d->tier) {      // the control reads every slice from where the pools are, slots play no part
        if ((st = check_tier(d, &tiered)) != PSA_OK) return st;
        d = &tiered;
    }
    if (d->batch == 0) return PSA_OK;
    if (!q || !out || !workspace) return PSA_ERR_INVALID_ARG;
    if (workspace_bytes < psa::dense_workspace_bytes(d)) return PSA_ERR_WORKSPACE_TOO_SMALL;
    hipError_t e = psa::launch_dense(d, q, out, lse, workspace, (hipStream_t)stream);
    return e == hipSuccess ? PSA_OK : PSA_ERR_LAUNCH;
}

size_t psa_tier_state_bytes(int64_t total_slices, int64_t num_slots) {
    if (total_slices < 1 || total_slices > INT32_MAX || num_slots < 1 || num_slots > PSA_TIER_MAX_SLOTS) return 0;
    return psa::tier_state_bytes(total_slices, num_slots);
}

size_t psa_tier_staging_bytes(int64_t staging_slices) {
    if (staging_slices < 1 || staging_slices > (1 << 24)) return 0;
    return psa::tier_staging_bytes(staging_slices);
}

psa_status psa_tier_init(const psa_tier *tier, void *stream) {
    if (!tier || !tier->state || (reinterpret_cast<uintptr_t>(tier->state) & 255u)) return PSA_ERR_INVALID_ARG;
    if (psa_tier_state_bytes(tier->total_slices, tier->num_slots) == 0) return PSA_ERR_INVALID_ARG;
    if (tier->staging && (reinterpret_cast<uintptr_t>(tier->staging) & 255u)) return PSA_ERR_INVALID_ARG;
    return psa::launch_tier_init(tier, (hipStream_t)stream) == hipSuccess ? PSA_OK : PSA_ERR_LAUNCH;
}

size_t psa_tier_update_workspace_bytes(const psa_kv_desc *d) {
    if (check_desc(d, false, false) != PSA_OK || !d->tier) return 0;
    if (psa_tier_state_bytes(d->tier->total_slices, d->tier->num_slots) == 0) return 0;
    return psa::tier_update_workspace_bytes(d);
}

psa_status psa_tier_update(const psa_kv_desc *d, const int32_t *order, const int32_t *blocks_read,
                           int64_t busy_first, int64_t busy_count, int32_t *stats_out, void *workspace,
                           size_t workspace_bytes, void *stream) {
    psa_status st = check_desc(d, true, true);
    if (st != PSA_OK) return st;
    psa_kv_desc tiered;
    if ((st = check_tier(d, &tiered)) != PSA_OK) return st;
    if (busy_count < 0) return PSA_ERR_INVALID_ARG;
    if (tiered.batch == 0) return PSA_OK;
    if (!order || !blocks_read || !workspace) return PSA_ERR_INVALID_ARG;
    if ((long long)tiered.batch * tiered.num_kv_heads * tiered.max_blocks_per_seq > INT32_MAX) return PSA_ERR_UNSUPPORTED;
    if (workspace_bytes < psa::tier_update_workspace_bytes(&tiered)) return PSA_ERR_WORKSPACE_TOO_SMALL;
    hipError_t e = psa::launch_tier_update(&tiered, order, blocks_read, busy_first, busy_count, stats_out, workspace,
                                           (hipStream_t)stream);
    return e == hipSuccess ? PSA_OK : PSA_ERR_LAUNCH;
}

psa_status psa_read_device_error(const void *workspace, int32_t *host_flags, void *stream) {
    if (!workspace || !host_flags) return PSA_ERR_INVALID_ARG;
    // word 1 of the workspace header holds the sticky bits
    hipError_t e = hipMemcpyAsync(host_flags, static_cast<const int32_t *>(workspace) + 1, sizeof(int32_t),
                                  hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    return e == hipSuccess ? PSA_OK : PSA_ERR_LAUNCH;
}

}  // extern "C"
