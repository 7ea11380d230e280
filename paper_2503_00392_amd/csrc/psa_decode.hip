// Host side of psa_decode_attention: workspace layout, launch plan and the kernel sequence
//   score (Algorithm 1 line 5) -> order (line 6) -> select (lines 7-18, key side and stop rule) ->
//   attend (value side of lines 10-12) -> finalize (line 19),
// all enqueued on one stream with no host involvement in between.
#include "psa_host.h"

namespace psa {

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Compute units of the current device (256 on MI355X); read once.
int compute_units() {
    static int cached = 0;
    if (cached == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cached = n;
    }
    return cached;
}

DecodePlan make_plan(const psa_kv_desc *d, const psa_tuning *t) {
    DecodePlan p;
    const int S = d->batch * d->num_kv_heads;
    p.chunk_blocks = (t && t->chunk_blocks) ? t->chunk_blocks : 32;
    if (t && t->window_chunks > 0) {
        p.window_chunks = t->window_chunks;
    } else {
        // about 96 MiB of key slices inside the streams' windows together (the chip holds 1024 workgroups of this
        // kernel, one 128 KiB chunk each; three quarters of that measured best: the fold widens the windows of the
        // streams that stay open longest), 2 to 24 chunks per stream
        const long long per_stream = (96ll << 20) / ((long long)(S > 0 ? S : 1) * p.chunk_blocks * kSliceBytes);
        p.window_chunks = per_stream < 2 ? 2 : (per_stream > 24 ? 24 : (int)per_stream);
    }
    p.spin_limit = (t && t->spin_limit > 0) ? t->spin_limit : (1 << 14);
    p.max_chunks = (d->max_blocks_per_seq + p.chunk_blocks - 1) / p.chunk_blocks;
    if (p.max_chunks < 1) p.max_chunks = 1;
    p.force_bitonic = t ? t->force_bitonic : 0;
    p.depth_hint = t ? t->depth_hint : nullptr;
    p.events = t ? static_cast<hipEvent_t *>(t->phase_events) : nullptr;
    return p;
}

struct WsLayout {
    size_t header, ctl, scores, order, ranked_page, agg, block_lse, logits, partial, value_items, total;
};

static WsLayout layout(const psa_kv_desc *d, const DecodePlan &p) {
    const size_t S = (size_t)d->batch * d->num_kv_heads;
    const size_t G = (size_t)(d->num_q_heads / d->num_kv_heads);
    const size_t MB = (size_t)d->max_blocks_per_seq;
    WsLayout L;
    size_t at = 0;
    L.header = at;      at = align_up(at + 512, 256);
    L.ctl = at;         at = align_up(at + S * sizeof(StreamCtl), 256);
    L.scores = at;      at = align_up(at + S * MB * 4, 256);
    L.order = at;       at = align_up(at + S * MB * 4, 256);
    L.ranked_page = at; at = align_up(at + S * MB * 4, 256);
    L.agg = at;         at = align_up(at + S * p.max_chunks * G * 8, 256);
    L.block_lse = at;   at = align_up(at + S * MB * G * 4, 256);
    L.logits = at;      at = align_up(at + S * MB * kPage * G * 4, 256);
    L.partial = at;     at = align_up(at + S * p.max_chunks * G * kPartialStride * 4, 256);
    L.value_items = at; at = align_up(at + S * p.max_chunks * 4, 256);
    L.total = at;
    return L;
}

size_t decode_workspace_bytes_plan(const psa_kv_desc *d, const DecodePlan &p) { return layout(d, p).total; }

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
    ws.block_lse = reinterpret_cast<float *>(base + L.block_lse);
    ws.logits = reinterpret_cast<float *>(base + L.logits);
    ws.partial = reinterpret_cast<float *>(base + L.partial);
    ws.value_items = reinterpret_cast<int32_t *>(base + L.value_items);
    ws.max_chunks = plan.max_chunks;
    ws.max_units = plan.max_chunks;
    const int G = d->num_q_heads / d->num_kv_heads;
    if (kv.batch == 0) return hipSuccess;
    hipEvent_t *ev = plan.events;
    hipError_t e;
    if (ev) (void)hipEventRecord(ev[0], st);
    if ((e = launch_score(kv, d->dtype, G, a.scorer, a.q, a.meta, ws, a.scores_out, st)) != hipSuccess) return e;
    if (ev) (void)hipEventRecord(ev[1], st);
    if ((e = launch_order(kv, ws, G, plan, a.budget_blocks, a.order_out, st)) != hipSuccess) return e;
    if (d->tier && (e = launch_tier_resolve(kv, d->tier, ws.ranked_page, st)) != hipSuccess) return e;
    if (ev) (void)hipEventRecord(ev[2], st);
    if ((e = launch_select(kv, d->dtype, G, a.q, ws, a.threshold, a.check_granularity, a.budget_blocks, plan, st)) != hipSuccess)
        return e;
    if (ev) (void)hipEventRecord(ev[3], st);
    if ((e = launch_attend(kv, d->dtype, G, ws, plan, st)) != hipSuccess) return e;
    if (ev) (void)hipEventRecord(ev[4], st);
    e = launch_finalize(kv, ws, G, plan.chunk_blocks, a.out, a.n_selected, a.mass_est, a.blocks_read, a.lse_out,
                        a.traffic_out, st);
    if (ev) (void)hipEventRecord(ev[5], st);
    return e;
}

}  // namespace psa
