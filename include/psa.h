/*
 * psa.h -- C ABI of the MI355X (gfx950) Progressive Sparse Attention decode library.
 *
 * The calls follow the paper's statement of the problem (arxiv 2503.00392): a decode-step query
 * attends a paged KV cache, blocks are scored from small per-block key metadata, ranked, and pulled
 * in that order into an exact attention accumulation until the accumulated attention weight passes
 * a threshold (Algorithm 1, Sec. 3.2).
 *
 * Conventions common to every call
 *   - Every pointer is a DEVICE pointer unless its comment says "host" (with a second tier the KV
 *     pools are host memory the GPU can address, see psa_tier).
 *   - The caller owns every buffer, the workspace included.  The library allocates no device
 *     memory and keeps no state between calls (the optional second tier keeps its tables in a
 *     buffer the caller owns, psa_tier.state); calls on distinct streams with distinct workspaces
 *     may overlap, calls sharing a workspace must be ordered by the stream.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Calls validate their arguments on the host, enqueue kernels and return.  No call
 *     synchronises the stream or copies to the host, except psa_read_device_error.  Outputs are
 *     valid once the caller has synchronised the stream.
 *   - Errors are return codes.  On any code other than PSA_OK nothing has been enqueued.
 *     What the host can see is checked there (null required pointer, shapes, threshold outside
 *     [0,1] or NaN, check_granularity < 1, workspace too small).  What only the device can see
 *     (a block-table entry outside [0,num_pages), a context longer than max_blocks_per_seq pages,
 *     a negative context length) is clamped by the kernels, which set a sticky bit in the workspace that psa_read_device_error returns.
 *   - Element type of Q, K, V and metadata: IEEE binary16 or bfloat16, 2 bytes.
 *   - Supported shapes: head_dim == 128, page_size == 16, num_q_heads / num_kv_heads in
 *     {1, 2, 4, 8}, max_blocks_per_seq <= 8192 for psa_decode_attention (128K tokens).
 *     Anything else returns PSA_ERR_UNSUPPORTED.
 */
#ifndef PSA_H
#define PSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PSA_OK = 0,
    PSA_ERR_INVALID_ARG = 1,
    PSA_ERR_UNSUPPORTED = 2,
    PSA_ERR_WORKSPACE_TOO_SMALL = 3,
    PSA_ERR_LAUNCH = 4
} psa_status;

typedef enum { PSA_F16 = 0, PSA_BF16 = 1 } psa_dtype;

/* Bits of the sticky device error word (psa_read_device_error). */
enum {
    PSA_DEVERR_PAGE_RANGE = 1,   /* block-table entry outside [0, num_pages): page 0 was used   */
    PSA_DEVERR_CTX_RANGE = 2,    /* ctx_len < 0 or > 16*max_blocks_per_seq: clamped             */
    PSA_DEVERR_STALLED = 4       /* the stop rule of a (request, KV head) gave up waiting for keys (seconds):
                                    its query heads' results are not valid.  Not expected to happen           */
};

/* How a block's criticality score is computed from its metadata (Algorithm 1, line 5: CS = q . B_meta).
 * Both read the same per-channel min/max metadata and take the maximum over the query heads that
 * share the KV head.
 *   PSA_SCORE_UPPER_BOUND    sum_c max(q_c kmin_c, q_c kmax_c) / sqrt(d): the largest scaled logit any
 *                            key inside the block's bounding cuboid can give (default)
 *   PSA_SCORE_CUBOID_CENTER  q . (kmin + kmax)/2 / sqrt(d): the scaled logit of the cuboid's centre, a
 *                            reading of the "cuboid-mean" metadata Sec. 3.1 names as its default
 *   PSA_SCORE_MEAN_KEY       q . mean / sqrt(d) over mean-key metadata (psa_build_block_means: one vector
 *                            per block, half the bytes of the cuboid): the mean of the block's scaled
 *                            logits.  Sec. 2.2 lists per-block vectors derived from the keys as what
 *                            selection algorithms score by; this is the smallest of them.  The `meta`
 *                            argument of the attention calls is then the means buffer.                */
typedef enum { PSA_SCORE_UPPER_BOUND = 0, PSA_SCORE_CUBOID_CENTER = 1, PSA_SCORE_MEAN_KEY = 2 } psa_scorer;

/*
 * Optional second tier (Sec. 3.1 KV cache manager, Sec. 3.4 unified memory management).  With a tier the
 * pools of a psa_kv_desc live in HOST memory that the GPU can address (pinned, e.g. hipHostMalloc), and
 * the GPU caches (page, KV head) "slices" -- one 4 KiB key slice and one 4 KiB value slice -- in ONE pool
 * of slots shared by all layers.  A slice has a global id: slice_base + page * num_kv_heads + h; the
 * layers that share a pool use disjoint id ranges inside [0, total_slices).
 * psa_decode_attention / psa_topk_attention read a slice from its slot if it has one and straight from
 * host memory (over the host link) if not; results do not depend on where a slice was read from.
 * psa_tier_update brings the pool up to date after a call (least recently used goes first).
 *   state      device, psa_tier_state_bytes(total_slices, num_slots) bytes, 256-byte aligned; the library's own
 *              tables (slice -> slot, slot -> slice, slot -> time of last use, clock); set up by
 *              psa_tier_init, owned by the caller, shared by every descriptor that names this pool
 *   slot_pool  device, num_slots * 8192 bytes, 16-byte aligned: slot s holds a key slice at s * 8192 and a
 *              value slice at s * 8192 + 4096, each [page_size][head_dim]
 *   staging    device or NULL, psa_tier_staging_bytes(staging_slices) bytes, 256-byte aligned, its first 256
 *              bytes zero before its first use: where the attention kernels leave a copy of every slice they
 *              read from host memory, so that the psa_tier_update that follows moves it into its slot from GPU
 *              memory and the slice crosses the host link once, not twice (Sec. 3.3 loads a missing block
 *              once).  Slices beyond staging_slices are simply fetched again by the update.  Unlike state and
 *              slot_pool this buffer belongs to ONE descriptor at a time: between a decode call that names it
 *              and the psa_tier_update of the same descriptor (which empties it) no other descriptor may use
 *              it, and the cache must not be appended to.  Layers whose attention and update overlap (two
 *              streams) alternate between two such buffers.  NULL: every missing slice is fetched by the update.
 */
#define PSA_TIER_MAX_SLOTS (1 << 26)   /* 512 GiB of slots: more than any GPU holds */
typedef struct {
    void *state;
    void *slot_pool;
    int64_t total_slices;       /* 1 .. 2^31 - 1                                                   */
    int64_t num_slots;          /* 1 .. PSA_TIER_MAX_SLOTS                                         */
    int64_t slice_base;         /* id of this descriptor's page 0, KV head 0                       */
    void *staging;              /* or NULL                                                         */
    int64_t staging_slices;     /* 1 .. 2^24 entries of 8 KiB (ignored without staging)            */
} psa_tier;

/* Shapes and layout of ONE layer's paged KV cache (PagedAttention layout, Sec. 2.1 "KV Cache"). */
typedef struct {
    int32_t batch;              /* decode requests, one query token each                          */
    int32_t num_q_heads;        /* Hq                                                             */
    int32_t num_kv_heads;       /* Hkv; Hq % Hkv == 0; G = Hq / Hkv query heads share a KV head   */
    int32_t head_dim;           /* d, must be 128                                                 */
    int32_t page_size;          /* tokens per KV block, must be 16                                */
    int32_t num_pages;          /* physical pages in each pool                                    */
    int32_t max_blocks_per_seq; /* row stride of block_table, >= 1 for the attention calls        */
    int32_t dtype;              /* psa_dtype of Q, K, V and metadata                              */
    const void *k_pool;         /* [num_pages][num_kv_heads][page_size][head_dim]                 */
    const void *v_pool;         /* same layout                                                    */
    const int32_t *block_table; /* [batch][max_blocks_per_seq]: logical block -> physical page    */
    const int32_t *ctx_lens;    /* [batch]: tokens of each request; need not be a multiple of 16  */
    const psa_tier *tier;       /* host pointer or NULL.  NULL: k_pool and v_pool are device memory and
                                   hold everything.  Otherwise they are GPU-addressable host memory and
                                   the slot pool caches slices of them (see psa_tier)              */
} psa_kv_desc;

/* Tuning knobs of psa_decode_attention; all zero = library defaults.  They change how much is read
 * speculatively and how work is cut, never which blocks are selected. */
typedef struct {
    int32_t chunk_blocks;   /* ranked blocks per work item: a multiple of 4 in 8..64 (default 32)      */
    int32_t window_chunks;  /* least number of chunks of one (request, KV head) read beyond the chunks
                               already folded into the stop rule; the window grows to a quarter of the
                               folded count, and to this number times the (request, KV head) pairs of the
                               call divided by those not yet finished, at most 256 (default: 96 MiB of
                               keys over all pairs, 2 to 24 chunks)                                    */
    int32_t spin_limit;     /* looks (about a microsecond apart) a workgroup takes at the window before it
                               reads its chunk regardless (default 1<<14); the wait only limits read-ahead  */
    int32_t force_bitonic;  /* 1: always rank with the bitonic network (testing); 0: automatic        */
    const int32_t *depth_hint; /* device pointer or NULL: [batch][num_kv_heads] blocks each (request, KV head)
                               is expected to need, e.g. blocks_read of the previous decode step of the
                               same layer (consecutive decode queries select similar sets).  The chunks
                               that cover it, plus a margin of a sixteenth and two chunks, are read at once
                               instead of window by window; a wrong hint costs time or traffic, never
                               correctness                                                            */
    void *phase_events;     /* host pointer: NULL, or hipEvent_t[6] the call records on `stream`
                               before scoring and after each of its kernels: scoring, ranking,
                               selection (key pass), attention (value pass), final merge
                               (profiling aid)                                                        */
} psa_tuning;

/* Bytes of workspace psa_decode_attention needs for this descriptor and tuning (NULL = defaults);
 * 0 on an invalid or unsupported descriptor. */
size_t psa_decode_workspace_bytes(const psa_kv_desc *desc, const psa_tuning *tuning);

/* Bytes of workspace psa_dense_attention needs for this descriptor (0 on an invalid one). */
size_t psa_dense_workspace_bytes(const psa_kv_desc *desc);

/*
 * Block metadata (Sec. 2.2 "KV Cache Selection": per-block vectors derived from the block's keys;
 * here the bounding cuboid, i.e. per-channel minimum and maximum; Sec. 3.1: created when a block
 * reaches capacity and kept in GPU memory).
 *   meta       out [num_pages][num_kv_heads][2][head_dim], desc->dtype; [..][0] = min, [..][1] = max.
 *              Exact: each entry is one of the block's own key bit patterns (-0 orders below +0).
 *   page_fill  [num_pages] valid tokens of each page (0..16), or NULL = every page is full.
 *              A page with 0 valid tokens gets min = max = +0.
 *   page_list  [num_listed] physical pages to (re)build, or NULL = all num_pages pages.  This is
 *              the per-step form: the pages that filled since the last decode step.
 * Only desc->k_pool, num_pages, num_kv_heads, head_dim, page_size and dtype are read.
 */
psa_status psa_build_block_metadata(const psa_kv_desc *desc, void *meta, const int32_t *page_fill,
                                    const int32_t *page_list, int32_t num_listed, void *stream);

/*
 * Incremental decode: appends one token per request to the paged cache and keeps the block metadata
 * current (Sec. 3.1: metadata is created on the GPU as a block fills).  For request r with length
 * c = ctx_lens[r] the token goes to slot c % 16 of page block_table[r][c / 16]; that page's metadata
 * becomes the min/max over its c % 16 + 1 valid tokens (bit for bit what psa_build_block_metadata
 * gives on the new cache); ctx_lens[r] becomes c + 1.
 *   desc     the call WRITES desc->k_pool, desc->v_pool and desc->ctx_lens (declared const in the
 *            struct because every other call only reads them); the block table must already hold a
 *            page for position c
 *   k_new    [batch][num_kv_heads][head_dim], desc->dtype: the new token's keys; v_new likewise
 *   meta     [num_pages][num_kv_heads][2][head_dim], updated in place
 *   status   [batch] int32 or NULL: 0 = appended; PSA_DEVERR_CTX_RANGE = the request's row of the
 *            block table is full (or its length is negative); PSA_DEVERR_PAGE_RANGE = the table entry
 *            is outside the pool.  In both cases nothing of that request is touched.
 * Not to be overlapped with another call that uses the same cache.
 */
psa_status psa_append_kv(const psa_kv_desc *desc, const void *k_new, const void *v_new, void *meta,
                         int32_t *status, void *stream);

/*
 * Mean-key metadata for PSA_SCORE_MEAN_KEY (Sec. 2.2 "KV Cache Selection": metadata vectors that stand for a
 * block's keys): per (page, KV head) and channel the mean of the page's valid keys, computed in binary64 and
 * rounded once, to nearest-even, to desc->dtype; a zero mean and a page without valid tokens give +0.
 *   means      out [num_pages][num_kv_heads][head_dim], desc->dtype
 *   page_fill, page_list, num_listed   as for psa_build_block_metadata
 * psa_append_kv does not maintain this buffer (a rounded mean cannot be updated in place exactly): after an
 * append, rebuild the pages that received a token with a page list.
 * Errors: as psa_build_block_metadata.
 */
psa_status psa_build_block_means(const psa_kv_desc *desc, void *means, const int32_t *page_fill,
                                 const int32_t *page_list, int32_t num_listed, void *stream);

/*
 * One decode step of Progressive Sparse Attention for one layer (Algorithm 1; Sec. 3.2 for the
 * microbatch size and for the batched form in which every query stops on its own).
 * Per (request, KV head): score every block from its metadata (line 5: the largest scaled logit
 * q.k/sqrt(d) any key inside [min,max] could give, maximised over the G query heads of the group),
 * rank the blocks (line 6; ties to the smaller logical block), then for each query head walk the
 * ranking, merging exact softmax attention block by block (lines 10-12) and stopping at the first
 * n that is a multiple of check_granularity (or the last block) where
 *   P_acc = AS_acc / (AS_acc + AS_min * N_left) > threshold            (lines 13-18).
 *   q            [batch][num_q_heads][head_dim], desc->dtype
 *   meta         as written by psa_build_block_metadata (pages' valid-token counts included); with
 *                PSA_SCORE_MEAN_KEY as written by psa_build_block_means
 *   threshold    epsilon in [0,1]; 1 never stops early, so the result is dense attention
 *   check_granularity  m >= 1 (Sec. 3.2 "microbatch")
 *   out          [batch][num_q_heads][head_dim] float32
 *   n_selected   [batch][num_q_heads] blocks attended by that query head (a prefix of the ranking)
 *   mass_est     [batch][num_q_heads] float32, P_acc at the stop (1 if every block was used)
 *   blocks_read  [batch][num_kv_heads] max of n_selected over the group; may be NULL
 *   lse_out      [batch][num_q_heads] float32, natural log of the sum of exp(scaled logit) over the
 *                tokens of the attended blocks (-inf for an empty request): what a caller needs to merge
 *                `out` with attention over other tokens, and, against psa_dense_attention's lse, the
 *                true share of the attention mass the selection holds; may be NULL
 *   order_out    [batch][num_kv_heads][max_blocks_per_seq] the ranking (logical blocks, -1 beyond
 *                the request's block count); may be NULL
 *   scores_out   [batch][num_kv_heads][max_blocks_per_seq] float32 criticality scores by logical
 *                block (untouched beyond the block count); may be NULL
 *   traffic_out  [batch][num_kv_heads][2] key slices and value slices actually loaded (keys are read
 *                a bounded window ahead of the stop, values only for selected blocks); may be NULL
 *   tuning       NULL = defaults
 * A request with ctx_len 0 gets out = 0, n_selected = 0, mass_est = 0.
 */
psa_status psa_decode_attention(const psa_kv_desc *desc, const void *q, const void *meta,
                                float threshold, int32_t check_granularity, int32_t scorer, float *out,
                                int32_t *n_selected, float *mass_est, int32_t *blocks_read,
                                float *lse_out, int32_t *order_out, float *scores_out, int32_t *traffic_out,
                                const psa_tuning *tuning, void *workspace, size_t workspace_bytes,
                                void *stream);

/*
 * psa_decode_attention for callers that cannot allocate device memory and have no workspace to bring: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same results
 * bit for bit as psa_decode_attention with the same arguments; the workspace is an array of
 * PSA_STATIC_SCRATCH_BYTES of device memory inside the library itself (every GPU the library runs on holds
 * its own copy until the process ends).  The call allocates nothing and frees nothing, on the host side of
 * the runtime or the device side; the first call on a GPU looks the array's address up (make that call
 * outside a graph capture).
 *   Arguments as for psa_decode_attention (no scores_out, no traffic_out, no workspace), plus
 *   device_error_out  device int32 or NULL: receives the sticky device error word of the call (an OR of
 *                     PSA_DEVERR_* bits, 0 = none) -- there is no workspace pointer to hand to
 *                     psa_read_device_error
 * Errors: those of psa_decode_attention; PSA_ERR_WORKSPACE_TOO_SMALL if this descriptor and tuning need more
 * than PSA_STATIC_SCRATCH_BYTES (psa_decode_workspace_bytes tells how much: about 43 MiB for 8 requests x 8
 * KV heads x 32K tokens with 4 query heads per KV head); PSA_ERR_UNSUPPORTED with a second tier.
 * All calls on one GPU share that GPU's array, whatever their streams: two calls whose kernels may overlap
 * in time race and give wrong results.  Order them (one stream, or events).  Nothing needs clearing between
 * calls: every call initialises what it reads.
 */
#define PSA_STATIC_SCRATCH_BYTES (64u << 20)
psa_status psa_decode_attention_static(const psa_kv_desc *desc, const void *q, const void *meta,
                                       float threshold, int32_t check_granularity, int32_t scorer, float *out,
                                       int32_t *n_selected, float *mass_est, int32_t *blocks_read,
                                       float *lse_out, int32_t *order_out, int32_t *device_error_out,
                                       const psa_tuning *tuning, void *stream);

/*
 * Fixed-budget control: what block-level dynamic sparse attention does without PSA (Sec. 1, Sec. 2.2
 * "KV Cache Selection": a fixed top-k, e.g. k = 64 or 128 blocks).  Same scoring and ranking as
 * psa_decode_attention; every query head then attends exactly the first min(k_blocks, N) ranked
 * blocks, and keys are read no further than that.  mass_est is P_acc of Algorithm 1 (lines 15-16)
 * evaluated at that point.  All other arguments, the workspace size and the error behaviour are those
 * of psa_decode_attention; k_blocks < 1 is PSA_ERR_INVALID_ARG.
 */
psa_status psa_topk_attention(const psa_kv_desc *desc, const void *q, const void *meta, int32_t k_blocks,
                              int32_t scorer, float *out, int32_t *n_selected, float *mass_est, int32_t *blocks_read,
                              float *lse_out, int32_t *order_out, float *scores_out, int32_t *traffic_out,
                              const psa_tuning *tuning, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Dense control: exact softmax attention over every block of the same paged layout
 * (Sec. 2.1: S = QK^T/sqrt(d), P = softmax(S), O = PV).
 *   out  [batch][num_q_heads][head_dim] float32
 *   lse  [batch][num_q_heads] float32 natural-log sum of exponentiated scaled logits; may be NULL
 */
psa_status psa_dense_attention(const psa_kv_desc *desc, const void *q, float *out, float *lse,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * Two-tier block store (Sec. 3.1, 3.4).  All of it runs on the GPU, on `stream`; the host is not in the loop.
 *
 * psa_tier_state_bytes: bytes of psa_tier.state for these sizes (0 if they are out of range).
 * psa_tier_staging_bytes: bytes of a psa_tier.staging buffer with room for this many slices (0 if out of range).
 * psa_tier_init: empties the pool (no slice has a slot, clock 0) and, if tier->staging is given, that staging
 *   buffer.  Only state, total_slices, num_slots and staging of `tier` are read.
 * psa_tier_update_workspace_bytes: bytes of scratch psa_tier_update needs for this descriptor (0 on an
 *   invalid one or one without a tier).
 * psa_tier_update: after a decode call on `desc` (same stream, or ordered after it), with that call's
 *   `order_out` and `blocks_read`: the slices the attention used -- the first blocks_read[r][h] ranked
 *   blocks of every (request, KV head) -- are marked used now; those without a slot are copied from host
 *   memory into slots, in the order (request, KV head, rank), taking empty slots first (lowest index
 *   first) and then the least recently used (ties: lowest slot index; slots unused for 65535 updates or
 *   more count as equally old).  Not taken: a slot used by this
 *   very update, and a slot whose slice id lies in [busy_first, busy_first + busy_count) -- name there the
 *   id range of the layer whose attention may run at the same time on another stream, whose slots are
 *   being read; busy_count = 0 for none.  If the misses outnumber the slots that may be taken, the first
 *   in that order are placed and the rest stay in host memory.  The clock advances by one per call.
 *   A page shared between two requests of the batch is not supported with a tier (its slices would
 *   be placed twice; nothing faults, one of the two slots is wasted until it ages out).
 *     order        device [batch][num_kv_heads][max_blocks_per_seq] int32, as written by the decode call
 *     blocks_read  device [batch][num_kv_heads] int32, as written by the decode call
 *     stats_out    device int32[5] or NULL: slices used that had a slot, that had none, slices placed,
 *                  slices that lost their slot, slices placed from the staging buffer (the others placed were
 *                  fetched from host memory by the update)
 *   Concurrency: calls that share a state must not overlap each other; a decode call may overlap an
 *   update only if its slices are in the update's busy range and it was enqueued after the previous
 *   update of its own layer completed.
 * Errors: PSA_ERR_INVALID_ARG (NULL pointers, sizes out of range, id range outside [0, total_slices),
 * pools the GPU cannot address), PSA_ERR_WORKSPACE_TOO_SMALL, PSA_ERR_LAUNCH.
 */
size_t psa_tier_state_bytes(int64_t total_slices, int64_t num_slots);
size_t psa_tier_staging_bytes(int64_t staging_slices);
psa_status psa_tier_init(const psa_tier *tier, void *stream);
size_t psa_tier_update_workspace_bytes(const psa_kv_desc *desc);
psa_status psa_tier_update(const psa_kv_desc *desc, const int32_t *order, const int32_t *blocks_read,
                           int64_t busy_first, int64_t busy_count, int32_t *stats_out, void *workspace,
                           size_t workspace_bytes, void *stream);

/*
 * Copies the sticky device error word of a workspace to the host and clears nothing.
 * Synchronises `stream`.  host_flags: host pointer, receives an OR of PSA_DEVERR_* bits.
 */
psa_status psa_read_device_error(const void *workspace, int32_t *host_flags, void *stream);

/* Static, human-readable name of a status code. */
const char *psa_status_string(psa_status status);

#ifdef __cplusplus
}
#endif
#endif /* PSA_H */
