// Shared device-side definitions of the PSA decode kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/psa.h"

namespace psa {

constexpr int kHeadDim = 128;     // channels per head
constexpr int kPage = 16;         // tokens per KV block
constexpr int kRowBytes = 256;    // one token's key (or value) for one head
constexpr int kSliceBytes = 4096; // one (page, KV head) K or V slice
constexpr int kMetaBytes = 512;   // one (page, KV head) metadata record: min[128] | max[128]
constexpr int kMaxBlocks = 8192;  // ranking limit per request (128K tokens)
constexpr int kMaxChunkBlocks = 64;   // key chunk and value unit, in blocks, at most

// 1/sqrt(128) * log2(e): logits are carried in log2 units so that exp is one v_exp_f32.
constexpr float kScaleLog2 = 0.08838834764831845f * 1.4426950408889634f;
constexpr float kScale = 0.08838834764831845f;
constexpr float kLn2 = 0.6931471805599453f;

// Kernel-side view of psa_kv_desc.
struct KvView {
    const uint8_t *k_pool;
    const uint8_t *v_pool;
    const int32_t *block_table;
    const int32_t *ctx_lens;
    int32_t batch, num_q_heads, num_kv_heads, num_pages, max_blocks;
    const uint8_t *slot_pool;   // second tier only: 8 KiB slots (key slice, value slice); else NULL
    // second tier with a staging buffer only (else staging == NULL): where slices read from host memory are
    // left for the update that follows
    uint8_t *staging;           // [256 B: entry counter][staging_cap slice ids][staging_cap x (key slice, value slice)]
    int32_t *staged_at;         // [total_slices] slice id -> staging entry, -1 = none (in the tier's state)
    long long slice_base;       // id of page 0, KV head 0
    int32_t staging_cap;
};

// Layout of a staging buffer.
__host__ __device__ __forceinline__ size_t staging_entries_offset(int cap) {
    return 256 + ((size_t)cap * 4 + 255) / 256 * 256;
}
__device__ __forceinline__ uint32_t *staging_count(uint8_t *st) { return reinterpret_cast<uint32_t *>(st); }
__device__ __forceinline__ int32_t *staging_ids(uint8_t *st) { return reinterpret_cast<int32_t *>(st + 256); }
__device__ __forceinline__ uint8_t *staging_entry(uint8_t *st, int cap, int idx) {
    return st + staging_entries_offset(cap) + (size_t)idx * (2 * 4096);
}

// Kernel-side view of a psa_tier and its state.
struct TierView {
    uint32_t *header;       // [64]: clock and the counters of the update in progress
    int32_t *slot_of;       // [total_slices] slice -> slot, -1 = host memory only
    int32_t *owner;         // [num_slots] slot -> slice, -1 = empty
    uint32_t *stamp;        // [num_slots] clock value of the slot's last use, 0 = never
    uint8_t *slot_pool;
    long long slice_base, total_slices;
    int num_slots;
    int32_t *staged_at;     // [total_slices] slice -> entry of the staging buffer in use, -1 = none
    uint8_t *staging;       // this descriptor's staging buffer or NULL
    int staging_cap;
};

// Where the key slice of ranked block `loc` of KV head h lives: loc >= 0 is a page of the pool, loc < 0
// is ~slot of the second tier's slot pool (whose value slice follows its key slice).
__device__ __forceinline__ const uint8_t *key_slice(const KvView &kv, int loc, int h) {
    return loc >= 0 ? kv.k_pool + ((size_t)loc * kv.num_kv_heads + h) * kSliceBytes
                    : kv.slot_pool + (size_t)(~loc) * (2 * kSliceBytes);
}
__device__ __forceinline__ const uint8_t *value_slice(const KvView &kv, int loc, int h) {
    return loc >= 0 ? kv.v_pool + ((size_t)loc * kv.num_kv_heads + h) * kSliceBytes
                    : kv.slot_pool + (size_t)(~loc) * (2 * kSliceBytes) + kSliceBytes;
}

// A wave that has just read the key slice of (page, KV head h) from host memory -- lane l holds bytes 16 l .. 16 l + 15
// of each of its four 1 KiB rows -- leaves a copy in the staging buffer, for the tier update that follows the call;
// the wave that later reads the value slice adds it to the same entry.  Entries beyond the buffer's capacity are
// not made (the update fetches those slices itself).
__device__ __forceinline__ void stage_key_slice(const KvView &kv, int page, int h, const uint4 (&rows)[4], int lane) {
    int entry = 0;
    if (lane == 0) entry = (int)atomicAdd(staging_count(kv.staging), 1u);
    entry = __builtin_amdgcn_readfirstlane(entry);
    if (entry < 0 || entry >= kv.staging_cap) return;
    uint8_t *e = staging_entry(kv.staging, kv.staging_cap, entry) + lane * 16;
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4 *>(e + i * 1024) = rows[i];
    if (lane == 0) {
        const long long id = kv.slice_base + (long long)page * kv.num_kv_heads + h;
        staging_ids(kv.staging)[entry] = (int)id;
        kv.staged_at[id] = entry;
    }
}
__device__ __forceinline__ void stage_value_slice(const KvView &kv, int page, int h, const uint4 (&rows)[4], int lane) {
    const int entry = kv.staged_at[kv.slice_base + (long long)page * kv.num_kv_heads + h];
    if (entry < 0 || entry >= kv.staging_cap) return;
    uint8_t *e = staging_entry(kv.staging, kv.staging_cap, entry) + kSliceBytes + lane * 16;
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4 *>(e + i * 1024) = rows[i];
}

// ---- workspace of psa_decode_attention -----------------------------------------------------
// "Stream" = one (request, KV head) pair: one ranking, G query heads.
// "Chunk" = `CB` consecutive ranked blocks: the unit in which keys are read and folded into the
// stop rule, and in which values are read.
//
// Per-stream control block of the progressive kernel: three 128-byte lines, so that the progress word
// that waiting workgroups poll, the traffic counter and the heads' stops never share a cache line
// (accesses to one line are served one after the other).
struct alignas(128) StreamCtl {
    // line 0: progress, written by the folding wave only, as ONE 64-bit store; polled by workgroups that
    // wait for the read-ahead window
    unsigned long long key_progress;    // bits 0-15: frontier = key chunks folded into the stop rule so far;
                                        // bits 16-31: the read-ahead window the fold grants beyond the frontier,
                                        // in chunks (0 = the launch's default);
                                        // high word: k_limit = key chunks worth reading (all of them, or what a
                                        // block budget covers, or what the stop rule can still reach; once the
                                        // fold has finished, what it used)
    int32_t pad0[30];
    // line 1: counters
    int32_t k_blocks;   // key slices loaded (traffic accounting)
    int32_t pad1[31];
    // line 2: the fold's result, written when it closes the stream
    unsigned long long stop[8];  // per head: (n << 32) | float bits of P_acc at the stop; ~0 = not stopped
    int32_t pad2[16];
};

struct DecodeWs {
    int32_t *header;        // [128]: word 1 = sticky error bits; word kValueCount (a cache line of its own) =
                            // number of entries of value_items; word kClosedStreams (again its own line) =
                            // streams whose stop rule has finished
    StreamCtl *ctl;         // [S]
    float *scores;          // [S][max_blocks]
    int32_t *order;         // [S][max_blocks]  ranked logical blocks
    int32_t *ranked_page;   // [S][max_blocks]  physical page of each ranked block
    unsigned long long *agg;  // [S][max_chunks][G]  (L_chunk, Lmin_chunk) as two floats, or kAggSentinel
    float *block_lse;       // [S][max_blocks][G]  log2 of each ranked block's AS (Algorithm 1 line 10)
    float *logits;          // [S][max_blocks][G][16]  scaled logits (log2 units) by ranked block; position
                            // 4*r + j of a (block, head) row holds token 4*j + r
    float *partial;         // [S][max_chunks][G][kPartialStride]
    int32_t *value_items;   // [S * max_chunks] value units to attend: stream * max_chunks + chunk, appended by
                            // each stream's fold when it closes the stream
    int32_t max_chunks;     // chunks per stream at most
    int32_t max_units;      // = max_chunks (stride of `partial`)
};
constexpr int kPartialStride = 132;  // M, l, pad, pad, acc[128]
constexpr int kMaxWindowChunks = 256; // chunks read beyond the fold's frontier, at most
constexpr int kValueCount = 32;      // index of the value-item counter in the workspace header
constexpr int kClosedStreams = 64;   // index of the closed-stream counter in the workspace header
// A chunk word holds (L_chunk, Lmin_chunk) as two floats once the chunk is published.  Before that
// it holds a NaN pattern no publisher writes: "not published".
constexpr unsigned long long kAggSentinel = 0xFFFFFFFFFFFFFFFFull;

__device__ __forceinline__ void set_error(int32_t *header, int bit) { atomicOr(&header[1], bit); }

// ---- 16-bit float helpers ------------------------------------------------------------------
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf2_t __attribute__((ext_vector_type(2)));

// acc + a.lo*b.lo + a.hi*b.hi, fp32 accumulate, on packed fp16 (DT 0) or bf16 (DT 1) pairs.
template <int DT>
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float acc) {
    if constexpr (DT == 0) {
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b),
                                      acc, false);
    } else {
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2_t, a),
                                               __builtin_bit_cast(bf2_t, b), acc, false);
    }
}

// D(16x16, fp32) += A(16x32) * B(32x16) on the matrix cores, 16-bit inputs.  Lane l supplies row
// l%16 of A and column l%16 of B, 8 consecutive k values each (k block l/16); it receives column
// l%16 of D, rows 4*(l/16) .. 4*(l/16)+3.
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
// Four floats written once and read once, by a later kernel, and four such floats read (see ld16_stream).
__device__ __forceinline__ void store_stream(float *p, f32x4_t v) {
    __builtin_nontemporal_store(v, reinterpret_cast<f32x4_t *>(p));
}
__device__ __forceinline__ f32x4_t load_stream(const float *p) {
    return __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(p));
}
template <int DT>
__device__ __forceinline__ f32x4_t mfma_16x16x32(const uint4 &a, const uint4 &b, f32x4_t c) {
    if constexpr (DT == 0) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a),
                                                      __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
}

template <int DT>
__device__ __forceinline__ float cvt_lo(uint32_t w) {
    if constexpr (DT == 0) {
        return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu));
    } else {
        return __builtin_bit_cast(float, w << 16);
    }
}
template <int DT>
__device__ __forceinline__ float cvt_hi(uint32_t w) {
    if constexpr (DT == 0) {
        return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
    } else {
        return __builtin_bit_cast(float, w & 0xffff0000u);
    }
}

// ---- cross-lane helpers ----------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
// Sum over the 16 lanes of a DPP row; every lane of the row gets the total.
__device__ __forceinline__ float row_sum16(float v) {
    v += dpp_f<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_f<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_f<0x141>(v);  // row_half_mirror
    v += dpp_f<0x140>(v);  // row_mirror
    return v;
}

// Maximum over the 16 lanes of a DPP row; every lane of the row gets it.
__device__ __forceinline__ float row_max16(float v) {
    v = fmaxf(v, dpp_f<0xB1>(v));
    v = fmaxf(v, dpp_f<0x4E>(v));
    v = fmaxf(v, dpp_f<0x141>(v));
    v = fmaxf(v, dpp_f<0x140>(v));
    return v;
}

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float log2_fast(float x) { return __builtin_amdgcn_logf(x); }

// log2(2^a + 2^b), safe for -inf operands.
__device__ __forceinline__ float lse2(float a, float b) {
    float hi = fmaxf(a, b), lo = fminf(a, b);
    if (hi == -INFINITY) return -INFINITY;
    return hi + log2_fast(1.0f + exp2_fast(lo - hi));
}

// Workgroup barrier that orders LDS traffic only: unlike __syncthreads() it does not wait for the
// wave's outstanding global loads, stores and atomics, so those stay in flight across it.  Use it
// where the waves of a workgroup communicate through LDS alone.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// 16-byte global load of 8 packed 16-bit values.
__device__ __forceinline__ uint4 ld16(const uint8_t *p) { return *reinterpret_cast<const uint4 *>(p); }

// The same for data that is read once (key and value slices, metadata records, the stored logits): marked
// non-temporal, so that hundreds of megabytes streaming through a launch do not push out of the caches what is
// used again -- queries, page lists, control words, the logits on their way to the next kernel.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld16_stream(const uint8_t *p) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ int clamp_page(int page, int num_pages, int32_t *header) {
    if ((unsigned)page >= (unsigned)num_pages) {
        set_error(header, PSA_DEVERR_PAGE_RANGE);
        return 0;
    }
    return page;
}

// Blocks of request r, clamped into [0, max_blocks]; reports a context outside the table.
__device__ __forceinline__ int ctx_clamped(const KvView &kv, int r, int32_t *header) {
    int ctx = kv.ctx_lens[r];
    if (ctx < 0) { set_error(header, PSA_DEVERR_CTX_RANGE); ctx = 0; }
    if (ctx > kv.max_blocks * kPage) { set_error(header, PSA_DEVERR_CTX_RANGE); ctx = kv.max_blocks * kPage; }
    return ctx;
}

__device__ __forceinline__ int ctx_clamped_quiet(const KvView &kv, int r) {
    const int ctx = kv.ctx_lens[r];
    return ctx < 0 ? 0 : (ctx > kv.max_blocks * kPage ? kv.max_blocks * kPage : ctx);
}
__device__ __forceinline__ int clamp_page_quiet(int page, int num_pages) {
    return (unsigned)page >= (unsigned)num_pages ? 0 : page;
}

// ---- packed 16-bit min/max on order-preserving keys (block metadata) --------------------------
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

// Two packed 16-bit floats -> keys whose unsigned order is the numeric order.
__device__ __forceinline__ uint32_t to_ordered(uint32_t w) {
    const uint32_t neg = ((w >> 15) & 0x00010001u) * 0xFFFFu;   // 0xFFFF in each negative half
    return w ^ (neg | 0x80008000u);
}
__device__ __forceinline__ uint32_t from_ordered(uint32_t k) {
    const uint32_t was_neg = (((~k) >> 15) & 0x00010001u) * 0xFFFFu;
    return k ^ (was_neg | 0x80008000u);
}
__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(ushort2_t, a),
                                                                  __builtin_bit_cast(ushort2_t, b)));
}
__device__ __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, a),
                                                                  __builtin_bit_cast(ushort2_t, b)));
}

// Chunks of a stream that are inside the read-ahead window from the start because the caller expects
// the stream to need them (0 without a hint).
__device__ __forceinline__ int hinted_chunks(const int32_t *depth_hint, int s, int N, int CB) {
    if (!depth_hint) return 0;
    const int h = depth_hint[s];
    return h <= 0 ? 0 : (min(h, N) + CB - 1) / CB;
}

}  // namespace psa
