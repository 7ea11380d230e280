// Block metadata: per (page, KV head), per channel, the minimum and maximum key over the page's
// valid tokens.  One wave reduces one 4 KiB key slice: 4 coalesced 1 KiB loads, packed 16-bit
// integer min/max on order-preserving keys (exact for fp16 and bf16 alike, -0 below +0), then a
// two-step exchange between the wave's four row groups.
#include "psa_attend.h"
#include "psa_host.h"

namespace psa {

// grid: ceil(units / 4) workgroups of 4 waves; unit = (listed page, KV head).
__global__ __launch_bounds__(256) void metadata_kernel(const uint8_t *__restrict__ k_pool,
                                                       uint8_t *__restrict__ meta,
                                                       const int32_t *__restrict__ page_fill,
                                                       const int32_t *__restrict__ page_list,
                                                       int num_units, int num_kv_heads, int num_pages) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, rg = lane >> 4, cl = lane & 15;
    const int unit = blockIdx.x * 4 + wave;
    if (unit >= num_units) return;
    const int listed = unit / num_kv_heads, h = unit % num_kv_heads;
    const int page = page_list ? page_list[listed] : listed;
    if ((unsigned)page >= (unsigned)num_pages) return;   // a listed page outside the pool is skipped
    int fill = page_fill ? page_fill[page] : kPage;
    fill = fill < 0 ? 0 : (fill > kPage ? kPage : fill);
    const size_t unit_off = (size_t)page * num_kv_heads + h;

    uint32_t lo[4], hi[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) { lo[j] = 0xFFFFFFFFu; hi[j] = 0u; }
    if (fill > 0) {
        Slice k = load_slice(k_pool + unit_off * kSliceBytes, lane);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (4 * i + rg < fill) {
                const uint32_t w[4] = {k.r[i].x, k.r[i].y, k.r[i].z, k.r[i].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t key = to_ordered(w[j]);
                    lo[j] = pk_min(lo[j], key);
                    hi[j] = pk_max(hi[j], key);
                }
            }
        }
    }
#pragma unroll
    for (int step = 16; step <= 32; step <<= 1) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            lo[j] = pk_min(lo[j], (uint32_t)__shfl_xor((int)lo[j], step));
            hi[j] = pk_max(hi[j], (uint32_t)__shfl_xor((int)hi[j], step));
        }
    }
    uint4 o;
    if (fill == 0) {
        o = make_uint4(0, 0, 0, 0);
    } else if (rg == 0) {
        o = make_uint4(from_ordered(lo[0]), from_ordered(lo[1]), from_ordered(lo[2]), from_ordered(lo[3]));
    } else {
        o = make_uint4(from_ordered(hi[0]), from_ordered(hi[1]), from_ordered(hi[2]), from_ordered(hi[3]));
    }
    // row group 0 writes the 256-byte min row, row group 1 the max row
    if (rg < 2) *reinterpret_cast<uint4 *>(meta + unit_off * kMetaBytes + rg * 256 + cl * 16) = o;
}

hipError_t launch_metadata(const psa_kv_desc *d, void *meta, const int32_t *page_fill,
                           const int32_t *page_list, int num_listed, hipStream_t st) {
    const long long units = (long long)(page_list ? num_listed : d->num_pages) * d->num_kv_heads;
    if (units == 0) return hipSuccess;
    const unsigned grid = (unsigned)((units + 3) / 4);
    metadata_kernel<<<grid, 256, 0, st>>>((const uint8_t *)d->k_pool, (uint8_t *)meta, page_fill, page_list,
                                          (int)units, d->num_kv_heads, d->num_pages);
    return hipGetLastError();
}

}  // namespace psa
