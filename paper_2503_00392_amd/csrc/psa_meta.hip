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

// Mean-key metadata: per (page, KV head) and channel, the mean of the page's valid keys, summed in binary64 (exact
// for any realistic keys, so the order of the additions does not show), divided by the count and rounded once, to
// nearest-even, to the cache's 16-bit type; a zero mean is +0.  One wave per slice, as above;
// out: [num_pages][num_kv_heads][128].
__device__ __forceinline__ double key_value(uint32_t bits16, int dtype) {
    if (dtype == 0) return (double)__builtin_bit_cast(_Float16, (uint16_t)bits16);
    return (double)__uint_as_float(bits16 << 16);
}

// x (zero, or a normal binary64 number no larger than the type's largest) to the 16-bit type: the significand is
// cut at the type's last place -- further left in the type's subnormal range -- and rounded to nearest, ties to even,
// in integer arithmetic; a carry out of the significand runs into the exponent field by itself.
__device__ __forceinline__ uint32_t round_to_16bit(double x, int dtype) {
    const int mant_bits = dtype ? 7 : 10, bias = dtype ? 127 : 15;
    const unsigned long long u = (unsigned long long)__double_as_longlong(x);
    const uint32_t sign = (uint32_t)(u >> 63) << 15;
    const int e = (int)((u >> 52) & 0x7ffull);
    if (e == 0) return (u << 1) == 0ull ? 0u : sign;           // zero is +0 (binary64 subnormals cannot occur)
    const int lead = e - 1023, emin = 1 - bias;
    const unsigned long long sig = (u & ((1ull << 52) - 1ull)) | (1ull << 52);
    const int shift = 52 - mant_bits + (lead < emin ? emin - lead : 0);
    if (shift > 62) return sign;                               // far below half the smallest subnormal
    unsigned long long kept = sig >> shift;
    const unsigned long long rest = sig & ((1ull << shift) - 1ull), half = 1ull << (shift - 1);
    if (rest > half || (rest == half && (kept & 1ull))) kept += 1ull;
    if (lead < emin) return sign | (uint32_t)kept;             // subnormal (or, after a carry, the smallest normal)
    return sign | (((uint32_t)(lead + bias) << mant_bits) + (uint32_t)(kept - (1ull << mant_bits)));
}

__global__ __launch_bounds__(256) void means_kernel(const uint8_t *__restrict__ k_pool, uint8_t *__restrict__ means,
                                                    const int32_t *__restrict__ page_fill,
                                                    const int32_t *__restrict__ page_list, int num_units,
                                                    int num_kv_heads, int num_pages, int dtype) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, rg = lane >> 4, cl = lane & 15;
    const int unit = blockIdx.x * 4 + wave;
    if (unit >= num_units) return;
    const int listed = unit / num_kv_heads, h = unit % num_kv_heads;
    const int page = page_list ? page_list[listed] : listed;
    if ((unsigned)page >= (unsigned)num_pages) return;   // a listed page outside the pool is skipped
    int fill = page_fill ? page_fill[page] : kPage;
    fill = fill < 0 ? 0 : (fill > kPage ? kPage : fill);
    const size_t unit_off = (size_t)page * num_kv_heads + h;
    double sum[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) sum[j] = 0.0;
    if (fill > 0) {
        Slice k = load_slice(k_pool + unit_off * kSliceBytes, lane);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (4 * i + rg < fill) {
                const uint32_t w[4] = {k.r[i].x, k.r[i].y, k.r[i].z, k.r[i].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    sum[2 * j] += key_value(w[j] & 0xffffu, dtype);
                    sum[2 * j + 1] += key_value(w[j] >> 16, dtype);
                }
            }
        }
    }
    // the four row groups' sums together (a lane's channels are those of the lanes 16, 32 and 48 further on)
#pragma unroll
    for (int step = 16; step <= 32; step <<= 1) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const long long mine = __double_as_longlong(sum[j]);
            const long long other = ((long long)__shfl_xor((int)(mine >> 32), step) << 32) |
                                    (long long)(unsigned)__shfl_xor((int)mine, step);
            sum[j] += __longlong_as_double(other);
        }
    }
    if (rg != 0) return;
    uint32_t o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const double a = fill > 0 ? sum[2 * j] / (double)fill : 0.0, b = fill > 0 ? sum[2 * j + 1] / (double)fill : 0.0;
        o[j] = round_to_16bit(a, dtype) | (round_to_16bit(b, dtype) << 16);
    }
    *reinterpret_cast<uint4 *>(means + unit_off * 256 + cl * 16) = make_uint4(o[0], o[1], o[2], o[3]);
}

hipError_t launch_means(const psa_kv_desc *d, void *means, const int32_t *page_fill, const int32_t *page_list,
                        int num_listed, hipStream_t st) {
    const long long units = (long long)(page_list ? num_listed : d->num_pages) * d->num_kv_heads;
    if (units == 0) return hipSuccess;
    const unsigned grid = (unsigned)((units + 3) / 4);
    means_kernel<<<grid, 256, 0, st>>>((const uint8_t *)d->k_pool, (uint8_t *)means, page_fill, page_list, (int)units,
                                       d->num_kv_heads, d->num_pages, (int)d->dtype);
    return hipGetLastError();
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
