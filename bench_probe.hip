// Streaming-read probe of bench.py -- a measurement aid, not part of libpsa: a plain kernel that reads a
// device buffer once, front to back, with 16-byte loads and keeps nothing.  It measures the read bandwidth
// the memory system actually delivers to a kernel of the simplest possible shape, the ceiling the decode
// path's rates are also quoted against (the published 8 TB/s is not reachable by any kernel).
// Built by __graft_entry__.build() into libbench_probe.so beside bench.py, which loads it through ctypes.
//   int bench_stream_read_probe(const void *src, size_t bytes, void *sink, void *stream)
//     src    device pointer, 16-byte aligned, read only; bytes is rounded down to a multiple of 16
//     sink   device pointer to 8 writable bytes (8-byte aligned) or NULL; practically never written
//     stream hipStream_t;  returns 0, 1 for a NULL or misaligned pointer, 4 if the launch failed
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

constexpr int kProbeThreads = 256;
constexpr int kProbeUnroll = 8;      // independent 16-byte loads in flight per thread

typedef uint32_t probe_word __attribute__((ext_vector_type(4)));      // 16 bytes, one load

__global__ __launch_bounds__(kProbeThreads) void read_probe_kernel(const probe_word *__restrict__ src, size_t n16,
                                                                    unsigned long long *sink) {
    uint32_t acc = 0;
    const size_t tile = (size_t)kProbeThreads * kProbeUnroll;           // 16-byte words per workgroup and turn
    for (size_t at = (size_t)blockIdx.x * tile; at < n16; at += (size_t)gridDim.x * tile) {
        probe_word v[kProbeUnroll];
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) {
            const size_t j = at + (size_t)u * kProbeThreads + threadIdx.x;
            v[u] = j < n16 ? __builtin_nontemporal_load(src + j) : probe_word{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    // a store that depends on every load (so none can be dropped) and all but never happens
    if (acc == 0x9e3779b9u && sink) *sink = acc;
}

}  // namespace

extern "C" int bench_stream_read_probe(const void *src, size_t bytes, void *sink, void *stream) {
    if (bytes < 16) return 0;
    if (!src || (reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(sink) & 7u)) return 1;
    const size_t n16 = bytes / 16;
    const size_t tile = (size_t)kProbeThreads * kProbeUnroll;
    size_t grid = (n16 + tile - 1) / tile;
    if (grid > 256 * 32) grid = 256 * 32;
    read_probe_kernel<<<(unsigned)grid, kProbeThreads, 0, (hipStream_t)stream>>>(
        static_cast<const probe_word *>(src), n16, static_cast<unsigned long long *>(sink));
    return hipGetLastError() == hipSuccess ? 0 : 4;
}
