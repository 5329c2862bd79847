// Measurement aid: a plain streaming read of two buffers with the same launch
// geometry and access pattern as the chunk kernel at 256 keys per chunk
// (256-thread workgroups, each walking 64 KiB of each buffer with non-temporal
// 128-bit loads, 4 KiB of each in flight per wavefront) and no arithmetic beyond an
// XOR.  Its rate is the ceiling a read-only kernel of this shape reaches.
#include "fd_internal.h"

namespace fd {
namespace {

constexpr int kTile = 65536;   // bytes of each buffer per workgroup

__global__ __launch_bounds__(256) void stream_read_kernel(const uint4 *a, const uint4 *b, unsigned *sink)
{
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 *pa = reinterpret_cast<const u32x4 *>(a) + (size_t)blockIdx.x * (kTile / 16) + threadIdx.x;
    const u32x4 *pb = reinterpret_cast<const u32x4 *>(b) + (size_t)blockIdx.x * (kTile / 16) + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
#pragma unroll 1
    for (int i = 0; i < kTile / 16 / 256; i += 4) {
        u32x4 x[4], y[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) x[u] = __builtin_nontemporal_load(pa + (size_t)(i + u) * 256);
#pragma unroll
        for (int u = 0; u < 4; ++u) y[u] = __builtin_nontemporal_load(pb + (size_t)(i + u) * 256);
#pragma unroll
        for (int u = 0; u < 4; ++u) acc ^= x[u] ^ y[u];
    }
    const unsigned r = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (r == 0x9e3779b9u) sink[0] = r;   // practically never true: keeps the loads alive
}

}  // namespace

hipError_t launch_stream_read(const void *a, const void *b, size_t bytes_each, unsigned *sink, hipStream_t s)
{
    const size_t tiles = bytes_each / kTile;
    if (tiles == 0) return hipSuccess;
    return launch(stream_read_kernel, dim3((unsigned)tiles), dim3(256), s,
                  static_cast<const uint4 *>(a), static_cast<const uint4 *>(b), sink);
}

}  // namespace fd
