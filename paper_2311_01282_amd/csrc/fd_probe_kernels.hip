// Measurement aid: a plain streaming read of two buffers with the same launch
// geometry and access pattern as the chunk kernel (256-thread workgroups, each
// walking 64 KiB of each buffer with 128-bit loads) and no arithmetic beyond an
// XOR.  Its rate is the ceiling a read-only kernel of this shape reaches.
#include "fd_internal.h"

namespace fd {
namespace {

constexpr int kTile = 65536;   // bytes of each buffer per workgroup

__global__ __launch_bounds__(256) void stream_read_kernel(const uint4 *a, const uint4 *b, unsigned *sink)
{
    const size_t base = (size_t)blockIdx.x * (kTile / 16) + threadIdx.x;
    uint4 acc = make_uint4(0, 0, 0, 0);
#pragma unroll 1
    for (int i = 0; i < kTile / 16 / 256; i += 8) {
        uint4 x[8], y[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = a[base + (size_t)(i + u) * 256];
#pragma unroll
        for (int u = 0; u < 8; ++u) y[u] = b[base + (size_t)(i + u) * 256];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            acc.x ^= x[u].x ^ y[u].x; acc.y ^= x[u].y ^ y[u].y;
            acc.z ^= x[u].z ^ y[u].z; acc.w ^= x[u].w ^ y[u].w;
        }
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
