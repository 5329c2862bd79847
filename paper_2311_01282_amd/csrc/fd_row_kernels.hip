// Chunk kernels that treat every query head as an independent row (VALU path).
//
// One workgroup of 4 wavefronts handles one (row, chunk).  A K or V row is 256
// bytes = 16 segments of 16 bytes; lane l of a wavefront owns segment l%16 of key
// (l/16) within a group of 4 consecutive keys, so one wavefront load instruction
// reads 1 KiB of contiguous cache memory with 128-bit loads.  The four wavefronts
// interleave groups, i.e. the workgroup walks the chunk front to back 4 KiB at a
// time.  The 16 lanes of a key reduce their 8-element partial dot products with
// DPP row operations (a DPP row is exactly 16 lanes), after which every one of
// the 16 lanes holds the key's logit and scales its own 8 elements of the V row.
//
//   unified kernel : Eq. 4 inner sums, no maximum, plus the range guard of
//                    Section 3 "Recomputation" (steps score, guard, exp+sums).
//   sync kernel    : the per-chunk part of the synchronized partial softmax,
//                    Eq. 2: m = max x, l = sum e^{x-m}, f.V = sum e^{x-m} v.
#include "fd_internal.h"

namespace fd {
namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ half2_t as_h2(uint32_t u) { return __builtin_bit_cast(half2_t, u); }

// fp32 dot product of 8 fp16 pairs; every product is exact in fp32.
__device__ __forceinline__ float dot8(const uint4 &a, const uint4 &b)
{
    float acc = 0.f;
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w};
    const uint32_t bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const half2_t x = as_h2(aw[i]), y = as_h2(bw[i]);
        acc = __builtin_fmaf((float)x.x, (float)y.x, acc);
        acc = __builtin_fmaf((float)x.y, (float)y.y, acc);
    }
    return acc;
}

// acc[0..7] += p * v[0..7]
__device__ __forceinline__ void axpy8(float (&acc)[8], float p, const uint4 &v)
{
    const uint32_t vw[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const half2_t x = as_h2(vw[i]);
        acc[2 * i]     = __builtin_fmaf(p, (float)x.x, acc[2 * i]);
        acc[2 * i + 1] = __builtin_fmaf(p, (float)x.y, acc[2 * i + 1]);
    }
}

template <int CTRL>
__device__ __forceinline__ float dpp_swap(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}

// Sum over the 16 lanes of a DPP row; every lane ends with the total.
__device__ __forceinline__ float row16_sum(float x)
{
    x += dpp_swap<0xB1>(x);   // quad_perm [1,0,3,2]  : lane ^ 1
    x += dpp_swap<0x4E>(x);   // quad_perm [2,3,0,1]  : lane ^ 2
    x += dpp_swap<0x141>(x);  // row_half_mirror      : other quad of the 8
    x += dpp_swap<0x140>(x);  // row_mirror           : other half of the 16
    return x;
}

template <int C>
struct ChunkLds {
    float acc[16][kHeadDim];   // [wave*4 + key-in-group][element]
    float x[C];                // logits of the chunk (synchronized scheme only)
    float den[16];
    float mx[4];
    int   flag[4];
};

// One (row, chunk).  SYNC == false: unified phi.  SYNC == true: chunk-local max.
template <int C, bool SYNC>
__device__ __forceinline__ void chunk_body(const Problem &p, int row, int c, ChunkLds<SYNC ? C : 1> &lds)
{
    constexpr int NG = C / 16;                 // groups of 16 keys (4 per wavefront) in the chunk
    constexpr int U = NG < 8 ? NG : 8;         // groups in flight per wavefront
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int seg = lane & 15, sub = lane >> 4;

    const int b = row / p.Hq;
    const int hq = row - b * p.Hq;
    const int hkv = hq / p.G;
    const int S = valid_len(p, b);
    const int start = c * C;
    const int nvalid = min(C, S - start);      // <= 0: no valid key in this chunk
    const size_t slot = (size_t)row * p.nc + c;

    if (nvalid <= 0) {                         // empty chunk: zero partials, no flag
        if (tid < kHeadDim) p.ws.num[slot * kHeadDim + tid] = 0.f;
        if (tid == 0) {
            p.ws.den[slot] = 0.f;
            if (SYNC) p.ws.mloc[slot] = -INFINITY; else p.ws.chunk_flags[slot] = 0;
        }
        return;
    }

    const uint4 qv = reinterpret_cast<const uint4 *>(p.q + (size_t)row * kHeadDim)[seg];
    const size_t kv_off = (((size_t)b * p.Hkv + hkv) * p.Smax + start) * kHeadDim;
    const uint4 *kp = reinterpret_cast<const uint4 *>(p.k + kv_off) + seg;
    const uint4 *vp = reinterpret_cast<const uint4 *>(p.v + kv_off) + seg;
    const int last = nvalid - 1;

    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float den = 0.f;
    float mc = 0.f;

    if constexpr (!SYNC) {
        const float nphi = -p.phi, lo = p.lo, hi = p.hi, scale = p.scale;
        bool bad = false;
#pragma unroll 1
        for (int g0 = 0; g0 < NG; g0 += U) {
            if (g0 * 16 >= nvalid) break;      // uniform: rest of the chunk is padding
            uint4 kk[U], vv[U];
            // Keys past the valid length re-read the last valid key (always in
            // bounds, never padding) and get weight zero below.
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int kidx = ((g0 + u) * 4 + wave) * 4 + sub;
                kk[u] = kp[(size_t)min(kidx, last) * 16];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int kidx = ((g0 + u) * 4 + wave) * 4 + sub;
                vv[u] = vp[(size_t)min(kidx, last) * 16];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int kidx = ((g0 + u) * 4 + wave) * 4 + sub;
                const bool valid = kidx <= last;
                const float x = row16_sum(dot8(qv, kk[u])) * scale;
                const float d = x + nphi;                       // x - phi
                bad |= valid && !(d > lo && d < hi);            // equality and NaN flag
                float e = __builtin_amdgcn_exp2f(d * kLog2e);   // e^{x - phi}
                e = valid ? e : 0.f;
                den += e;
                axpy8(acc, e, vv[u]);
            }
        }
        const unsigned long long any_bad = __ballot(bad);
        if (lane == 0) lds.flag[wave] = any_bad != 0ull;
    } else {
        // Pass 1: logits of the whole chunk into LDS, and their maximum.
        float m = -INFINITY;
        const float scale = p.scale;
#pragma unroll 1
        for (int g0 = 0; g0 < NG; g0 += U) {
            if (g0 * 16 >= nvalid) break;      // uniform: rest of the chunk is padding
            uint4 kk[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int kidx = ((g0 + u) * 4 + wave) * 4 + sub;
                kk[u] = kp[(size_t)min(kidx, last) * 16];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int kidx = ((g0 + u) * 4 + wave) * 4 + sub;
                float x = row16_sum(dot8(qv, kk[u])) * scale;
                x = kidx <= last ? x : -INFINITY;
                if (seg == 0) lds.x[kidx] = x;
                m = fmaxf(m, x);
            }
        }
        // chunk maximum: over the 4 keys of the lane's column, then the 4 wavefronts
        m = fmaxf(m, __shfl_xor(m, 16));
        m = fmaxf(m, __shfl_xor(m, 32));
        if (lane == 0) lds.mx[wave] = m;
        __syncthreads();
        mc = fmaxf(fmaxf(lds.mx[0], lds.mx[1]), fmaxf(lds.mx[2], lds.mx[3]));
        // Pass 2: e^{x - m} and the V products.
#pragma unroll 1
        for (int g0 = 0; g0 < NG; g0 += U) {
            if (g0 * 16 >= nvalid) break;
            uint4 vv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int kidx = ((g0 + u) * 4 + wave) * 4 + sub;
                vv[u] = vp[(size_t)min(kidx, last) * 16];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int kidx = ((g0 + u) * 4 + wave) * 4 + sub;
                const float e = __builtin_amdgcn_exp2f((lds.x[kidx] - mc) * kLog2e);   // 0 for padding
                den += e;
                axpy8(acc, e, vv[u]);
            }
        }
    }

    // Workgroup reduction: 16 partial vectors (4 wavefronts x 4 keys per group).
    float4 *dst = reinterpret_cast<float4 *>(&lds.acc[wave * 4 + sub][seg * 8]);
    dst[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
    dst[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
    if (seg == 0) lds.den[wave * 4 + sub] = den;
    __syncthreads();
    if (tid < kHeadDim) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) s += lds.acc[i][tid];
        p.ws.num[slot * kHeadDim + tid] = s;
    } else if (tid == kHeadDim) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) s += lds.den[i];
        p.ws.den[slot] = s;
        if (SYNC) p.ws.mloc[slot] = mc;
        else p.ws.chunk_flags[slot] = (lds.flag[0] | lds.flag[1] | lds.flag[2] | lds.flag[3]) ? 1 : 0;
    }
}

template <int C>
__global__ __launch_bounds__(kThreads) void partial_unified_kernel(const Problem p)
{
    __shared__ ChunkLds<1> lds;
    const int w = blockIdx.x;
    chunk_body<C, false>(p, w / p.nc, w % p.nc, lds);
}

// use_list == false: every (row, chunk), one per workgroup.
// use_list == true : only the rows in ws.list[0 .. *ws.count); the grid is fixed
// and workgroups stride over (flagged row, chunk) items, so the launch needs no
// host knowledge of the count and exits at once when nothing is flagged.
template <int C>
__global__ __launch_bounds__(kThreads) void partial_sync_kernel(const Problem p, const int use_list)
{
    __shared__ ChunkLds<C> lds;
    if (!use_list) {
        const int w = blockIdx.x;
        chunk_body<C, true>(p, w / p.nc, w % p.nc, lds);
        return;
    }
    const long long items = (long long)(*p.ws.count) * p.nc;
    for (long long w = blockIdx.x; w < items; w += gridDim.x) {
        const int row = p.ws.list[w / p.nc];
        chunk_body<C, true>(p, row, (int)(w % p.nc), lds);
        __syncthreads();                        // lds is reused by the next item
    }
}

template <template <int> class Launcher, typename... Args>
hipError_t dispatch_chunk(int C, Args... args)
{
    switch (C) {
        case 64:   return Launcher<64>::run(args...);
        case 128:  return Launcher<128>::run(args...);
        case 256:  return Launcher<256>::run(args...);
        case 512:  return Launcher<512>::run(args...);
        case 1024: return Launcher<1024>::run(args...);
        default:   return hipErrorInvalidValue;
    }
}

template <int C> struct UnifiedLauncher {
    static hipError_t run(const Problem &p, hipStream_t s)
    {
        const unsigned grid = (unsigned)((long long)p.rows * p.nc);
        if (grid == 0) return hipSuccess;
        return launch(partial_unified_kernel<C>, dim3(grid), dim3(kThreads), s, p);
    }
};

template <int C> struct SyncLauncher {
    static hipError_t run(const Problem &p, bool use_list, hipStream_t s)
    {
        const long long all = (long long)p.rows * p.nc;
        if (all == 0) return hipSuccess;
        const long long cap = 4096;             // resident capacity is 256 CUs x a few workgroups
        const unsigned grid = (unsigned)(use_list ? (all < cap ? all : cap) : all);
        return launch(partial_sync_kernel<C>, dim3(grid), dim3(kThreads), s, p, use_list ? 1 : 0);
    }
};

}  // namespace

hipError_t launch_partial_unified(const Problem &p, hipStream_t s)
{
    return dispatch_chunk<UnifiedLauncher>(p.C, p, s);
}

hipError_t launch_partial_sync(const Problem &p, bool use_list, hipStream_t s)
{
    return dispatch_chunk<SyncLauncher>(p.C, p, use_list, s);
}

}  // namespace fd
