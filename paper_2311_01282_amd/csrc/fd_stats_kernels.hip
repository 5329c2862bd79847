// Statistics of the softmax inputs (Section 3, the distribution of x_i from which the
// unified scaling factor and its bounds are chosen): a fixed-width histogram of every
// valid scaled logit x = s <q, k_j>, plus their minimum and maximum.  Reads K (256 B
// per key and KV head, once per block of query heads that share it), nothing else of size.
//
// A fixed grid of workgroups strides over (head block, 256-key tile) items; the lane layout
// and the dot product are those of the chunk kernels (fd_chunk.h).  Counts go to an
// LDS histogram first and reach the device histogram as 64-bit integer atomic adds
// when the workgroup is done: integer sums, so the result does not depend on order.
#include "fd_chunk.h"

namespace fd {
namespace {

constexpr int kStatsTile = 256;      // keys per item
constexpr int kStatsThreads = 256;

// float minimum / maximum through integer atomics (the IEEE order of same-sign floats is
// the order of their bit patterns, reversed for negatives).  NaN never reaches here.
__device__ __forceinline__ void atomic_max_float(float *addr, float v)
{
    if (v >= 0.f) atomicMax(reinterpret_cast<int *>(addr), __builtin_bit_cast(int, v));
    else atomicMin(reinterpret_cast<unsigned *>(addr), __builtin_bit_cast(unsigned, v));
}
__device__ __forceinline__ void atomic_min_float(float *addr, float v)
{
    if (v >= 0.f) atomicMin(reinterpret_cast<int *>(addr), __builtin_bit_cast(int, v));
    else atomicMax(reinterpret_cast<unsigned *>(addr), __builtin_bit_cast(unsigned, v));
}

// GT = query heads handled per K tile: 1 for ungrouped heads; 4 when heads share a KV
// head, so that the tile is fetched once per four of them (the other fetches of a larger
// group hit in L2).  An item is (sequence, KV head, block of GT heads, 256-key tile).
template <int GT>
__global__ __launch_bounds__(kStatsThreads) void logit_histogram_kernel(
    const Problem p, const float x_min, const float inv_width, const int n_bins,
    unsigned long long *__restrict__ hist, float *__restrict__ min_max)
{
    static_assert(GT <= 16, "one lane of a key's 16 per head");
    extern __shared__ unsigned lds_hist[];              // n_bins + 2 counters, then 8 floats
    float *lds_mm = reinterpret_cast<float *>(lds_hist + n_bins + 2);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seg = lane & 15, sub = lane >> 4;
    for (int i = tid; i < n_bins + 2; i += kStatsThreads) lds_hist[i] = 0u;
    __syncthreads();

    constexpr int UP = 4;                                // groups of 4 keys per wavefront and stage
    constexpr int NBLK = kStatsTile / (16 * UP);         // stages per tile
    const int tiles = (p.Smax + kStatsTile - 1) / kStatsTile;
    const int hblocks = (p.G + GT - 1) / GT;
    const long long items = (long long)p.B * p.Hkv * hblocks * tiles;
    float lo = INFINITY, hi = -INFINITY;
    for (long long it = blockIdx.x; it < items; it += gridDim.x) {
        const int t = (int)(it % tiles);
        const long long r = it / tiles;
        const int hb = (int)(r % hblocks);
        const int gi = (int)(r / hblocks);               // (sequence, KV head)
        const int b = gi / p.Hkv, hkv = gi - b * p.Hkv;
        const int nvalid = min(kStatsTile, valid_len(p, b) - t * kStatsTile);
        if (nvalid <= 0) continue;                       // uniform over the workgroup
        const int last = nvalid - 1;
        const int h0 = hb * GT, nh = min(GT, p.G - h0);  // heads h0 .. h0 + nh - 1 of the group
        const int row0 = b * p.Hq + hkv * p.G + h0;
        u32x4 qv[GT];
#pragma unroll
        for (int g = 0; g < GT; ++g)
            qv[g] = reinterpret_cast<const u32x4 *>(p.q + (size_t)(row0 + min(g, nh - 1)) * kHeadDim)[seg];
        const u32x4 *kp = reinterpret_cast<const u32x4 *>(
                              p.k + (((size_t)b * p.Hkv + hkv) * p.Smax + (size_t)t * kStatsTile) * kHeadDim) + seg;
        auto key_of = [&](int g) { return (g * 4 + wave) * 4 + sub; };
        auto issue = [&](int blk, u32x4 (&kk)[UP]) {
#pragma unroll
            for (int u = 0; u < UP; ++u) kk[u] = load_stream(kp + (size_t)min(key_of(blk * UP + u), last) * 16);
        };
        auto count = [&](int blk, const u32x4 (&kk)[UP]) {
#pragma unroll
            for (int u = 0; u < UP; ++u) {
                const bool valid = key_of(blk * UP + u) <= last;
                // every lane of the key's 16 ends up with all GT logits; lane `seg` bins head `seg`
                float x = row16_sum(dot8(qv[0], kk[u])) * p.scale;
#pragma unroll
                for (int g = 1; g < GT; ++g) {
                    const float xg = row16_sum(dot8(qv[g], kk[u])) * p.scale;
                    x = seg == g ? xg : x;
                }
                if (seg < nh && valid) {
                    int slot;
                    if (x != x) {
                        slot = n_bins + 1;
                    } else {
                        const float tq = floorf((x - x_min) * inv_width);
                        slot = tq < 0.f ? 0 : (tq >= (float)n_bins ? n_bins + 1 : (int)tq + 1);
                        lo = fminf(lo, x);
                        hi = fmaxf(hi, x);
                    }
                    atomicAdd(&lds_hist[slot], 1u);
                }
            }
        };
        // two stages in flight; loads past the last valid key re-read it and are not counted
        const int nblk = min(NBLK, (nvalid + 16 * UP - 1) / (16 * UP));
        u32x4 kA[UP], kB[UP];
        issue(0, kA);
        int blk = 0;
#pragma unroll 1
        for (; blk + 2 < nblk; blk += 2) {
            issue(blk + 1, kB);
            count(blk, kA);
            issue(blk + 2, kA);
            count(blk + 1, kB);
        }
        if (blk + 2 == nblk) {
            issue(blk + 1, kB);
            count(blk, kA);
            count(blk + 1, kB);
        } else {
            count(blk, kA);
        }
    }
    // workgroup minimum / maximum: wavefront reduction, then four values through LDS
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, o));
        hi = fmaxf(hi, __shfl_xor(hi, o));
    }
    if (lane == 0) { lds_mm[wave] = lo; lds_mm[4 + wave] = hi; }
    __syncthreads();
    for (int i = tid; i < n_bins + 2; i += kStatsThreads) {
        const unsigned n = lds_hist[i];
        if (n) atomicAdd(&hist[i], (unsigned long long)n);
    }
    if (tid == 0 && min_max) {
        lo = fminf(fminf(lds_mm[0], lds_mm[1]), fminf(lds_mm[2], lds_mm[3]));
        hi = fmaxf(fmaxf(lds_mm[4], lds_mm[5]), fmaxf(lds_mm[6], lds_mm[7]));
        if (lo <= hi) {                                  // at least one logit that is not NaN was seen
            atomic_min_float(&min_max[0], lo);
            atomic_max_float(&min_max[1], hi);
        }
    }
}

}  // namespace

hipError_t launch_logit_histogram(const Problem &p, float x_min, float bin_width, int n_bins,
                                  unsigned long long *hist, float *min_max, hipStream_t s)
{
    const int gt = p.G > 1 ? 4 : 1;
    const long long items = (long long)p.B * p.Hkv * ((p.G + gt - 1) / gt) * ((p.Smax + kStatsTile - 1) / kStatsTile);
    if (items == 0) return hipSuccess;
    // Few workgroups: every one of them ends with up to n_bins + 2 atomic adds on the same
    // addresses, and those serialize (2048 workgroups cost 25 % more time than 512 on a
    // 1 GiB cache).  The grouped variant does four dot products per key and needs more
    // wavefronts to cover them.
    const long long cap = p.G > 1 ? 1024 : 512;
    const unsigned grid = (unsigned)(items < cap ? items : cap);
    const size_t lds = (size_t)(n_bins + 2) * sizeof(unsigned) + 8 * sizeof(float);
    const float inv_width = 1.0f / bin_width;
    void *args[] = {(void *)&p, (void *)&x_min, (void *)&inv_width, (void *)&n_bins, (void *)&hist, (void *)&min_max};
    const void *fn = p.G > 1 ? reinterpret_cast<const void *>(&logit_histogram_kernel<4>)
                             : reinterpret_cast<const void *>(&logit_histogram_kernel<1>);
    return hipLaunchKernel(fn, dim3(grid), dim3(kStatsThreads), args, lds, s);
}

}  // namespace fd
