// Small kernels of the multi-kernel chain: flag reduction, the outer sums of
// Eq. 4 (atomic-free: one workgroup owns one output row), and the synchronized
// merge of Eq. 2 for recomputed rows.  Plus the ticket clear of fd_workspace_init.
#include "fd_chunk.h"

namespace fd {
namespace {

__global__ __launch_bounds__(256) void clear_tickets_kernel(int32_t *ticket, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) ticket[i] = 0;
}

// The row epilogue as a launch of its own (one workgroup per row), used when the
// chunk kernels run without electing a finisher.
__global__ __launch_bounds__(256) void row_epilogue_kernel(const Problem p)
{
    __shared__ __attribute__((aligned(16))) float scratch[8 * kHeadDim + 16];
    const int row = blockIdx.x;
    // one batch of argument loads at the top instead of one per first use
    asm volatile("" ::"s"(p.ws.num), "s"(p.ws.meta), "s"(p.ws.row_flags), "s"(p.seq_lens), "s"(p.out), "s"(p.nc),
                 "s"(p.Hq), "s"(p.C), "s"(p.Smax));
    // every slot of the row holds defined values, so the loads need not wait for the length
    row_epilogue<4, false>(p, row, p.nc, [&] { return (valid_len(p, row / p.Hq) + p.C - 1) / p.C; }, scratch);
}

// The same for rows of at most 8 chunks: 8 rows per workgroup, 32 threads per row walking
// the row's chunks in registers (no LDS, no barrier, an eighth of the workgroups).
__global__ __launch_bounds__(256) void rows8_epilogue_kernel(const Problem p)
{
    const int row0 = blockIdx.x * 8;
    rows_epilogue<false>(p, row0, min(8, p.rows - row0), [&](int row) { return (valid_len(p, row / p.Hq) + p.C - 1) / p.C; });
}

// Chunk flags -> row flags, ascending list of flagged rows, their count.
// A single workgroup: the compaction is a block-wide prefix sum, no atomics.
__global__ __launch_bounds__(1024) void flag_reduce_kernel(const Problem p)
{
    __shared__ int wave_cnt[16];
    __shared__ int base_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) base_s = 0;
    __syncthreads();
    for (int r0 = 0; r0 < p.rows; r0 += 1024) {
        const int row = r0 + tid;
        int f = 0;
        if (row < p.rows) {
            const int S = valid_len(p, row / p.Hq);
            const int nb = (S + p.C - 1) / p.C;
            const uint8_t *cf = p.ws.chunk_flags + (size_t)row * p.nc;
            for (int c = 0; c < nb; ++c) f |= cf[c];
            f = f ? 1 : 0;
            p.ws.row_flags[row] = (uint8_t)f;
        }
        const unsigned long long mask = __ballot(f);
        const int before = __popcll(mask & ((1ull << lane) - 1ull));
        if (lane == 0) wave_cnt[wave] = __popcll(mask);
        __syncthreads();
        int off = base_s, total = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < wave) off += wave_cnt[w];
            total += wave_cnt[w];
        }
        if (f) p.ws.list[off + before] = row;
        __syncthreads();
        if (tid == 0) base_s += total;
        __syncthreads();
    }
    if (tid == 0) *p.ws.count = base_s;
}

// Eq. 4 outer accumulation and the division, for rows that raised no flag.
__global__ __launch_bounds__(kHeadDim) void combine_unified_kernel(const Problem p)
{
    const int row = blockIdx.x, t = threadIdx.x;
    if (p.ws.row_flags[row]) return;            // recomputed by the synchronized scheme
    const int S = valid_len(p, row / p.Hq);
    const int nb = (S + p.C - 1) / p.C;
    const float *num = p.ws.num + (size_t)row * p.nc * kHeadDim + t;
    const float *den = p.ws.den + (size_t)row * p.nc;
    float s = 0.f, l = 0.f;
#pragma unroll 8
    for (int c = 0; c < nb; ++c) {
        s += num[(size_t)c * kHeadDim];
        l += den[c];
    }
    p.out[(size_t)row * kHeadDim + t] = nb > 0 ? to_half_bits(s / l) : (uint16_t)0;
}

// Eq. 2: m = max_c m_c, result = sum_c e^{m_c - m} (f.V)_c / sum_c e^{m_c - m} l_c.
__global__ __launch_bounds__(kHeadDim) void combine_sync_kernel(const Problem p, const int use_list)
{
    const int t = threadIdx.x;
    const int n = use_list ? *p.ws.count : p.rows;
    for (int i = blockIdx.x; i < n; i += gridDim.x) {
        const int row = use_list ? p.ws.list[i] : i;
        const int S = valid_len(p, row / p.Hq);
        const int nb = (S + p.C - 1) / p.C;
        const float *num = p.ws.num + (size_t)row * p.nc * kHeadDim + t;
        const float *den = p.ws.den + (size_t)row * p.nc;
        const float *mloc = p.ws.mloc + (size_t)row * p.nc;
        float m = -INFINITY;
        for (int c = 0; c < nb; ++c) m = fmaxf(m, mloc[c]);
        float s = 0.f, l = 0.f;
#pragma unroll 4
        for (int c = 0; c < nb; ++c) {
            const float a = __builtin_amdgcn_exp2f((mloc[c] - m) * kLog2e);
            s = __builtin_fmaf(a, num[(size_t)c * kHeadDim], s);
            l = __builtin_fmaf(a, den[c], l);
        }
        p.out[(size_t)row * kHeadDim + t] = nb > 0 ? to_half_bits(s / l) : (uint16_t)0;
    }
}

}  // namespace

hipError_t launch_clear_tickets(int32_t *ticket, size_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const size_t blocks = (n + 255) / 256;
    return launch(clear_tickets_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), s, ticket, n);
}

hipError_t launch_row_epilogue(const Problem &p, hipStream_t s)
{
    if (p.rows == 0) return hipSuccess;
    if (p.nc <= 8) return launch(rows8_epilogue_kernel, dim3((p.rows + 7) / 8), dim3(256), s, p);
    return launch(row_epilogue_kernel, dim3(p.rows), dim3(256), s, p);
}

hipError_t launch_flag_reduce(const Problem &p, hipStream_t s)
{
    return launch(flag_reduce_kernel, dim3(1), dim3(1024), s, p);
}

hipError_t launch_combine_unified(const Problem &p, hipStream_t s)
{
    if (p.rows == 0) return hipSuccess;
    return launch(combine_unified_kernel, dim3(p.rows), dim3(kHeadDim), s, p);
}

hipError_t launch_combine_sync(const Problem &p, bool use_list, hipStream_t s)
{
    if (p.rows == 0) return hipSuccess;
    const int grid = use_list ? (p.rows < 512 ? p.rows : 512) : p.rows;
    return launch(combine_sync_kernel, dim3(grid), dim3(kHeadDim), s, p, use_list ? 1 : 0);
}

}  // namespace fd
