// Small kernels: the flag reduction of fd_list_flagged_rows, the synchronized merge of
// Eq. 2 (fd_decode_attn_sync; third launch of the literal chain), the row epilogue as a
// launch of its own, and the counter clear of fd_workspace_init.
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

// Eq. 2: m = max_c m_c, result = sum_c e^{m_c - m} (f.V)_c / sum_c e^{m_c - m} l_c.
__global__ __launch_bounds__(kHeadDim) void combine_sync_kernel(const Problem p)
{
    const int t = threadIdx.x;
    const int row = blockIdx.x;
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

// Third launch of the literal chain.  Blocks 0 .. gridDim.x - 2 stride over the rows and finish the
// flagged ones: Eq. 2 over the row's recomputed partial vectors, m = max_c m_c, result =
// sum_c e^{m_c - m} (f.V)_c / sum_c e^{m_c - m} l_c.  The last block turns the row flags into the
// ascending list of flagged rows and their count (prefix sums over ballots, no atomics).
__global__ __launch_bounds__(kHeadDim) void chain_finish_kernel(const Problem p)
{
    const int t = threadIdx.x;
    const int workers = (int)gridDim.x - 1;
    if ((int)blockIdx.x == workers) {
        __shared__ int cnt[2];
        const int lane = t & 63, wave = t >> 6;
        int base = 0;
        for (int r0 = 0; r0 < p.rows; r0 += kHeadDim) {
            const int row = r0 + t;
            const int f = row < p.rows ? (int)p.ws.row_flags[row] : 0;
            const unsigned long long mask = __ballot(f);
            if (lane == 0) cnt[wave] = __popcll(mask);
            __syncthreads();
            const int before = (wave ? cnt[0] : 0) + __popcll(mask & ((1ull << lane) - 1ull));
            if (f) p.ws.list[base + before] = row;
            base += cnt[0] + cnt[1];
            __syncthreads();
        }
        if (t == 0) *p.ws.count = base;
        return;
    }
    for (int row = blockIdx.x; row < p.rows; row += workers) {
        if (!p.ws.row_flags[row]) continue;
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

hipError_t launch_chain_finish(const Problem &p, hipStream_t s)
{
    if (p.rows == 0) return hipSuccess;
    return launch(chain_finish_kernel, dim3((p.rows < 1024 ? p.rows : 1024) + 1), dim3(kHeadDim), s, p);
}

hipError_t launch_combine_sync(const Problem &p, hipStream_t s)
{
    if (p.rows == 0) return hipSuccess;
    return launch(combine_sync_kernel, dim3(p.rows), dim3(kHeadDim), s, p);
}

}  // namespace fd
