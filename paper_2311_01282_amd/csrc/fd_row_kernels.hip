// Chunk kernels that treat every query head as an independent row (VALU path).
// One workgroup of NW wavefronts handles one (row, chunk); see fd_chunk.h for the
// lane layout.
//
//   decode_fused_kernel    : the whole method in one launch.  Every workgroup
//       computes its chunk's Eq. 4 inner sums under the range guard; a chunk whose
//       guard fired is recomputed on the spot with its own maximum (Eq. 2); the
//       workgroup that finishes a row last (elected by a small tree of arrival
//       counters) runs the row epilogue.
//   partial_unified_kernel : Eq. 4 inner sums + guard only (first launch of the chain).
//   chain_combine_kernel   : row flags; Eq. 4 outer sums for clean rows, per-chunk
//       synchronized recomputation for flagged rows (second launch of the chain).
//   partial_sync_kernel    : per-chunk part of the synchronized scheme, for all rows.
#include "fd_chunk.h"

namespace fd {
namespace {

// Wavefronts per workgroup and pipeline depth per chunk size, from a sweep on
// MI355X at the 8K-context shape: 8 wavefronts pay off once a chunk holds at
// least 512 keys; 4 groups (4 KiB of K and of V per wavefront) per pipeline stage.
template <int C> struct Tune {
    static constexpr int NW = C >= 512 ? 8 : 4;
    static constexpr int NG = C / (4 * NW);
    static constexpr int UP = NG < 4 ? NG : 4;
};

// ELECT: the launch is small enough for the in-kernel hand-over.
// PAGED: K and V are page pools addressed through the sequence's block table.
// EARLY: the first loads go out before the sequence length has arrived -- for launches of at
//        most one workgroup per compute unit, where every workgroup starts with the launch and
//        the length load is on its critical path.  In a larger launch the later workgroups
//        start behind somebody else's stream anyway, and where the launch covers more than the
//        sequences hold (max_seq beyond the lengths) many of them are chunks without keys,
//        which then leave without reading any.
template <int C, bool ELECT, bool PAGED = false, bool EARLY = false>
__global__ __launch_bounds__(Tune<C>::NW * 64) void decode_fused_kernel(const Problem p)
{
    static_assert(!EARLY || (ELECT && !PAGED), "early loads: in-kernel hand-over, contiguous cache");
    constexpr int NW = Tune<C>::NW, UP = Tune<C>::UP;
    __shared__ ChunkLds<NW, C> lds;
    const int tid = threadIdx.x;
    if constexpr (ELECT) fetch_arguments_now(p);
    // Workgroups are dealt to the 8 XCDs round-robin by index.  In a launch that hands its rows
    // over inside the kernel all chunks of a row go to the same XCD (row % 8), so the row's counters
    // and partial results stay in one L2 instead of bouncing between eight; a launch that leaves the
    // epilogue to a second one spreads them (row_slot).  Placement only affects speed: every
    // hand-over below is device-coherent wherever the workgroups land.
    // Order within that: row-major -- all chunks of rows 0..7, then of rows 8..15, ... -- except in
    // the launches of at most one workgroup per compute unit (EARLY), which go chunk-major and whose
    // order hardly matters (every workgroup is resident at once).  Chunk-major order -- chunk 0 of
    // every row, then chunk 1, ... -- used to serve every launch of up to 1024 workgroups, because it
    // dispatches the chunks past the end of the sequences last (8192 keys in a cache of 16384: 33.5 ->
    // 29 us); but it confines a round of the chip to one slice of every row, and for rows of a
    // power-of-two stride that costs up to 20 % on some boxes (2 x 32 rows of 8192 keys, 1024-key
    // chunks: 54.3 us against 44.7 row-major on the same box; 1 x 32 rows of 16384 keys, 512-key chunks:
    // 51.1 against 46.3; other boxes: 45.8 either way), where row-major with the in-kernel hand-over
    // loses 4 % on the half-empty cache (24.2 -> 25.2 us, 25.9 -> 26.8 us at a quarter).
    const int groups8 = (p.rows + 7) >> 3;
    const int j = blockIdx.x >> 3;
    constexpr bool CM = EARLY;                 // chunk-major in the one-round launches only (see below)
    const int c = CM ? j / groups8 : j % p.nc;
    const int row = row_slot(p, blockIdx.x & 7, c) + 8 * (CM ? j - c * groups8 : j / p.nc);
    if (row >= p.rows) return;
    FD_PHASE(0);
    int S;
    const bool flagged = chunk_body<C, NW, UP, false, C, EARLY, PAGED>(p, row, c, lds, &S);
    FD_PHASE(3);
    const int nb = (S + p.C - 1) / p.C;        // chunks of this row that hold a valid key
    if (c >= nb) {                             // padding chunk: zero partials were written
        if (nb == 0 && c == 0 && ELECT) {    // empty sequence: nobody else owns the row
            if (tid < kHeadDim) p.out[(size_t)row * kHeadDim + tid] = 0;
            if (tid == 0) p.ws.row_flags[row] = 0;
        }
        return;
    }
    if (flagged) {                             // Section 3 "Recomputation", for this partial vector
        __syncthreads();
        chunk_body<C, NW, UP, true, C, false, PAGED>(p, row, c, lds);
    }

    if (!ELECT) return;                        // a row-epilogue launch follows
    // Publish this chunk's results (written through by chunk_body), then arrive; the
    // last arrival owns the row and reads the others' results past the caches.
    wait_stores_performed();
    __syncthreads();
    FD_PHASE(4);
    if (tid == 0) lds.last = arrive_and_elect(p, row, c, nb);
    __syncthreads();
    FD_PHASE(5);
    if (!lds.last) return;
    // up to 8 chunks: 32 threads walk them in registers (one round trip, no LDS, no barrier)
    if (nb <= 8) group_epilogue(p, row, 1, nb);
    else row_epilogue<NW, true>(p, row, nb, [nb] { return nb; }, &lds.acc[0][0]);
#ifdef FD_PHASE_PROBE
    wait_stores_performed();
    FD_PHASE(7);
#endif
}

// First launch of the literal chain: Eq. 4 inner sums and the range guard, nothing else (no
// recomputation, no hand-over).  Same workgroup shape, workgroup order and early loads as the
// fused kernel: SMALL = a launch of at most 1024 workgroups (kernel arguments fetched in one batch),
// EARLY = of at most 256 (chunk-major order, first loads before the sequence length has arrived).
template <int C, bool SMALL, bool EARLY>
__global__ __launch_bounds__(Tune<C>::NW * 64) void partial_unified_kernel(const Problem p)
{
    static_assert(!EARLY || SMALL, "early loads belong to the small launches");
    constexpr int NW = Tune<C>::NW, UP = Tune<C>::UP;
    __shared__ ChunkLds<NW, 1> lds;
    if constexpr (SMALL) fetch_arguments_now(p);
    const int groups8 = (p.rows + 7) >> 3;
    const int j = blockIdx.x >> 3;
    const int c = EARLY ? j / groups8 : j % p.nc;              // the fused kernel's orders
    const int row = row_slot(p, blockIdx.x & 7, c) + 8 * (EARLY ? j - c * groups8 : j / p.nc);
    if (row >= p.rows) return;
    chunk_body<C, NW, UP, false, 1, EARLY, false>(p, row, c, lds);
}

// Second launch of the literal chain, over (row, chunk) items: every item first forms its row's
// flag, the OR of the row's chunk flags (Section 3 "Recomputation": one logit out of range
// condemns the whole vector).
//   row clean   : the item of chunk 0 adds the row's partial sums and divides -- Eq. 4 outer
//                 sums, fixed order, no atomics; the other items have nothing to do;
//   row flagged : every item recomputes its chunk by the synchronized partial softmax -- chunk
//                 maximum m, l = sum e^{x-m}, f.V -- into the chunk's slot (Eq. 2, per partial
//                 vector); the third launch merges them.
// The grid is bounded; workgroups stride over the items.
template <int C> struct ChainTune {
    static constexpr int NW = 8;
    static constexpr int NG = C / (4 * NW);
    static constexpr int UP = NG < 8 ? NG : 8;
};
template <int C>
__global__ __launch_bounds__(ChainTune<C>::NW * 64) void chain_combine_kernel(const Problem p)
{
    constexpr int NW = ChainTune<C>::NW, UP = ChainTune<C>::UP;
    constexpr int KB = NW * 2;                  // items per batch: one per half wavefront
    __shared__ ChunkLds<NW, C> lds;
    __shared__ int item_flag[KB];
    const int tid = threadIdx.x, half = tid >> 5, j = tid & 31;
    const long long items = (long long)p.rows * p.nc;
    // Workgroups stride over the items (the chunks of a flagged row go to different workgroups) and
    // take them in batches of KB: the row flags of a whole batch are fetched at once -- 32 threads
    // per item OR the row's chunk flags -- so a batch of clean rows costs one memory round trip.
    // All nc slots are read: chunks without a valid key carry flag 0 and zero sums, so neither the
    // decision nor the outer sums need the sequence length.
    for (long long w0 = blockIdx.x; w0 < items; w0 += (long long)KB * gridDim.x) {
        const long long mine = w0 + (long long)half * gridDim.x;
        int f = 0;
        if (mine < items) {
            const uint8_t *cf = p.ws.chunk_flags + (size_t)(mine / p.nc) * p.nc;
            for (int i = j; i < p.nc; i += 32) f |= cf[i];
        }
        const unsigned long long any = __ballot(f != 0);
        if (j == 0) item_flag[half] = ((any >> (32 * (half & 1))) & 0xffffffffull) != 0ull;
        __syncthreads();
        for (int k = 0; k < KB; ++k) {
            const long long w = w0 + (long long)k * gridDim.x;
            if (w >= items) break;
            const int row = (int)(w / p.nc), c = (int)(w % p.nc);
            const int flagged = item_flag[k];
            if (c == 0 && tid == 0) p.ws.row_flags[row] = flagged ? 1 : 0;
            if (flagged) {
                chunk_body<C, NW, UP, true>(p, row, c, lds);                // (a chunk without keys leaves at once)
                __syncthreads();                                             // lds is reused by the next item
            } else if (c == 0) {
                // 4 slices of 128 threads; slice s adds chunks s, s+4, ...; the slices are added in order
                const int slice = tid >> 7, t = tid & 127;
                const float *num = p.ws.num + (size_t)row * p.nc * kHeadDim + t;
                const float *den = p.ws.den + (size_t)row * p.nc;
                float s = 0.f, l = 0.f;
#pragma unroll 4
                for (int i = slice; i < p.nc; i += 4) {
                    s += num[(size_t)i * kHeadDim];
                    l += den[i];
                }
                lds.acc[slice][t] = s;
                if (t == 0) lds.den[slice] = l;
                __syncthreads();
                if (tid < kHeadDim) {
                    const float st = ((lds.acc[0][t] + lds.acc[1][t]) + lds.acc[2][t]) + lds.acc[3][t];
                    const float lt = ((lds.den[0] + lds.den[1]) + lds.den[2]) + lds.den[3];
                    // an empty sequence has no term at all: zeros
                    p.out[(size_t)row * kHeadDim + t] = lt > 0.f ? to_half_bits(st / lt) : (uint16_t)0;
                }
                __syncthreads();
            }
        }
        __syncthreads();                        // item_flag is rewritten by the next batch
    }
}

// The synchronized partial softmax of every (row, chunk), one per workgroup (fd_decode_attn_sync).
template <int C>
__global__ __launch_bounds__(256) void partial_sync_kernel(const Problem p)
{
    constexpr int UP = C / 16 < 8 ? C / 16 : 8;
    __shared__ ChunkLds<4, C> lds;
    const int w = blockIdx.x;
    chunk_body<C, 4, UP, true>(p, w / p.nc, w % p.nc, lds);
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
        case 2048: return Launcher<2048>::run(args...);
        case 4096: return Launcher<4096>::run(args...);
        default:   return hipErrorInvalidValue;
    }
}

template <int C> struct FusedLauncher {
    static hipError_t run(const Problem &p0, hipStream_t s)
    {
        const unsigned grid = (unsigned)(8ll * ((p0.rows + 7) / 8) * p0.nc);
        if (grid == 0) return hipSuccess;
        Problem p = p0;
        p.scatter |= !p.elect;                     // no hand-over inside the launch: every XCD reads from every row
        if (p.block_table)
            return p.elect ? launch(decode_fused_kernel<C, true, true>, dim3(grid), dim3(Tune<C>::NW * 64), s, p)
                           : launch(decode_fused_kernel<C, false, true>, dim3(grid), dim3(Tune<C>::NW * 64), s, p);
        if (p.elect && grid <= (unsigned)kComputeUnits)
            return launch(decode_fused_kernel<C, true, false, true>, dim3(grid), dim3(Tune<C>::NW * 64), s, p);
        return p.elect ? launch(decode_fused_kernel<C, true>, dim3(grid), dim3(Tune<C>::NW * 64), s, p)
                       : launch(decode_fused_kernel<C, false>, dim3(grid), dim3(Tune<C>::NW * 64), s, p);
    }
};

template <int C> struct UnifiedLauncher {
    static hipError_t run(const Problem &p0, hipStream_t s)
    {
        const unsigned grid = (unsigned)(8ll * ((p0.rows + 7) / 8) * p0.nc);
        if (grid == 0) return hipSuccess;
        Problem p = p0;
        p.scatter |= grid > 1024u;                 // no hand-over in this launch; measured on large grids only
        const dim3 block(Tune<C>::NW * 64);
        if (grid <= (unsigned)kComputeUnits) return launch(partial_unified_kernel<C, true, true>, dim3(grid), block, s, p);
        if (grid <= 1024u) return launch(partial_unified_kernel<C, true, false>, dim3(grid), block, s, p);
        return launch(partial_unified_kernel<C, false, false>, dim3(grid), block, s, p);
    }
};

template <int C> struct ChainCombineLauncher {
    static hipError_t run(const Problem &p, hipStream_t s)
    {
        const long long items = (long long)p.rows * p.nc;
        if (items == 0) return hipSuccess;
        // two workgroups of 8 wavefronts fit a compute unit: one round of the chip, striding over the items
        const unsigned grid = (unsigned)(items < 512 ? items : 512);
        return launch(chain_combine_kernel<C>, dim3(grid), dim3(ChainTune<C>::NW * 64), s, p);
    }
};

template <int C> struct SyncLauncher {
    static hipError_t run(const Problem &p, hipStream_t s)
    {
        const long long all = (long long)p.rows * p.nc;
        if (all == 0) return hipSuccess;
        return launch(partial_sync_kernel<C>, dim3((unsigned)all), dim3(256), s, p);
    }
};

}  // namespace

#ifdef FD_PHASE_PROBE
// Probe build only: copies the phase log of the last fused per-row launch to the host
// (synchronizes the device).  `n` = number of 64-bit stamps wanted, <= 4096 * 8.
extern "C" int fd_phase_probe_read(unsigned long long *host_dst, size_t n)
{
    if (!host_dst || n > (size_t)kPhaseMaxGrid * kPhaseSlots) return 1;
    if (hipDeviceSynchronize() != hipSuccess) return 6;
    return hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(fd_phase_log), n * sizeof(unsigned long long), 0,
                               hipMemcpyDeviceToHost) == hipSuccess ? 0 : 6;
}
#endif

hipError_t launch_decode_fused(const Problem &p, hipStream_t s)
{
    return dispatch_chunk<FusedLauncher>(chunk_capacity(p.C), p, s);
}

hipError_t launch_partial_unified(const Problem &p, hipStream_t s)
{
    return dispatch_chunk<UnifiedLauncher>(chunk_capacity(p.C), p, s);
}

hipError_t launch_chain_combine(const Problem &p, hipStream_t s)
{
    return dispatch_chunk<ChainCombineLauncher>(chunk_capacity(p.C), p, s);
}

hipError_t launch_partial_sync(const Problem &p, hipStream_t s)
{
    return dispatch_chunk<SyncLauncher>(chunk_capacity(p.C), p, s);
}

}  // namespace fd
