// Internal declarations shared by the libfdattn translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace fd {

constexpr int kComputeUnits = 256; // of an MI355X
constexpr int kHeadDim = 128;      // fp16 elements per K/V row = 256 bytes = 16 x 16-byte segments

// Chunk lengths are multiples of 16 from 64 to 4096 keys; the kernels are compiled for these
// capacities and a chunk runs on the smallest one that holds it.
inline int chunk_capacity(int len)
{
    int cap = 64;
    while (cap < len) cap *= 2;
    return cap;
}
constexpr float kLog2e = 1.4426950408889634f;

// One record per (row, chunk) slot, read by the row epilogue with a single 16-byte
// load: the slot's denominator, the reference its sums are scaled by (phi, or the
// chunk maximum after a recomputation) and whether the chunk's guard fired.
struct alignas(16) SlotMeta {
    float den, ref;
    int flagged, pad;
};

// Views into the caller's workspace.
struct WsView {
    float   *num;          // [rows, nc, 128]  sum e^{x-phi} v   (or f.V of the synchronized scheme)
    float   *den;          // [rows, nc]       sum e^{x-phi}     (or l)
    float   *mloc;         // [rows, nc]       chunk maximum m (synchronized scheme only)
    uint8_t *chunk_flags;  // [rows, nc]
    SlotMeta *meta;        // [rows, nc]  (den, reference, flag) handed to the row epilogue
    uint8_t *row_flags;    // [rows]  (room for rows * nc)
    int32_t *list;         // [rows]  flagged rows, ascending (room for rows * nc)
    int32_t *count;        // [1]     number of flagged rows
    int32_t *ticket;       // [rows, nc]  arrival counters (a small tree per row) of the fused kernels; zero between
                           // calls; they end where the workspace ends, whatever the shape
};

struct Problem {
    const uint16_t *q, *k, *v;
    const int32_t  *seq_lens;
    uint16_t       *out;
    WsView ws;
    int B, Hq, Hkv, G, Smax, C, nc, rows;
    float scale, phi, lo, hi;
    int chunk_major; // workgroup order of the grouped kernel, set at launch: 1 = chunk 0 of every row, then chunk 1, ...
    int elect;     // 1: chunk kernels elect a finisher per row and run the row epilogue themselves;
                   // 0: a separate row-epilogue launch follows (no per-workgroup hand-over latency)
    // Fused append (null otherwise): this step's K and V rows, [B, Hkv, D].  Sequence b then
    // has seq_lens[b] resident keys plus the new one at position seq_lens[b] (if the cache
    // has room); the new rows are taken from here, never from the cache, and are also
    // written into the cache through k_store / v_store (the cache pointers, writable).
    const uint16_t *k_new, *v_new;
    uint16_t *k_store, *v_store;
    // Paged cache (null otherwise): k and v are then pools [n_pages, Hkv, page, D] and token t of
    // sequence b lives in row t % page of page block_table[b * pages_per_seq + t / page];
    // page = 1 << page_shift.  Smax is the logical capacity pages_per_seq * page.
    const int32_t *block_table;
    int pages_per_seq, page_shift, n_pages;
    // Which XCD (workgroup index modulo 8) serves which row of a block of 8 rows (or head groups):
    //   0: row r on XCD r % 8, all its chunks on that one XCD;
    //   1: chunk c of row r on XCD (r + c) % 8 -- every XCD reads from every row.
    // Set at launch: 1 for the launches that leave the row epilogue to a second launch (see
    // row_slot below); the probe build can force 1 everywhere (tests of the hand-over).
    int scatter;
};

// XCD slot (workgroup index modulo 8) -> the row, or head group, within its block of 8 that the
// workgroup serves: the slot itself, or the slot rotated by the chunk.  With rows on fixed XCDs an
// XCD only ever reads addresses that agree in the bits just above the row stride, and for some row
// strides (4096 keys = 1 MiB: a batch of 16 x 32 rows) the memory system then serves it from a part
// of its channels only: 74 % of the HBM peak against 85 % with the rows spread (batch 16 x 4096
// keys, 1024-key chunks; 4 x 16384: 81 -> 85 %; 1 x 65536: 79 -> 83 %; shapes that were fast stay
// fast).  Launches that hand over between workgroups keep a row on one XCD (measured: no
// difference there, and the counters of a row then live in one L2).
__device__ __forceinline__ int row_slot(const Problem &p, int slot, int c)
{
    return p.scatter ? (slot - c) & 7 : slot;
}

// Number of keys resident in the cache: the clamped entry of seq_lens.
__device__ __forceinline__ int clamp_len(const Problem &p, int raw)
{
    raw = raw < 0 ? 0 : raw;
    return raw > p.Smax ? p.Smax : raw;
}
// Keys a row attends over: the resident ones plus the appended one, if any and if it fits.
__device__ __forceinline__ int effective_len(const Problem &p, int resident)
{
    return resident + ((p.k_new != nullptr) & (resident < p.Smax));
}
__device__ __forceinline__ int valid_len(const Problem &p, int b)
{
    return effective_len(p, clamp_len(p, p.seq_lens[b]));
}

// Launch that reports its own error code (the runtime's "last error" slot is shared
// with every other HIP user in the process and may hold a stale, unrelated value).
template <typename... KArgs>
inline hipError_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t s,
                         typename std::common_type<KArgs>::type... args)
{
    void *argv[] = {static_cast<void *>(&args)...};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, argv, 0, s);
}

// fd_row_kernels.hip : one query head per workgroup (VALU path)
hipError_t launch_decode_fused(const Problem &p, hipStream_t s);
hipError_t launch_partial_unified(const Problem &p, hipStream_t s);
hipError_t launch_chain_combine(const Problem &p, hipStream_t s);
hipError_t launch_partial_sync(const Problem &p, hipStream_t s);
// fd_reduce_kernels.hip : flag reduction, the synchronized merge, the chain's last launch, the row epilogue
hipError_t launch_flag_reduce(const Problem &p, hipStream_t s);
hipError_t launch_chain_finish(const Problem &p, hipStream_t s);
hipError_t launch_combine_sync(const Problem &p, hipStream_t s);
hipError_t launch_clear_tickets(int32_t *ticket, size_t n, hipStream_t s);
hipError_t launch_row_epilogue(const Problem &p, hipStream_t s);
// fd_gqa_kernels.hip : one KV head (a group of query heads) per workgroup (MFMA path)
hipError_t launch_decode_fused_gqa(const Problem &p, hipStream_t s);
// fd_stats_kernels.hip : histogram of the scaled logits (uses q, k, seq_lens and the shape only)
hipError_t launch_logit_histogram(const Problem &p, float x_min, float bin_width, int n_bins,
                                  unsigned long long *hist, float *min_max, hipStream_t s);
// fd_prefill_kernels.hip : prompt phase (causal attention of all prompt tokens at once)
struct PrefillProblem {
    const uint16_t *q, *k, *v;   // q [B, Hq, Smax, D]; k, v [B, Hkv, Smax, D]
    const int32_t *seq_lens;
    uint16_t *out;               // [B, Hq, Smax, D]
    uint16_t *vt;                // workspace: V transposed per KV head, tiled [Spad / 32][4][D][8 keys], fp16
    uint8_t *tile_flags;         // workspace: [B, Hq, tiles]
    int B, Hq, Hkv, G, Smax, Spad, tiles;   // Spad = Smax rounded up to 64; tiles = Spad / 64
    float scale, phi, lo, hi;
};
hipError_t launch_prefill(const PrefillProblem &p, hipStream_t s);

}  // namespace fd
