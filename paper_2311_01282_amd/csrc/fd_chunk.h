// Device code shared by the chunk kernels: the per-(row, chunk) body of the VALU
// path and the row epilogue (outer sums / synchronized merge).
//
// Lane layout of the VALU path.  A K or V row is 256 bytes = 16 segments of 16
// bytes; lane l of a wavefront owns segment l%16 of key (l/16) within a group of
// 4 consecutive keys, so one wavefront load instruction reads 1 KiB of contiguous
// cache memory with 128-bit loads.  The four wavefronts of a workgroup interleave
// groups, i.e. the workgroup walks the chunk front to back 4 KiB at a time.  The
// 16 lanes of a key reduce their 8-element partial dot products with DPP row
// operations (a DPP row is exactly 16 lanes), after which every one of the 16
// lanes holds the key's logit and scales its own 8 elements of the V row.
// K and V are read exactly once and never reused, so they are loaded with
// non-temporal loads straight into registers; LDS only carries the final
// cross-wavefront reduction.
#pragma once

#include <type_traits>

#include "fd_internal.h"

namespace fd {

// Phase probe (a build of its own, -DFD_PHASE_PROBE, never the product library): thread 0 of
// every workgroup of the per-row fused kernel stamps the device's constant-rate clock (100 MHz)
// at fixed points into a log that fd_phase_probe_read copies out.  Slots: 0 kernel entered,
// 1 first block's data used, 2 chunk loop done, 3 workgroup's sums reduced and stores issued,
// 4 stores performed, 5 arrival counted, 6 (finisher) partial results loaded and merged, 7
// (finisher) output stored and performed.
#ifdef FD_PHASE_PROBE
constexpr int kPhaseSlots = 8, kPhaseMaxGrid = 4096;
static __device__ unsigned long long fd_phase_log[kPhaseMaxGrid * kPhaseSlots];
#define FD_PHASE(i)                                                                                         \
    do {                                                                                                    \
        __builtin_amdgcn_sched_barrier(0);                                                                  \
        if (threadIdx.x == 0 && blockIdx.x < (unsigned)kPhaseMaxGrid)                                       \
            fd_phase_log[(size_t)blockIdx.x * kPhaseSlots + (i)] = wall_clock64();                          \
        __builtin_amdgcn_sched_barrier(0);                                                                  \
    } while (0)
#else
#define FD_PHASE(i) do { } while (0)
#endif

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// (bit-casting a vector ELEMENT in place is unreliable: take the element by value first)
__device__ __forceinline__ half2_t as_h2(uint32_t u) { return __builtin_bit_cast(half2_t, u); }
__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }

// 128-bit streaming load: the data is used once, keep it from displacing other lines.
__device__ __forceinline__ u32x4 load_stream(const u32x4 *p) { return __builtin_nontemporal_load(p); }

// fp32 dot product of 8 fp16 pairs; every product is exact in fp32.
__device__ __forceinline__ float dot8(const u32x4 &a, const u32x4 &b)
{
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const half2_t x = as_h2(a[i]), y = as_h2(b[i]);
        acc = __builtin_fmaf((float)x.x, (float)y.x, acc);
        acc = __builtin_fmaf((float)x.y, (float)y.y, acc);
    }
    return acc;
}

// acc[0..7] += p * v[0..7]
__device__ __forceinline__ void axpy8(float (&acc)[8], float p, const u32x4 &v)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const half2_t x = as_h2(v[i]);
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

// Device-coherent accesses for results that another workgroup of the SAME launch
// reads (the per-chunk partial results and the per-row ticket).  Each XCD has its
// own L2, so such data is written through and read past the L2 ("agent scope"
// relaxed atomics); ordinary cached accesses would need an L2 write-back fence per
// workgroup, which costs about a microsecond each and serializes per XCD.
template <typename T>
__device__ __forceinline__ void store_coherent(T *p, T v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ T load_coherent(const T *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The (den, reference, flag) record of a slot, written through as two 8-byte words.
__device__ __forceinline__ void store_meta(const Problem &p, size_t slot, float den, float ref, int flagged)
{
    unsigned long long *w = reinterpret_cast<unsigned long long *>(&p.ws.meta[slot]);
    store_coherent(&w[0], (unsigned long long)__builtin_bit_cast(unsigned, den) |
                              ((unsigned long long)__builtin_bit_cast(unsigned, ref) << 32));
    store_coherent(&w[1], (unsigned long long)(unsigned)flagged);
}

// Four consecutive floats written through as two 8-byte words (16-byte aligned).
__device__ __forceinline__ void store_coherent4(float *ptr, float a, float b, float c, float d)
{
    unsigned long long *w = reinterpret_cast<unsigned long long *>(ptr);
    store_coherent(&w[0], (unsigned long long)__builtin_bit_cast(unsigned, a) | ((unsigned long long)__builtin_bit_cast(unsigned, b) << 32));
    store_coherent(&w[1], (unsigned long long)__builtin_bit_cast(unsigned, c) | ((unsigned long long)__builtin_bit_cast(unsigned, d) << 32));
}

// Wait until this thread's earlier stores are performed (vector memory counter at
// zero); with write-through stores this is the release half of the hand-over.
__device__ __forceinline__ void wait_stores_performed()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

__device__ __forceinline__ uint16_t to_half_bits(float x)
{
    return __builtin_bit_cast(uint16_t, (_Float16)x);   // round to nearest even
}

// LDS of one workgroup of NW wavefronts.  XN = number of logits kept for the
// synchronized scheme.
template <int NW, int XN>
struct ChunkLds {
    float acc[NW * 4][kHeadDim];   // [wave*4 + key-in-group][element]; reused by the row epilogue
    float x[XN];
    float den[NW * 4];
    float mx[NW];
    int   flag[NW];
    int   last;
};

// One (row, chunk) on the VALU path, by a workgroup of NW wavefronts.
//   SYNC == false : unified scaling factor phi -- Eq. 4 inner sums and the range
//                   guard of Section 3 "Recomputation".  Writes num, den,
//                   chunk_flags and mloc = phi (the reference the sums are scaled by).
//   SYNC == true  : the chunk's part of the synchronized partial softmax, Eq. 2:
//                   m = max x, l = sum e^{x-m}, f.V = sum e^{x-m} v.  Writes num,
//                   den, mloc = m and leaves chunk_flags alone; `sync_flag` is what the
//                   slot's record tells the row epilogue about the guard.
// UP = groups of 4 keys per wavefront per pipeline stage.
// Returns (uniformly over the workgroup) whether the guard fired (false for SYNC).
// Pins the kernel arguments the chunk loop needs into scalar registers at this point,
// so that their loads leave in one batch at the top of the kernel.  Left alone the
// compiler fetches each cache line of the argument block where it is first used --
// behind the early-exit test, behind the index arithmetic -- and a fresh wavefront
// then pays three dependent memory latencies instead of one.
__device__ __forceinline__ void fetch_arguments_now(const Problem &p)
{
    asm volatile("" ::"s"(p.q), "s"(p.k), "s"(p.v), "s"(p.seq_lens), "s"(p.Hq), "s"(p.G), "s"(p.Hkv), "s"(p.Smax),
                 "s"(p.nc), "s"(p.rows));
}

// The sequence length through a vector load, in two halves.  Scalar loads return out
// of order, so waiting for any of them waits for all: a scalar length load would be
// waited for together with the kernel arguments, before the first K/V load can go
// out.  Vector loads return in order; this one stays in flight behind the loads
// issued between the two halves.  (The opaque zero keeps the compiler from proving
// the address uniform and turning the load back into a scalar one.)
__device__ __forceinline__ int seq_len_issue(const Problem &p, int b)
{
    int zero;
    asm("v_mov_b32 %0, 0" : "=v"(zero));
    return p.seq_lens[b + zero];
}
__device__ __forceinline__ int seq_len_finish(const Problem &p, int raw)
{
    return clamp_len(p, __builtin_amdgcn_readfirstlane(raw));     // resident keys
}

// Where the rows of a chunk's keys are, in 16-byte units from the start of K (or V; both are
// laid out alike): consecutive rows of the caller's buffer, or -- paged cache -- row t % page of
// the page the sequence's table names for t / page.  A chunk spans at most 64 pages (the
// entry points see to it); each lane fetches one table entry when the chunk starts and a lane
// exchange hands every lane the page of the key it is about to load.  Entries of pages that
// hold no valid key may be anything: they are clamped into the pool and what they bring in is
// never used.
template <bool PAGED> struct KvRows {
    size_t base;             // first row of the chunk (contiguous), 0 (paged)
    int pages, first, start, shift, hkv, Hkv;
    __device__ __forceinline__ KvRows(const Problem &p, int b, int hkv_, int start_, int lane)
        : base(PAGED ? 0 : (((size_t)b * p.Hkv + hkv_) * p.Smax + start_) * 16), pages(0), first(0), start(start_),
          shift(p.page_shift), hkv(hkv_), Hkv(p.Hkv)
    {
        if constexpr (PAGED) {
            first = start_ >> shift;
            const int entry = p.block_table[(size_t)b * p.pages_per_seq + min(first + lane, p.pages_per_seq - 1)];
            pages = min(max(entry, 0), p.n_pages - 1);
        }
    }
    // First row, relative to `base`, of the 16 keys key0 .. key0 + 15 (key0 a multiple of 16, the same
    // for the whole wavefront): they share a page, which one lane-to-scalar read finds.
    __device__ __forceinline__ size_t block16(int key0) const
    {
        if constexpr (PAGED) {
            const int t = start + key0;
            const int page = __builtin_amdgcn_readlane(pages, (t >> shift) - first);
            return ((((size_t)page * Hkv + hkv) << shift) + (size_t)(t & ((1 << shift) - 1))) * 16;
        } else {
            return (size_t)key0 * 16;
        }
    }
    // row of chunk-relative key `key` from the start of the buffer or pool (for the store of an appended row)
    __device__ __forceinline__ size_t absolute(int key) const { return base + (*this)(key); }
    // row of chunk-relative key `key`, relative to `base`
    __device__ __forceinline__ size_t operator()(int key) const
    {
        if constexpr (PAGED) {
            const int t = start + key;
            const int page = __builtin_amdgcn_ds_bpermute(((t >> shift) - first) << 2, pages);
            return ((((size_t)page * Hkv + hkv) << shift) + (size_t)(t & ((1 << shift) - 1))) * 16;
        } else {
            return (size_t)key * 16;
        }
    }
};

// EARLY (unified scheme only): the first block's loads are issued before the
// sequence length has arrived, clamped to the chunk's extent in the padded buffer
// instead of to the last valid key; what they bring in from beyond the valid
// length is replaced by zeros before use.  Takes the length load off the critical
// path of a short launch; a padding chunk then reads one block for nothing, so
// large ragged launches leave it off.
template <int C, int NW, int UP, bool SYNC, int XN, bool EARLY = false, bool PAGED = false>
__device__ __forceinline__ bool chunk_body(const Problem &p, int row, int c, ChunkLds<NW, XN> &lds, int *len_out = nullptr,
                                           int sync_flag = 1)
{
    static_assert(!(EARLY && SYNC), "early loads belong to the unified scheme");
    static_assert(!(EARLY && PAGED), "the page table has to arrive before the first load");
    static_assert(!SYNC || XN >= C, "the synchronized scheme keeps the chunk's logits in LDS");
    constexpr int NG = C / (4 * NW);           // groups of 4 keys each wavefront handles
    static_assert(NG >= 1 && NG % UP == 0, "chunk, wavefront count and stage depth must divide");
    constexpr int NBLK = NG / UP;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int seg = lane & 15, sub = lane >> 4;

    const int b = row / p.Hq;
    const int hq = row - b * p.Hq;
    const int hkv = hq / p.G;
    int S_raw = 0;
    if constexpr (EARLY) S_raw = seq_len_issue(p, b);
    const int len = p.C;                       // keys per chunk (<= C, the kernel's capacity)
    const int start = c * len;
    const size_t slot = (size_t)row * p.nc + c;

    const u32x4 qv = reinterpret_cast<const u32x4 *>(p.q + (size_t)row * kHeadDim)[seg];
    const KvRows<PAGED> at(p, b, hkv, start, lane);
    const u32x4 *kp = reinterpret_cast<const u32x4 *>(p.k) + at.base + seg;
    const u32x4 *vp = reinterpret_cast<const u32x4 *>(p.v) + at.base + seg;
    // key handled by this lane in group g of the chunk: the NW wavefronts interleave
    auto key_of = [&](int g) { return (g * NW + wave) * 4 + sub; };
    u32x4 kA[UP], vA[UP];
    if constexpr (EARLY) {
        const int cap = min(len, p.Smax - start) - 1;   // the chunk's last key inside the buffer (start < Smax)
#pragma unroll
        for (int u = 0; u < UP; ++u) kA[u] = load_stream(kp + at(min(key_of(u), cap)));
#pragma unroll
        for (int u = 0; u < UP; ++u) vA[u] = load_stream(vp + at(min(key_of(u), cap)));
    }

    if constexpr (EARLY) __builtin_amdgcn_sched_barrier(0);   // the loads above go out before the length is awaited
    const int S_res = EARLY ? seq_len_finish(p, S_raw) : clamp_len(p, p.seq_lens[b]);
    const int S = effective_len(p, S_res);
    if (len_out) *len_out = S;
    const int nvalid = min(len, S - start);    // <= 0: no valid key in this chunk
    const int nres = min(len, S_res - start);  // of them resident in the cache
    // A fused append puts the new key at offset jn of exactly one chunk of the row.
    const int jn = S_res - start;
    const bool owner = (S != S_res) & (jn >= 0) & (jn < len);
    // where the appended row goes (all lanes take part in the page lookup of a paged cache)
    const size_t row_new = at.absolute(owner ? jn : 0);
    // With early loads an empty chunk takes the ordinary path below (no block beyond the
    // first is touched, every key is masked): a branch here would pull the loads behind it.
    if (!EARLY && nvalid <= 0) {               // empty chunk: zero partials, no flag
        if (tid < kHeadDim) p.ws.num[slot * kHeadDim + tid] = 0.f;
        if (tid == 0) {
            p.ws.den[slot] = 0.f;
            p.ws.mloc[slot] = SYNC ? -INFINITY : p.phi;
            store_meta(p, slot, 0.f, p.phi, 0);
            if (!SYNC) p.ws.chunk_flags[slot] = 0;
        }
        return false;
    }

    const int last = nres - 1;                 // last resident key; the appended one is handled apart
    // blocks (of UP groups per wavefront) that hold at least one resident key
    const int nblk = min(NBLK, (nres + UP * NW * 4 - 1) / (UP * NW * 4));
    // the appended rows of this row's KV head
    const u32x4 *knp = reinterpret_cast<const u32x4 *>(p.k_new + ((size_t)b * p.Hkv + hkv) * kHeadDim) + seg;
    const u32x4 *vnp = reinterpret_cast<const u32x4 *>(p.v_new + ((size_t)b * p.Hkv + hkv) * kHeadDim) + seg;

    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float den = 0.f;
    float mc = p.phi;

    if constexpr (!SYNC) {
        // Software pipeline over blocks of UP groups: the loads of block i+1 are in
        // flight while block i is reduced.  Keys past the valid length re-read the
        // last valid key (always in bounds, never padding) and get weight zero.
        const float nphi = -p.phi, lo = p.lo, hi = p.hi, scale = p.scale;
        bool bad = false;
        // Rows of more than 32 chunks: every workgroup starts its chunk at a different block and wraps
        // around (the sums do not care about the order).  The workgroups of such a launch start at
        // addresses a power of two apart and walk them in step, and for some shapes the memory system
        // serves that badly: 1 x 32 rows x 131072 keys in 1024-key chunks 462 -> 338 us, 2 x 131072
        // 718 -> 652, 1 x 131072 in 2048-key chunks 333 -> 317; the shapes that were fine lose up to
        // 1.4 % (4 x 65536), and with 32 chunks per row or fewer (4 x 32768: 321 -> 330 us) it only costs.
        const int rot = (!EARLY && p.nc > 32 && nblk > 1) ? (int)((unsigned)(c * 3 + row) % (unsigned)nblk) : 0;
        auto phys = [&](int blk) { const int b = blk + rot; return b >= nblk ? b - nblk : b; };
        auto issue = [&](int blk0, u32x4 (&kk)[UP], u32x4 (&vv)[UP]) {
            const int blk = phys(blk0);
#pragma unroll
            for (int u = 0; u < UP; ++u) kk[u] = load_stream(kp + at(min(key_of(blk * UP + u), last)));
#pragma unroll
            for (int u = 0; u < UP; ++u) vv[u] = load_stream(vp + at(min(key_of(blk * UP + u), last)));
        };
        auto reduce = [&](int blk0, const u32x4 (&kk)[UP], const u32x4 (&vv)[UP]) {
            const int blk = phys(blk0);
#pragma unroll
            for (int u = 0; u < UP; ++u) {
                const bool valid = key_of(blk * UP + u) <= last;
                const float x = row16_sum(dot8(qv, kk[u])) * scale;
                const float d = x + nphi;                       // x - phi
                bad |= valid & !((d > lo) & (d < hi));          // equality and NaN flag
                float e = __builtin_amdgcn_exp2f(d * kLog2e);   // e^{x - phi}
                e = valid ? e : 0.f;
                den += e;
                axpy8(acc, e, vv[u]);
            }
        };
        u32x4 kB[UP], vB[UP];
        int blk = 0;
        if constexpr (EARLY) {
            // Block 0 is already in flight.  Block 1 goes out before block 0 is touched
            // (clamped into the chunk even when no key is valid), then the loop keeps two
            // blocks in flight; loads past the last block re-read the last valid key.
            if constexpr (NBLK > 1) {
#pragma unroll
                for (int u = 0; u < UP; ++u) kB[u] = load_stream(kp + at(max(min(key_of(UP + u), last), 0)));
#pragma unroll
                for (int u = 0; u < UP; ++u) vB[u] = load_stream(vp + at(max(min(key_of(UP + u), last), 0)));
            }
#pragma unroll
            for (int u = 0; u < UP; ++u)
                if (key_of(u) > last) vA[u] = u32x4{0u, 0u, 0u, 0u};   // padding may hold anything
#ifdef FD_PHASE_PROBE
            // (probe build only: the first block peeled so that its arrival can be stamped)
            if (blk + 2 < nblk) {
                reduce(blk, kA, vA);
                FD_PHASE(1);
                issue(blk + 2, kA, vA);
                reduce(blk + 1, kB, vB);
                issue(blk + 3, kB, vB);
                blk += 2;
            }
#endif
#pragma unroll 1
            for (; blk + 2 < nblk; blk += 2) {
                reduce(blk, kA, vA);
                issue(blk + 2, kA, vA);
                reduce(blk + 1, kB, vB);
                issue(blk + 3, kB, vB);
            }
            reduce(blk, kA, vA);
            if constexpr (NBLK > 1) {
                if (blk + 1 < nblk) reduce(blk + 1, kB, vB);
            }
        } else if (nres > 0) {                     // (a chunk may hold the appended key only)
            // The steady-state loop issues unconditionally (a load inside a branch
            // would force a full wait at the join); the last one or two blocks are peeled.
            issue(0, kA, vA);
#pragma unroll 1
            for (; blk + 2 < nblk; blk += 2) {
                issue(blk + 1, kB, vB);
                reduce(blk, kA, vA);
                issue(blk + 2, kA, vA);
                reduce(blk + 1, kB, vB);
            }
            if (blk + 2 == nblk) {
                issue(blk + 1, kB, vB);
                reduce(blk, kA, vA);
                reduce(blk + 1, kB, vB);
            } else {
                reduce(blk, kA, vA);
            }
        }
        if (owner && wave == 0 && sub == 0) {
            // The appended key: one more term of Eq. 4, taken from the step's own K/V rows by
            // the 16 lanes of the first key column, which also put the rows into the cache.
            const u32x4 kn = *knp, vn = *vnp;
            const float d = row16_sum(dot8(qv, kn)) * scale + nphi;
            bad |= !((d > lo) & (d < hi));
            const float e = __builtin_amdgcn_exp2f(d * kLog2e);
            den += e;
            axpy8(acc, e, vn);
            if (hq == hkv * p.G) {                  // one writer per KV head
                reinterpret_cast<u32x4 *>(p.k_store)[row_new + seg] = kn;
                reinterpret_cast<u32x4 *>(p.v_store)[row_new + seg] = vn;
            }
        }
        const unsigned long long any_bad = __ballot(bad);
        if (lane == 0) lds.flag[wave] = any_bad != 0ull;
    } else {
        // Pass 1: logits of the whole chunk into LDS, and their maximum.  An appended key
        // takes its place at offset jn with the logit of the step's own K row; loads of
        // non-resident positions are clamped into the chunk and their values replaced.
        float m = -INFINITY;
        const float scale = p.scale;
        const int jnew = owner ? jn : -1;
        u32x4 vn = {0u, 0u, 0u, 0u};
        float x_new = -INFINITY;
        if (owner) {
            x_new = row16_sum(dot8(qv, *knp)) * scale;
            vn = *vnp;
        }
        const int nblk_all = min(NBLK, (nvalid + UP * NW * 4 - 1) / (UP * NW * 4));
#pragma unroll 1
        for (int blk = 0; blk < nblk_all; ++blk) {
            u32x4 kk[UP];
#pragma unroll
            for (int u = 0; u < UP; ++u) kk[u] = load_stream(kp + at(max(min(key_of(blk * UP + u), last), 0)));
#pragma unroll
            for (int u = 0; u < UP; ++u) {
                const int kidx = key_of(blk * UP + u);
                float x = row16_sum(dot8(qv, kk[u])) * scale;
                x = kidx <= last ? x : (kidx == jnew ? x_new : -INFINITY);
                if (seg == 0) lds.x[kidx] = x;
                m = fmaxf(m, x);
            }
        }
        // chunk maximum: over the 4 keys of the lane's column, then the wavefronts
        m = fmaxf(m, __shfl_xor(m, 16));
        m = fmaxf(m, __shfl_xor(m, 32));
        if (lane == 0) lds.mx[wave] = m;
        __syncthreads();
        mc = lds.mx[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) mc = fmaxf(mc, lds.mx[w]);
        // Pass 2: e^{x - m} and the V products.
#pragma unroll 1
        for (int blk = 0; blk < nblk_all; ++blk) {
            u32x4 vv[UP];
#pragma unroll
            for (int u = 0; u < UP; ++u) vv[u] = load_stream(vp + at(max(min(key_of(blk * UP + u), last), 0)));
#pragma unroll
            for (int u = 0; u < UP; ++u) {
                const int kidx = key_of(blk * UP + u);
                const float e = __builtin_amdgcn_exp2f((lds.x[kidx] - mc) * kLog2e);   // 0 for padding
                den += e;
                // the appended V row for its key, and for every key when no resident row was
                // there to clamp to (weight zero then, but the cache may hold anything)
                axpy8(acc, e, ((kidx == jnew) | (nres <= 0)) ? vn : vv[u]);
            }
        }
        if (owner && hq == hkv * p.G && wave == 0 && sub == 0 && p.k_store) {
            // a recomputed chunk of the fused kernels has stored the rows already; the
            // synchronized entry points come here first
            reinterpret_cast<u32x4 *>(p.k_store)[row_new + seg] = *knp;
            reinterpret_cast<u32x4 *>(p.v_store)[row_new + seg] = vn;
        }
    }

    if constexpr (!SYNC) FD_PHASE(2);
    // Workgroup reduction: NW*4 partial vectors (NW wavefronts x 4 keys per group).
    // LDS row layout: elements 8s..8s+3 at 4s, elements 8s+4..8s+7 at 64 + 4((s + 4) & 15). Both the
    // 16-byte writes here and the 4-byte reads below then touch every bank once per pass.
    float *arow = lds.acc[wave * 4 + sub];
    *reinterpret_cast<float4 *>(&arow[4 * seg]) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    *reinterpret_cast<float4 *>(&arow[64 + 4 * ((seg + 4) & 15)]) = make_float4(acc[4], acc[5], acc[6], acc[7]);
    if (seg == 0) lds.den[wave * 4 + sub] = den;
    __syncthreads();
    bool flagged = false;
    if constexpr (!SYNC) {
#pragma unroll
        for (int w = 0; w < NW; ++w) flagged |= lds.flag[w] != 0;
    }
    if (tid < kHeadDim) {
        const int es = tid >> 3;                   // element tid sits in 16-byte segment es
        const int pos = (tid & 4) ? 64 + 4 * ((es + 4) & 15) + (tid & 3) : 4 * es + (tid & 3);
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < NW * 4; ++i) s += lds.acc[i][pos];
        store_coherent(&p.ws.num[slot * kHeadDim + tid], s);
    } else if (tid == kHeadDim) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < NW * 4; ++i) s += lds.den[i];
        store_coherent(&p.ws.den[slot], s);
        store_coherent(&p.ws.mloc[slot], mc);
        // the flag the row epilogue ORs into the row flag: the guard's; a recomputed chunk carries what its caller
        // says (1 when the guard sent it here, 0 when it is redone for another reason)
        store_meta(p, slot, s, mc, SYNC ? sync_flag : (int)flagged);
        if (!SYNC) p.ws.chunk_flags[slot] = flagged ? 1 : 0;
    }
    return flagged;
}

// Row epilogue, run by the one workgroup that owns the row's output (its first 256
// threads do the arithmetic): the synchronized update of Eq. 2 over the row's
// partial results, each scaled by its own reference r_c -- phi for chunks summed
// with the unified factor, the chunk maximum for recomputed ones:
//     m = max_c r_c,   out = sum_c e^{r_c-m} num_c / sum_c e^{r_c-m} den_c,
// evaluated in one pass with a running maximum (partial sums are merged by the same
// rule).  For a row without flags every r_c is phi, every factor is exactly 1 and
// the expression IS the plain outer sum of Eq. 4, so one code path serves both.
// Work split: 8 slices of 32 threads; slice k takes chunks k, k+8, ...; a thread
// owns 4 consecutive output elements, so a chunk costs it one 16-byte load of the
// numerator and one of the slot record.  Fixed summation order: no atomics on data,
// same bits on every run.
// Slots [0, n_load) are loaded (all of them hold defined values: chunks without a
// valid key carry zeros), slots [0, nb) enter the result; passing n_load = nc lets
// the loads start before the sequence length is known.
// COHERENT: the partial results come from other workgroups of the same launch and
// are read past the caches; false is for a launch of its own.
// `scratch` is >= 8 * 128 + 16 floats of LDS.
template <int NW, bool COHERENT, typename NbFn>
__device__ __forceinline__ void row_epilogue(const Problem &p, int row, int n_load, NbFn nb_fn, float *scratch)
{
    auto ld16 = [](const void *ptr) {
        if constexpr (COHERENT) {
            const unsigned long long *w = static_cast<const unsigned long long *>(ptr);
            const unsigned long long a = load_coherent(&w[0]), b = load_coherent(&w[1]);
            return u32x4{(unsigned)a, (unsigned)(a >> 32), (unsigned)b, (unsigned)(b >> 32)};
        } else {
            return *static_cast<const u32x4 *>(ptr);
        }
    };
    const int tid = threadIdx.x;
    const int slice = (tid >> 5) & 7, t4 = tid & 31;
    const bool worker = NW * 64 <= 256 || tid < 256;
    const size_t r0 = (size_t)row * p.nc;
    const float *num = p.ws.num + r0 * kHeadDim + 4 * t4;
    const SlotMeta *meta = p.ws.meta + r0;

    // Within a batch the loads are unconditional and clamped to the last loaded slot (a load
    // inside a divergent branch would force a full wait where the branch rejoins); slots
    // outside the row are masked in the arithmetic.  The batch is sized to the row -- 1, 2 or
    // 4 chunks per thread -- and rows of more than 32 chunks keep two batches in flight.
    float m = -INFINITY, l = 0.f;
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    int f = 0;
    int nb = 0;
    if (worker) {
        const int cap = max(n_load - 1, 0);
        auto issue = [&](int c0, auto &nv, auto &mv, auto n) {
#pragma unroll
            for (int i = 0; i < decltype(n)::value; ++i) {
                const int c = min(c0 + 8 * i + slice, cap);
                nv[i] = ld16(num + (size_t)c * kHeadDim);
                mv[i] = ld16(meta + c);
            }
        };
        auto process = [&](int c0, const auto &nv, const auto &mv, auto n) {
            constexpr int N = decltype(n)::value;
            float r[N], bm = -INFINITY;
#pragma unroll
            for (int i = 0; i < N; ++i) {
                const bool in_row = c0 + 8 * i + slice < nb;
                r[i] = in_row ? as_f32(mv[i][1]) : -INFINITY;
                bm = fmaxf(bm, r[i]);
                f |= in_row ? (int)mv[i][2] : 0;
            }
            if (bm > m) {                       // rescale what was summed so far (never for unflagged rows)
                const float a = __builtin_amdgcn_exp2f((m - bm) * kLog2e);   // 0 on the first batch
#pragma unroll
                for (int e = 0; e < 4; ++e) s[e] *= a;
                l *= a;
                m = bm;
            }
#pragma unroll
            for (int i = 0; i < N; ++i) {
                // exactly 1 when r_c == m; 0 for slots outside the row (their sums are finite)
                const float a = r[i] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((r[i] - m) * kLog2e);
#pragma unroll
                for (int e = 0; e < 4; ++e) s[e] = __builtin_fmaf(a, as_f32(nv[i][e]), s[e]);
                l = __builtin_fmaf(a, as_f32(mv[i][0]), l);
            }
        };
        auto single = [&](auto n) {             // the whole row in one batch of N chunks per thread
            u32x4 nv[decltype(n)::value], mv[decltype(n)::value];
            issue(0, nv, mv, n);
            nb = nb_fn();                       // may be a load of its own, in flight with the batch
            process(0, nv, mv, n);
        };
        if (n_load <= 8) {
            single(std::integral_constant<int, 1>{});
        } else if (n_load <= 16) {
            single(std::integral_constant<int, 2>{});
        } else if (n_load <= 32) {
            single(std::integral_constant<int, 4>{});
        } else {
            constexpr std::integral_constant<int, 4> n{};
            u32x4 nA[4], mA[4], nB[4], mB[4];
            issue(0, nA, mA, n);
            nb = nb_fn();
            for (int c0 = 0; c0 < n_load; c0 += 64) {
                issue(c0 + 32, nB, mB, n);
                process(c0, nA, mA, n);
                issue(c0 + 64, nA, mA, n);
                if (c0 + 32 < n_load) process(c0 + 32, nB, mB, n);
            }
        }
    } else {
        nb = nb_fn();
    }
    // merge the 8 slices (slice order), divide, round to fp16
    float *S = scratch, *L = scratch + 8 * kHeadDim, *M = L + 8;
    if (worker) {
        *reinterpret_cast<float4 *>(&S[slice * kHeadDim + 4 * t4]) = make_float4(s[0], s[1], s[2], s[3]);
        if (t4 == 0) { L[slice] = l; M[slice] = m; }
    }
    const int rf = __syncthreads_or(f);
    FD_PHASE(6);
    if (tid < 32) {
        float mm = M[0];
#pragma unroll
        for (int k = 1; k < 8; ++k) mm = fmaxf(mm, M[k]);
        float o[4] = {0.f, 0.f, 0.f, 0.f}, lt = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float a = M[k] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((M[k] - mm) * kLog2e);   // 1 for unflagged rows
            const float4 v = *reinterpret_cast<const float4 *>(&S[k * kHeadDim + 4 * tid]);
            o[0] = __builtin_fmaf(a, v.x, o[0]); o[1] = __builtin_fmaf(a, v.y, o[1]);
            o[2] = __builtin_fmaf(a, v.z, o[2]); o[3] = __builtin_fmaf(a, v.w, o[3]);
            lt = __builtin_fmaf(a, L[k], lt);
        }
        uint2 h = make_uint2(0u, 0u);
        if (nb > 0) {
            h.x = (unsigned)to_half_bits(o[0] / lt) | ((unsigned)to_half_bits(o[1] / lt) << 16);
            h.y = (unsigned)to_half_bits(o[2] / lt) | ((unsigned)to_half_bits(o[3] / lt) << 16);
        }
        *reinterpret_cast<uint2 *>(p.out + (size_t)row * kHeadDim + 4 * tid) = h;
    }
    if (tid == 0) p.ws.row_flags[row] = rf ? 1 : 0;
}

// The row epilogue for the G <= 16 rows of one head group at once, by 256 threads or more:
// thread (h, t) = (tid / 32, tid % 32) owns elements 4t..4t+3 of row row0 + h and walks
// that row's nb partial results in chunk order with a running maximum of the
// references (Eq. 2; every factor is exactly 1 for an unflagged row, which makes it
// the plain sum of Eq. 4).  No thread needs another's data: one memory round trip
// per 4 chunks, two batches in flight, no LDS and no barrier.  Loads pass the caches
// (the partial results come from other workgroups of the same launch).
// COHERENT = false and a per-row chunk count serve a launch of its own over arbitrary rows.
template <bool COHERENT = true, typename NbFn>
__device__ __forceinline__ void rows_epilogue(const Problem &p, int row0, int G, NbFn nb_of)
{
    const int tid = threadIdx.x, t4 = tid & 31;
    auto ld16 = [](const void *ptr) {
        if constexpr (COHERENT) {
            const unsigned long long *w = static_cast<const unsigned long long *>(ptr);
            const unsigned long long a = load_coherent(&w[0]), b = load_coherent(&w[1]);
            return u32x4{(unsigned)a, (unsigned)(a >> 32), (unsigned)b, (unsigned)(b >> 32)};
        } else {
            return *static_cast<const u32x4 *>(ptr);
        }
    };
    for (int h = tid >> 5; h < G; h += (int)(blockDim.x >> 5)) {
        const int row = row0 + h;
        const int nb = nb_of(row);
        if (nb <= 0) {                          // (only a launch of its own gets here: empty sequence)
            *reinterpret_cast<uint2 *>(p.out + (size_t)row * kHeadDim + 4 * t4) = make_uint2(0u, 0u);
            if (t4 == 0) p.ws.row_flags[row] = 0;
            continue;
        }
        const size_t r0 = (size_t)row * p.nc;
        const float *num = p.ws.num + r0 * kHeadDim + 4 * t4;
        const SlotMeta *meta = p.ws.meta + r0;
        const int cap = nb - 1;                 // nb >= 1: the caller holds one of the row's chunks
        float m = -INFINITY, l = 0.f;
        float s[4] = {0.f, 0.f, 0.f, 0.f};
        int f = 0;
        auto issue = [&](int c0, u32x4 (&nv)[4], u32x4 (&mv)[4]) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c = min(c0 + i, cap);
                nv[i] = ld16(num + (size_t)c * kHeadDim);
                mv[i] = ld16(meta + c);
            }
        };
        auto process = [&](int c0, const u32x4 (&nv)[4], const u32x4 (&mv)[4]) {
            float r[4], bm = -INFINITY;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool in_row = c0 + i < nb;
                r[i] = in_row ? as_f32(mv[i][1]) : -INFINITY;
                bm = fmaxf(bm, r[i]);
                f |= in_row ? (int)mv[i][2] : 0;
            }
            if (bm > m) {
                const float a = __builtin_amdgcn_exp2f((m - bm) * kLog2e);   // 0 on the first batch
#pragma unroll
                for (int e = 0; e < 4; ++e) s[e] *= a;
                l *= a;
                m = bm;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float a = r[i] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((r[i] - m) * kLog2e);
#pragma unroll
                for (int e = 0; e < 4; ++e) s[e] = __builtin_fmaf(a, as_f32(nv[i][e]), s[e]);
                l = __builtin_fmaf(a, as_f32(mv[i][0]), l);
            }
        };
        u32x4 nA[4], mA[4], nB[4], mB[4];
        issue(0, nA, mA);
        if (nb <= 4) {
            process(0, nA, mA);
        } else {
            for (int c0 = 0; c0 < nb; c0 += 8) {
                issue(c0 + 4, nB, mB);
                process(c0, nA, mA);
                issue(c0 + 8, nA, mA);
                if (c0 + 4 < nb) process(c0 + 4, nB, mB);
            }
        }
        FD_PHASE(6);
        uint2 o;
        o.x = (unsigned)to_half_bits(s[0] / l) | ((unsigned)to_half_bits(s[1] / l) << 16);
        o.y = (unsigned)to_half_bits(s[2] / l) | ((unsigned)to_half_bits(s[3] / l) << 16);
        *reinterpret_cast<uint2 *>(p.out + (size_t)row * kHeadDim + 4 * t4) = o;
        if (t4 == 0) p.ws.row_flags[row] = f ? 1 : 0;
    }
}
__device__ __forceinline__ void group_epilogue(const Problem &p, int row0, int G, int nb)
{
    rows_epilogue<true>(p, row0, G, [nb](int) { return nb; });
}

// Elects the workgroup that completes a row: a radix-8 tree of arrival counters
// over the row's nb chunks.  Same-address device-scope atomics complete one after
// another (about 0.13 us each on MI355X), so a flat counter costs nb of them on the
// critical path when the workgroups of a row finish together; the tree costs at
// most 8 per level plus one memory round trip per level.  Called by one thread after the workgroup's results are performed.
// Returns true for exactly one caller per row, after every other chunk arrived.
// Counters are zero before and after (the last arrival at a node resets it).
__device__ __forceinline__ bool arrive_and_elect(const Problem &p, int row, int c, int nb)
{
    constexpr int LR = 3, R = 1 << LR;
    int32_t *node = p.ws.ticket + (size_t)row * p.nc;
    int idx = c, n = nb;
    while (n > 1) {
        const int parent = idx >> LR;
        const int children = min(R, n - (parent << LR));
        const int t = __hip_atomic_fetch_add(&node[parent], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (t != children - 1) return false;
        store_coherent(&node[parent], 0);
        n = (n + R - 1) >> LR;
        node += n;
        idx = parent;
    }
    return true;
}

}  // namespace fd
