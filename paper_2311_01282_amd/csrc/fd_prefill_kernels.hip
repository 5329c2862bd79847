// Prompt (prefill) phase with the asynchronized softmax of Section 3: every token of a
// prompt attends to itself and the tokens before it (Eq. 1 under the causal mask), all
// weights taken against the unified scaling factor phi.  Partial sums over successive key
// tiles then simply add (Eq. 4): no running maximum, and the output accumulators are never
// rescaled while the keys stream by.  A 128-query tile whose guard fires is redone on the
// spot with the synchronized scheme (running maximum per query, Eq. 2).
//
// Matrix-core mapping (16x16x32 MFMA; lane = (n, g) = (lane % 16, lane / 16)):
//   scores   S^T[key][query] = K . Q^T      A = 16 keys of the K tile in LDS, B = Q^T held in
//            registers for the whole kernel.  Row 4g + r of key block t is key
//            k0 + 8g + 4t + r: with that permutation the two score tiles of a 32-key
//            step leave lane (n, g) holding keys k0 + 8g .. 8g + 7 of query n -- exactly
//            the B operand of the second product, no data movement.
//   weights  P = e^{s S^T - phi}, fp32, guard, causal mask.  They go to the matrix cores as fp16
//            hi + lo pairs (22 significant bits).  fp16 has the precision but not the range of
//            e^{x - phi} over the admissible x - phi, so every query carries a scale of its own,
//            2^{k_q}, fixed after its first key step so that the largest weight seen there becomes
//            2^4: numerator and denominator of a query are both scaled by it and it cancels in the
//            division; being constant over the keys of a query it leaves the sums of Eq. 4 as
//            they are -- partial sums still just add, nothing is ever rescaled.  A query whose later
//            logits exceed its first step's maximum by more than 2^11.9 would overflow fp16: its
//            tile is redone with the synchronized scheme, like a tile whose guard fired (but
//            without raising the guard's flag).
//   output   O^T[d][query] = V^T . P^T       A = V^T from a transposed copy of V that a
//            small pass writes first (keys contiguous per d, so the loop transposes
//            nothing); V is fp16 as it is.  Two MFMAs per tile (V Ph + V Pl).
// K and V^T tiles are loaded from global memory straight into LDS, once per workgroup, and
// shared by its four wavefronts (double-buffered; layouts free of bank conflicts for the
// 16-byte operand reads).
#include "fd_chunk.h"

namespace fd {

namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr float kFirstStepLog2 = 4.f;     // a query's largest weight of its first key step becomes 2^4 ...
constexpr float kOverflowLog2 = 15.9f;    // ... and no later weight may reach 2^16 (fp16 ends at 65504)

constexpr int kQB = 2;            // 16-query blocks per wavefront (1: 401, 2: 471-500 TFLOP/s at 8K)
constexpr int kWaveQ = 16 * kQB;  // queries per wavefront
constexpr int kQTile = 4 * kWaveQ; // query rows per workgroup
constexpr int kStep = 32;        // keys per wavefront step
constexpr int kVAhead = 1;    // V^T operand tiles read from LDS ahead of the MFMAs that use them

// V^T of one KV head is stored tile by tile, in the order the attention kernel consumes it:
// [32-key step][8-key chunk g][d][8 keys], so the 8 KiB a step needs are contiguous (whole
// cache lines, and the image of the LDS tile).  Element offset of keys key .. key + 7 (key a
// multiple of 8) of row d within the head:
__device__ __forceinline__ size_t vt_offset(int key, int d)
{
    return (size_t)(key >> 5) * (32 * kHeadDim) + (size_t)((((key >> 3) & 3) * kHeadDim + d) << 3);
}

// ---- pass 0: V [B,Hkv,Smax,D] fp16 -> tiled V^T (Spad keys) fp16, zero beyond the prompt ----
__global__ __launch_bounds__(256) void transpose_v_kernel(const PrefillProblem p)
{
    __shared__ uint16_t tile[64][kHeadDim + 2];
    const int gi = blockIdx.y;                          // (sequence, KV head)
    const int b = gi / p.Hkv;
    const int k0 = blockIdx.x * 64;
    int S = p.seq_lens[b];
    S = S < 0 ? 0 : (S > p.Smax ? p.Smax : S);
    const int tid = threadIdx.x;
    // 64 keys x 128 d: thread reads 8 d of one key (16 bytes), 4 times
    for (int i = tid; i < 64 * 16; i += 256) {
        const int key = i >> 4, c = i & 15;
        u32x4 w = {0u, 0u, 0u, 0u};
        if (k0 + key < S) w = *reinterpret_cast<const u32x4 *>(p.v + ((size_t)gi * p.Smax + k0 + key) * kHeadDim + 8 * c);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t x = w[j];
            tile[key][8 * c + 2 * j] = (uint16_t)(x & 0xffffu);
            tile[key][8 * c + 2 * j + 1] = (uint16_t)(x >> 16);
        }
    }
    __syncthreads();
    // thread writes 8 keys of one d (16 bytes), 4 times; consecutive threads take consecutive d,
    // which are consecutive 16-byte pieces of the tiled layout
    for (int i = tid; i < kHeadDim * 8; i += 256) {
        const int d = i & (kHeadDim - 1), kc = i >> 7;
        uint32_t o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            o[j] = (uint32_t)tile[8 * kc + 2 * j][d] | ((uint32_t)tile[8 * kc + 2 * j + 1][d] << 16);
        const size_t at = (size_t)gi * kHeadDim * p.Spad + vt_offset(k0 + 8 * kc, d);
        *reinterpret_cast<u32x4 *>(p.vt + at) = u32x4{o[0], o[1], o[2], o[3]};
    }
}

// 16 bytes per lane from global memory into LDS without passing through registers: lane l's
// bytes land at lds_base + 16 l (lds_base is the same for the whole wavefront).
__device__ __forceinline__ void load_to_lds(const void *global, void *lds_base)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)global,
                                     (__attribute__((address_space(3))) void *)lds_base, 16, 0, 0);
}

// ---- the attention kernel ----
// A workgroup owns 128 queries of one head: wavefront w the 32 queries i0 + 32w .. +31 (two
// blocks of 16).  The K and V^T tiles of a 32-key step are loaded once per workgroup into LDS
// (double-buffered, one barrier per step) and read from there by all four wavefronts as MFMA A
// operands; Q^T stays in registers as the B operand.  Every output row belongs to one wavefront:
// nothing is reduced across wavefronts, and with the unified phi nothing is ever rescaled.
// A 16-byte LDS access of a wavefront is served 16 lanes per cycle, and the 16 are not
// consecutive lanes: lanes 0-3, 12-15, 20-27 share a cycle, lanes 4-11, 16-19, 28-31 the next
// (measured with a two-lane probe; likewise for the upper half).  In terms of lane = 16g + n a
// cycle holds every n once, taken from two different g.  A layout is conflict-free when the
// 16-byte unit (address / 16 mod 16) of lane (n, g) is a function of n alone and a permutation
// of it (the V^T layout below), or n ^ g (the K layout).
constexpr int kKStride = 256;    // bytes per K row in LDS (16 chunks of 16 bytes, XOR-swizzled)
struct PrefillLds {
    alignas(16) unsigned char k[2][kStep * kKStride];          // 2 x 8 KiB
    alignas(16) unsigned char v[2][4 * kHeadDim * 16];         // 2 x 8 KiB: [8-key chunk g][d][16 bytes], unit = d % 16
    int bad[4], redo[4];
};
// V^T: the 16 bytes of keys 8g .. 8g + 7 of row d
__device__ __forceinline__ int v_slot(int d, int g) { return (g * kHeadDim + d) << 4; }

// K row r, 16-byte chunk c -> byte offset.  Lane (n, g) reads row r(n) in {0..3, 8..11, 16..19,
// 24..27} (+4 for the second key block), chunk 4 kb + g: XOR with (r & 3) | ((r >> 3) & 3) << 2
// (= n for those rows) puts it in unit (4 kb + g) ^ n; a row's 16 chunks stay a permutation of
// themselves, so the row-wise writes are conflict-free too.
__device__ __forceinline__ int k_slot(int r, int c)
{
    return r * kKStride + ((c ^ ((r & 3) | (((r >> 3) & 3) << 2))) << 4);
}

// One 128-query tile.  ONLINE == false: unified scaling factor (Eq. 4); returns true when the tile
// has to be redone with the synchronized scheme -- its guard fired (recorded in tile_flags) or a
// weight left the range of the fp16 operands (not recorded: the result is the same either way).
// ONLINE == true: the synchronized scheme (running maximum per query, Eq. 2); always stores.
template <bool ONLINE>
__device__ __forceinline__ bool tile_all(const PrefillProblem &p, PrefillLds &lds, int b, int hq, int i0, int S)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int hkv = hq / p.G;
    const size_t kv_head = (size_t)b * p.Hkv + hkv;
    const uint16_t *qbase = p.q + (((size_t)b * p.Hq + hq) * p.Smax) * kHeadDim;
    const uint16_t *kbase = p.k + kv_head * p.Smax * kHeadDim;
    const uint16_t *vt = p.vt + kv_head * kHeadDim * p.Spad;
    const float c1 = p.scale * kLog2e, c0 = -p.phi * kLog2e;      // log2 of e^{s x - phi} = c1 x + c0
    const float lo2 = p.lo * kLog2e, hi2 = p.hi * kLog2e;
    const int w0 = i0 + kWaveQ * wave;                       // first query of this wavefront
    // -1.0 in a register the compiler cannot see through: keeps e - (float)hi a single mixed-precision
    // fused multiply-add (fp16 operand read in place) instead of a conversion and a subtraction
    float neg1;
    asm("v_mov_b32 %0, -1.0" : "=v"(neg1));

    // Q^T as the B operand: lane (n, g) holds d = 32 kb + 8g .. +7 of query w0 + 16 qb + n
    f16x8 qB[kQB][4];
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) {
        const int row = min(w0 + 16 * qb + n, p.Smax - 1);
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
            qB[qb][kb] = __builtin_bit_cast(f16x8, *reinterpret_cast<const u32x4 *>(qbase + (size_t)row * kHeadDim + 32 * kb + 8 * g));
    }
    f32x4 acc[8][kQB];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb) acc[dt][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
    float den[kQB], mrun[kQB];
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) { den[qb] = 0.f; mrun[qb] = -INFINITY; }
    // unified scheme: running extremes of log2 of the SCALED weights (guard, fp16 range) and the
    // queries' scale exponents k_q, folded into the additive constant of the logit
    float zlo[kQB], zhi[kQB], kq[kQB], c0q[kQB];
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) { zlo[qb] = INFINITY; zhi[qb] = -INFINITY; kq[qb] = 0.f; c0q[qb] = c0; }

    // key steps: the workgroup walks 0 .. nsteps - 1 (keys some query of the tile sees); this
    // wavefront computes while a key of the step is visible to one of its queries
    const int last_q = min(i0 + kQTile, S) - 1;
    const int nsteps = last_q / kStep + 1;
    const int my_last_q = min(w0 + kWaveQ, S) - 1;           // < w0 when the wavefront has no query
    const int my_steps = my_last_q >= w0 ? my_last_q / kStep + 1 : 0;

    // Cooperative tile fetch, global memory straight into LDS (no staging registers): a wavefront's
    // load instruction fills 1 KiB of LDS, lane l the 16 bytes at l * 16 from the wavefront's base,
    // each lane from a global address of its own.  Thread t moves chunks t and t + 256 of each of
    // the K and V^T tiles.  The V^T tile in memory is the image of the LDS tile; for K the lane
    // whose LDS slot is (row r, physical chunk c') fetches logical chunk c' ^ key(r).
    auto fetch = [&](int s, int buf) {
        const int k0 = s * kStep;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int id = tid + 256 * i;
            const int base = (256 * i + 64 * wave) << 4;         // the wavefront's 1 KiB of each tile
            const int r = id >> 4, c = (id & 15) ^ ((r & 3) | (((r >> 3) & 3) << 2));
            const uint16_t *gk = kbase + (size_t)min(k0 + r, p.Smax - 1) * kHeadDim + 8 * c;
            const size_t at = (size_t)s * (kStep * kHeadDim) + 8 * id;
            load_to_lds(gk, &lds.k[buf][base]);
            load_to_lds(vt + at, &lds.v[buf][base]);
        }
    };
    // the loads of this wavefront have landed in LDS
    auto fetched = [&]() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };
    // scores -> weights (fp16 hi / lo B operands) for one query block; log2 domain
    auto weights = [&](auto masked, bool first, int qb, const f32x4 (&sc)[2], f16x8 &pB, f16x8 &pBl, int k0) {
        constexpr bool MASKED = decltype(masked)::value;
        const int qrow = w0 + 16 * qb + n;
        float z[8];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) z[4 * t + r] = __builtin_fmaf(sc[t][r], c1, c0q[qb]);
        bool ok[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) ok[j] = true;
        if constexpr (MASKED) {
            const int kmax = qrow < S ? qrow : -1;                       // last key this query sees
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                ok[j] = k0 + 8 * g + j <= kmax;                          // j = 4t + r: key k0 + 8g + j
                z[j] = ok[j] ? z[j] : -INFINITY;                         // weight 0
            }
        }
        float shift = 0.f;
        if constexpr (ONLINE) {
            float m = fmaxf(fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])), fmaxf(fmaxf(z[4], z[5]), fmaxf(z[6], z[7])));
            m = fmaxf(m, __shfl_xor(m, 16));
            m = fmaxf(m, __shfl_xor(m, 32));
            const float mnew = fmaxf(mrun[qb], m);
            if (mnew > mrun[qb]) {                                   // rescale what was summed so far
                const float alpha = mrun[qb] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mrun[qb] - mnew);
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) acc[dt][qb] *= alpha;
                den[qb] *= alpha;
                mrun[qb] = mnew;
            }
            shift = mnew == -INFINITY ? 0.f : mnew;
        } else {
            if (first) {
                // The query's scale: its largest weight of this first step becomes 2^kFirstStepLog2.
                // The four lane groups of a query hold different keys: they agree on the maximum first.
                float m = fmaxf(fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])), fmaxf(fmaxf(z[4], z[5]), fmaxf(z[6], z[7])));
                m = fmaxf(m, __shfl_xor(m, 16));
                m = fmaxf(m, __shfl_xor(m, 32));
                const float k = (m == -INFINITY || m != m) ? 0.f : kFirstStepLog2 - m;      // no visible key, or NaN: leave as is
                kq[qb] = k;
                c0q[qb] = c0 + k;
#pragma unroll
                for (int j = 0; j < 8; ++j) z[j] += k;
            }
            // Guard: running extremes over all keys of the query, compared with the bounds (shifted by
            // k_q) once, after the last step (three-input min / max: four instructions each per step).
            float hi_run = zhi[qb], lo_run = zlo[qb];
#pragma unroll
            for (int j = 0; j < 8; j += 2) {
                hi_run = fmaxf(fmaxf(z[j], z[j + 1]), hi_run);
                lo_run = fminf(fminf(ok[j] ? z[j] : INFINITY, ok[j + 1] ? z[j + 1] : INFINITY), lo_run);
            }
            zhi[qb] = hi_run;
            zlo[qb] = lo_run;
        }
        unsigned hi[4], lo[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float e0 = __builtin_amdgcn_exp2f(z[2 * j] - shift), e1 = __builtin_amdgcn_exp2f(z[2 * j + 1] - shift);
            den[qb] += e0 + e1;
            // hi = the weight cut to fp16 (11 bits), lo = what that leaves (exact in fp32) cut to fp16
            const f16x2 h = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(e0, e1));
            const _Float16 h0 = h.x, h1 = h.y;
            const float l0 = __builtin_fmaf((float)h0, neg1, e0), l1 = __builtin_fmaf((float)h1, neg1, e1);
            hi[j] = __builtin_bit_cast(unsigned, h);
            lo[j] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(l0, l1));
        }
        pB = __builtin_bit_cast(f16x8, u32x4{hi[0], hi[1], hi[2], hi[3]});
        pBl = __builtin_bit_cast(f16x8, u32x4{lo[0], lo[1], lo[2], lo[3]});
    };
    // one step of this wavefront on the tiles in LDS buffer `buf`
    auto compute = [&](auto masked, int s, int buf) {
        const int k0 = s * kStep;
        // scores: row m = n of key block t is key k0 + 8 (n >> 2) + 4t + (n & 3), so that the two
        // score tiles leave lane (n, g) holding keys k0 + 8g .. 8g + 7 of query n
        f32x4 sc[kQB][2];
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb)
#pragma unroll
            for (int t = 0; t < 2; ++t) sc[qb][t] = f32x4{0.f, 0.f, 0.f, 0.f};
        // all eight K operands of the step first (their LDS latency overlaps), then the MFMAs
        u32x4 ka[2][4];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int r = 8 * (n >> 2) + 4 * t + (n & 3);
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) ka[t][kb] = *reinterpret_cast<const u32x4 *>(&lds.k[buf][k_slot(r, 4 * kb + g)]);
        }
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int qb = 0; qb < kQB; ++qb)
                    sc[qb][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, ka[t][kb]), qB[qb][kb], sc[qb][t], 0, 0, 0);
        // O^T += V^T P^T with P = Ph + Pl: V Ph + V Pl.  The A operand of tile dt + 1 is read from LDS
        // while the MFMAs of tile dt run; that of tile 0 before the weights are computed.
        u32x4 a_v[kVAhead + 1];
        auto read_v = [&](int dt, int slot) { a_v[slot] = *reinterpret_cast<const u32x4 *>(&lds.v[buf][v_slot(16 * dt + n, g)]); };
#pragma unroll
        for (int dt = 0; dt < kVAhead; ++dt) read_v(dt, dt);
        f16x8 pB[kQB], pBl[kQB];
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb) weights(masked, s == 0, qb, sc[qb], pB[qb], pBl[qb], k0);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            if (dt + kVAhead < 8) read_v(dt + kVAhead, (dt + kVAhead) % (kVAhead + 1));
            const f16x8 v8 = __builtin_bit_cast(f16x8, a_v[dt % (kVAhead + 1)]);
#pragma unroll
            for (int qb = 0; qb < kQB; ++qb) acc[dt][qb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(v8, pB[qb], acc[dt][qb], 0, 0, 0);
#pragma unroll
            for (int qb = 0; qb < kQB; ++qb) acc[dt][qb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(v8, pBl[qb], acc[dt][qb], 0, 0, 0);
            // keep the order: the next tile's LDS read, then this tile's four MFMAs
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 2 * kQB, 0);
        }
    };

    fetch(0, 0);
    fetched();
    __syncthreads();
#pragma unroll 1
    for (int s = 0; s < nsteps; ++s) {
        const int buf = s & 1;
        // the other buffer was last read in step s - 1, which every wavefront has left
        if (s + 1 < nsteps) fetch(s + 1, buf ^ 1);       // uniform over the workgroup
        const bool full = s < my_steps && s * kStep + kStep - 1 <= w0 && w0 + kWaveQ <= S;
        if (s < my_steps) {                              // uniform over the wavefront
            // steps entirely below this wavefront's first query, all 32 of whose queries exist, need no mask
            if (full) compute(std::false_type{}, s, buf);
            else compute(std::true_type{}, s, buf);
        }
        fetched();
        __syncthreads();
    }
    // the four lane groups of a query hold disjoint keys: total per query
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) {
        den[qb] += __shfl_xor(den[qb], 16);
        den[qb] += __shfl_xor(den[qb], 32);
    }
    if constexpr (!ONLINE) {
        // strict guard on x - phi (the extremes carry the query's scale exponent); a NaN logit, which
        // minimum and maximum skip, shows as a NaN denominator.  Apart from the guard: a weight at or
        // beyond 2^kOverflowLog2 does not fit the fp16 operands.
        bool bad = false, range = false;
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb) {
            bad |= (zhi[qb] >= hi2 + kq[qb]) | (zlo[qb] <= lo2 + kq[qb]) | (den[qb] != den[qb]);
            range |= zhi[qb] >= kOverflowLog2;
        }
        const unsigned long long any_bad = __ballot(bad), any_range = __ballot(range);
        if (lane == 0) { lds.bad[wave] = any_bad != 0ull; lds.redo[wave] = (any_bad | any_range) != 0ull; }
        __syncthreads();
        // one flag byte per 64 queries
        constexpr int kFlagTiles = kQTile / 64, kWavesPerFlag = 4 / kFlagTiles;
        if (tid < kFlagTiles) {
            const int t64 = i0 / 64 + tid;
            int f = 0;
#pragma unroll
            for (int w = 0; w < kWavesPerFlag; ++w) f |= lds.bad[tid * kWavesPerFlag + w];
            if (t64 < p.tiles) p.tile_flags[((size_t)b * p.Hq + hq) * p.tiles + t64] = f != 0;
        }
        if ((lds.redo[0] | lds.redo[1] | lds.redo[2] | lds.redo[3]) != 0) return true;   // uniform: the tile is redone, nothing stored
    }
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) {
        const int row = w0 + 16 * qb + n;
        if (row >= p.Smax) continue;
        const bool live = row < S;
        const float inv = live ? 1.f / den[qb] : 0.f;
        uint16_t *o = p.out + (((size_t)b * p.Hq + hq) * p.Smax + row) * kHeadDim;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            uint2 h = make_uint2(0u, 0u);
            if (live) {
                h.x = (unsigned)to_half_bits(acc[dt][qb][0] * inv) | ((unsigned)to_half_bits(acc[dt][qb][1] * inv) << 16);
                h.y = (unsigned)to_half_bits(acc[dt][qb][2] * inv) | ((unsigned)to_half_bits(acc[dt][qb][3] * inv) << 16);
            }
            *reinterpret_cast<uint2 *>(o + 16 * dt + 4 * g) = h;
        }
    }
    return false;
}

__global__ __launch_bounds__(256, 2) void prefill_kernel(const PrefillProblem p)
{
    __shared__ PrefillLds lds;
    // Workgroups are dealt to the 8 XCDs round-robin by index; each XCD has its own L2.  All
    // tiles of the query heads that share one KV head go to the same XCD, one KV head after the
    // other, so that the K and V^T an XCD streams at any time belong to one head and its tiles
    // walk the keys together (the reads then hit in that L2 instead of going to memory eight
    // times).  Within a head, heavy tiles (late queries see more keys) first.
    const int qtiles = (p.Smax + kQTile - 1) / kQTile;
    const int j = blockIdx.x >> 3;
    const int per_group = p.G * qtiles;
    const int gi = (blockIdx.x & 7) + 8 * (j / per_group);       // (sequence, KV head)
    if (gi >= p.B * p.Hkv) return;
    const int r = j % per_group;
    const int qt = qtiles - 1 - r % qtiles;
    const int b = gi / p.Hkv;
    const int hq = (gi - b * p.Hkv) * p.G + r / qtiles;
    const int i0 = qt * kQTile;
    int S = p.seq_lens[b];
    S = S < 0 ? 0 : (S > p.Smax ? p.Smax : S);
    if (i0 >= S) {                                       // no prompt token in this tile: zeros, no flag
        uint16_t *o = p.out + (((size_t)b * p.Hq + hq) * p.Smax + i0) * kHeadDim;
        const int rows = min(kQTile, p.Smax - i0);
        for (int i = threadIdx.x; i < rows * (kHeadDim / 8); i += 256)
            reinterpret_cast<u32x4 *>(o)[i] = u32x4{0u, 0u, 0u, 0u};
        if (threadIdx.x < kQTile / 64 && i0 / 64 + (int)threadIdx.x < p.tiles)
            p.tile_flags[((size_t)b * p.Hq + hq) * p.tiles + i0 / 64 + threadIdx.x] = 0;
        return;
    }
    if (tile_all<false>(p, lds, b, hq, i0, S)) {         // Section 3 "Recomputation", for this tile
        __syncthreads();
        tile_all<true>(p, lds, b, hq, i0, S);
    }
}

}  // namespace

hipError_t launch_prefill(const PrefillProblem &p, hipStream_t s)
{
    if (p.B == 0) return hipSuccess;
    hipError_t e = launch(transpose_v_kernel, dim3(p.Spad / 64, p.B * p.Hkv), dim3(256), s, p);
    if (e != hipSuccess) return e;
    const long long groups8 = ((long long)p.B * p.Hkv + 7) / 8 * 8;
    const int qtiles = (p.Smax + kQTile - 1) / kQTile;
    return launch(prefill_kernel, dim3((unsigned)(groups8 * p.G * qtiles)), dim3(256), s, p);
}

}  // namespace fd
