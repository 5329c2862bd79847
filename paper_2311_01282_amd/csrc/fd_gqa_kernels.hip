// Grouped-query chunk kernel (MFMA path): the G <= 16 query heads that share one
// KV head are processed together, so every K and V element is read from HBM once
// per group instead of once per query head.  With G = 8 the work is 8 flop per KV
// byte, more than the vector ALUs sustain at HBM rate once fp16->fp32 conversions
// are counted, hence the matrix cores:
//
//   scores   S^T[key][head] = sum_d K[key][d] Q[head][d]
//            v_mfma_f32_16x16x32_f16: A = a 16-key block of K, B = Q padded to 16
//            heads (zero rows), 4 instructions per block (d = 4 x 32).
//   weights  P = e^{s S^T - phi} in fp32, in place in the accumulator layout
//            (lane (head, g) holds keys g, 4+g, 8+g, 12+g of the block) -- Eq. 4, no maximum.
//            fp16 has neither the range of e^{x-phi} over the admissible x - phi nor, with 11
//            bits, the precision, so P goes to the matrix cores as fp16 hi + lo pairs (22 bits)
//            under a scale 2^k of the (wavefront, head)'s own: k, an integer, is fixed after the
//            wavefront's first 16-key block so that the head's largest weight there lies in
//            [2^3, 2^4]; it is constant over the keys the wavefront sums, so the sums of Eq. 4 stay
//            plain sums, and it is taken out again (exactly: a power of two) before the
//            wavefronts' tiles are added.  V is fp16 and is used as it is:
//   P.V      out[head][d] += sum_key P[head][key] V[key][d]
//            v_mfma_f32_16x16x16_f16, two per tile (P_hi V + P_lo V): A = P, whose four weights
//            per lane are exactly contraction indices 4g..4g+3 when index 4g + r stands for key
//            4r + g; B = V, where lane (n, g) loads the 16 bytes d = 8n..8n+7 of the same keys
//            4r + g (r = 0..3) and feeds element e of the four rows to accumulator tile e (d = 8n
//            + e), so V needs no transpose, only a byte permute per pair of rows: 16 matrix
//            instructions per 16-key block.  (Earlier forms: fp32 16x16x4, 32 instructions of 16
//            passes; then bf16 with P in three and V in two pieces, 40 instructions and about 4
//            vector-ALU operations per V element for the split.)
//            A weight at or beyond 2^15.9 -- a logit more than 8 above the largest of the
//            wavefront's first block -- does not fit: that (head, chunk) is redone on the per-row
//            path like a flagged one, but without the flag.
//
// K reaches the A layout through a per-wavefront LDS tile (coalesced 1 KiB global
// loads in, 16-byte reads out, XOR-swizzled so both directions are bank-conflict
// free).  One workgroup = 4 wavefronts = one (sequence, KV head, chunk); the
// wavefronts interleave 16-key blocks.  The rest of the method -- guard, on-the-spot
// recomputation of a flagged (head, chunk) with the synchronized scheme, election of
// the workgroup that completes the group, row epilogue -- is shared with the per-row
// kernels (fd_chunk.h).
#include "fd_chunk.h"

namespace fd {
namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// NW wavefronts per workgroup (4 or 8; the launcher uses 4).
template <int NW>
struct GqaLds {
    // K staging (NW wavefronts x 4 KiB) during the main loop, then the reduction tile
    // [wave][head][d] (NW x 8 KiB), then (rarely) the per-row recomputation's workspace:
    // never live together.
    alignas(16) float tile[NW * 16 * kHeadDim];
    float den[NW][64];
    float e_new[16];                 // weight of an appended key per head (0 when there is none)
    int   f_new[16];                 // ... and whether it left the bounds
    unsigned long long bad[NW], over[NW];
    int last;
};

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

constexpr float kFirstBlockLog2 = 4.f;    // a head's largest weight of the wavefront's first block lies in [2^3, 2^4] ...
constexpr float kOverflowLog2 = 15.9f;    // ... and no later weight may reach 2^16 (fp16 ends at 65504)

template <int C, bool PAGED = false, int NW = 4>
__global__ __launch_bounds__(NW * 64, NW == 4 ? 3 : 1) void decode_fused_gqa_kernel(const Problem p)
{
    static_assert(NW == 4 || NW == 8, "the appended key's lane assignment covers 16 heads with 4 wavefronts");
    static_assert(sizeof(ChunkLds<NW, C>) <= sizeof(GqaLds<NW>::tile), "recompute workspace must fit the tile");
    constexpr int kGqaThreads = NW * 64;
    constexpr int UP = C / (4 * NW) < 8 ? C / (4 * NW) : 8;    // stage depth of the per-row recomputation
    __shared__ GqaLds<NW> lds;
    constexpr int NBLK = C / 16;               // 16-key blocks in the chunk
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;    // n: head (scores) / 16-byte segment (loads); g: lane group
    const int G = p.G;

    // All chunks of a KV-head group go to the same XCD (see decode_fused_kernel).
    const int groups = p.B * p.Hkv;
    // chunk-major in a launch of up to 1024 workgroups, so that chunks past the end of the
    // sequences come last; row-major beyond (see decode_fused_kernel)
    const int groups8 = (groups + 7) >> 3;
    const int j = blockIdx.x >> 3;
    const int c = p.chunk_major ? j / groups8 : j % p.nc;
    const int gi = row_slot(p, blockIdx.x & 7, c) + 8 * (p.chunk_major ? j - c * groups8 : j / p.nc);
    if (gi >= groups) return;
    const int b = gi / p.Hkv;
    const int row0 = b * p.Hq + (gi - b * p.Hkv) * G;       // first query row of the group
    const int S_res = clamp_len(p, p.seq_lens[b]);          // keys resident in the cache
    const int S = effective_len(p, S_res);                  // plus the appended one, if any
    const int len = p.C;                                    // keys per chunk (<= C, the kernel's capacity)
    const int nb = (S + len - 1) / len;
    const int start = c * len;
    const int nvalid = min(len, S - start);
    const int nres = min(len, S_res - start);
    const bool owner = (S != S_res) & (S_res >= start) & (S_res < start + len);   // this chunk takes the appended key

    if (nvalid <= 0) {                         // padding chunk: zero partials, no flag
        for (int i = tid; i < G * kHeadDim; i += kGqaThreads)
            p.ws.num[((size_t)(row0 + i / kHeadDim) * p.nc + c) * kHeadDim + (i & (kHeadDim - 1))] = 0.f;
        if (tid < G) {
            const size_t slot = (size_t)(row0 + tid) * p.nc + c;
            p.ws.den[slot] = 0.f; p.ws.mloc[slot] = p.phi;
            p.ws.chunk_flags[slot] = 0; store_meta(p, slot, 0.f, p.phi, 0);
            if (nb == 0 && c == 0 && p.elect) p.ws.row_flags[row0 + tid] = 0;
        }
        if (nb == 0 && c == 0 && p.elect)      // empty sequence: nobody else owns these rows
            for (int i = tid; i < G * kHeadDim; i += kGqaThreads) p.out[(size_t)row0 * kHeadDim + i] = 0;
        return;
    }

    // Q as the B operand: lane (n, g) holds d = 32kb + 8g .. +7 of head n; heads >= G are zero rows.
    f16x8 qb[4];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
        u32x4 t = {0u, 0u, 0u, 0u};
        if (n < G) t = *reinterpret_cast<const u32x4 *>(p.q + (size_t)(row0 + n) * kHeadDim + 32 * kb + 8 * g);
        qb[kb] = __builtin_bit_cast(f16x8, t);
    }

    const KvRows<PAGED> at(p, b, gi - b * p.Hkv, start, lane);   // rows of the chunk's keys (contiguous or paged)
    const u32x4 *kp = reinterpret_cast<const u32x4 *>(p.k) + at.base + n;
    const u32x4 *vp = reinterpret_cast<const u32x4 *>(p.v) + at.base + n;
    const int last = nres - 1;                 // last resident key; the appended one joins at the reduction
    const float nphi = -p.phi, lo = p.lo, hi = p.hi, scale = p.scale;
    u32x4 *kst = reinterpret_cast<u32x4 *>(lds.tile) + wave * 256;     // this wavefront's 16 x 16 slots

    f32x4 acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};
    float den = 0.f;
    bool bad = false;
    const bool head_on = n < G;
    float kq = 0.f;                            // scale exponent of (this wavefront, head n), set by the first block
    float zmax = -INFINITY;                    // largest log2 of a scaled weight of head n so far
    float neg1;                                // -1.0 the compiler cannot fold: keeps e - (float)hi one mixed-precision FMA
    asm("v_mov_b32 %0, -1.0" : "=v"(neg1));

    // Keys past the valid length re-read the last valid key and get weight zero.
    auto issue = [&](int blk, u32x4 (&kk)[4], u32x4 (&vv)[4]) {
        const int k0 = blk * 16;
        if constexpr (PAGED) {
            // the block holds a resident key (k0 <= last), so a clamped key stays inside it: one page per block
            const size_t blk0 = at.block16(k0);
#pragma unroll
            for (int r = 0; r < 4; ++r) kk[r] = load_stream(kp + blk0 + (size_t)(min(k0 + 4 * r + g, last) - k0) * 16);
#pragma unroll
            for (int r = 0; r < 4; ++r) vv[r] = load_stream(vp + blk0 + (size_t)(min(k0 + 4 * r + g, last) - k0) * 16);
            return;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) kk[r] = load_stream(kp + at(min(k0 + 4 * r + g, last)));
#pragma unroll
        for (int r = 0; r < 4; ++r) vv[r] = load_stream(vp + at(min(k0 + 4 * r + g, last)));
    };
    auto reduce = [&](int blk, bool first, const u32x4 (&kk)[4], const u32x4 (&vv)[4]) {
        const int k0 = blk * 16;
        // K block -> LDS row (4i + g), 16-byte slot n ^ row; then out in the A layout.
        // Row i of the A operand is key pk = 4(i%4) + i/4 of the block, so that score
        // register r of lane group g belongs to key 4r + g -- the key whose V row the
        // same lane group fetched with load r (1 KiB contiguous per load).
        // Swizzle key swz(r) = the two 2-bit halves of r swapped: the read of lane (n, g) then
        // lands in 16-byte unit (4 kb + g) ^ n, which is conflict-free on this chip (a 16-byte
        // LDS access serves 16 lanes a cycle, every n once, from two lane groups g; measured:
        // no conflict cycles).
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = 4 * i + g;
            kst[r * 16 + (n ^ (i | (g << 2)))] = kk[i];
        }
        const int pk = 4 * (n & 3) + (n >> 2);
        const int pswz = n;                            // swz(pk) = (pk >> 2) | ((pk & 3) << 2) = n
        f32x4 sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
            const f16x8 ka = __builtin_bit_cast(f16x8, kst[pk * 16 + ((4 * kb + g) ^ pswz)]);
            sc = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka, qb[kb], sc, 0, 0, 0);
        }
        // sc[r] = <q_head n, k_key>, key = k0 + 4r + g.  Guard on x - phi, then the scaled weight.
        float dd[4];
        bool valid[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            valid[r] = k0 + 4 * r + g <= last;
            dd[r] = sc[r] * scale + nphi;
            bad |= valid[r] & head_on & !((dd[r] > lo) & (dd[r] < hi));
        }
        if (first) {
            // the head's scale: the four lane groups of a head hold different keys and agree on the maximum first
            float m = -INFINITY;
#pragma unroll
            for (int r = 0; r < 4; ++r) m = fmaxf(m, valid[r] ? dd[r] * kLog2e : -INFINITY);
            m = fmaxf(m, __shfl_xor(m, 16));
            m = fmaxf(m, __shfl_xor(m, 32));
            kq = m > -INFINITY ? kFirstBlockLog2 - ceilf(m) : 0.f;      // (no finite logit: the guard has fired anyway)
        }
        float pw[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float z = __builtin_fmaf(dd[r], kLog2e, kq);
            zmax = fmaxf(zmax, valid[r] ? z : -INFINITY);
            const float e = __builtin_amdgcn_exp2f(z);
            pw[r] = valid[r] ? e : 0.f;
            den += pw[r];
        }
        // P as the A operand of the 16x16x16 product: lane (head n, g) holds contraction indices
        // 4g .. 4g+3, which stand for keys g, 4+g, 8+g, 12+g -- its own four weights.
        // hi = the weight cut to fp16, lo = what that leaves (exact in fp32) cut to fp16: 22 bits.
        const f16x2 h01 = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(pw[0], pw[1]));
        const f16x2 h23 = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(pw[2], pw[3]));
        const _Float16 h0 = h01.x, h1 = h01.y, h2 = h23.x, h3 = h23.y;
        const float l0 = __builtin_fmaf((float)h0, neg1, pw[0]), l1 = __builtin_fmaf((float)h1, neg1, pw[1]);
        const float l2 = __builtin_fmaf((float)h2, neg1, pw[2]), l3 = __builtin_fmaf((float)h3, neg1, pw[3]);
        const f16x4 p_hi = __builtin_bit_cast(f16x4, make_uint2(__builtin_bit_cast(unsigned, h01), __builtin_bit_cast(unsigned, h23)));
        const f16x4 p_lo = __builtin_bit_cast(f16x4, make_uint2(__builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(l0, l1)),
                                                              __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(l2, l3))));
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            // dword w of the four V rows holds elements d = 8n + 2w (low halves) and 8n + 2w + 1 (high
            // halves): the B operands of accumulator tiles 2w and 2w + 1 are the low, resp. high, halves
            // of rows 0..3 (v_perm_b32: two halves of two registers into one)
            const uint32_t v0 = vv[0][w], v1 = vv[1][w], v2 = vv[2][w], v3 = vv[3][w];
            const f16x4 b_even = __builtin_bit_cast(f16x4, make_uint2(__builtin_amdgcn_perm(v1, v0, 0x05040100u), __builtin_amdgcn_perm(v3, v2, 0x05040100u)));
            const f16x4 b_odd = __builtin_bit_cast(f16x4, make_uint2(__builtin_amdgcn_perm(v1, v0, 0x07060302u), __builtin_amdgcn_perm(v3, v2, 0x07060302u)));
            // the small product first
            acc[2 * w] = __builtin_amdgcn_mfma_f32_16x16x16f16(p_lo, b_even, acc[2 * w], 0, 0, 0);
            acc[2 * w + 1] = __builtin_amdgcn_mfma_f32_16x16x16f16(p_lo, b_odd, acc[2 * w + 1], 0, 0, 0);
            acc[2 * w] = __builtin_amdgcn_mfma_f32_16x16x16f16(p_hi, b_even, acc[2 * w], 0, 0, 0);
            acc[2 * w + 1] = __builtin_amdgcn_mfma_f32_16x16x16f16(p_hi, b_odd, acc[2 * w + 1], 0, 0, 0);
        }
    };
    // This wavefront's blocks are wave, wave + NW, ...; nmine of them hold a valid key.
    // Two-stage software pipeline, steady state free of branches around loads.
    const int nblk_valid = min(NBLK, (nres + 15) / 16);
    const int nmine = nblk_valid > wave ? (nblk_valid - wave + NW - 1) / NW : 0;
    if (nmine > 0) {
        // Rows of more than 32 chunks: the wavefront starts at a different one of its blocks in every
        // workgroup and wraps around (as in the per-row kernel: workgroups that start a power of two
        // apart and advance in step are served badly by the memory system for some shapes; 1 x 64/8
        // heads x 262144 keys: 188 us against 161 for the same bytes as 4 x 65536).  Whichever block
        // comes first fixes the scale of the fp16 weights.
        const int rot = (p.nc > 32 && nmine > 1) ? (int)((unsigned)(c * 3 + gi) % (unsigned)nmine) : 0;
        auto blk_of = [&](int i) { const int t = i + rot; return wave + NW * (t >= nmine ? t - nmine : t); };
        u32x4 kA[4], vA[4], kB[4], vB[4];
        issue(blk_of(0), kA, vA);
        int i = 0;
#pragma unroll 1
        for (; i + 2 < nmine; i += 2) {
            issue(blk_of(i + 1), kB, vB);
            __builtin_amdgcn_sched_barrier(0);     // keep the prefetch ahead of the arithmetic
            reduce(blk_of(i), i == 0, kA, vA);
            issue(blk_of(i + 2), kA, vA);
            __builtin_amdgcn_sched_barrier(0);
            reduce(blk_of(i + 1), false, kB, vB);
        }
        if (i + 2 == nmine) {
            issue(blk_of(i + 1), kB, vB);
            __builtin_amdgcn_sched_barrier(0);
            reduce(blk_of(i), i == 0, kA, vA);
            reduce(blk_of(i + 1), false, kB, vB);
        } else {
            reduce(blk_of(i), i == 0, kA, vA);
        }
        // Take the scales out again (exact: integer powers of two).  den belongs to head n; acc[e][r]
        // to head 4g + r, whose exponent sits in the lanes with n = 4g + r.
        den *= __builtin_amdgcn_exp2f(-kq);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float inv = __builtin_amdgcn_exp2f(-__shfl(kq, 4 * g + r));
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e][r] *= inv;
        }
    }

    // ---- the appended key, if this chunk takes it: one more term of Eq. 4 per head ----
    // Lane group (wave, g) of the first four wavefronts handles head 4 wave + g on the vector ALU: weight e^{x - phi}
    // and guard from the step's own K row.  The weights go to LDS and enter the sums at
    // the reduction below, multiplied with the step's V row.
    float e_new = 0.f;
    int f_new = 0;
    const size_t row_new = at.absolute(owner ? S_res - start : 0);   // where the appended row goes (all lanes look the page up)
    if (owner) {
        const int hh = 4 * wave + g;
        const size_t at_new = (size_t)gi * kHeadDim;
        const u32x4 kn = reinterpret_cast<const u32x4 *>(p.k_new + at_new)[n];
        const u32x4 qh = reinterpret_cast<const u32x4 *>(p.q + (size_t)(row0 + min(hh, G - 1)) * kHeadDim)[n];
        const float d = row16_sum(dot8(qh, kn)) * scale + nphi;
        if (hh < G) {                          // (never for a wavefront past the fourth: hh >= 16)
            f_new = !((d > lo) & (d < hi));
            e_new = __builtin_amdgcn_exp2f(d * kLog2e);
        }
        if (wave == 0 && g == 0) {             // 16 lanes put the rows into the cache
            reinterpret_cast<u32x4 *>(p.k_store)[row_new + n] = kn;
            reinterpret_cast<u32x4 *>(p.v_store)[row_new + n] = reinterpret_cast<const u32x4 *>(p.v_new + at_new)[n];
        }
    }

    // ---- workgroup reduction and publication of the G rows' partial results ----
    const unsigned long long bad_mask = __ballot(bad);
    const unsigned long long over_mask = __ballot(head_on & (zmax >= kOverflowLog2));   // a weight beyond the fp16 operand
    __syncthreads();                           // every wavefront is done with its K staging
    // acc[e][r] is (head 4g + r, d = 8n + e) of this wavefront's partial tile.
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int h = 4 * g + r;
        if (h < G) {
            // Row layout in LDS: elements 8n..8n+3 at 4n, elements 8n+4..8n+7 at 64 + 4n, so that
            // consecutive lanes write consecutive 16-byte slots (no bank conflicts).
            float4 *dst = reinterpret_cast<float4 *>(&lds.tile[(wave * 16 + h) * kHeadDim + 4 * n]);
            dst[0] = make_float4(acc[0][r], acc[1][r], acc[2][r], acc[3][r]);
            dst[16] = make_float4(acc[4][r], acc[5][r], acc[6][r], acc[7][r]);
        }
    }
    lds.den[wave][lane] = den;
    if (lane == 0) { lds.bad[wave] = bad_mask; lds.over[wave] = over_mask; }
    if (n == 0 && wave < 4) { lds.e_new[4 * wave + g] = e_new; lds.f_new[4 * wave + g] = f_new; }
    __syncthreads();
    unsigned long long any = 0, any_over = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) { any |= lds.bad[w]; any_over |= lds.over[w]; }
    // head h was flagged iff one of its 4 lanes (h, h+16, h+32, h+48) in any wavefront says so
    unsigned flagged_heads = (unsigned)((any | (any >> 16) | (any >> 32) | (any >> 48)) & 0xffffull);
#pragma unroll
    for (int h = 0; h < 16; ++h) flagged_heads |= (unsigned)(lds.f_new[h] != 0) << h;
    // heads whose sums have to be redone: the flagged ones, and those with a weight that did not fit
    const unsigned redo_heads = flagged_heads | (unsigned)((any_over | (any_over >> 16) | (any_over >> 32) | (any_over >> 48)) & 0xffffull);
    auto den_of = [&](int h) {                 // Eq. 4's denominator of head h over this chunk
        float s = lds.e_new[h];
#pragma unroll
        for (int w = 0; w < NW; ++w)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) s += lds.den[w][h + 16 * q4];
        return s;
    };
    // A sequence of one chunk whose guard stayed quiet is complete here: its rows' results are
    // this workgroup's own sums, so they go out directly instead of through the workspace and
    // the epilogue (same arithmetic: the epilogue's factors are exactly 1 for such a row).
    const bool solo = p.elect && nb == 1 && !redo_heads;
    // 4 consecutive elements per thread: one 16-byte LDS read per wavefront tile, 16 bytes out
    for (int i = 4 * tid; i < G * kHeadDim; i += 4 * kGqaThreads) {
        float4 o = *reinterpret_cast<const float4 *>(&lds.tile[i]);
#pragma unroll
        for (int w = 1; w < NW; ++w) {         // wavefront order
            const float4 t = *reinterpret_cast<const float4 *>(&lds.tile[w * 16 * kHeadDim + i]);
            o.x += t.x; o.y += t.y; o.z += t.z; o.w += t.w;
        }
        const int q = i & (kHeadDim - 1);      // LDS position -> element index (see the layout above)
        const int d0 = 2 * (q & 63) + 4 * (q >> 6);
        if (owner) {                           // + e_new[head] * v_new[d0 .. d0 + 3]
            const float en = lds.e_new[i / kHeadDim];
            const uint2 vn = *reinterpret_cast<const uint2 *>(p.v_new + (size_t)gi * kHeadDim + d0);
            const half2_t v01 = as_h2(vn.x), v23 = as_h2(vn.y);
            o.x = __builtin_fmaf(en, (float)v01.x, o.x); o.y = __builtin_fmaf(en, (float)v01.y, o.y);
            o.z = __builtin_fmaf(en, (float)v23.x, o.z); o.w = __builtin_fmaf(en, (float)v23.y, o.w);
        }
        if (solo) {
            const float l = den_of(i / kHeadDim);
            uint2 h;
            h.x = (unsigned)to_half_bits(o.x / l) | ((unsigned)to_half_bits(o.y / l) << 16);
            h.y = (unsigned)to_half_bits(o.z / l) | ((unsigned)to_half_bits(o.w / l) << 16);
            *reinterpret_cast<uint2 *>(p.out + (size_t)(row0 + i / kHeadDim) * kHeadDim + d0) = h;
        }
        float *dst = &p.ws.num[((size_t)(row0 + i / kHeadDim) * p.nc + c) * kHeadDim + d0];
        if (p.elect && !solo) {      // read by another workgroup of this launch: write through
            store_coherent4(dst, o.x, o.y, o.z, o.w);
        } else {
            *reinterpret_cast<float4 *>(dst) = o;
        }
    }
    if (tid < G) {
        const float s = den_of(tid);
        const size_t slot = (size_t)(row0 + tid) * p.nc + c;
        const int f = (flagged_heads >> tid) & 1;
        store_coherent(&p.ws.den[slot], s);
        store_coherent(&p.ws.mloc[slot], p.phi);
        store_meta(p, slot, s, p.phi, f);
        p.ws.chunk_flags[slot] = (uint8_t)f;
        if (solo) p.ws.row_flags[row0 + tid] = 0;
    }
    if (solo) return;

    // Section 3 "Recomputation": a (head, chunk) whose guard fired is redone with the
    // synchronized scheme on the per-row path (rare; re-reads this chunk only).  So is one whose
    // weights did not fit the fp16 operands; its slot record then says "not flagged".
    if (redo_heads) {
        wait_stores_performed();               // the stores above must not overtake the rewrite
        for (int h = 0; h < G; ++h) {
            if (!((redo_heads >> h) & 1)) continue;
            __syncthreads();
            chunk_body<C, NW, UP, true, C, false, PAGED>(p, row0 + h, c, *reinterpret_cast<ChunkLds<NW, C> *>(lds.tile), nullptr,
                                                         (int)((flagged_heads >> h) & 1));
        }
    }

    if (!p.elect) return;                      // a row-epilogue launch follows
    // Publish, arrive, and let the last arrival of the group finish its G rows.
    wait_stores_performed();
    __syncthreads();
    if (tid == 0) lds.last = arrive_and_elect(p, row0, c, nb);
    __syncthreads();
    if (!lds.last) return;
    group_epilogue(p, row0, G, nb);
}

template <int C> struct GqaLauncher {
    static hipError_t run(const Problem &p0, hipStream_t s)
    {
        const long long groups = (long long)p0.B * p0.Hkv;
        const unsigned grid = (unsigned)(8ll * ((groups + 7) / 8) * p0.nc);
        if (grid == 0) return hipSuccess;
        Problem p = p0;
        p.chunk_major = grid <= 1024u;
        p.scatter |= !p.elect;                     // no hand-over inside the launch: every XCD reads from every head group
        // 4 wavefronts per workgroup.  (8 were measured for launches of at most one workgroup per
        // compute unit: within 2 % either way at 256 workgroups, 12 % faster only for a lone
        // 4096-key chunk, which fd_pick_chunk never chooses.)
        if (p.block_table) return launch(decode_fused_gqa_kernel<C, true, 4>, dim3(grid), dim3(256), s, p);
        return launch(decode_fused_gqa_kernel<C, false, 4>, dim3(grid), dim3(256), s, p);
    }
};

}  // namespace

hipError_t launch_decode_fused_gqa(const Problem &p, hipStream_t s)
{
    switch (chunk_capacity(p.C)) {
        case 64:   return GqaLauncher<64>::run(p, s);
        case 128:  return GqaLauncher<128>::run(p, s);
        case 256:  return GqaLauncher<256>::run(p, s);
        case 512:  return GqaLauncher<512>::run(p, s);
        case 1024: return GqaLauncher<1024>::run(p, s);
        case 2048: return GqaLauncher<2048>::run(p, s);
        case 4096: return GqaLauncher<4096>::run(p, s);
        default:   return hipErrorInvalidValue;
    }
}

}  // namespace fd
