// C-ABI entry points of libfdattn: argument checks, workspace carving, launch order.
#include "../../include/fdattn.h"
#include "fd_internal.h"

#include <cfloat>
#include <cmath>
#include <mutex>

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Layout {
    size_t num, den, mloc, chunk_flags, meta, row_flags, list, count, data_end, ticket_bytes, total;
    long long rows, nc;
};

// Bytes of the data sections (everything but the arrival counters) and of the arrival
// counters for `slots` (row, chunk) pairs.  Both depend on the slot count alone and grow with
// it -- the per-row arrays are sized by slots >= rows -- which is what lets one workspace
// serve different shapes: data sections grow upwards from offset 0, the counters sit at the
// END of the workspace, and for any two shapes that fit the same workspace the data of one
// never reaches the counters of the other.
inline size_t data_bytes(size_t slots, Layout *L = nullptr)
{
    Layout tmp;
    if (!L) L = &tmp;
    size_t off = 0;
    L->num = off;          off = align_up(off + slots * fd::kHeadDim * sizeof(float));
    L->den = off;          off = align_up(off + slots * sizeof(float));
    L->mloc = off;         off = align_up(off + slots * sizeof(float));
    L->chunk_flags = off;  off = align_up(off + slots);
    L->meta = off;         off = align_up(off + slots * sizeof(fd::SlotMeta));
    L->row_flags = off;    off = align_up(off + slots);
    L->list = off;         off = align_up(off + slots * sizeof(int32_t));
    L->count = off;        off = align_up(off + sizeof(int32_t));
    L->data_end = off;
    return off;
}
inline size_t ticket_bytes(size_t slots) { return align_up(slots * sizeof(int32_t)); }

// FD_OK and a filled layout, or the reason the shape cannot be served.
fd_status plan(const fd_shape *sh, Layout *L)
{
    if (!sh) return FD_ERR_NULL;
    if (sh->batch < 0 || sh->n_q_heads <= 0 || sh->n_kv_heads <= 0 || sh->head_dim <= 0 ||
        sh->max_seq <= 0 || sh->chunk <= 0)
        return FD_ERR_SHAPE;
    if (sh->n_q_heads % sh->n_kv_heads != 0) return FD_ERR_SHAPE;
    if (!std::isfinite(sh->scale)) return FD_ERR_SHAPE;
    if (sh->head_dim != fd::kHeadDim) return FD_ERR_UNSUPPORTED;
    if (sh->chunk < 64 || sh->chunk > 4096 || sh->chunk % 16 != 0) return FD_ERR_UNSUPPORTED;
    const long long rows = (long long)sh->batch * sh->n_q_heads;
    const long long nc = ((long long)sh->max_seq + sh->chunk - 1) / sh->chunk;
    if (rows * nc >= (1ll << 31)) return FD_ERR_UNSUPPORTED;
    const size_t slots = (size_t)(rows * nc);
    data_bytes(slots, L);
    L->ticket_bytes = ticket_bytes(slots);
    L->total = L->data_end + L->ticket_bytes;
    L->rows = rows;
    L->nc = nc;
    return FD_OK;
}

fd_status check_ws(const Layout &L, fd_workspace ws)
{
    if (!ws.ptr || ((uintptr_t)ws.ptr % kAlign) != 0 || ws.bytes < L.total) return FD_ERR_WORKSPACE;
    return FD_OK;
}

// End of the workspace as the counters see it: the last 256-byte boundary inside it.
inline char *ws_end(fd_workspace ws) { return static_cast<char *>(ws.ptr) + ws.bytes / kAlign * kAlign; }

// The arrival-counter region that fd_workspace_init clears: large enough for every shape
// this workspace can hold (the largest slot count whose data and counters still fit).
inline size_t max_ticket_bytes(size_t ws_bytes)
{
    size_t lo = 0, hi = (size_t)1 << 31;            // slots: lo fits, hi does not
    if (data_bytes(0) + ticket_bytes(0) > ws_bytes) return 0;
    while (hi - lo > 1) {
        const size_t mid = lo + (hi - lo) / 2;
        if (data_bytes(mid) + ticket_bytes(mid) <= ws_bytes) lo = mid; else hi = mid;
    }
    return ticket_bytes(lo);
}

fd::WsView view(const Layout &L, fd_workspace ws)
{
    char *base = static_cast<char *>(ws.ptr);
    fd::WsView w;
    w.num = reinterpret_cast<float *>(base + L.num);
    w.den = reinterpret_cast<float *>(base + L.den);
    w.mloc = reinterpret_cast<float *>(base + L.mloc);
    w.chunk_flags = reinterpret_cast<uint8_t *>(base + L.chunk_flags);
    w.meta = reinterpret_cast<fd::SlotMeta *>(base + L.meta);
    w.row_flags = reinterpret_cast<uint8_t *>(base + L.row_flags);
    w.list = reinterpret_cast<int32_t *>(base + L.list);
    w.count = reinterpret_cast<int32_t *>(base + L.count);
    w.ticket = reinterpret_cast<int32_t *>(ws_end(ws) - L.ticket_bytes);
    return w;
}

inline bool misaligned(const void *p) { return ((uintptr_t)p % 16) != 0; }

#ifdef FD_PHASE_PROBE
int g_probe_scatter = 0;       // probe build only: see Problem::scatter
#endif

fd_status make_problem(const fd_shape *sh, const void *q, const void *k, const void *v,
                       const int32_t *seq_lens, void *out, bool need_out, fd_workspace ws,
                       fd::Problem *p)
{
    Layout L;
    fd_status st = plan(sh, &L);
    if (st != FD_OK) return st;
    if (!q || !k || !v || !seq_lens || (need_out && !out)) return FD_ERR_NULL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || (need_out && misaligned(out)) ||
        ((uintptr_t)seq_lens % 4) != 0)
        return FD_ERR_SHAPE;
    st = check_ws(L, ws);
    if (st != FD_OK) return st;
    p->q = static_cast<const uint16_t *>(q);
    p->k = static_cast<const uint16_t *>(k);
    p->v = static_cast<const uint16_t *>(v);
    p->seq_lens = seq_lens;
    p->out = static_cast<uint16_t *>(out);
    p->ws = view(L, ws);
    p->B = sh->batch; p->Hq = sh->n_q_heads; p->Hkv = sh->n_kv_heads;
    p->G = sh->n_q_heads / sh->n_kv_heads;
    p->Smax = sh->max_seq; p->C = sh->chunk; p->nc = (int)L.nc; p->rows = (int)L.rows;
    p->scale = sh->scale; p->phi = 0.f; p->lo = 0.f; p->hi = 0.f;
    p->elect = 0;
    p->chunk_major = 0;
    p->k_new = p->v_new = nullptr;
    p->k_store = p->v_store = nullptr;
    p->block_table = nullptr;
    p->pages_per_seq = 0; p->page_shift = 0; p->n_pages = 0;
    p->scatter = 0;
#ifdef FD_PHASE_PROBE
    p->scatter = g_probe_scatter;          // (probe build: spread the rows over the XCDs in every launch)
#endif
    return FD_OK;
}

fd_status set_guard(fd::Problem *p, float phi, fd_bounds b)
{
    if (!std::isfinite(phi) || !std::isfinite(b.lo) || !std::isfinite(b.hi) || !(b.lo < b.hi))
        return FD_ERR_BOUNDS;
    p->phi = phi; p->lo = b.lo; p->hi = b.hi;
    return FD_OK;
}

// Whether the chunk kernel should finish the rows itself (one launch) or leave that
// to a second, tiny launch.  Electing a finisher costs every workgroup two memory
// round trips at its end (results performed, arrival counter); a second launch costs
// about 3 us once.  Small grids are latency-bound, so they fuse; large grids keep
// their workgroups streaming and pay the launch.
inline int elect_in_kernel(long long workgroups, long long limit = 1024, bool and_also = true)
{
    return workgroups <= limit && and_also;
}

// The per-row kernel: one launch up to 1024 workgroups, unless the launch is long -- more than one
// round of the chip over 320 MiB or more of cache -- where the second launch wins (whole call, one
// launch / two, same box: 2 x 32 rows x 16384 keys 90.0 / 84.7 us, 4 x 32 x 8192 85.4 / 83.6, 1 x 32 x
// 32768 91.3 / 83.7, 1 x 32 x 24000 68.9 / 65.0; at 256 MiB they tie: 44.7 / 44.5, 46.2 / 45.7, 46.3 /
// 44.8) at the price of a cache that is mostly empty (1 x 32 x 32768 holding 8192 keys: 26.8 / 31.4 us).
inline int elect_per_row(const fd::Problem &p)
{
    const long long workgroups = (long long)p.rows * p.nc;
    const long long cache_bytes = (long long)p.B * p.Hkv * p.Smax * fd::kHeadDim * 2 * 2;
    return elect_in_kernel(workgroups, 1024, workgroups <= 256 || cache_bytes < (320ll << 20));
}

// The grouped kernel: its elected workgroup finishes the G rows of its head group by itself,
// walking each row's chunks in order, which is the cheaper way up to 8 chunks per row and 256
// workgroups; beyond either the second launch (one workgroup per row, 8 chunk slices in
// parallel) wins: whole call, one launch / two, 64 query on 8 KV heads -- 25.7 / 26.4 us at 4
// chunks per row, 17.4 / 17.2 at 8, 18.9 / 17.7 at 16, 18.0 / 15.3 at 24, 30.3 / 27.2 at 32.
inline int elect_grouped(const fd::Problem &p)
{
    return elect_in_kernel((long long)p.B * p.Hkv * p.nc, 256, p.nc <= 8);
}

#define FD_TRY(expr) do { if ((expr) != hipSuccess) return FD_ERR_HIP; } while (0)

// A problem description that carries only the shape and the workspace views.
fd_status make_ws_problem(const fd_shape *sh, fd_workspace ws, fd::Problem *p)
{
    Layout L;
    fd_status st = plan(sh, &L);
    if (st != FD_OK) return st;
    st = check_ws(L, ws);
    if (st != FD_OK) return st;
    *p = fd::Problem{};
    p->ws = view(L, ws);
    p->B = sh->batch; p->Hq = sh->n_q_heads; p->Hkv = sh->n_kv_heads;
    p->G = sh->n_q_heads / sh->n_kv_heads;
    p->Smax = sh->max_seq; p->C = sh->chunk; p->nc = (int)L.nc; p->rows = (int)L.rows;
    p->scale = sh->scale;
    return FD_OK;
}

}  // namespace

extern "C" {

size_t fd_workspace_bytes(const fd_shape *shape)
{
    Layout L;
    return plan(shape, &L) == FD_OK ? L.total : 0;
}

// Chunk size from the shape alone (shape->chunk is ignored).  Fitted to sweeps on MI355X
// (per-row kernel: batch 1 .. 32 x 1K .. 32K keys; grouped kernel: batch 1 .. 64): one
// workgroup streams one chunk, so a chunk should be as long as possible (fewer partial
// results, fewer hand-overs) while the launch still covers the 256 CUs.
//   per-row kernel: at least four chunks per row and at most 2048 keys per chunk (a row in one
//     or two pieces, or very long pieces, hide less latency: 18.3 us against 14.7 for 4 x 32
//     rows of 1K keys cut in two instead of four); a large batch, whose sequences may differ in
//     length (8 sequences or more), gets enough workgroups per CU (about 16) to even out ragged
//     rows, but never chunks below 256 keys for that; otherwise the longest chunk that still
//     gives 256 workgroups -- for a batch, 2048 keys only where that makes the launch a single
//     round of the chip, else at most 1024.  Within 6 % of the best chunk on every shape of the sweeps.
//   grouped kernel: 1/G as many workgroups, each with four wavefronts' worth of loads in flight
//     and a heavy tail (reduction over the group's heads); it is fastest with one workgroup
//     per CU -- a single launch that finishes its rows itself -- so: the fewest chunks, of up to
//     4096 keys, that still give 256 workgroups and fill their last round of the chip
//     (B x 64/8 heads x 4096 keys: 25.2 us at 1024 keys against 29.2 at 256 for B = 8; 80.8 at
//     4096 against 87.6 at 1024 for B = 32).
//   Both: max_seq is cut into equal chunks (a multiple of 16 keys, a power of two only where
//     max_seq divides that way) so that launches of a few rounds of the chip fill their last one.
int32_t fd_pick_chunk(const fd_shape *shape)
{
    if (!shape) return 0;
    fd_shape sh = *shape;
    sh.chunk = 64;
    Layout L;
    if (plan(&sh, &L) != FD_OK) return 0;
    static const int32_t sizes[] = {4096, 2048, 1024, 512, 256, 128, 64};
    const int group = sh.n_q_heads / sh.n_kv_heads;
    const bool grouped = group >= 2 && group <= 16;   // the shapes that run on the grouped kernel
    const long long units = (long long)sh.batch * (grouped ? sh.n_kv_heads : sh.n_q_heads);
    auto workgroups = [&](int32_t c) { return units * (((long long)sh.max_seq + c - 1) / c); };
    auto largest_with = [&](long long want, int32_t shortest, int32_t longest) -> int32_t {
        for (int32_t c : sizes)
            if (c >= shortest && c <= longest && workgroups(c) >= want) return c;
        return 0;
    };
    int32_t c = 0;
    auto fill_of = [](long long w) { return (double)w / (256.0 * (double)((w + 255) / 256)); };
    if (grouped) {
        // the fewest (longest, equal) chunks whose workgroups fill whole rounds of the 256 CUs to 90 %
        // (384 workgroups would leave half the chip idle in their second round: 139 us against 128 us
        // with 768); a length is a multiple of 16 keys, not necessarily a power of two
        double best = 0.0;
        long long alt_nb = 0, nb_taken = 0;
        int32_t alt = 0;
        for (long long nb = ((long long)sh.max_seq + 4095) / 4096; nb <= ((long long)sh.max_seq + 63) / 64; ++nb) {
            const long long len = (((long long)sh.max_seq + nb - 1) / nb + 15) / 16 * 16;
            if (len < 64) break;
            const long long w = workgroups((int32_t)len);
            if (w < 256) {
                // a single round that is 90 % full: remembered, see below
                if (w >= 231 && !alt) { alt = (int32_t)len; alt_nb = nb; }
                continue;
            }
            const double fill = fill_of(w);
            if (fill >= 0.9) { c = (int32_t)len; nb_taken = nb; break; }
            if (fill > best) { best = fill; c = (int32_t)len; nb_taken = nb; }
        }
        // ... and taken when it needs at most two thirds of the chunks (5 x 8 head groups x 3000 keys:
        // 6 chunks of 512, 240 workgroups, 16.6 us, against 12 of 256, 480 workgroups, 18.4 us)
        if (alt && (!c || 3 * alt_nb <= 2 * nb_taken)) c = alt;
    } else {
        const int32_t quarter = sh.max_seq / 4;
        const int32_t longest = quarter >= 2048 ? 2048 : (quarter < 64 ? 64 : quarter);
        // many sequences, whose lengths may differ: enough workgroups per CU to even them out
        if (sh.batch >= 8) c = largest_with(4096, 256, longest < 1024 ? longest : 1024);
        if (!c) c = largest_with(256, 64, longest);
        // Chunks of 2048 keys pay when they make the launch a single round of the chip, and for a single
        // sequence at any length (1 x 32 rows x 131072 keys: 315 us against 372 with 1024, 65536: 160
        // against 171 -- a row of 64 or more chunks streams badly); a batch whose 2048-key chunks give
        // more than one round does as well or better with 1024 (2 x 16384: 83.3 against 83.9 us; 3 x 8192:
        // 63.8 against 67.2 with the equal chunks of 1648 that 2048 would become; 4 x 32768: a tie).
        if (c == 2048 && sh.batch >= 2 && workgroups(2048) > 256) c = 1024;
    }
    if (!c) c = largest_with(256, 64, grouped ? 4096 : 1024);
    if (!c) c = 64;
    // A launch of one to four rounds of the chip that leaves its last round less than 90 % full
    // (288 workgroups: 32 CUs stream two chunks while 224 wait) gets chunks of equal length, a
    // multiple of 16 keys that need not be a power of two, in the number that fills whole rounds:
    // 32 rows of 9216 keys run as 8 x 1152 keys instead of 9 x 1024 (34.8 -> 27 us).  Fewest (longest)
    // chunks first, within a factor of two of the choice above.
    const long long w0 = workgroups(c);
    if (w0 > 256 && w0 <= 1024 && fill_of(w0) < 0.9) {
        const long long nb0 = ((long long)sh.max_seq + c - 1) / c;
        const int32_t cap = grouped ? 4096 : 2048;
        double best = fill_of(w0);
        for (long long nb = nb0 / 2 > 0 ? nb0 / 2 : 1; nb <= 2 * nb0; ++nb) {
            const long long len = (((long long)sh.max_seq + nb - 1) / nb + 15) / 16 * 16;
            if (len < 64 || len > cap) continue;
            const double fill = fill_of(workgroups((int32_t)len));
            if (fill >= 0.9) { c = (int32_t)len; break; }
            if (fill > best + 0.05) { best = fill; c = (int32_t)len; }
        }
    }
    return c;
}

// The chunk kernel of fd_decode_attn / fd_decode_attn_gqa alone: no election, no
// row epilogue.
static fd_status partial_only(const fd_shape *shape, const void *q, const void *k_cache,
                              const void *v_cache, const int32_t *seq_lens, float phi,
                              fd_bounds bounds, fd_workspace ws, void *stream, bool grouped)
{
    fd::Problem p;
    fd_status st = make_problem(shape, q, k_cache, v_cache, seq_lens, nullptr, false, ws, &p);
    if (st != FD_OK) return st;
    st = set_guard(&p, phi, bounds);
    if (st != FD_OK) return st;
    if (grouped && (p.G < 2 || p.G > 16)) return FD_ERR_UNSUPPORTED;
    if (p.rows == 0) return FD_OK;
    p.elect = 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    FD_TRY(grouped ? fd::launch_decode_fused_gqa(p, s) : fd::launch_decode_fused(p, s));
    return FD_OK;
}

fd_status fd_decode_attn_partial(const fd_shape *shape, const void *q, const void *k_cache,
                                 const void *v_cache, const int32_t *seq_lens, float phi,
                                 fd_bounds bounds, fd_workspace ws, void *stream)
{
    return partial_only(shape, q, k_cache, v_cache, seq_lens, phi, bounds, ws, stream, false);
}

fd_status fd_decode_attn_gqa_partial(const fd_shape *shape, const void *q, const void *k_cache,
                                     const void *v_cache, const int32_t *seq_lens, float phi,
                                     fd_bounds bounds, fd_workspace ws, void *stream)
{
    return partial_only(shape, q, k_cache, v_cache, seq_lens, phi, bounds, ws, stream, true);
}

fd_status fd_workspace_init(const fd_shape *shape, fd_workspace ws, void *stream)
{
    Layout L;
    fd_status st = plan(shape, &L);
    if (st != FD_OK) return st;
    st = check_ws(L, ws);
    if (st != FD_OK) return st;
    // every counter any shape could use in this workspace, not just this shape's
    const size_t bytes = max_ticket_bytes(ws.bytes);
    FD_TRY(fd::launch_clear_tickets(reinterpret_cast<int32_t *>(ws_end(ws) - bytes), bytes / sizeof(int32_t),
                                    static_cast<hipStream_t>(stream)));
    return FD_OK;
}

fd_status fd_decode_attn(const fd_shape *shape, const void *q, const void *k_cache,
                         const void *v_cache, const int32_t *seq_lens, float phi,
                         fd_bounds bounds, void *out, fd_workspace ws, void *stream)
{
    fd::Problem p;
    fd_status st = make_problem(shape, q, k_cache, v_cache, seq_lens, out, true, ws, &p);
    if (st != FD_OK) return st;
    st = set_guard(&p, phi, bounds);
    if (st != FD_OK) return st;
    if (p.rows == 0) return FD_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    p.elect = elect_per_row(p);
    FD_TRY(fd::launch_decode_fused(p, s));
    if (!p.elect) FD_TRY(fd::launch_row_epilogue(p, s));
    return FD_OK;
}

fd_status fd_decode_attn_gqa(const fd_shape *shape, const void *q, const void *k_cache,
                             const void *v_cache, const int32_t *seq_lens, float phi,
                             fd_bounds bounds, void *out, fd_workspace ws, void *stream)
{
    fd::Problem p;
    fd_status st = make_problem(shape, q, k_cache, v_cache, seq_lens, out, true, ws, &p);
    if (st != FD_OK) return st;
    st = set_guard(&p, phi, bounds);
    if (st != FD_OK) return st;
    if (p.G < 2 || p.G > 16) return FD_ERR_UNSUPPORTED;
    if (p.rows == 0) return FD_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // the grouped kernel holds fewer workgroups per CU, so the election hurts it sooner
    p.elect = elect_grouped(p);
    FD_TRY(fd::launch_decode_fused_gqa(p, s));
    if (!p.elect) FD_TRY(fd::launch_row_epilogue(p, s));
    return FD_OK;
}

fd_status fd_decode_attn_append(const fd_shape *shape, const void *q, const void *k_new, const void *v_new,
                                void *k_cache, void *v_cache, const int32_t *seq_lens, float phi,
                                fd_bounds bounds, void *out, fd_workspace ws, void *stream)
{
    fd::Problem p;
    fd_status st = make_problem(shape, q, k_cache, v_cache, seq_lens, out, true, ws, &p);
    if (st != FD_OK) return st;
    st = set_guard(&p, phi, bounds);
    if (st != FD_OK) return st;
    if (!k_new || !v_new) return FD_ERR_NULL;
    if (misaligned(k_new) || misaligned(v_new)) return FD_ERR_SHAPE;
    if (p.rows == 0) return FD_OK;
    p.k_new = static_cast<const uint16_t *>(k_new);
    p.v_new = static_cast<const uint16_t *>(v_new);
    p.k_store = static_cast<uint16_t *>(k_cache);
    p.v_store = static_cast<uint16_t *>(v_cache);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (p.G >= 2 && p.G <= 16) {
        p.elect = elect_grouped(p);
        FD_TRY(fd::launch_decode_fused_gqa(p, s));
    } else {
        p.elect = elect_per_row(p);
        FD_TRY(fd::launch_decode_fused(p, s));
    }
    if (!p.elect) FD_TRY(fd::launch_row_epilogue(p, s));
    return FD_OK;
}

// Shared by the two paged entry points: checks and fields of the paged cache.
static fd_status set_paged(fd::Problem *p, const fd_shape *shape, const int32_t *block_table, int32_t page_size, int32_t n_pages)
{
    if (!block_table) return FD_ERR_NULL;
    if (((uintptr_t)block_table % 4) != 0) return FD_ERR_SHAPE;
    // a power of two; a chunk may span at most 64 pages (one table entry per lane)
    if (page_size < 16 || (page_size & (page_size - 1)) != 0 || n_pages < 1 || shape->max_seq % page_size != 0 ||
        // a chunk's pages are looked up by the 64 lanes of a wavefront; a chunk that neither divides
        // nor is divided by the page may start anywhere in one (at a multiple of 16)
        (shape->chunk % page_size == 0 || page_size % shape->chunk == 0 ? shape->chunk : shape->chunk + page_size - 16) >
            64 * (long long)page_size)
        return FD_ERR_SHAPE;
    p->block_table = block_table;
    p->pages_per_seq = shape->max_seq / page_size;
    p->page_shift = __builtin_ctz((unsigned)page_size);
    p->n_pages = n_pages;
    return FD_OK;
}

static fd_status run_fused(fd::Problem &p, hipStream_t s)
{
    if (p.G >= 2 && p.G <= 16) {
        p.elect = elect_grouped(p);
        FD_TRY(fd::launch_decode_fused_gqa(p, s));
    } else {
        p.elect = elect_per_row(p);
        FD_TRY(fd::launch_decode_fused(p, s));
    }
    if (!p.elect) FD_TRY(fd::launch_row_epilogue(p, s));
    return FD_OK;
}

fd_status fd_decode_attn_paged(const fd_shape *shape, const void *q, const void *k_pool, const void *v_pool,
                               const int32_t *block_table, int32_t page_size, int32_t n_pages,
                               const int32_t *seq_lens, float phi, fd_bounds bounds, void *out,
                               fd_workspace ws, void *stream)
{
    fd::Problem p;
    fd_status st = make_problem(shape, q, k_pool, v_pool, seq_lens, out, true, ws, &p);
    if (st != FD_OK) return st;
    st = set_guard(&p, phi, bounds);
    if (st != FD_OK) return st;
    st = set_paged(&p, shape, block_table, page_size, n_pages);
    if (st != FD_OK) return st;
    if (p.rows == 0) return FD_OK;
    return run_fused(p, static_cast<hipStream_t>(stream));
}

fd_status fd_decode_attn_paged_append(const fd_shape *shape, const void *q, const void *k_new, const void *v_new,
                                      void *k_pool, void *v_pool, const int32_t *block_table, int32_t page_size,
                                      int32_t n_pages, const int32_t *seq_lens, float phi, fd_bounds bounds,
                                      void *out, fd_workspace ws, void *stream)
{
    fd::Problem p;
    fd_status st = make_problem(shape, q, k_pool, v_pool, seq_lens, out, true, ws, &p);
    if (st != FD_OK) return st;
    st = set_guard(&p, phi, bounds);
    if (st != FD_OK) return st;
    st = set_paged(&p, shape, block_table, page_size, n_pages);
    if (st != FD_OK) return st;
    if (!k_new || !v_new) return FD_ERR_NULL;
    if (misaligned(k_new) || misaligned(v_new)) return FD_ERR_SHAPE;
    if (p.rows == 0) return FD_OK;
    p.k_new = static_cast<const uint16_t *>(k_new);
    p.v_new = static_cast<const uint16_t *>(v_new);
    p.k_store = static_cast<uint16_t *>(k_pool);
    p.v_store = static_cast<uint16_t *>(v_pool);
    return run_fused(p, static_cast<hipStream_t>(stream));
}

// ---- fd_decode_attn_static: the workspace lives in the library's own device memory ----
//
// `static_scratch` is the array's host-side stand-in: in host code the name is not a device
// address.  The address on the current device comes from hipGetSymbolAddress, once per device
// (every GPU holds its own copy of the array at its own address), and only that pointer is
// handed to kernels.
static __device__ __align__(256) unsigned char static_scratch[FD_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
void *g_static_ptr[kMaxDevices] = {};

// Device address of static_scratch on the current device.  First call on a device: looks the
// address up and enqueues one clear of the arrival-counter region on `s` (the array starts
// zeroed with the code object; the clear makes the precondition explicit).  Allocates nothing.
fd_status static_scratch_on_current_device(hipStream_t s, void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FD_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(static_scratch)) != hipSuccess || !ptr) return FD_ERR_HIP;
        if (((uintptr_t)ptr % kAlign) != 0) return FD_ERR_HIP;
        const fd_workspace ws{ptr, (size_t)FD_STATIC_SCRATCH_BYTES};
        const size_t bytes = max_ticket_bytes(ws.bytes);
        if (fd::launch_clear_tickets(reinterpret_cast<int32_t *>(ws_end(ws) - bytes), bytes / sizeof(int32_t), s) != hipSuccess)
            return FD_ERR_HIP;
        g_static_ptr[dev] = ptr;
    }
    *out = g_static_ptr[dev];
    return FD_OK;
}
}  // namespace

fd_status fd_decode_attn_static(const fd_shape *shape, const void *q, const void *k_cache, const void *v_cache,
                                const int32_t *seq_lens, float phi, fd_bounds bounds, void *out, void *stream)
{
    Layout L;
    fd_status st = plan(shape, &L);
    if (st != FD_OK) return st;
    if (L.total > (size_t)FD_STATIC_SCRATCH_BYTES) return FD_ERR_STATIC_LIMIT;
    // every host-side check comes before the first touch of the device
    if (!q || !k_cache || !v_cache || !seq_lens || !out) return FD_ERR_NULL;
    if (misaligned(q) || misaligned(k_cache) || misaligned(v_cache) || misaligned(out) || ((uintptr_t)seq_lens % 4) != 0)
        return FD_ERR_SHAPE;
    if (!std::isfinite(phi) || !std::isfinite(bounds.lo) || !std::isfinite(bounds.hi) || !(bounds.lo < bounds.hi))
        return FD_ERR_BOUNDS;
    hipStream_t s = static_cast<hipStream_t>(stream);
    void *ptr = nullptr;
    st = static_scratch_on_current_device(s, &ptr);
    if (st != FD_OK) return st;
    const fd_workspace ws{ptr, (size_t)FD_STATIC_SCRATCH_BYTES};
    fd::Problem p;
    st = make_problem(shape, q, k_cache, v_cache, seq_lens, out, true, ws, &p);
    if (st != FD_OK) return st;
    st = set_guard(&p, phi, bounds);
    if (st != FD_OK) return st;
    if (p.rows == 0) return FD_OK;
    return run_fused(p, s);
}

fd_status fd_decode_attn_multikernel(const fd_shape *shape, const void *q, const void *k_cache,
                                     const void *v_cache, const int32_t *seq_lens, float phi,
                                     fd_bounds bounds, void *out, fd_workspace ws, void *stream)
{
    fd::Problem p;
    fd_status st = make_problem(shape, q, k_cache, v_cache, seq_lens, out, true, ws, &p);
    if (st != FD_OK) return st;
    st = set_guard(&p, phi, bounds);
    if (st != FD_OK) return st;
    if (p.rows == 0) return FD_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    FD_TRY(fd::launch_partial_unified(p, s));
    FD_TRY(fd::launch_chain_combine(p, s));
    FD_TRY(fd::launch_chain_finish(p, s));
    return FD_OK;
}

fd_status fd_list_flagged_rows(const fd_shape *shape, const int32_t *seq_lens, fd_workspace ws, void *stream)
{
    fd::Problem p;
    fd_status st = make_ws_problem(shape, ws, &p);
    if (st != FD_OK) return st;
    if (!seq_lens) return FD_ERR_NULL;
    p.seq_lens = seq_lens;
    FD_TRY(fd::launch_flag_reduce(p, static_cast<hipStream_t>(stream)));
    return FD_OK;
}

fd_status fd_decode_attn_sync(const fd_shape *shape, const void *q, const void *k_cache,
                              const void *v_cache, const int32_t *seq_lens,
                              void *out, fd_workspace ws, void *stream)
{
    fd::Problem p;
    fd_status st = make_problem(shape, q, k_cache, v_cache, seq_lens, out, true, ws, &p);
    if (st != FD_OK) return st;
    if (p.rows == 0) return FD_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    FD_TRY(fd::launch_partial_sync(p, s));
    FD_TRY(fd::launch_combine_sync(p, s));
    return FD_OK;
}

fd_status fd_get_flags(const fd_shape *shape, fd_workspace ws,
                       const uint8_t **chunk_flags, const uint8_t **row_flags,
                       const int32_t **n_flagged, const int32_t **flagged_rows)
{
    Layout L;
    fd_status st = plan(shape, &L);
    if (st != FD_OK) return st;
    st = check_ws(L, ws);
    if (st != FD_OK) return st;
    const fd::WsView w = view(L, ws);
    if (chunk_flags) *chunk_flags = w.chunk_flags;
    if (row_flags) *row_flags = w.row_flags;
    if (n_flagged) *n_flagged = w.count;
    if (flagged_rows) *flagged_rows = w.list;
    return FD_OK;
}

fd_status fd_get_partials(const fd_shape *shape, fd_workspace ws,
                          const float **num, const float **den)
{
    Layout L;
    fd_status st = plan(shape, &L);
    if (st != FD_OK) return st;
    st = check_ws(L, ws);
    if (st != FD_OK) return st;
    const fd::WsView w = view(L, ws);
    if (num) *num = w.num;
    if (den) *den = w.den;
    return FD_OK;
}

fd_status fd_logit_histogram(const fd_shape *shape, const void *q, const void *k_cache,
                             const int32_t *seq_lens, float x_min, float bin_width, int32_t n_bins,
                             uint64_t *hist, float *min_max, void *stream)
{
    if (!shape) return FD_ERR_NULL;
    fd_shape sh = *shape;
    sh.chunk = 64;                                   // the split plays no part in the statistics
    Layout L;
    fd_status st = plan(&sh, &L);
    if (st != FD_OK) return st;
    if (!q || !k_cache || !seq_lens || !hist) return FD_ERR_NULL;
    if (misaligned(q) || misaligned(k_cache) || ((uintptr_t)seq_lens % 4) != 0 || ((uintptr_t)hist % 8) != 0 ||
        ((uintptr_t)min_max % 4) != 0)
        return FD_ERR_SHAPE;
    if (!std::isfinite(x_min) || !std::isfinite(bin_width) || !(bin_width > 0.f)) return FD_ERR_BOUNDS;
    if (n_bins < 1 || n_bins > 4096) return FD_ERR_UNSUPPORTED;
    fd::Problem p{};
    p.q = static_cast<const uint16_t *>(q);
    p.k = static_cast<const uint16_t *>(k_cache);
    p.seq_lens = seq_lens;
    p.B = sh.batch; p.Hq = sh.n_q_heads; p.Hkv = sh.n_kv_heads; p.G = sh.n_q_heads / sh.n_kv_heads;
    p.Smax = sh.max_seq; p.rows = (int)L.rows; p.scale = sh.scale;
    FD_TRY(fd::launch_logit_histogram(p, x_min, bin_width, n_bins, reinterpret_cast<unsigned long long *>(hist),
                                      min_max, static_cast<hipStream_t>(stream)));
    return FD_OK;
}

// Host-side choice of phi and the bounds from a histogram (Section 3: the range that
// holds more than a given fraction of the x_i; phi = a when e^{b-a} fits float32; no
// unified factor when the range is too wide).
fd_status fd_calibrate(const uint64_t *hist, int32_t n_bins, float x_min, float bin_width, double coverage,
                       float margin, float phi_position, int32_t max_seq, fd_calibration *out)
{
    if (!hist || !out) return FD_ERR_NULL;
    if (n_bins < 1 || max_seq < 1) return FD_ERR_SHAPE;
    if (!std::isfinite(x_min) || !std::isfinite(bin_width) || !(bin_width > 0.f) || !std::isfinite(margin) ||
        !(margin >= 0.f) || !(coverage > 0.0 && coverage <= 1.0) || !(phi_position >= 0.f && phi_position <= 1.f))
        return FD_ERR_BOUNDS;
    *out = fd_calibration{};
    unsigned long long total = 0;
    for (int32_t i = 0; i < n_bins + 2; ++i) total += hist[i];
    if (total == 0) return FD_OK;                    // nothing seen: apply = 0
    const unsigned long long tail = (unsigned long long)std::floor((1.0 - coverage) * (double)total / 2.0);
    // walk inwards from both ends while the mass left outside stays within the allowance
    int32_t e_lo = -1, e_hi = -1;
    unsigned long long below = hist[0];              // logits under edge 0
    for (int32_t e = 0; e <= n_bins && below <= tail; ++e) {
        e_lo = e;
        if (e < n_bins) below += hist[e + 1];
    }
    unsigned long long above = hist[n_bins + 1];     // logits at or over edge n_bins
    for (int32_t e = n_bins; e >= 0 && above <= tail; --e) {
        e_hi = e;
        if (e > 0) above += hist[e];
    }
    if (e_lo < 0 || e_hi < 0) return FD_OK;          // the window itself cuts off too much: apply = 0
    if (e_hi <= e_lo) {                              // all mass inside the allowance: keep one bin
        e_hi = e_lo + 1 < n_bins ? e_lo + 1 : n_bins;
        e_lo = e_hi - 1;
    }
    const double w = (double)bin_width, x0 = (double)x_min;
    const double x_lo = x0 + e_lo * w - (double)margin, x_hi = x0 + e_hi * w + (double)margin;
    const double range = x_hi - x_lo;
    // e^{range} x the longest sequence x the largest fp16 magnitude of V must fit float32
    const double limit = std::log((double)FLT_MAX) - std::log((double)max_seq) - std::log(65504.0);
    const double phi = x_lo + (double)phi_position * range;
    unsigned long long inside = 0;
    for (int32_t i = e_lo; i < e_hi; ++i) inside += hist[i + 1];
    out->apply = range <= limit ? 1 : 0;
    out->phi = (float)phi;
    out->bounds.lo = (float)(x_lo - phi);
    out->bounds.hi = (float)(x_hi - phi);
    out->x_lo = (float)x_lo;
    out->x_hi = (float)x_hi;
    out->covered = (double)inside / (double)total;
    return FD_OK;
}

namespace {
struct PrefillLayout { size_t vt, flags, total; int spad, tiles; };
fd_status plan_prefill(const fd_shape *shape, PrefillLayout *P)
{
    if (!shape) return FD_ERR_NULL;
    fd_shape sh = *shape;
    sh.chunk = 64;                                   // the prompt phase has its own tiling
    Layout L;
    fd_status st = plan(&sh, &L);
    if (st != FD_OK) return st;
    P->spad = (sh.max_seq + 63) / 64 * 64;
    P->tiles = P->spad / 64;
    const size_t vt = (size_t)sh.batch * sh.n_kv_heads * fd::kHeadDim * P->spad * sizeof(uint16_t);
    size_t off = 0;
    P->vt = off;     off = align_up(off + vt);
    P->flags = off;  off = align_up(off + (size_t)sh.batch * sh.n_q_heads * P->tiles);
    P->total = off;
    return FD_OK;
}
}  // namespace

size_t fd_prefill_workspace_bytes(const fd_shape *shape)
{
    PrefillLayout P;
    return plan_prefill(shape, &P) == FD_OK ? P.total : 0;
}

fd_status fd_prefill_attn(const fd_shape *shape, const void *q, const void *k_cache, const void *v_cache,
                          const int32_t *seq_lens, float phi, fd_bounds bounds, void *out,
                          fd_workspace ws, void *stream)
{
    PrefillLayout P;
    fd_status st = plan_prefill(shape, &P);
    if (st != FD_OK) return st;
    if (!q || !k_cache || !v_cache || !seq_lens || !out) return FD_ERR_NULL;
    if (misaligned(q) || misaligned(k_cache) || misaligned(v_cache) || misaligned(out) || ((uintptr_t)seq_lens % 4) != 0)
        return FD_ERR_SHAPE;
    if (!std::isfinite(phi) || !std::isfinite(bounds.lo) || !std::isfinite(bounds.hi) || !(bounds.lo < bounds.hi))
        return FD_ERR_BOUNDS;
    if (!ws.ptr || ((uintptr_t)ws.ptr % kAlign) != 0 || ws.bytes < P.total) return FD_ERR_WORKSPACE;
    if (shape->n_q_heads > 65535 || shape->batch > 65535 || (long long)shape->batch * shape->n_kv_heads > 65535)
        return FD_ERR_UNSUPPORTED;                   // grid dimensions
    fd::PrefillProblem p{};
    char *base = static_cast<char *>(ws.ptr);
    p.q = static_cast<const uint16_t *>(q);
    p.k = static_cast<const uint16_t *>(k_cache);
    p.v = static_cast<const uint16_t *>(v_cache);
    p.seq_lens = seq_lens;
    p.out = static_cast<uint16_t *>(out);
    p.vt = reinterpret_cast<uint16_t *>(base + P.vt);
    p.tile_flags = reinterpret_cast<uint8_t *>(base + P.flags);
    p.B = shape->batch; p.Hq = shape->n_q_heads; p.Hkv = shape->n_kv_heads; p.G = p.Hq / p.Hkv;
    p.Smax = shape->max_seq; p.Spad = P.spad; p.tiles = P.tiles;
    p.scale = shape->scale; p.phi = phi; p.lo = bounds.lo; p.hi = bounds.hi;
    FD_TRY(fd::launch_prefill(p, static_cast<hipStream_t>(stream)));
    return FD_OK;
}

fd_status fd_prefill_get_flags(const fd_shape *shape, fd_workspace ws, const uint8_t **tile_flags)
{
    PrefillLayout P;
    fd_status st = plan_prefill(shape, &P);
    if (st != FD_OK) return st;
    if (!ws.ptr || ((uintptr_t)ws.ptr % kAlign) != 0 || ws.bytes < P.total) return FD_ERR_WORKSPACE;
    if (tile_flags) *tile_flags = reinterpret_cast<const uint8_t *>(static_cast<char *>(ws.ptr) + P.flags);
    return FD_OK;
}

#ifdef FD_PHASE_PROBE
// Probe build only (not in the product library, not in the header): deal the chunks of a row to
// different XCDs from the next call on.
void fd_phase_probe_scatter(int on) { g_probe_scatter = on ? 1 : 0; }
#endif

const char *fd_status_str(fd_status status)
{
    switch (status) {
        case FD_OK: return "FD_OK";
        case FD_ERR_NULL: return "FD_ERR_NULL: a required pointer is NULL";
        case FD_ERR_SHAPE: return "FD_ERR_SHAPE: invalid shape, scale or pointer alignment";
        case FD_ERR_BOUNDS: return "FD_ERR_BOUNDS: need finite phi and lo < hi";
        case FD_ERR_WORKSPACE: return "FD_ERR_WORKSPACE: workspace NULL, misaligned or too small";
        case FD_ERR_UNSUPPORTED: return "FD_ERR_UNSUPPORTED: shape not supported by this build";
        case FD_ERR_HIP: return "FD_ERR_HIP: the HIP runtime refused a launch";
        case FD_ERR_STATIC_LIMIT:
            return "FD_ERR_STATIC_LIMIT: the shape needs more scratch than fd_decode_attn_static holds "
                   "(fd_workspace_bytes(shape) > FD_STATIC_SCRATCH_BYTES); use fd_decode_attn with a workspace";
    }
    return "unknown fd_status";
}

}  // extern "C"
