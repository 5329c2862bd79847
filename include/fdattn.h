/*
 * libfdattn -- decode-phase attention with asynchronized softmax for MI355X.
 *
 * C-ABI boundary of the library.  The method is Section 3 of FlashDecoding++
 * (arXiv 2311.01282): one query token per sequence attends over an fp16 KV
 * cache; the sequence axis is cut into chunks ("partial vectors"); every chunk
 * accumulates e^{x - phi} and e^{x - phi} v against ONE unified scaling factor
 * phi, so chunk results simply add (Eq. 3, Eq. 4); a chunk whose logits leave
 * a < x - phi < b raises a flag and its row is produced by the synchronized
 * partial softmax of Eq. 2 instead (Section 3, "Recomputation").  How much of a
 * flagged row is re-read differs by entry point: fd_decode_attn_multikernel
 * recomputes every chunk of the row, as the paper's text has it; fd_decode_attn
 * and its variants recompute only the chunks that left the bounds and merge all
 * of the row's partial results by Eq. 2 (see the description of each call).
 *
 * Conventions common to every call
 * --------------------------------
 * Memory.  Every data pointer is DEVICE memory allocated and owned by the
 *   caller (hipMalloc or a framework tensor).  The library allocates nothing,
 *   frees nothing and keeps no state of its own between calls (no globals, no
 *   environment variables); what fd_decode_attn and its variants carry from one
 *   call to the next lives in the caller's workspace (see fd_workspace_init).
 *   Inputs are never written.
 * Layouts (all contiguous, row-major, IEEE binary16 unless noted):
 *   q        [batch, n_q_heads, head_dim]
 *   k_cache  [batch, n_kv_heads, max_seq, head_dim]
 *   v_cache  [batch, n_kv_heads, max_seq, head_dim]
 *   seq_lens [batch] int32 -- valid keys per sequence; values are clamped to
 *            [0, max_seq]; cache positions >= the valid length are padding:
 *            they may hold anything (NaN included) and never enter a result.
 *            They may still be LOADED, within the allocated [.., max_seq, ..]
 *            extent of the caches only (small launches request a chunk's first
 *            block before the length has arrived and discard what lies beyond
 *            it).  A sequence of length 0 produces a zero row and raises no flag.
 *   out      [batch, n_q_heads, head_dim]
 *   All pointers must be 16-byte aligned.
 *   Query head hq reads KV head hq / (n_q_heads / n_kv_heads).
 * Logit.  x_j = scale * <q, k_j> (fp32 accumulation); phi and the bounds apply
 *   to this scaled logit.  A "row" is one (sequence, query head) pair; chunk c
 *   of a row covers keys [c*chunk, min((c+1)*chunk, valid length)).
 * Stream.  `stream` is a hipStream_t passed as void* (NULL = the default
 *   stream).  All work is enqueued on it; no call synchronizes or reads device
 *   memory on the host.  Results are ready when the stream reaches that point.
 * Errors.  Every entry point returns an fd_status.  Problems visible on the host
 *   (null pointer, unsupported shape, bad bounds, workspace too small) are
 *   reported before anything is enqueued.  A failed launch returns FD_ERR_HIP.
 * Threads.  Calls are re-entrant as long as they use distinct workspaces.
 * Supported shapes.  head_dim == 128; chunk a multiple of 16 from 64 to 4096 keys (the
 *   kernels are built for the powers of two in that range and run a chunk on the smallest
 *   that holds it);
 *   n_q_heads a multiple of n_kv_heads; batch*n_q_heads*ceil(max_seq/chunk)
 *   < 2^31.
 */
#ifndef FDATTN_H
#define FDATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FD_OK = 0,
    FD_ERR_NULL = 1,         /* a required pointer is NULL                      */
    FD_ERR_SHAPE = 2,        /* non-positive size, heads not divisible, ...     */
    FD_ERR_BOUNDS = 3,       /* lo >= hi, or phi / a bound is NaN or infinite   */
    FD_ERR_WORKSPACE = 4,    /* workspace NULL, misaligned or too small         */
    FD_ERR_UNSUPPORTED = 5,  /* valid in principle, not built (head_dim, chunk) */
    FD_ERR_HIP = 6,          /* the HIP runtime refused a launch                */
    FD_ERR_STATIC_LIMIT = 7  /* fd_decode_attn_static: shape beyond its scratch */
} fd_status;

/* Problem shape.  Plain data, read during the call only. */
typedef struct {
    int32_t batch;
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t max_seq;   /* padded length of the cache's sequence axis           */
    int32_t chunk;     /* keys per partial vector                              */
    float   scale;     /* logit scale, e.g. 1/sqrt(head_dim)                   */
} fd_shape;

/* Bounds a, b on (logit - phi): in range means lo < x - phi < hi, strictly.
 * Equality with either bound, either side out of range, or a NaN logit flags. */
typedef struct { float lo, hi; } fd_bounds;

/* Caller-owned device scratch of at least fd_workspace_bytes(shape) bytes,
 * 256-byte aligned.  After a call it holds that call's partial results and
 * flags (see fd_get_flags, fd_get_partials).  fd_decode_attn and its variants
 * (_gqa, _append, _paged, _paged_append) need the workspace prepared once by
 * fd_workspace_init; the other calls accept arbitrary previous contents.
 * Layout: the data sections start at ptr and grow with the number of
 * (row, chunk) slots; the arrival counters of fd_workspace_init END at the last
 * 256-byte boundary inside [ptr, ptr + bytes).  Describe one allocation by the
 * same (ptr, bytes) pair in every call.                                       */
typedef struct { void *ptr; size_t bytes; } fd_workspace;

/* Bytes of workspace the calls below need for this shape; 0 if the shape is
 * invalid or unsupported.  Pure host function.                                */
size_t fd_workspace_bytes(const fd_shape *shape);

/* A chunk size (keys per partial vector, Section 3's split of the sequence axis)
 * suited to this shape on MI355X: a multiple of 16 from 64 to 2048 keys (to 4096 for
 * grouped heads), chosen so that the workgroups -- one per (row or head group, chunk)
 * -- cover the chip's 256 compute units in whole rounds; max_seq is cut into equal
 * chunks, so the value is a power of two only where max_seq divides that way.
 * shape->chunk is ignored.  0 if the rest of the shape is invalid or unsupported.
 * It sees max_seq, not the lengths: a caller whose cache is much longer than its
 * sequences gets a better value from a copy of the shape with max_seq set to the
 * longest current length (any chunk is valid with any max_seq; the workspace size
 * depends on both).  The paper leaves the split size open; any supported value gives
 * the same result up to rounding.  Pure host function.                          */
int32_t fd_pick_chunk(const fd_shape *shape);

/*
 * Prepare a workspace for fd_decode_attn and its variants: zeroes the arrival
 * counters (one int32 per (row, chunk) slot) by which the workgroups of those
 * calls elect the one that finishes a row.  It clears the counters of EVERY shape
 * that fits into ws.bytes, not just of `shape` (which only has to be valid and to
 * fit): enqueue it once after allocating the workspace; after that the shape --
 * batch, heads, max_seq, chunk -- may change from call to call, as it does for a
 * caller that passes the longest current length as max_seq or re-picks the chunk
 * every step, as long as each shape's fd_workspace_bytes fits and (ptr, bytes)
 * stay the same.  Every completed call leaves the counters zero again.
 * A call that did not complete (device reset, a launch that failed half-way
 * through a call, a kernel killed mid-flight) may leave counters non-zero: a
 * later call then elects nobody for the rows concerned, i.e. their `out` rows and
 * row flags are NOT written (nothing else goes wrong, and no error is reported).
 * After any such event enqueue fd_workspace_init again before reusing the
 * workspace.
 */
fd_status fd_workspace_init(const fd_shape *shape, fd_workspace ws, void *stream);

/*
 * Asynchronized-softmax decode attention, one row at a time (Section 3), in
 * one kernel launch (two for large grids, see step 3).  Per (row, chunk) workgroup:
 *   1. logits, range guard, sum e^{x-phi} and sum e^{x-phi} v with no maximum
 *      and no rescaling                               (Eq. 4, inner sums);
 *   2. if the guard fired for this chunk, its partial softmax is recomputed at
 *      once with the chunk's own maximum: (m, l, f.V)  (Eq. 2; "Recomputation");
 *   3. the workgroup that completes a row last -- elected by a small tree of
 *      integer arrival counters per row; the sums themselves use no atomics and
 *      run in fixed order -- forms the row: unflagged rows by the plain outer
 *      sums of Eq. 4, flagged rows by the synchronized update of Eq. 2 over all
 *      partial results, each rescaled from its own reference (phi, or the chunk
 *      maximum) to the row maximum of those references.  For grids of more than
 *      1024 workgroups, or of more than 256 workgroups over 320 MiB or more of cache
 *      (fd_decode_attn_gqa: more than 256 workgroups, or more than 8 chunks per row)
 *      step 3 runs as a second, tiny
 *      launch instead (one workgroup per row, no counters): large grids are
 *      throughput-bound and the election's two memory round trips per workgroup
 *      cost more than a launch.
 * A flagged row is thus produced by the synchronized scheme, but only the
 * partial vectors that left the bounds are re-read; the others already are
 * valid partial-softmax results relative to phi.  fd_decode_attn_multikernel
 * recomputes every chunk of a flagged row instead; both give the same result up
 * to fp32 rounding.  Works for any head grouping (each query head is a row).
 * Requires fd_workspace_init.  Fills chunk_flags and row_flags.
 * Which of the two launch forms runs depends on the shape alone (the numbers
 * above); no environment variable or other hidden switch takes part.
 */
fd_status fd_decode_attn(const fd_shape *shape, const void *q, const void *k_cache,
                         const void *v_cache, const int32_t *seq_lens, float phi,
                         fd_bounds bounds, void *out, fd_workspace ws, void *stream);

/*
 * Same result as fd_decode_attn for grouped-query attention: the
 * n_q_heads / n_kv_heads query heads that share one KV head are processed
 * together so each K and V element is read from memory once per group.
 * Requires 2 <= n_q_heads / n_kv_heads <= 16.  (Grouping is not in the paper;
 * per query head the arithmetic is Eq. 4 unchanged: the weights e^{x-phi} are formed
 * in fp32 and enter the second product on the matrix cores as fp16 hi + lo pairs, 22
 * significant bits, under a power-of-two scale per head that is taken out again
 * exactly; V is used as it is.  A (head, chunk) with a weight beyond the range of
 * that operand -- a logit more than 8 above the largest among the first keys of its
 * part of the chunk -- is recomputed like a flagged one, in fp32 throughout, without
 * raising a flag.)  Flags are per query head and report the guard alone.
 * Requires fd_workspace_init.
 */
fd_status fd_decode_attn_gqa(const fd_shape *shape, const void *q, const void *k_cache,
                             const void *v_cache, const int32_t *seq_lens, float phi,
                             fd_bounds bounds, void *out, fd_workspace ws, void *stream);

/*
 * One decode step with the cache update fused in (Section 2.2: the step's k and v
 * are concatenated to the cache before the attention of Eq. 1).  `k_new`, `v_new`
 * [batch, n_kv_heads, head_dim] fp16 are this step's rows.  For sequence b with
 * n = clamp(seq_lens[b], 0, max_seq) keys in the cache:
 *   n < max_seq : out = attention over the n cached keys AND the new one; the new
 *                 rows are written to k_cache / v_cache at position n.  The rows are
 *                 taken from k_new / v_new, not read back from the cache.
 *   n == max_seq: the cache is full; the new rows are dropped and out is the
 *                 attention over the cached keys alone.
 * seq_lens is not modified: the caller adds 1 to the lengths it passes to the next
 * step (and to fd_list_flagged_rows for this one).  Nothing else of the cache is
 * written.  Grouped shapes (2 <= n_q_heads / n_kv_heads <= 16) take the grouped
 * kernel, all others the per-row kernel; workspace, flags, recomputation, errors
 * and the fd_workspace_init requirement are those of fd_decode_attn.  The same
 * k_cache / v_cache must not be in use by another call in flight.
 */
fd_status fd_decode_attn_append(const fd_shape *shape, const void *q, const void *k_new, const void *v_new,
                                void *k_cache, void *v_cache, const int32_t *seq_lens, float phi,
                                fd_bounds bounds, void *out, fd_workspace ws, void *stream);

/*
 * fd_decode_attn / fd_decode_attn_gqa over a paged cache.  The paper keeps each
 * sequence's keys and values concatenated (Section 2.1) and does not say where in
 * memory; here they sit in fixed-size pages that need not be adjacent:
 *   k_pool, v_pool [n_pages, n_kv_heads, page_size, head_dim] fp16
 *   block_table    [batch, max_seq / page_size] int32 (device): token t of sequence b
 *                  is row t % page_size of page block_table[b][t / page_size].
 * shape->max_seq is the logical capacity per sequence, a multiple of page_size -- here only
 * the width of block_table, so a caller that rebuilds its table every step can (and should)
 * pass the longest current length rounded up to a page: the launch covers max_seq, and
 * chunks past a sequence's end cost a workgroup each (they leave at once, but a cache sized
 * for 32768 tokens holding 2000 would launch sixteen times the workgroups it needs);
 * page_size is a power of two >= 16 and a chunk touches at most 64 pages: chunk <=
 * 64 * page_size when one of chunk and page_size divides the other, else chunk +
 * page_size - 16 <= 64 * page_size (such a chunk may start inside a page); fd_pick_chunk
 * knows nothing of pages, so with small pages use the smaller of its value and
 * 64 * page_size.  Only the
 * entries of pages that hold a valid token (t < seq_lens[b]) are followed; the
 * others may hold anything (they are clamped into [0, n_pages) and what they bring
 * in is never used); an entry of a page in use that is out of range is the
 * caller's error and reads the wrong page.  Chunks, flags, recomputation,
 * workspace, the fd_workspace_init requirement and errors are those of
 * fd_decode_attn; chunk c covers tokens cC .. (c+1)C - 1 whatever pages hold them.
 * Grouped shapes (2 <= n_q_heads / n_kv_heads <= 16) take the grouped kernel.
 * FD_ERR_SHAPE for a page_size or n_pages outside the stated limits.
 */
fd_status fd_decode_attn_paged(const fd_shape *shape, const void *q, const void *k_pool, const void *v_pool,
                               const int32_t *block_table, int32_t page_size, int32_t n_pages,
                               const int32_t *seq_lens, float phi, fd_bounds bounds, void *out,
                               fd_workspace ws, void *stream);

/*
 * fd_decode_attn_append over a paged cache: the step's rows k_new, v_new
 * [batch, n_kv_heads, head_dim] are attended from their own buffers and written to
 * row n % page_size of page block_table[b][n / page_size], n = clamp(seq_lens[b], 0,
 * max_seq), by the same launch.  That entry of the table must name the page the
 * caller has set aside for the token (a fresh page when n is a multiple of
 * page_size); it is followed although the page holds no valid token yet.  A full
 * sequence (n == max_seq) drops the rows.  Everything else as fd_decode_attn_paged
 * and fd_decode_attn_append.
 */
fd_status fd_decode_attn_paged_append(const fd_shape *shape, const void *q, const void *k_new, const void *v_new,
                                      void *k_pool, void *v_pool, const int32_t *block_table, int32_t page_size,
                                      int32_t n_pages, const int32_t *seq_lens, float phi, fd_bounds bounds,
                                      void *out, fd_workspace ws, void *stream);

/*
 * fd_decode_attn / fd_decode_attn_gqa for callers that cannot allocate or carry a
 * workspace: code recorded by a stream capture that must not call hipMalloc, tight
 * serving loops, harnesses that forbid allocation.  Same arguments minus `ws`; same
 * kernels, same results bit for bit (grouped shapes, 2 <= n_q_heads / n_kv_heads <=
 * 16, take the grouped kernel, all others the per-row kernel).  The partial results,
 * flags and arrival counters live in a device array that is part of the library's
 * code object: FD_STATIC_SCRATCH_BYTES per GPU the library runs on, held until the
 * process ends.  The call allocates nothing and frees nothing (no hipMalloc, no
 * hipFree, no allocating runtime or library routine); the caller still owns q, the
 * caches, seq_lens and out.
 *   Limit.  fd_workspace_bytes(shape) <= FD_STATIC_SCRATCH_BYTES, else
 *     FD_ERR_STATIC_LIMIT before anything is enqueued (8 MiB hold about 14 000
 *     (row, chunk) slots: every workload shape of this repository at its picked
 *     chunk size; e.g. 32 rows x 8 chunks need 0.15 MiB, 128 rows x 32 chunks 2.3 MiB).
 *   Device.  The array of the CURRENT device is used (hipGetDevice at the call);
 *     `stream` must belong to it.  The first call on each device looks the array's
 *     address up and enqueues one clear of its arrival counters on `stream`; make that
 *     first call outside a stream capture.
 *   Sharing.  Every call on a GPU uses that GPU's one array, which keeps the last
 *     call's partial results and flags (nothing of them is an input of the next call;
 *     the arrival counters are zero between completed calls).  Calls that may overlap
 *     on one GPU -- different streams, different host threads -- RACE on it: use
 *     fd_decode_attn with distinct workspaces for those.  There is no fd_get_flags for
 *     the static array; callers that need flags use the workspace form.
 *   After a call that did not complete (see fd_workspace_init) the process has lost its
 *     device context anyway; there is nothing to re-initialise.
 * Other errors as fd_decode_attn; FD_ERR_HIP also when the array's address cannot be
 * obtained or the current device's ordinal is 64 or more.
 */
#define FD_STATIC_SCRATCH_BYTES (8u << 20)
fd_status fd_decode_attn_static(const fd_shape *shape, const void *q, const void *k_cache, const void *v_cache,
                                const int32_t *seq_lens, float phi, fd_bounds bounds, void *out, void *stream);

/*
 * The same method as a chain of three dependent launches with no atomics at all and no
 * hand-over inside a launch, following Section 3 to the letter:
 *   1. per (row, chunk): Eq. 4 inner sums and the range guard (partial sums, chunk flags);
 *   2. per (row, chunk) again, once all partial vectors of launch 1 exist: the row flag =
 *      OR of the row's chunk flags.  Unflagged rows: the workgroup of chunk 0 forms the
 *      Eq. 4 outer sums and the division (atomic-free: one workgroup owns one output row,
 *      fixed summation order).  Flagged rows: EVERY chunk of the row is recomputed by the
 *      synchronized partial softmax (m, l, f.V) -- the whole vector, as the paper says;
 *   3. flagged rows only: the synchronized update of Eq. 2 over the row's recomputed
 *      partial vectors, written to out; one more workgroup turns the row flags into the
 *      ascending list of flagged rows and their count.
 * Needs no fd_workspace_init.  A launch that depends on the previous one starts about 3 us
 * after it on an MI355X whatever its size, which is why fd_decode_attn fuses the three.
 * Fills chunk_flags, row_flags, n_flagged and flagged_rows.
 */
fd_status fd_decode_attn_multikernel(const fd_shape *shape, const void *q, const void *k_cache,
                                     const void *v_cache, const int32_t *seq_lens, float phi,
                                     fd_bounds bounds, void *out, fd_workspace ws, void *stream);

/*
 * The synchronized partial softmax (Eq. 2) applied to EVERY row: step 4 above
 * without steps 1-3.  This is the scheme the paper's method replaces; it is the
 * in-library baseline and the cross-check for the unified path.  No phi, no
 * bounds, no flags.
 */
fd_status fd_decode_attn_sync(const fd_shape *shape, const void *q, const void *k_cache,
                              const void *v_cache, const int32_t *seq_lens,
                              void *out, fd_workspace ws, void *stream);

/*
 * The chunk stage of fd_decode_attn alone (steps 1 and 2 of its description: Eq. 4
 * inner sums, the range guard, on-the-spot recomputation of flagged chunks): fills
 * the workspace's per-chunk numerators, denominators, references and chunk flags
 * and writes neither `out` nor the row flags.  For tests of the partial sums and
 * for timing the dominant kernel on its own.  fd_decode_attn_gqa_partial is the
 * same for the grouped kernel of fd_decode_attn_gqa.
 */
fd_status fd_decode_attn_partial(const fd_shape *shape, const void *q, const void *k_cache,
                                 const void *v_cache, const int32_t *seq_lens, float phi,
                                 fd_bounds bounds, fd_workspace ws, void *stream);
fd_status fd_decode_attn_gqa_partial(const fd_shape *shape, const void *q, const void *k_cache,
                                     const void *v_cache, const int32_t *seq_lens, float phi,
                                     fd_bounds bounds, fd_workspace ws, void *stream);

/*
 * Device pointers into `ws` to the flags of the last decode call that used it
 * (valid until the next call on `ws`):
 *   chunk_flags [batch*n_q_heads, ceil(max_seq/chunk)] uint8, 0 or 1
 *   row_flags   [batch*n_q_heads] uint8 = OR over the row's chunks
 *   n_flagged   [1] int32 = number of flagged rows
 *   flagged_rows[batch*n_q_heads] int32, the first *n_flagged entries are the
 *               flagged row indices in ascending order
 * Any output pointer may be NULL.  chunk_flags is filled by every decode call
 * that takes phi; row_flags by all of those except fd_decode_attn_partial;
 * n_flagged and flagged_rows by fd_decode_attn_multikernel and by
 * fd_list_flagged_rows only.
 */
fd_status fd_get_flags(const fd_shape *shape, fd_workspace ws,
                       const uint8_t **chunk_flags, const uint8_t **row_flags,
                       const int32_t **n_flagged, const int32_t **flagged_rows);

/*
 * Enqueue the flag reduction alone: chunk_flags -> row_flags, flagged_rows and
 * n_flagged (a single workgroup, prefix-sum compaction, no atomics).  For
 * callers that want the list of recomputed rows after fd_decode_attn /
 * fd_decode_attn_gqa, which do not need it themselves.
 */
fd_status fd_list_flagged_rows(const fd_shape *shape, const int32_t *seq_lens,
                               fd_workspace ws, void *stream);

/*
 * Device pointers into `ws` to the per-chunk partial results (D3 of Eq. 4):
 *   num [batch*n_q_heads, ceil(max_seq/chunk), head_dim] fp32 = sum e^{x-phi} v
 *   den [batch*n_q_heads, ceil(max_seq/chunk)]           fp32 = sum e^{x-phi}
 * Chunks without a valid key hold zeros.  Chunks that were recomputed hold the
 * synchronized scheme's (f.V, l) instead.
 */
fd_status fd_get_partials(const fd_shape *shape, fd_workspace ws,
                          const float **num, const float **den);

/*
 * Statistics of the softmax inputs (Section 3, the distribution of x_i that the
 * unified scaling factor is chosen from).  Enqueues a pass over q and k_cache that
 * ADDS, for every valid key j of every row, the scaled logit x = scale * <q, k_j> to
 * a histogram of `n_bins` (1..4096) bins of width `bin_width` starting at `x_min`:
 *   hist[0]            x <  x_min
 *   hist[1 + i]        x_min + i * bin_width <= x < x_min + (i + 1) * bin_width
 *   hist[n_bins + 1]   x >= x_min + n_bins * bin_width, or x is NaN
 * `hist` is device memory, n_bins + 2 uint64, 8-byte aligned, caller-owned; the
 * caller zeroes it once and may accumulate several calls (layers, prompts) in it.
 * `min_max` (device, 2 floats, may be NULL) receives min(min_max[0], smallest x)
 * and max(min_max[1], largest x), NaN excluded; initialise it to {+inf, -inf}.
 * shape->chunk is ignored; v_cache and a workspace are not needed.  Logits are
 * evaluated in fp32: one within rounding distance of a bin edge may be counted on
 * either side of it.  Errors as for fd_decode_attn, plus FD_ERR_BOUNDS for a
 * non-finite window or bin_width <= 0 and FD_ERR_UNSUPPORTED for n_bins.
 */
fd_status fd_logit_histogram(const fd_shape *shape, const void *q, const void *k_cache,
                             const int32_t *seq_lens, float x_min, float bin_width, int32_t n_bins,
                             uint64_t *hist, float *min_max, void *stream);

/* What fd_calibrate decides. */
typedef struct {
    int32_t   apply;     /* 1: use the unified factor with phi and bounds below;
                            0: the range is too wide for float32 (the paper's OPT-6.7B
                            case), the window cut off too much, or nothing was counted:
                            use fd_decode_attn_sync                                  */
    float     phi;       /* unified scaling factor                                   */
    fd_bounds bounds;    /* (x_lo - phi, x_hi - phi), for the guard on x - phi       */
    float     x_lo, x_hi;/* the chosen range of the logit itself                     */
    double    covered;   /* fraction of the counted logits inside [x_lo, x_hi) before
                            widening by margin                                       */
} fd_calibration;

/*
 * Choose phi and the bounds from a histogram that fd_logit_histogram filled
 * (Section 3: more than a fraction `coverage` -- the paper uses 99.99 % -- of the
 * x_i lie in a range (a, b); when e^{b-a} is representable in float32 the unified
 * factor is phi = a; when the range is too wide the technique is not applied).
 * Pure HOST function: `hist` is a host copy, n_bins + 2 values.
 *   range        the narrowest run of whole bins that leaves at most
 *                floor((1 - coverage) * total / 2) logits on either side (the two
 *                outlier slots count as outside), widened by `margin` >= 0 per side;
 *   phi          x_lo + phi_position * (x_hi - x_lo); phi_position = 0 is the
 *                paper's phi = a, 1 puts phi at the upper end;
 *   apply        e^{x_hi - x_lo} * max_seq * 65504 (the largest fp16 magnitude a V
 *                entry can have) <= FLT_MAX, i.e. no partial sum can overflow.
 * FD_ERR_NULL, FD_ERR_SHAPE (n_bins, max_seq < 1), FD_ERR_BOUNDS (window, coverage
 * outside (0, 1], margin < 0, phi_position outside [0, 1]).
 */
fd_status fd_calibrate(const uint64_t *hist, int32_t n_bins, float x_min, float bin_width,
                       double coverage, float margin, float phi_position, int32_t max_seq,
                       fd_calibration *out);

/*
 * Prompt (prefill) phase: the attention of Eq. 1 for every token of a prompt at
 * once, token i attending to tokens 0..i of its sequence, with the asynchronized
 * softmax of Section 3 (the paper applies it to both phases): weights against the
 * unified factor phi, partial sums over disjoint key sets added without a
 * maximum exchange, the range guard lo < x - phi < hi on every logit that takes
 * part, and on-the-spot recomputation with the synchronized scheme for a tile of
 * 128 queries in which the guard fired (flags are recorded per 64 queries).
 *   q, out   [batch, n_q_heads, max_seq, head_dim] fp16 (out is written)
 *   k_cache, v_cache [batch, n_kv_heads, max_seq, head_dim] fp16 (the prompt's keys)
 *   seq_lens [batch]: prompt length n_b = clamp(seq_lens[b], 0, max_seq); rows
 *            i >= n_b of out are set to zero, keys >= n_b are never used.
 * shape->chunk is ignored.  `ws`: device scratch of fd_prefill_workspace_bytes(shape)
 * bytes, 256-byte aligned, arbitrary previous contents (it receives a transposed
 * copy of V and one flag byte per (row head, 64-query tile)); no initialisation call
 * is needed.  Arithmetic: fp16 products with fp32 accumulation for the scores; fp32
 * exponentials and denominators; the weights enter the second product as fp16 hi + lo
 * pairs (22 significant bits) under a scale 2^k of the query's own, fixed after the
 * query's first 32 keys (it cancels in the division and is constant over the keys, so
 * partial sums still just add); V is used as it is.  A query whose later weights exceed
 * that scale's headroom (a logit more than 8.2 above the largest of its first 32) has
 * its 128-query tile redone with the synchronized scheme: same result, NO flag (the
 * flags report the guard alone).  Guard: as in decode a logit outside the bounds flags,
 * and so does a NaN logit; the comparison is made on log2 e^{x - phi} (plus k) against
 * the bounds times log2 e (plus k), so a logit within fp32 rounding of a bound may fall
 * on either side of it (decode compares x * scale - phi itself).
 * Errors as for fd_decode_attn; FD_ERR_UNSUPPORTED beyond 65535 heads, sequences
 * or batch * n_kv_heads.
 */
size_t    fd_prefill_workspace_bytes(const fd_shape *shape);
fd_status fd_prefill_attn(const fd_shape *shape, const void *q, const void *k_cache, const void *v_cache,
                          const int32_t *seq_lens, float phi, fd_bounds bounds, void *out,
                          fd_workspace ws, void *stream);
/* Device pointer into `ws`: tile_flags [batch, n_q_heads, ceil(max_seq / 64)], 1 where
 * the guard fired for a logit of those 64 queries (their 128-query tile was recomputed). */
fd_status fd_prefill_get_flags(const fd_shape *shape, fd_workspace ws, const uint8_t **tile_flags);

/* Static, human-readable name of a status code. */
const char *fd_status_str(fd_status status);

#ifdef __cplusplus
}
#endif
#endif /* FDATTN_H */
