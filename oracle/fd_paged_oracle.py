"""Plain numpy oracle for decode attention over a paged KV cache.

TEST INFRASTRUCTURE ONLY (like ``fd_oracle``): the checker for the library's
``fd_decode_attn_paged``.  It imports nothing from the GPU package.

What the paper fixes: the keys and values of the tokens generated so far are kept
and concatenated per sequence (Section 2.1, the KV cache); attention is Eq. 1 over
that sequence.  How the cache is laid out in memory is not the paper's subject.  A
paged cache stores it in fixed-size pages that need not be adjacent:

    pool   [n_pages, Hkv, page_size, D]   (K and V each)
    table  [B, pages_per_seq] int32       page of the pool that holds tokens
                                          j * page_size .. (j + 1) * page_size - 1 of sequence b

So the oracle is the definition written out: put every sequence's pages back in
order (``gather_pages``), then the exact attention / flag oracle of ``fd_oracle``
on the resulting contiguous cache.  Table entries of pages that hold no valid
token are never followed (they may be anything); those positions read as NaN.
"""
import numpy as np

from . import fd_oracle


def gather_pages(pool, table, page_size, seq_lens):
    """pool [n_pages, Hkv, P, D], table [B, T] -> contiguous [B, Hkv, T * P, D] (float16).

    Only pages that hold at least one valid token (position < seq_lens[b], clamped to
    T * P) are copied; every other position is NaN.
    """
    pool = np.asarray(pool)
    table = np.asarray(table)
    n_pages, Hkv, P, D = pool.shape
    assert P == page_size
    B, T = table.shape
    out = np.full((B, Hkv, T * P, D), np.float16(np.nan), dtype=np.float16)
    for b in range(B):
        n = int(min(max(int(seq_lens[b]), 0), T * P))
        for j in range((n + P - 1) // P):
            pid = int(table[b, j])
            assert 0 <= pid < n_pages, "table entry of a page in use is out of range"
            out[b, :, j * P:(j + 1) * P, :] = pool[pid]
    return out


def attn_exact(q, k_pool, v_pool, table, page_size, seq_lens, scale, nthreads=1):
    """Exact fp64 attention of each row over its sequence's tokens, [B, Hq, D]."""
    k = gather_pages(k_pool, table, page_size, seq_lens)
    v = gather_pages(v_pool, table, page_size, seq_lens)
    return fd_oracle.attn_exact(q, k, v, np.minimum(np.asarray(seq_lens), k.shape[2]).astype(np.int32), scale, nthreads=nthreads)


def flags(q, k_pool, table, page_size, seq_lens, scale, phi, lo, hi, chunk, nthreads=1):
    """Chunk flags, row flags and row margins of the range guard (chunks count logical positions)."""
    k = gather_pages(k_pool, table, page_size, seq_lens)
    return fd_oracle.flags(q, k, np.minimum(np.asarray(seq_lens), k.shape[2]).astype(np.int32), scale, phi, lo, hi, chunk,
                           nthreads=nthreads)
