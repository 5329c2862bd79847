"""Pins of the paged-cache oracle (CPU only).  ``gather_pages`` is checked against an
index formula written out independently (token t of sequence b lives in row t % P of page
table[b][t // P]), against the contiguous oracle on the unpaged case, and through
invariances: where the pages sit in the pool, and what unused pages hold, cannot matter."""
import numpy as np
import pytest

from oracle import fd_oracle, fd_paged_oracle as po
from paper_2311_01282_amd import synth


def small_case(seed, B=3, Hq=4, Hkv=2, Smax=96, lens=(96, 37, 0)):
    return synth.make_case(B=B, Hq=Hq, Hkv=Hkv, D=128, Smax=Smax, seed=seed, seq_lens=list(lens))


@pytest.mark.parametrize("P", [4, 16, 32])
def test_gather_follows_the_table_token_by_token(P):
    case = small_case(11)
    k_pool, v_pool, table = synth.to_pages(case, P, seed=5)
    dense = po.gather_pages(k_pool, table, P, case["seq_lens"])
    for b in range(case["B"]):
        n = int(case["seq_lens"][b])
        for t in range(n):                               # the definition, one token at a time
            want = k_pool[table[b, t // P], :, t % P, :]
            assert np.array_equal(dense[b, :, t, :], want)
            assert np.array_equal(want, case["k"][b, :, t, :])
        # pages without a valid token are not followed: NaN there
        first_free = -(-n // P) * P
        assert np.isnan(dense[b, :, first_free:, :].astype(np.float32)).all()


def test_identity_table_is_the_contiguous_cache():
    case = small_case(12, B=2, lens=(64, 64), Smax=64)
    P = 16
    T = case["Smax"] // P
    # pool = the contiguous cache cut into pages in order
    k_pool = case["k"].reshape(2, 2, T, P, 128).transpose(0, 2, 1, 3, 4).reshape(2 * T, 2, P, 128).copy()
    table = np.arange(2 * T, dtype=np.int32).reshape(2, T)
    assert np.array_equal(po.gather_pages(k_pool, table, P, case["seq_lens"]), case["k"])


@pytest.mark.parametrize("P", [8, 32])
def test_paged_attention_equals_contiguous_attention(P):
    case = small_case(13)
    k_pool, v_pool, table = synth.to_pages(case, P, seed=6)
    got = po.attn_exact(case["q"], k_pool, v_pool, table, P, case["seq_lens"], case["scale"])
    want = fd_oracle.attn_exact(case["q"], case["k"], case["v"], case["seq_lens"], case["scale"])
    assert np.array_equal(got, want)
    assert not got[2].any()                              # empty sequence: zeros


def test_placement_in_the_pool_and_unused_pages_do_not_matter():
    case = small_case(14)
    P = 16
    a = synth.to_pages(case, P, seed=1, spare_pages=1)
    b = synth.to_pages(case, P, seed=2, spare_pages=9, poison_unused=False)
    assert not np.array_equal(a[2], b[2])                # different places
    ra = po.attn_exact(case["q"], a[0], a[1], a[2], P, case["seq_lens"], case["scale"])
    rb = po.attn_exact(case["q"], b[0], b[1], b[2], P, case["seq_lens"], case["scale"])
    assert np.array_equal(ra, rb)
    # entries of pages that hold no valid token may be anything
    t = b[2].copy()
    t[t < 0] = 12345
    assert np.array_equal(po.attn_exact(case["q"], b[0], b[1], t, P, case["seq_lens"], case["scale"]), rb)


def test_brute_force_one_row():
    # two pages of two tokens, stored in reverse order; the softmax written out by hand
    rng = np.random.default_rng(3)
    D, P = 128, 2
    q = rng.standard_normal((1, 1, D)).astype(np.float16)
    k_pool = rng.standard_normal((3, 1, P, D)).astype(np.float16)
    v_pool = rng.standard_normal((3, 1, P, D)).astype(np.float16)
    table = np.array([[2, 0]], dtype=np.int32)
    sl = np.array([3], dtype=np.int32)                   # tokens: (page 2, row 0), (page 2, row 1), (page 0, row 0)
    toks = [(2, 0), (2, 1), (0, 0)]
    scale = 0.125
    x = [scale * float(np.dot(q[0, 0].astype(np.float64), k_pool[p, 0, r].astype(np.float64))) for p, r in toks]
    w = np.exp(np.array(x) - max(x))
    want = sum(wi * v_pool[p, 0, r].astype(np.float64) for wi, (p, r) in zip(w, toks)) / w.sum()
    got = po.attn_exact(q, k_pool, v_pool, table, P, sl, scale)
    assert np.allclose(got[0, 0], want, rtol=1e-13, atol=1e-15)


def test_flags_count_logical_positions():
    case = small_case(15, B=1, Hq=2, Hkv=2, Smax=128, lens=(100,))
    case["k"][0, 1, 70] = (40.0 * case["q"][0, 1].astype(np.float64) / np.linalg.norm(case["q"][0, 1].astype(np.float64))).astype(np.float16)
    P = 16
    k_pool, v_pool, table = synth.to_pages(case, P, seed=8)
    cf, rf, margin = po.flags(case["q"], k_pool, table, P, case["seq_lens"], case["scale"], 3.0, -60.0, 20.0, 64)
    want = fd_oracle.flags(case["q"], case["k"], case["seq_lens"], case["scale"], 3.0, -60.0, 20.0, 64)
    assert np.array_equal(cf, want[0]) and np.array_equal(rf, want[1])
    assert cf[0, 1].tolist() == [0, 1] and cf[0, 0].sum() == 0      # token 70 sits in chunk 1, whatever page holds it


def test_lengths_beyond_the_capacity_are_clamped():
    # seq_lens above the table's capacity (and below zero) are clamped, as everywhere in the library
    case = small_case(16, B=2, Hq=2, Hkv=2, Smax=64, lens=(64, 64))
    P = 16
    k_pool, v_pool, table = synth.to_pages(case, P, seed=9)
    want = po.attn_exact(case["q"], k_pool, v_pool, table, P, np.array([64, 64]), case["scale"])
    got = po.attn_exact(case["q"], k_pool, v_pool, table, P, np.array([1000, 64]), case["scale"])
    assert np.array_equal(got, want)
    neg = po.attn_exact(case["q"], k_pool, v_pool, table, P, np.array([-5, 64]), case["scale"])
    assert not neg[0].any() and np.array_equal(neg[1], want[1])
