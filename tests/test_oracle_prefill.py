"""Pins for the prefill oracle (``oracle/fd_prefill_oracle.c``): brute force with
every index written out, closed forms, the causal property, and the reduction of
one prompt row to the (separately pinned) decode oracle.  No expected value
comes from the prefill oracle itself or from the GPU path."""
import math

import numpy as np
import pytest

from oracle import fd_prefill_oracle as pf


def draw(B, Hq, Hkv, S, D, seed):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, Hq, S, D)).astype(np.float16)
    k = rng.standard_normal((B, Hkv, S, D)).astype(np.float16)
    v = rng.standard_normal((B, Hkv, S, D)).astype(np.float16)
    return q, k, v


def test_brute_force_tiny():
    B, Hq, Hkv, S, D = 2, 4, 2, 5, 3
    q, k, v = draw(B, Hq, Hkv, S, D, 1)
    sl = np.array([5, 3], dtype=np.int32)
    scale = 0.7
    s = float(np.float32(scale))
    rows = pf.all_rows(B, Hq, S)
    out, _, _ = pf.prefill_rows(q, k, v, sl, scale, rows)
    out = out.reshape(B, Hq, S, D)
    for b in range(B):
        for h in range(Hq):
            for i in range(S):
                if i >= sl[b]:
                    assert not out[b, h, i].any()
                    continue
                xs = [s * sum(float(q[b, h, i, t]) * float(k[b, h // 2, j, t]) for t in range(D)) for j in range(i + 1)]
                den = sum(math.exp(x) for x in xs)                      # Eq. 1 literally, no max subtraction
                for t in range(D):
                    want = sum(math.exp(xs[j]) * float(v[b, h // 2, j, t]) for j in range(i + 1)) / den
                    assert out[b, h, i, t] == pytest.approx(want, rel=1e-12, abs=1e-14)


def test_first_token_returns_its_own_value_row():
    q, k, v = draw(1, 2, 2, 7, 16, 2)
    out, _, _ = pf.prefill_rows(q, k, v, [7], 0.3, [[0, 0, 0], [0, 1, 0]])
    assert np.array_equal(out[0], v[0, 0, 0].astype(np.float64))
    assert np.array_equal(out[1], v[0, 1, 0].astype(np.float64))


def test_zero_queries_give_prefix_means_of_v():
    q, k, v = draw(1, 1, 1, 9, 8, 3)
    q[:] = 0
    out, _, _ = pf.prefill_rows(q, k, v, [9], 1.0, pf.all_rows(1, 1, 9))
    vd = v[0, 0].astype(np.float64)
    for i in range(9):
        np.testing.assert_allclose(out[i], vd[:i + 1].mean(axis=0), rtol=1e-13, atol=1e-15)


def test_future_tokens_do_not_matter():
    q, k, v = draw(1, 2, 1, 12, 8, 4)
    rows = pf.all_rows(1, 2, 12)
    base, _, _ = pf.prefill_rows(q, k, v, [12], 0.5, rows)
    k2, v2 = k.copy(), v.copy()
    k2[0, 0, 7:] = np.float16(np.nan)                                   # poison tokens 7..11
    v2[0, 0, 7:] = np.float16(np.inf)
    out, _, _ = pf.prefill_rows(q, k2, v2, [12], 0.5, rows)
    out, base = out.reshape(2, 12, 8), base.reshape(2, 12, 8)
    assert np.array_equal(out[:, :7], base[:, :7])                      # rows 0..6 never see them
    assert not np.isfinite(out[:, 7:]).all()


def test_each_row_is_decode_attention_over_its_prefix(oracle):
    # row i of a prompt = the decode step of Eq. 1 with query q_i over a cache of i + 1 keys
    B, Hq, Hkv, S, D = 2, 4, 2, 40, 32
    q, k, v = draw(B, Hq, Hkv, S, D, 5)
    sl = np.array([40, 23], dtype=np.int32)
    out, _, _ = pf.prefill_rows(q, k, v, sl, 0.2, pf.all_rows(B, Hq, S), nthreads=4)
    out = out.reshape(B, Hq, S, D)
    for i in (0, 1, 17, 22, 23, 39):
        lens = np.where(i < sl, i + 1, 0).astype(np.int32)
        want = oracle.attn_exact(np.ascontiguousarray(q[:, :, i, :]), k, v, lens, 0.2)
        np.testing.assert_allclose(out[:, :, i, :], want, rtol=1e-12, atol=1e-14)


def test_guard_is_strict_and_sees_only_causal_logits():
    # scale 1, q = e_0, k_j = x_j e_0: the logits of row i are x_0..x_i exactly
    D, x = 4, [1.0, 2.0, 5.0, 2.5, -4.0, 3.0]
    S = len(x)
    q = np.zeros((1, 1, S, D), dtype=np.float16)
    q[..., 0] = 1
    k = np.zeros((1, 1, S, D), dtype=np.float16)
    k[0, 0, :, 0] = x
    v = np.ones((1, 1, S, D), dtype=np.float16)
    # phi = 2, bounds (-3, 3): d = x - 2 = -1, 0, 3 (on the bound: flags), 0.5, -6 (flags), 1
    _, flag, margin = pf.prefill_rows(q, k, v, [S], 1.0, pf.all_rows(1, 1, S), phi=2.0, lo=-3.0, hi=3.0)
    assert flag.tolist() == [0, 0, 1, 1, 1, 1]                          # from token 2 on, every row sees x_2
    assert margin.tolist() == [2.0, 2.0, 0.0, 0.0, 0.0, 0.0]
    _, flag, _ = pf.prefill_rows(q, k, v, [2], 1.0, pf.all_rows(1, 1, S), phi=2.0, lo=-3.0, hi=3.0)
    assert flag.tolist() == [0, 0, 0, 0, 0, 0]                          # tokens beyond the prompt: no rows, no flags
