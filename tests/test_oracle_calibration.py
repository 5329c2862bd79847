"""Pins for the calibration oracle (``oracle/fd_calibration_oracle.py``): the
range the paper prints for Llama2-7B, closed-form quantiles, brute force on tiny
inputs and a distribution whose law is known.  No expected value below comes
from the oracle itself or from the GPU path."""
import math
import os

import numpy as np
import pytest

from oracle import fd_calibration_oracle as cal

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                key, val = line.split("=")
                out[key.strip()] = float(val)
    return out


@pytest.fixture(autouse=True)
def _built(oracle):
    return oracle


def keys_for_logits(x, D=8):
    """q = e_0, K[j] = x_j e_0 with scale 1: the logits are exactly x (fp16-representable x)."""
    x = np.asarray(x, dtype=np.float16)
    q = np.zeros((1, 1, D), dtype=np.float16)
    q[0, 0, 0] = 1
    k = np.zeros((1, 1, x.size, D), dtype=np.float16)
    k[0, 0, :, 0] = x
    return q, k, np.array([x.size], dtype=np.int32)


def test_histogram_of_hand_placed_logits():
    # window [-2, 2) in 4 bins of width 1; edges belong to the bin above them
    x = [-3.0, -2.0, -1.5, -1.0, 0.0, 0.5, 1.0, 1.999, 2.0, 7.0, -2.0005]
    q, k, sl = keys_for_logits(x)
    hist, lo, hi, _ = cal.logit_histogram(q, k, sl, 1.0, -2.0, 1.0, 4)
    # slots: below | [-2,-1) | [-1,0) | [0,1) | [1,2) | at-or-above
    # fp16 rounds 1.999 to 1.9990234 (inside [1,2)) and -2.0005 to -2.0 (spacing there is 2^-9; edge -> first bin)
    assert hist.tolist() == [1, 3, 1, 2, 2, 2]
    assert lo == -3.0 and hi == 7.0


def test_histogram_counts_only_valid_keys_and_every_row():
    rng = np.random.default_rng(5)
    B, Hq, Hkv, S, D = 3, 4, 2, 50, 16
    q = rng.standard_normal((B, Hq, D)).astype(np.float16)
    k = rng.standard_normal((B, Hkv, S, D)).astype(np.float16)
    k[1, :, 20:] = np.nan                                   # padding of sequence 1: never read
    sl = np.array([50, 20, 0], dtype=np.int32)
    hist, lo, hi, _ = cal.logit_histogram(q, k, sl, 0.25, -8.0, 0.5, 32)
    assert hist.sum() == Hq * (50 + 20 + 0)
    assert hist[-1] == 0 and math.isfinite(lo) and math.isfinite(hi)
    # brute force, every index written out
    want = np.zeros(34, dtype=np.int64)
    for b in range(B):
        for h in range(Hq):
            for j in range(int(sl[b])):
                x = 0.25 * sum(float(q[b, h, t]) * float(k[b, h // 2, j, t]) for t in range(D))
                i = math.floor((x + 8.0) / 0.5)
                want[0 if i < 0 else (33 if i >= 32 else i + 1)] += 1
    assert hist.tolist() == want.tolist()


def test_histogram_nan_logits_land_in_the_last_slot():
    q, k, sl = keys_for_logits([0.0, 1.0, 2.0])
    k[0, 0, 1, 0] = np.nan
    hist, lo, hi, _ = cal.logit_histogram(q, k, sl, 1.0, -4.0, 1.0, 8)
    assert hist[-1] == 1 and hist.sum() == 3 and lo == 0.0 and hi == 2.0


def test_histogram_follows_the_normal_law():
    # fixed q, K ~ N(0, 1): x_j = s <q, k_j> ~ N(0, s^2 |q|^2) up to fp16 rounding of K
    rng = np.random.default_rng(11)
    D, S = 128, 200000
    q = rng.standard_normal((1, 1, D)).astype(np.float16)
    k = rng.standard_normal((1, 1, S, D)).astype(np.float16)
    s = 1.0 / math.sqrt(D)
    sigma = s * float(np.linalg.norm(q.astype(np.float64)))
    hist, _, _, _ = cal.logit_histogram(q, k, np.array([S], dtype=np.int32), s, -4.0, 0.25, 32, nthreads=8)
    edges = -4.0 + 0.25 * np.arange(33)
    cdf = np.array([0.5 * (1 + math.erf(e / (sigma * math.sqrt(2)))) for e in edges])
    emp = (hist[0] + np.concatenate(([0], np.cumsum(hist[1:33])))) / S
    # Dvoretzky-Kiefer-Wolfowitz: P(sup |F_n - F| > eps) <= 2 exp(-2 n eps^2); eps for 1e-9
    eps = math.sqrt(math.log(2 / 1e-9) / (2 * S))
    assert np.abs(emp - cdf).max() < eps + 2e-3             # 2e-3: fp16 rounding of the keys


def test_near_edge_counts():
    x = [0.0, 0.001, 0.999, 1.0, 1.5]
    q, k, sl = keys_for_logits(x)
    _, _, _, near = cal.logit_histogram(q, k, sl, 1.0, 0.0, 1.0, 2, edge_eps=0.01)
    # edges 0, 1, 2; fp16(0.001) = 0.0010004, fp16(0.999) = 0.99902
    assert near.tolist() == [2, 2, 0]


def test_llama2_range_from_the_paper():
    g = read_golden("sec3_llama2_range.txt")
    # a histogram with bin edges at multiples of 0.1 whose mass outside (a, b) is below 0.01 %
    x_min, w, n = -40.0, 0.1, 800
    hist = np.zeros(n + 2, dtype=np.int64)
    centre = np.arange(n) * w + x_min + w / 2
    inside = (centre > g["a"]) & (centre < g["b"])
    hist[1:n + 1][inside] = 1000000
    hist[1:n + 1][~inside] = 1                       # 567 of 233 000 567 logits outside: 2.4e-6
    r = cal.calibrate(hist, x_min, w, g["coverage"], 0.0, 0.0, 4096)
    assert r["apply"] == int(g["apply"])
    assert r["x_lo"] == pytest.approx(g["a"], abs=1e-4) and r["x_hi"] == pytest.approx(g["b"], abs=1e-4)
    assert r["phi"] == pytest.approx(g["phi"], abs=1e-4)          # phi = a
    assert r["lo"] == pytest.approx(0.0, abs=1e-9) and r["hi"] == pytest.approx(g["b"] - g["a"], abs=1e-4)
    assert r["covered"] >= g["coverage"]


def test_uniform_histogram_has_closed_form_quantiles():
    # 1000 bins of 1000 logits on [0, 100): coverage 0.98 leaves 1 % = 10 bins per side
    hist = np.zeros(1002, dtype=np.int64)
    hist[1:1001] = 1000
    r = cal.calibrate(hist, 0.0, 0.1, 0.98, 0.5, 0.25, 1024)
    assert r["x_lo"] == pytest.approx(1.0 - 0.5) and r["x_hi"] == pytest.approx(99.0 + 0.5)
    assert r["covered"] == pytest.approx(0.98)
    rng = 99.5 - 0.5
    assert r["phi"] == pytest.approx(0.5 + 0.25 * rng)
    assert r["lo"] == pytest.approx(-0.25 * rng) and r["hi"] == pytest.approx(0.75 * rng)
    # e^{99} overflows float32 by itself: not applicable
    assert r["apply"] == 0


def test_apply_threshold_is_the_float32_range():
    # range R is applicable iff e^R * max_seq * 65504 <= FLT_MAX
    for max_seq in (1, 1024, 32768):
        limit = math.log(3.4028234663852886e38) - math.log(max_seq) - math.log(65504.0)
        for R_bins, want in ((int(limit) - 1, 1), (int(limit) + 2, 0)):
            hist = np.zeros(202, dtype=np.int64)
            hist[1:R_bins + 1] = 5
            r = cal.calibrate(hist, 0.0, 1.0, 1.0, 0.0, 0.0, max_seq)
            assert (r["x_lo"], r["x_hi"]) == (0.0, float(R_bins))
            assert r["apply"] == want, (max_seq, R_bins)


def test_window_too_narrow_or_empty_means_do_not_apply():
    hist = np.zeros(12, dtype=np.int64)
    assert cal.calibrate(hist, 0.0, 1.0, 0.9999, 0.0, 0.0, 128)["apply"] == 0
    hist[1:11] = 100
    hist[11] = 50                                    # 4.8 % of the logits beyond the window
    assert cal.calibrate(hist, 0.0, 1.0, 0.9999, 0.0, 0.0, 128)["apply"] == 0
    assert cal.calibrate(hist, 0.0, 1.0, 0.90, 0.0, 0.0, 128)["apply"] == 1


def test_calibrated_guard_flags_no_more_than_the_allowed_fraction(oracle):
    from paper_2311_01282_amd import synth
    case = synth.make_case(B=2, Hq=4, Hkv=4, D=128, Smax=3000, seq_lens=[3000, 1777], seed=77)
    hist, _, _, _ = cal.logit_histogram(case["q"], case["k"], case["seq_lens"], case["scale"], -16.0, 0.125, 256, nthreads=4)
    r = cal.calibrate(hist, -16.0, 0.125, 0.99, 0.0, 0.0, 3000)
    assert r["apply"] == 1
    _, x = oracle.attn_exact(case["q"], case["k"], case["v"], case["seq_lens"], case["scale"], nthreads=4, return_logits=True)
    xs = np.concatenate([x[0, :, :3000].ravel(), x[1, :, :1777].ravel()])
    d = xs - r["phi"]
    outside = int(((d <= r["lo"]) | (d >= r["hi"])).sum())
    assert outside <= 0.01 * xs.size + 2             # at most (1 - coverage) of the logits, up to edge ties
    assert outside >= 0.01 * xs.size - 2 * hist.max()  # and the interval is the narrowest run of whole bins
