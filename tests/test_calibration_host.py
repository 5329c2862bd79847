"""fd_calibrate (a pure host function of the C-ABI library) against the numpy
calibration oracle on seeded random histograms and on the paper's Llama2-7B
range.  No GPU needed."""
import math
import os

import numpy as np
import pytest

from oracle import fd_calibration_oracle as cal

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def fdattn():
    lib = os.path.join(ROOT, "paper_2311_01282_amd", "libfdattn.so")
    if not os.path.exists(lib):          # build only if nothing is built
        from paper_2311_01282_amd import build
        build.build()
    from paper_2311_01282_amd import fdattn as mod
    return mod


def same(got, want):
    assert got.apply == want["apply"]
    if not want["apply"] and want["x_hi"] == want["x_lo"] == 0.0:
        return
    for a, b in ((got.phi, want["phi"]), (got.bounds.lo, want["lo"]), (got.bounds.hi, want["hi"]),
                 (got.x_lo, want["x_lo"]), (got.x_hi, want["x_hi"])):
        assert a == pytest.approx(b, rel=1e-6, abs=1e-5)
    assert got.covered == pytest.approx(want["covered"], abs=1e-12)


def test_random_histograms(fdattn):
    rng = np.random.default_rng(2024)
    for trial in range(300):
        n = int(rng.integers(1, 400))
        kind = trial % 4
        if kind == 0:      # bell-shaped
            centre, width = rng.uniform(0, n), rng.uniform(0.5, n / 3 + 1)
            hist = (1e6 * np.exp(-0.5 * ((np.arange(n + 2) - centre) / width) ** 2)).astype(np.int64)
        elif kind == 1:    # sparse
            hist = rng.integers(0, 3, n + 2) * rng.integers(0, 2, n + 2)
        elif kind == 2:    # heavy outlier slots
            hist = rng.integers(0, 1000, n + 2)
            hist[0] = rng.integers(0, 20000)
            hist[-1] = rng.integers(0, 20000)
        else:              # flat
            hist = np.full(n + 2, int(rng.integers(1, 50)))
        x_min = float(np.float32(rng.uniform(-50, 10)))
        w = float(np.float32(rng.choice([0.0625, 0.125, 0.25, 0.5, 1.0])))
        coverage = float(rng.choice([0.5, 0.9, 0.99, 0.9999, 1.0]))
        margin = float(np.float32(rng.choice([0.0, 0.5, 2.0])))
        pos = float(np.float32(rng.choice([0.0, 0.25, 1.0])))
        max_seq = int(rng.choice([1, 1024, 32768]))
        want = cal.calibrate(hist, x_min, w, coverage, margin, pos, max_seq)
        got = fdattn.fd_calibrate(hist.tolist(), n, x_min, w, coverage, margin, pos, max_seq)
        same(got, want)


def test_llama2_range_from_the_paper(fdattn):
    # Section 3: -16.8 < x_i < 6.5 for more than 99.99 % of the x_i; phi = a; applied
    x_min, w, n = -40.0, 0.1, 800
    hist = np.ones(n + 2, dtype=np.int64)
    centre = np.arange(n) * w + x_min + w / 2
    hist[1:n + 1][(centre > -16.8) & (centre < 6.5)] = 1000000
    got = fdattn.fd_calibrate(hist.tolist(), n, x_min, w, 0.9999, 0.0, 0.0, 4096)
    assert got.apply == 1
    assert got.phi == pytest.approx(-16.8, abs=1e-4) and got.x_hi == pytest.approx(6.5, abs=1e-4)
    assert got.bounds.lo == pytest.approx(0.0, abs=1e-6) and got.bounds.hi == pytest.approx(23.3, abs=1e-4)


def test_bad_arguments(fdattn):
    h = [0, 5, 5, 0]
    for args in ((0, 0.0, 1.0, 0.99, 0.0, 0.0, 128),            # n_bins
                 (2, 0.0, 1.0, 0.99, 0.0, 0.0, 0),              # max_seq
                 (2, 0.0, 0.0, 0.99, 0.0, 0.0, 128),            # bin_width
                 (2, math.nan, 1.0, 0.99, 0.0, 0.0, 128),       # window
                 (2, 0.0, 1.0, 0.0, 0.0, 0.0, 128),             # coverage
                 (2, 0.0, 1.0, 1.5, 0.0, 0.0, 128),
                 (2, 0.0, 1.0, 0.99, -1.0, 0.0, 128),           # margin
                 (2, 0.0, 1.0, 0.99, 0.0, 2.0, 128)):           # phi_position
        with pytest.raises(fdattn.FdError):
            fdattn.fd_calibrate(h if args[0] else [0, 0], max(args[0], 0), *args[1:])
    # an empty histogram is not an error: nothing to apply
    assert fdattn.fd_calibrate([0, 0, 0, 0], 2, 0.0, 1.0, 0.99, 0.0, 0.0, 128).apply == 0
