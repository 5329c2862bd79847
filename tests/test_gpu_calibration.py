"""fd_logit_histogram on the GPU against the calibration oracle, and the whole
calibration loop: histogram -> fd_calibrate -> fd_decode_attn with the chosen
phi and bounds.

The histogram is integer work, but the logit that decides the bin is fp32 on
the GPU and fp64 in the oracle: a logit within rounding distance of a bin edge
may land on either side.  What is unique is compared exactly (the total, and
every cumulative count up to the number of logits the oracle finds within
EDGE_EPS of that edge); EDGE_EPS is far above the fp32 error of a 128-term dot
product of N(0,1) values (about 1e-5) and far below the bin width."""
import numpy as np
import pytest
import torch

from oracle import fd_calibration_oracle as cal
from paper_2311_01282_amd import fdattn, synth

pytestmark = pytest.mark.gpu
EDGE_EPS = 2e-4


@pytest.fixture(scope="module")
def H():
    import fd_harness
    return fd_harness


def gpu_histogram(case, x_min, w, n_bins, calls=1):
    dev = torch.device("cuda:0")
    q = torch.from_numpy(case["q"]).to(dev)
    k = torch.from_numpy(case["k"]).to(dev)
    sl = torch.from_numpy(np.asarray(case["seq_lens"], dtype=np.int32)).to(dev)
    hist = torch.zeros(n_bins + 2, dtype=torch.int64, device=dev)
    mm = torch.tensor([float("inf"), float("-inf")], dtype=torch.float32, device=dev)
    shape = fdattn.make_shape(case["B"], case["Hq"], case["Hkv"], case["D"], case["Smax"], 0, case["scale"])
    stream = torch.cuda.current_stream(dev).cuda_stream
    for _ in range(calls):
        fdattn.fd_logit_histogram(shape, q.data_ptr(), k.data_ptr(), sl.data_ptr(), x_min, w, n_bins,
                                  hist.data_ptr(), mm.data_ptr(), stream)
    torch.cuda.synchronize()
    return hist.cpu().numpy(), mm.cpu().numpy()


def check_histogram(got, want, near):
    n_bins = want.size - 2
    assert got.sum() == want.sum()
    cum_got = got[0] + np.concatenate(([0], np.cumsum(got[1:n_bins + 1])))
    cum_want = want[0] + np.concatenate(([0], np.cumsum(want[1:n_bins + 1])))
    assert (np.abs(cum_got - cum_want) <= near).all(), "counts differ by more than the logits near an edge"


@pytest.mark.parametrize("B,Hq,Hkv,Smax,lens", [
    (1, 4, 4, 256, None),
    (2, 8, 8, 1000, [1000, 333]),
    (3, 8, 2, 777, [777, 1, 0]),           # grouped heads, a single key, an empty sequence
    (2, 12, 2, 600, [600, 411]),           # groups of 6 heads: a full block of 4 and a partial one
    (1, 32, 32, 4096, None),
    (8, 16, 16, 4700, None),               # 2432 (row, tile) items: more than the 2048 workgroups of the grid
])
def test_histogram_matches_oracle(B, Hq, Hkv, Smax, lens):
    case = synth.make_case(B=B, Hq=Hq, Hkv=Hkv, D=128, Smax=Smax, seq_lens=lens, seed=900 + Smax, poison_padding=True)
    x_min, w, n_bins = -6.0, 0.125, 96
    want, lo, hi, near = cal.logit_histogram(case["q"], case["k"], case["seq_lens"], case["scale"], x_min, w, n_bins,
                                             nthreads=8, edge_eps=EDGE_EPS)
    got, mm = gpu_histogram(case, x_min, w, n_bins)
    check_histogram(got, want, near)
    assert near.sum() < 0.01 * want.sum()                      # the tolerance is not what makes it pass
    assert mm[0] == pytest.approx(lo, abs=1e-4) and mm[1] == pytest.approx(hi, abs=1e-4)


def test_histogram_accumulates_and_keeps_outliers_apart():
    case = synth.make_case(B=1, Hq=4, Hkv=4, D=128, Smax=512, seed=31)
    # a narrow window: most logits fall into the two outlier slots
    want, _, _, near = cal.logit_histogram(case["q"], case["k"], case["seq_lens"], case["scale"], -0.5, 0.25, 4,
                                           edge_eps=EDGE_EPS)
    got, _ = gpu_histogram(case, -0.5, 0.25, 4, calls=3)
    assert got.sum() == 3 * want.sum() and got[0] > 0 and got[-1] > 0
    check_histogram(got, 3 * want, 3 * near)


def test_nan_logits_are_counted_in_the_last_slot():
    case = synth.make_case(B=1, Hq=2, Hkv=2, D=128, Smax=300, seed=32)
    case["k"][0, 1, 17, 5] = np.float16(np.nan)
    want, lo, hi, near = cal.logit_histogram(case["q"], case["k"], case["seq_lens"], case["scale"], -6.0, 0.5, 24,
                                             edge_eps=EDGE_EPS)
    got, mm = gpu_histogram(case, -6.0, 0.5, 24)
    check_histogram(got, want, near)
    assert got[-1] >= 1 and np.isfinite(mm).all()


def test_calibration_loop_end_to_end(oracle, H):
    # statistics of one layer -> phi and bounds -> decode with them: nothing flagged beyond the
    # allowance, and the output is the exact attention
    case = synth.make_config("c0_b1_h32_s1024")
    x_min, w, n_bins = -16.0, 0.125, 256
    hist, mm = gpu_histogram(case, x_min, w, n_bins)
    c = fdattn.fd_calibrate(hist.tolist(), n_bins, x_min, w, 0.9999, 4.0, 0.0, case["Smax"])
    want_c = cal.calibrate(cal.logit_histogram(case["q"], case["k"], case["seq_lens"], case["scale"], x_min, w, n_bins,
                                               nthreads=8)[0], x_min, w, 0.9999, 4.0, 0.0, case["Smax"])
    assert c.apply == 1 and want_c["apply"] == 1
    assert abs(c.phi - want_c["phi"]) <= w + 1e-6              # at most one bin apart (edge ties)
    assert c.x_lo <= mm[0] and mm[1] <= c.x_hi                 # margin 4 covers every logit seen
    dc = H.DeviceCase(case, chunk=256)
    got = dc.run("fd_decode_attn", phi=c.phi, bounds=(c.bounds.lo, c.bounds.hi))
    H.assert_close(got, oracle.attn_exact(case["q"], case["k"], case["v"], case["seq_lens"], case["scale"], nthreads=8),
                   "calibrated phi")
    assert dc.flags()[2] == 0


def test_histogram_rejects_bad_arguments():
    dev = torch.device("cuda:0")
    buf = torch.zeros(4096, dtype=torch.int64, device=dev)
    sh = fdattn.make_shape(1, 4, 4, 128, 256, 0, 0.1)
    p = buf.data_ptr()
    for args, code in (((sh, 0, p, p, 0.0, 1.0, 8, p), fdattn.FD_ERR_NULL),
                       ((sh, p, p, p, 0.0, 0.0, 8, p), fdattn.FD_ERR_BOUNDS),
                       ((sh, p, p, p, float("nan"), 1.0, 8, p), fdattn.FD_ERR_BOUNDS),
                       ((sh, p, p, p, 0.0, 1.0, 0, p), fdattn.FD_ERR_UNSUPPORTED),
                       ((sh, p, p, p, 0.0, 1.0, 5000, p), fdattn.FD_ERR_UNSUPPORTED),
                       ((fdattn.make_shape(1, 4, 3, 128, 256, 0, 0.1), p, p, p, 0.0, 1.0, 8, p), fdattn.FD_ERR_SHAPE)):
        with pytest.raises(fdattn.FdError) as e:
            fdattn.fd_logit_histogram(*args)
        assert e.value.status == code
