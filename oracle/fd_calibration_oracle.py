"""Plain numpy oracle for the offline choice of the unified scaling factor.

TEST INFRASTRUCTURE ONLY (like ``fd_oracle``): the checker for the library's
logit histogram kernel and its host-side calibration rule.  It imports nothing
from the GPU package.

What the paper fixes (Section 3, the paragraph on the statistical distribution
of the softmax inputs x_i): more than 99.99 % of the x_i of a model fall in a
range (a, b); when e^{b-a} and e^{a-b} are representable in float32 the unified
factor can be set to phi = a; when the range is too wide (the OPT-6.7B case) the
technique is not applied.  The guard of "Recomputation" is then a < x - phi < b
on the shifted logit.  Everything else is this build's reading, listed where
the library documents ``fd_calibrate``:

* ``logit_histogram`` -- the definition: every valid scaled logit
  x = s <q, k_j> of every row, counted into fixed-width bins
  [x_min + i w, x_min + (i+1) w), i < n_bins; slot 0 counts x below the window,
  slot n_bins + 1 counts x at or above its end and NaN.  Logits come from
  ``fd_oracle.attn_exact`` (fp64, exactly widened fp16 inputs).
* ``calibrate``       -- from such a histogram: the narrowest run of whole bins
  that leaves at most (1 - coverage) / 2 of the mass on either side, widened by
  ``margin``; phi = x_lo + phi_position (x_hi - x_lo) (phi_position = 0 is the
  paper's phi = a); bounds (x_lo - phi, x_hi - phi) on x - phi; ``apply`` says
  whether the widest exponent, times the longest sequence, times the largest
  fp16 magnitude of V, still fits float32.
"""
import math

import numpy as np

from . import fd_oracle

FLT_MAX = 3.4028234663852886e38
HALF_MAX = 65504.0


def logit_histogram(q, k, seq_lens, scale, x_min, bin_width, n_bins, nthreads=1, edge_eps=0.0):
    """Returns (hist [n_bins + 2] int64, x_lo, x_hi, near [n_bins + 1] int64).

    ``near[e]`` counts the logits within ``edge_eps`` of edge e (x_min + e w): the only
    logits an fp32 evaluation may legitimately put on the other side of that edge.
    x_lo / x_hi are the smallest / largest valid logit (+inf / -inf when there is none).
    """
    k = np.asarray(k)
    _, x = fd_oracle.attn_exact(q, k, k, seq_lens, scale, nthreads=nthreads, return_logits=True)
    B, Hq, Smax = x.shape
    sl = np.clip(np.asarray(seq_lens, dtype=np.int64), 0, Smax)
    valid = np.arange(Smax)[None, None, :] < sl[:, None, None]
    xs = x[np.broadcast_to(valid, x.shape)]
    hist = np.zeros(n_bins + 2, dtype=np.int64)
    x_min = float(np.float32(x_min))
    w = float(np.float32(bin_width))
    nan = np.isnan(xs)
    t = np.floor((xs[~nan] - x_min) / w)
    idx = np.where(t < 0, 0, np.where(t >= n_bins, n_bins + 1, t + 1)).astype(np.int64)
    np.add.at(hist, idx, 1)
    hist[n_bins + 1] += int(nan.sum())
    edges = x_min + w * np.arange(n_bins + 1)
    near = np.zeros(n_bins + 1, dtype=np.int64)
    if edge_eps > 0 and xs.size:
        fin = np.sort(xs[~nan])
        near = (np.searchsorted(fin, edges + edge_eps, side="right") -
                np.searchsorted(fin, edges - edge_eps, side="left")).astype(np.int64)
    lo = float(xs[~nan].min()) if (~nan).any() else math.inf
    hi = float(xs[~nan].max()) if (~nan).any() else -math.inf
    return hist, lo, hi, near


def calibrate(hist, x_min, bin_width, coverage, margin, phi_position, max_seq):
    """Returns a dict: apply, phi, lo, hi (bounds on x - phi), x_lo, x_hi, covered."""
    hist = np.asarray(hist, dtype=np.int64)
    n_bins = hist.size - 2
    x_min = float(np.float32(x_min))
    w = float(np.float32(bin_width))
    total = int(hist.sum())
    res = {"apply": 0, "phi": 0.0, "lo": 0.0, "hi": 0.0, "x_lo": 0.0, "x_hi": 0.0, "covered": 0.0}
    if total == 0:
        return res
    tail = int(math.floor((1.0 - coverage) * total / 2.0))     # logits allowed outside, per side
    # below[e] = logits under edge e, above[e] = logits at or over edge e, e = 0 .. n_bins
    below = hist[0] + np.concatenate(([0], np.cumsum(hist[1:n_bins + 1])))
    above = total - below
    ok_lo = np.flatnonzero(below <= tail)
    ok_hi = np.flatnonzero(above <= tail)
    if ok_lo.size == 0 or ok_hi.size == 0:
        return res                                             # the window itself cuts off too much
    e_lo, e_hi = int(ok_lo.max()), int(ok_hi.min())
    if e_hi <= e_lo:                                           # degenerate: everything in the tails' slack
        e_hi = min(e_lo + 1, n_bins)
        e_lo = e_hi - 1
    x_lo = x_min + e_lo * w - margin
    x_hi = x_min + e_hi * w + margin
    rng = x_hi - x_lo
    limit = math.log(FLT_MAX) - math.log(max(int(max_seq), 1)) - math.log(HALF_MAX)
    phi = x_lo + phi_position * rng
    res.update(apply=int(rng <= limit), phi=phi, lo=x_lo - phi, hi=x_hi - phi, x_lo=x_lo, x_hi=x_hi,
               covered=float(below[e_hi] - below[e_lo]) / total)
    return res
