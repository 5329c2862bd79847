"""fd_prefill_attn on the GPU against the prefill oracle: causal attention of all
prompt tokens, the tile flags of the range guard, recomputation of flagged tiles.
Small cases check every output row; larger ones a seeded sample of rows (the
fp64 oracle costs O(S^2 D) per head) plus every row of the first and the last
tile."""
import numpy as np
import pytest
import torch

from oracle import fd_prefill_oracle as pf
from paper_2311_01282_amd import fdattn, synth

pytestmark = pytest.mark.gpu
LO, HI = synth.BOUNDS


@pytest.fixture(scope="module")
def H():
    import fd_harness
    return fd_harness


def close(H, got, want, what):
    """The decode tolerance: 2e-3 absolute, 1e-2 relative against max(|oracle|, 1e-3)."""
    return H.assert_close(got, want, what)


def draw(B, Hq, Hkv, Smax, lens, seed, poison=True):
    rng = np.random.default_rng(seed)
    D = 128
    q = rng.standard_normal((B, Hq, Smax, D)).astype(np.float16)
    k = rng.standard_normal((B, Hkv, Smax, D)).astype(np.float16)
    v = rng.standard_normal((B, Hkv, Smax, D)).astype(np.float16)
    sl = np.asarray(lens if lens is not None else [Smax] * B, dtype=np.int32)
    if poison:                                   # keys and queries beyond the prompt hold NaN
        for b in range(B):
            k[b, :, sl[b]:] = np.float16(np.nan)
            v[b, :, sl[b]:] = np.float16(np.nan)
            q[b, :, sl[b]:] = np.float16(np.nan)
    return q, k, v, sl


def run_gpu(q, k, v, sl, scale, phi=synth.PHI, bounds=synth.BOUNDS):
    dev = torch.device("cuda:0")
    B, Hq, Smax, D = q.shape
    Hkv = k.shape[1]
    tq, tk, tv = (torch.from_numpy(a).to(dev) for a in (q, k, v))
    tsl = torch.from_numpy(sl).to(dev)
    out = torch.full((B, Hq, Smax, D), float("nan"), dtype=torch.float16, device=dev)
    shape = fdattn.make_shape(B, Hq, Hkv, D, Smax, 0, scale)
    nws = fdattn.fd_prefill_workspace_bytes(shape)
    assert nws > 0
    ws = torch.full((nws,), 0xA5, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    fdattn.fd_prefill_attn(shape, tq.data_ptr(), tk.data_ptr(), tv.data_ptr(), tsl.data_ptr(), phi, bounds,
                           out.data_ptr(), ws.data_ptr(), nws, stream)
    torch.cuda.synchronize()
    tiles = -(-Smax // 64)
    addr = fdattn.fd_prefill_get_flags(shape, ws.data_ptr(), nws)
    off = addr - ws.data_ptr()
    flags = ws[off:off + B * Hq * tiles].cpu().numpy().reshape(B, Hq, tiles)
    return out.cpu().numpy().astype(np.float64), flags


def tile_flags_from_rows(rows, flag, B, Hq, Smax):
    tiles = -(-Smax // 64)
    tf = np.zeros((B, Hq, tiles), dtype=np.uint8)
    for (b, h, i), f in zip(rows, flag):
        if f:
            tf[b, h, i // 64] = 1
    return tf


@pytest.mark.parametrize("B,Hq,Hkv,Smax,lens", [
    (1, 1, 1, 64, None),                     # one tile
    (1, 2, 2, 200, [200]),                   # ragged maximum length, diagonal tiles
    (2, 4, 4, 320, [320, 77]),               # a short prompt in a long buffer
    (3, 4, 2, 256, [256, 1, 0]),             # shared KV heads; one token; empty prompt
    (1, 8, 1, 130, [129]),
])
def test_every_row_matches_oracle(H, B, Hq, Hkv, Smax, lens):
    q, k, v, sl = draw(B, Hq, Hkv, Smax, lens, seed=7000 + Smax)
    scale = float(np.float32(1.0 / np.sqrt(128.0)))
    rows = pf.all_rows(B, Hq, Smax)
    want, flag, margin = pf.prefill_rows(q, k, v, sl, scale, rows, phi=synth.PHI, lo=LO, hi=HI, nthreads=8)
    assert margin.min() > 1e-2 and not flag.any()
    got, tf = run_gpu(q, k, v, sl, scale)
    close(H, got.reshape(-1, 128), want, "prefill %s" % ((B, Hq, Hkv, Smax),))
    assert not tf.any()
    for b in range(B):                       # rows beyond the prompt are zero
        assert not got[b, :, sl[b]:].any()


def test_long_prompt_sampled_rows(H):
    B, Hq, Hkv, Smax = 2, 8, 8, 2048
    q, k, v, sl = draw(B, Hq, Hkv, Smax, [2048, 1500], seed=7100)
    scale = float(np.float32(1.0 / np.sqrt(128.0)))
    rng = np.random.default_rng(1)
    rows = [(b, h, i) for b in range(B) for h in range(Hq) for i in list(range(64)) + list(range(sl[b] - 64, sl[b]))]
    rows += [(int(rng.integers(B)), int(rng.integers(Hq)), int(rng.integers(1500))) for _ in range(600)]
    rows = np.asarray(rows, dtype=np.int32)
    want, flag, margin = pf.prefill_rows(q, k, v, sl, scale, rows, phi=synth.PHI, lo=LO, hi=HI, nthreads=16)
    assert margin.min() > 1e-2 and not flag.any()
    got, tf = run_gpu(q, k, v, sl, scale)
    close(H, got[rows[:, 0], rows[:, 1], rows[:, 2]], want, "prefill 2048")
    assert not tf.any() and np.isfinite(got).all()
    assert not got[1, :, 1500:].any()


def test_flagged_tiles_are_recomputed(H):
    # one key is made to overflow for one query head: every later token of that head sees it, so
    # all tiles from its position on are flagged and recomputed; earlier tiles and other heads are not
    B, Hq, Hkv, Smax = 1, 4, 4, 320
    q, k, v, sl = draw(B, Hq, Hkv, Smax, [300], seed=7200)
    scale = float(np.float32(1.0 / np.sqrt(128.0)))
    pos = 150
    # aim the key at the queries of head 2 from token 150 on: k = 36 * mean direction is not enough in
    # general, so give those queries a common component along a fixed unit vector u and put k = gamma u
    u = np.zeros(128)
    u[5] = 1.0
    q[0, 2, pos:300, 5] = np.float16(12.0)             # <q, u> = 12
    k[0, 2, pos] = (36.0 * u).astype(np.float16)       # logit = 12 * 36 / sqrt(128) = 38.2 > phi + 20
    rows = pf.all_rows(B, Hq, Smax)
    want, flag, margin = pf.prefill_rows(q, k, v, sl, scale, rows, phi=synth.PHI, lo=LO, hi=HI, nthreads=8)
    assert margin.min() > 1e-2
    want_tf = tile_flags_from_rows(rows, flag, B, Hq, Smax)
    assert want_tf[0, 2].tolist() == [0, 0, 1, 1, 1] and want_tf.sum() == 3
    got, tf = run_gpu(q, k, v, sl, scale)
    assert np.array_equal(tf, want_tf)
    close(H, got.reshape(-1, 128), want, "prefill with recomputation")


@pytest.mark.parametrize("logit,phi,bounds", [(16.0, 3.0, (LO, HI)), (21.0, 3.0, (LO, HI)), (0.0, -16.8, (0.0, 23.3)),
                                              (10.0, -16.8, (0.0, 40.0)), (-40.0, 3.0, (LO, HI))])
def test_weights_beyond_the_fp16_operand_range_stay_exact_and_unflagged(H, logit, phi, bounds):
    """The kernel hands its weights to the matrix cores as fp16 pairs under a per-query scale fixed after the
    query's first 32 keys.  A later key whose weight exceeds that scale's headroom (2^11.9 above the first
    step's maximum) while staying INSIDE the guard's bounds must not change what the caller sees: no flag (the
    guard did not fire), and the exact result (the tile is redone with the synchronized scheme).  Cases: a key
    13 .. 18 above the other logits; the paper's choice of phi at the lower end of the range (every exponent
    positive, weights up to e^21), without and with such a key; and the opposite, first keys far ABOVE the
    rest of the prompt (the later weights underflow the operands and are negligible, no redo needed)."""
    B, Hq, Hkv, Smax = 1, 4, 4, 320
    q, k, v, sl = draw(B, Hq, Hkv, Smax, [300], seed=7500)
    scale = float(np.float32(1.0 / np.sqrt(128.0)))
    u = np.zeros(128)
    u[7] = 1.0
    if logit == 0:
        pass                                               # ordinary logits, only phi and the bounds differ
    elif logit > 0:
        pos = 150                                          # beyond the first key step of every query
        q[0, 1, pos:300, 7] = np.float16(8.0)              # <q, u> = 8 for the later queries of head 1
        k[0, 1, pos] = (logit * np.sqrt(128.0) / 8.0 * u).astype(np.float16)
    else:
        q[0, 1, :300, 7] = np.float16(8.0)                 # the first 32 keys carry +|logit| for every query of head 1
        k[0, 1, :32, 7] = np.float16(-logit * np.sqrt(128.0) / 8.0)
        phi = 3.0 - logit                                  # ... and phi sits above them: inside the bounds
    rows = pf.all_rows(B, Hq, Smax)
    want, flag, margin = pf.prefill_rows(q, k, v, sl, scale, rows, phi=phi, lo=bounds[0], hi=bounds[1], nthreads=8)
    assert margin.min() > 1e-2 and not flag.any()          # inside (lo, hi): the guard stays quiet
    got, tf = run_gpu(q, k, v, sl, scale, phi=phi, bounds=bounds)
    assert not tf.any()
    close(H, got.reshape(-1, 128), want, "weights beyond the fp16 operand range, logit %g phi %g" % (logit, phi))


def test_nan_logit_flags_its_tiles(H):
    # a NaN inside a key of the prompt makes every logit against it NaN: the guard flags those
    # rows (a NaN is outside every range); rows before the key, and other heads, are untouched
    B, Hq, Hkv, Smax = 1, 2, 2, 256
    q, k, v, sl = draw(B, Hq, Hkv, Smax, [230], seed=7400)
    scale = float(np.float32(1.0 / np.sqrt(128.0)))
    k[0, 1, 70, 5] = np.float16(np.nan)
    rows = pf.all_rows(B, Hq, Smax)
    want, flag, _ = pf.prefill_rows(q, k, v, sl, scale, rows, phi=synth.PHI, lo=LO, hi=HI, nthreads=8)
    want_tf = tile_flags_from_rows(rows, flag, B, Hq, Smax)
    assert want_tf[0, 0].sum() == 0 and want_tf[0, 1].tolist() == [0, 1, 1, 1]
    got, tf = run_gpu(q, k, v, sl, scale)
    assert np.array_equal(tf, want_tf)
    got = got.reshape(-1, 128)
    clean = np.isfinite(want).all(axis=1)
    assert clean.sum() == Smax + 70 + (Smax - 230)      # head 0, head 1 before the key, rows past the prompt
    close(H, got[clean], want[clean], "prefill rows that do not see the NaN key")
    assert np.isnan(got[~clean]).all()


def test_lower_bound_flags_too(H):
    # phi far above the logits: every logit is below phi + lo, every tile with a token is flagged,
    # and the synchronized scheme still gives the exact result
    B, Hq, Hkv, Smax = 1, 2, 2, 192
    q, k, v, sl = draw(B, Hq, Hkv, Smax, [130], seed=7300)
    scale = float(np.float32(1.0 / np.sqrt(128.0)))
    rows = pf.all_rows(B, Hq, Smax)
    want, flag, margin = pf.prefill_rows(q, k, v, sl, scale, rows, phi=100.0, lo=LO, hi=HI, nthreads=8)
    assert margin.min() > 1e-2
    got, tf = run_gpu(q, k, v, sl, scale, phi=100.0)
    assert np.array_equal(tf, tile_flags_from_rows(rows, flag, B, Hq, Smax)) and tf.sum() == 2 * 3
    close(H, got.reshape(-1, 128), want, "prefill, all tiles recomputed")


def test_prefill_can_be_captured_and_replayed(H):
    # two launches on the caller's stream and nothing else: a stream capture of the call replays,
    # also when a tile is flagged and recomputed inside the kernel
    B, Hq, Hkv, Smax = 1, 4, 2, 512
    q, k, v, sl = draw(B, Hq, Hkv, Smax, [500], seed=7500)
    scale = float(np.float32(1.0 / np.sqrt(128.0)))
    q[0, 1, 300:500, 7] = np.float16(12.0)
    k[0, 0, 300] = 0
    k[0, 0, 300, 7] = np.float16(36.0)                 # head 1 overflows from token 300 on
    eager, tf = run_gpu(q, k, v, sl, scale)
    assert tf[0, 1].sum() > 0 and tf[0, 0].sum() == 0
    dev = torch.device("cuda:0")
    tq, tk, tv = (torch.from_numpy(a).to(dev) for a in (q, k, v))
    tsl = torch.from_numpy(sl).to(dev)
    out = torch.full((B, Hq, Smax, 128), float("nan"), dtype=torch.float16, device=dev)
    shape = fdattn.make_shape(B, Hq, Hkv, 128, Smax, 0, scale)
    nws = fdattn.fd_prefill_workspace_bytes(shape)
    ws = torch.full((nws,), 0x5A, dtype=torch.uint8, device=dev)
    side = torch.cuda.Stream(device=dev)
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream(dev))
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            fdattn.fd_prefill_attn(shape, tq.data_ptr(), tk.data_ptr(), tv.data_ptr(), tsl.data_ptr(), synth.PHI, synth.BOUNDS,
                                   out.data_ptr(), ws.data_ptr(), nws, side.cuda_stream)
    torch.cuda.synchronize()
    for i in range(3):
        out.fill_(float("nan"))
        ws.fill_(0x11 * (i + 1))                        # the workspace needs no particular contents
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().astype(np.float64), eager), "replay %d differs from the eager call" % i
    del graph


def test_prefill_rejects_bad_arguments():
    dev = torch.device("cuda:0")
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device=dev)
    p = buf.data_ptr()
    sh = fdattn.make_shape(1, 2, 2, 128, 64, 0, 0.1)
    n = fdattn.fd_prefill_workspace_bytes(sh)
    for args, code in (((sh, 0, p, p, p, 3.0, (-60.0, 20.0), p, p, n), fdattn.FD_ERR_NULL),
                       ((sh, p, p, p, p, 3.0, (5.0, 5.0), p, p, n), fdattn.FD_ERR_BOUNDS),
                       ((sh, p, p, p, p, 3.0, (-60.0, 20.0), p, p, n - 1), fdattn.FD_ERR_WORKSPACE),
                       ((fdattn.make_shape(1, 2, 2, 64, 64, 0, 0.1), p, p, p, p, 3.0, (-60.0, 20.0), p, p, n), fdattn.FD_ERR_UNSUPPORTED)):
        with pytest.raises(fdattn.FdError) as e:
            fdattn.fd_prefill_attn(*args)
        assert e.value.status == code


def test_short_prompts_sweep(H):
    """Rows of a handful of keys are where the bf16 hi + lo weights show (the first query tile carries them with all 24 bits for that reason):
    200 seeded short prompts (lengths 1 .. 320, so that queries just past the first tile are covered too), every row
    against the oracle at the decode tolerance."""
    scale = float(np.float32(1.0 / np.sqrt(128.0)))
    for seed in range(100, 300):
        rng = np.random.default_rng(seed)
        B = int(rng.integers(1, 4)); Hkv = int(rng.choice([1, 2, 4])); Hq = Hkv * int(rng.choice([1, 2, 4]))
        Smax = int(rng.integers(16, 200 if seed < 250 else 321))
        lens = [int(x) for x in rng.integers(1, Smax + 1, size=B)]
        q, k, v, sl = draw(B, Hq, Hkv, Smax, lens, seed=90000 + seed)
        rows = pf.all_rows(B, Hq, Smax)
        want, flag, margin = pf.prefill_rows(q, k, v, sl, scale, rows, phi=synth.PHI, lo=LO, hi=HI, nthreads=8)
        got, tf = run_gpu(q, k, v, sl, scale)
        close(H, got.reshape(-1, 128), want, "short prompts, seed %d %s" % (seed, (B, Hq, Hkv, Smax, lens)))
