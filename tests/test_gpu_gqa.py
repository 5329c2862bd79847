"""Grouped-query path (MFMA kernel): parity with the fp64 oracle, with the
per-row path on explicitly repeated K/V, flags per query head, recomputation."""
import numpy as np
import pytest

from paper_2311_01282_amd import synth

pytestmark = pytest.mark.gpu
LO, HI = synth.BOUNDS


@pytest.fixture(scope="module")
def H():
    import fd_harness
    return fd_harness


def exact(oracle, case):
    return oracle.attn_exact(case["q"], case["k"], case["v"], case["seq_lens"], case["scale"], nthreads=8)


def num_bound(case, oden):
    """Error bound of a chunk's numerator sum_k P_k V_k: the kernel feeds P to the matrix cores as
    fp16 hi + lo pairs (22 bits of the fp32 weight; V is fp16 as it is), accumulates in fp32 and
    computes P itself in fp32 (a few 1e-6 relative): 1e-5 * sum_k P_k |V_k|, bounded here by the
    chunk's denominator times the largest |V|."""
    return 1e-5 * np.abs(case["v"].astype(np.float64)[np.isfinite(case["v"])]).max() * oden


CASES = [
    # B, Hq, Hkv, Smax, lens, chunk
    (2, 16, 2, 1024, [1024, 777], 256),     # the benchmark's group of 8
    (1, 8, 2, 600, [555], 64),              # group of 4, small chunks, ragged tail
    (2, 6, 3, 1500, [1500, 17], 512),       # group of 2, a 17-key sequence
    (1, 16, 1, 2100, [2050], 1024),         # group of 16 (the tile is full), one short last chunk
    (3, 12, 4, 700, [0, 700, 1], 128),      # group of 3 (not a power of two), an empty sequence
    (2, 16, 2, 5000, [5000, 2049], 2048),   # long chunks: a ragged last one, one key in a chunk
    (2, 16, 2, 9000, [8999, 4097], 4096),   # the longest chunk
    (4, 16, 2, 4096, [4096, 3000, 1, 0], 4096),   # every sequence fits one chunk: results leave without the epilogue
    (3, 12, 4, 256, [256, 100, 255], 256),  # the same with groups of 3
    (2, 16, 2, 700, [700, 200], 512),       # a sequence of two chunks next to one of a single chunk
    (8, 64, 8, 1024, [1024, 100, 300, 1, 0, 513, 512, 900], 256),   # 256 workgroups, ragged: many chunks past the ends
    (10, 64, 8, 1024, None, 256),           # 320 workgroups: the row epilogue as a second launch
    (2, 16, 2, 3000, [3000, 1111], 1152),   # a chunk length that is no power of two (capacity 2048)
    (1, 8, 2, 600, [555], 80),              # ... of 80 keys (capacity 128)
    (2, 16, 2, 9000, [8999, 4097], 3008),   # ... of 3008 keys (capacity 4096)
]


@pytest.mark.parametrize("B,Hq,Hkv,Smax,lens,chunk", CASES)
def test_gqa_matches_oracle_and_per_row_path(oracle, H, B, Hq, Hkv, Smax, lens, chunk):
    if lens is None:
        lens = [Smax - 53 * b for b in range(B)]
    case = synth.make_case(B=B, Hq=Hq, Hkv=Hkv, D=128, Smax=Smax, seed=400 + Smax + chunk, seq_lens=lens,
                           poison_padding=True)
    want = exact(oracle, case)
    ocf, orf, margin = oracle.flags(case["q"], case["k"], case["seq_lens"], case["scale"], synth.PHI, LO, HI, chunk)
    assert margin.min() > 1e-2 and not orf.any()
    dc = H.DeviceCase(case, chunk=chunk)
    got = dc.run("fd_decode_attn_gqa")
    H.assert_close(got, want, "gqa")
    cf, rf, n, rows = dc.flags()
    assert np.array_equal(cf, ocf) and np.array_equal(rf, orf) and n == 0
    # the per-row path on K/V repeated for every query head must agree row by row
    G = Hq // Hkv
    rep = dict(case)
    rep["k"] = np.ascontiguousarray(np.repeat(case["k"], G, axis=1))
    rep["v"] = np.ascontiguousarray(np.repeat(case["v"], G, axis=1))
    rep["Hkv"] = Hq
    got_rows = H.DeviceCase(rep, chunk=chunk).run("fd_decode_attn")
    assert np.abs(got - got_rows).max() <= 1e-3
    H.assert_close(dc.run("fd_decode_attn"), want, "per-row path on shared KV heads")


def test_gqa_partial_sums_match_eq4(oracle, H):
    """The per-chunk numerators and denominators the MFMA kernel leaves behind."""
    case = synth.make_case(B=2, Hq=16, Hkv=2, D=128, Smax=1300, seed=410, seq_lens=[1300, 515],
                           poison_padding=True)
    _, onum, oden = oracle.attn_unified(case["q"], case["k"], case["v"], case["seq_lens"], case["scale"],
                                        synth.PHI, 256, return_partials=True)
    dc = H.DeviceCase(case, chunk=256)
    dc.run("fd_decode_attn_gqa")
    num, den = dc.partials()
    np.testing.assert_allclose(den, oden, rtol=2e-5, atol=0)
    assert (np.abs(num - onum) <= num_bound(case, oden)[..., None]).all()


@pytest.mark.parametrize("Smax,lens,chunk", [(2048, [2048, 1111], 256), (8192, [8192, 5000], 4096), (3000, [3000, 1700], 1152)])
def test_gqa_flags_are_per_query_head_and_rows_recomputed(oracle, H, Smax, lens, chunk):
    case = synth.make_case(B=2, Hq=16, Hkv=2, D=128, Smax=Smax, seed=420, seq_lens=lens,
                           poison_padding=True)
    planted = synth.plant_keys(case, 3, 36.0, seed=421, allow_shared_kv=True)
    want = exact(oracle, case)
    ocf, orf, margin = oracle.flags(case["q"], case["k"], case["seq_lens"], case["scale"], synth.PHI, LO, HI, chunk)
    assert margin.min() > 1e-2
    for b, h, _ in planted:
        assert orf[b, h]
    assert orf.sum() < orf.size                     # other heads of the groups stay unflagged
    dc = H.DeviceCase(case, chunk=chunk)
    for _ in range(2):                              # twice: the arrival counters must reset
        got = dc.run("fd_decode_attn_gqa")
        H.assert_close(got, want, "gqa + recompute")
        cf, rf, n, rows = dc.flags()
        assert np.array_equal(cf, ocf) and np.array_equal(rf, orf)
        assert n == int(orf.sum()) and rows.tolist() == np.flatnonzero(orf.reshape(-1)).tolist()
    for b, h, pos in planted:
        np.testing.assert_allclose(got[b, h], case["v"][b, h // 8, pos].astype(np.float64), atol=2e-3)
    # every row flagged through tight bounds: everything comes from the synchronized scheme
    got = dc.run("fd_decode_attn_gqa", phi=0.0, bounds=(-0.5, 0.5))
    assert dc.flags()[1].all()
    H.assert_close(got, want, "gqa, all rows recomputed")


def test_gqa_rejects_ungrouped_shapes(H):
    from paper_2311_01282_amd import fdattn
    case = synth.make_case(B=1, Hq=4, Hkv=4, D=128, Smax=256, seed=430)
    dc = H.DeviceCase(case, chunk=256)
    with pytest.raises(fdattn.FdError) as e:
        dc.run("fd_decode_attn_gqa")
    assert e.value.status == fdattn.FD_ERR_UNSUPPORTED


def test_gqa_single_chunk_sequences_publish_partials_and_recompute(oracle, H):
    """Sequences of one chunk: the partial sums still reach the workspace, and a head whose guard
    fires takes the ordinary route (recomputation, then the epilogue) while its neighbours do not."""
    case = synth.make_case(B=3, Hq=16, Hkv=2, D=128, Smax=2048, seed=430, seq_lens=[2048, 900, 33],
                           poison_padding=True)
    planted = synth.plant_keys(case, 2, 36.0, seed=431, allow_shared_kv=True)
    want = exact(oracle, case)
    ocf, orf, margin = oracle.flags(case["q"], case["k"], case["seq_lens"], case["scale"], synth.PHI, LO, HI, 2048)
    assert margin.min() > 1e-2 and 0 < orf.sum() < orf.size
    dc = H.DeviceCase(case, chunk=2048)
    got = dc.run("fd_decode_attn_gqa")
    H.assert_close(got, want, "gqa, single chunk")
    cf, rf, n, rows = dc.flags()
    assert np.array_equal(cf, ocf) and np.array_equal(rf, orf) and n == int(orf.sum())
    # partial sums of the unflagged (head, chunk) pairs are Eq. 4's
    _, onum, oden = oracle.attn_unified(case["q"], case["k"], case["v"], case["seq_lens"], case["scale"],
                                        synth.PHI, 2048, return_partials=True)
    num, den = dc.partials()
    keep = ~ocf.astype(bool)
    np.testing.assert_allclose(den[keep], oden[keep], rtol=2e-5, atol=0)
    assert (np.abs(num - onum)[keep] <= num_bound(case, oden)[keep][..., None]).all()


@pytest.mark.parametrize("phi", [40.0, -15.0])
def test_gqa_weights_at_both_ends_of_the_admissible_range(oracle, H, phi):
    """Every weight e^{x - phi} near e^-40 (phi = 40) or near e^+15 (phi = -15): inside the bounds, so
    nothing is flagged, and far outside what fp16 could hold -- the matrix-core operands (fp16 pairs under a
    scale of the head's own) must carry them; one key per sequence dominates its row as well."""
    case = synth.make_case(B=2, Hq=16, Hkv=2, D=128, Smax=1500, seed=440, seq_lens=[1500, 700], poison_padding=True)
    synth.plant_keys(case, 2, 4.5, seed=441, allow_shared_kv=True)       # logit about 4.5: inside the bounds for both phi
    want = exact(oracle, case)
    ocf, orf, margin = oracle.flags(case["q"], case["k"], case["seq_lens"], case["scale"], phi, LO, HI, 512)
    assert margin.min() > 1e-2 and not orf.any()
    dc = H.DeviceCase(case, chunk=512)
    got = dc.run("fd_decode_attn_gqa", phi=phi)
    H.assert_close(got, want, "gqa, phi %g" % phi)
    cf, rf, n, rows = dc.flags()
    assert not cf.any() and not rf.any() and n == 0
    # and through the per-row kernel, whose arithmetic is fp32 throughout
    assert np.abs(got - dc.run("fd_decode_attn", phi=phi)).max() <= 1e-3


@pytest.mark.parametrize("gamma,chunk", [(14.0, 512), (17.0, 2048), (14.0, 64)])
def test_gqa_weights_beyond_the_fp16_operand_range_stay_exact_and_unflagged(oracle, H, gamma, chunk):
    """The grouped kernel hands its weights to the matrix cores as fp16 pairs under a scale fixed after each
    wavefront's first 16 keys.  A later key whose logit is 10 .. 18 above the rest, yet INSIDE the bounds, does
    not fit that scale: its (head, chunk) must be redone on the per-row path -- exact result, and no flag, for
    the guard did not fire.  (Where the key falls into a wavefront's first block the scale adapts instead.)"""
    case = synth.make_case(B=3, Hq=16, Hkv=2, D=128, Smax=2048, seed=450, seq_lens=[2048, 1300, 90], poison_padding=True)
    planted = synth.plant_keys(case, 8, gamma, seed=451 + chunk, allow_shared_kv=True)
    assert len(planted) == 8
    want = exact(oracle, case)
    ocf, orf, margin = oracle.flags(case["q"], case["k"], case["seq_lens"], case["scale"], synth.PHI, LO, HI, chunk)
    assert margin.min() > 1e-2 and not orf.any()          # logit - phi about 7 .. 16: inside (-60, 20)
    x = [float(case["q"][b, h].astype(np.float64) @ case["k"][b, h // 8, pos].astype(np.float64)) * case["scale"] for b, h, pos in planted]
    assert min(x) > 9.5                                    # ... and 8 or more above every other logit of its row
    dc = H.DeviceCase(case, chunk=chunk)
    for _ in range(2):
        got = dc.run("fd_decode_attn_gqa")
        H.assert_close(got, want, "gqa, weights beyond the fp16 operand range")
        cf, rf, n, rows = dc.flags()
        assert not cf.any() and not rf.any() and n == 0
    assert np.abs(got - dc.run("fd_decode_attn")).max() <= 1e-3
