"""GPU parity at sizes the oracle finishes in seconds: every element of the
output, the flag set and the per-chunk partial sums, against the fp64 oracle on
the same seeded inputs.  Shapes span several workgroup tiles and ragged tails."""
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


SMALL = [
    # B, Hq, Hkv, Smax, lens, chunk
    (1, 4, 4, 1024, None, 256),                       # config-0 shape, fewer heads
    (2, 3, 3, 1000, [1000, 777], 256),                # ragged tail inside a chunk
    (3, 2, 2, 600, [1, 63, 600], 64),                 # tiny rows, many chunks
    (2, 2, 2, 2048, [2048, 1025], 1024),              # largest chunk, one key in the last
    (2, 2, 2, 1536, [0, 1300], 512),                  # an empty sequence
    (1, 8, 2, 700, [700], 128),                       # grouped heads through the per-row path
    (2, 4, 4, 5000, [5000, 2049], 2048),              # long chunks: a ragged last one, one key in a chunk
    (2, 4, 4, 9000, [8999, 4097], 4096),              # the longest chunk
    (2, 32, 32, 2048, [1500, 900], 256),              # 512 workgroups: in-kernel hand-over without early loads
    (3, 32, 32, 1024, [1024, 1, 300], 128),           # 768 workgroups, most of them past the sequences' ends
    (1, 16, 16, 4096, [700], 256),                    # 256 workgroups (early loads), a cache six times the sequence
    (2, 4, 4, 3000, [3000, 1700], 1152),              # a chunk length that is no power of two (capacity 2048)
    (1, 4, 4, 1000, [1000], 80),                      # ... of 80 keys (capacity 128): 13 chunks
    (2, 2, 2, 9000, [9000, 4100], 3008),              # ... of 3008 keys (capacity 4096)
]


UNIFIED = ["fd_decode_attn", "fd_decode_attn_multikernel"]


@pytest.mark.parametrize("B,Hq,Hkv,Smax,lens,chunk", SMALL)
def test_unified_and_sync_match_oracle(oracle, H, B, Hq, Hkv, Smax, lens, chunk):
    case = synth.make_case(B=B, Hq=Hq, Hkv=Hkv, D=128, Smax=Smax, seed=100 + Smax + chunk,
                           seq_lens=lens, poison_padding=True)
    want = exact(oracle, case)
    dc = H.DeviceCase(case, chunk=chunk)
    ocf, orf, margin = oracle.flags(case["q"], case["k"], case["seq_lens"], case["scale"], synth.PHI, LO, HI, chunk)
    assert margin.min() > 1e-2
    for entry in UNIFIED:
        got = dc.run(entry)
        H.assert_close(got, want, entry)
        cf, rf, n, rows = dc.flags()
        assert np.array_equal(cf, ocf) and np.array_equal(rf, orf) and n == 0 and len(rows) == 0
    got_sync = dc.run("fd_decode_attn_sync")
    H.assert_close(got_sync, want, "sync")
    assert np.abs(got - got_sync).max() <= 1e-3


@pytest.mark.parametrize("chunk", [64, 256, 1024, 208])
def test_partial_sums_match_eq4(oracle, H, chunk):
    case = synth.make_case(B=2, Hq=2, Hkv=2, D=128, Smax=1300, seed=200 + chunk, seq_lens=[1300, 515],
                           poison_padding=True)
    _, onum, oden = oracle.attn_unified(case["q"], case["k"], case["v"], case["seq_lens"], case["scale"],
                                        synth.PHI, chunk, return_partials=True)
    dc = H.DeviceCase(case, chunk=chunk)
    dc.run_partial()
    num, den = dc.partials()
    np.testing.assert_allclose(den, oden, rtol=2e-5, atol=0)
    np.testing.assert_allclose(num, onum, rtol=0, atol=2e-5 * np.abs(oden).max())
    assert not dc.chunk_flags().any()


def test_planted_keys_flag_and_recompute(oracle, H):
    """Rows holding a key whose logit exceeds phi + hi are flagged (exactly the
    chunk that holds it), listed in ascending order and recomputed; all rows match."""
    case = synth.make_case(B=3, Hq=4, Hkv=4, D=128, Smax=2048, seed=300, seq_lens=[2048, 1500, 300],
                           poison_padding=True)
    planted = synth.plant_keys(case, 3, 36.0, seed=301)
    want = exact(oracle, case)
    ocf, orf, margin = oracle.flags(case["q"], case["k"], case["seq_lens"], case["scale"], synth.PHI, LO, HI, 256)
    assert margin.min() > 1e-2 and orf.sum() == 3
    dc = H.DeviceCase(case, chunk=256)
    outs = {}
    for entry in UNIFIED + UNIFIED[:1]:            # the fused call twice: its tickets must reset
        got = outs[entry] = dc.run(entry)
        H.assert_close(got, want, entry + " + recompute")
        cf, rf, n, rows = dc.flags()
        assert np.array_equal(cf, ocf) and np.array_equal(rf, orf)
        assert n == 3 and rows.tolist() == sorted(b * 4 + h for b, h, _ in planted)
        for b, h, pos in planted:                  # closed form: the row is its planted key's V row
            np.testing.assert_allclose(got[b, h], case["v"][b, h, pos].astype(np.float64), atol=2e-3)
    assert np.abs(outs[UNIFIED[0]] - outs[UNIFIED[1]]).max() <= 1e-3
    # gamma = 12 stays inside the bounds: nothing may be flagged
    case2 = synth.make_case(B=3, Hq=4, Hkv=4, D=128, Smax=2048, seed=300, seq_lens=[2048, 1500, 300])
    synth.plant_keys(case2, 3, 12.0, seed=301)
    dc2 = H.DeviceCase(case2, chunk=256)
    got2 = dc2.run("fd_decode_attn")
    H.assert_close(got2, exact(oracle, case2), "gamma 12")
    assert dc2.flags()[2] == 0


def test_every_row_flagged_and_lower_bound(oracle, H):
    """Tight bounds flag every row (both sides of the guard): the whole output then
    comes from the synchronized scheme."""
    case = synth.make_case(B=2, Hq=3, Hkv=3, D=128, Smax=900, seed=310, seq_lens=[900, 257])
    want = exact(oracle, case)
    dc = H.DeviceCase(case, chunk=128)
    for phi, bounds in ((3.0, (-1.5, 20.0)), (0.0, (-60.0, 0.75)), (0.0, (-0.5, 0.5))):
        ocf, orf, margin = oracle.flags(case["q"], case["k"], case["seq_lens"], case["scale"], phi,
                                        bounds[0], bounds[1], 128)
        assert orf.all()
        near = margin.min() <= 1e-4     # a logit within rounding distance of a bound: flags not comparable
        for entry in UNIFIED:
            got = dc.run(entry, phi=phi, bounds=bounds)
            cf, rf, n, rows = dc.flags()
            assert near or (np.array_equal(cf, ocf) and np.array_equal(rf, orf))
            assert n == int(rf.sum()) and rows.tolist() == np.flatnonzero(rf.reshape(-1)).tolist()
            H.assert_close(got, want, entry + ", all rows recomputed")


def test_guard_equality_flags(oracle, H):
    """Logits exactly on a bound must flag.  q = 8 e_1 and scale = 1/8 make the
    logit equal to the key's first element exactly in fp32."""
    S = 512
    case = synth.make_case(B=1, Hq=4, Hkv=4, D=128, Smax=S, seed=320)
    case["scale"] = 0.125
    case["q"][:] = 0; case["q"][:, :, 0] = 8.0
    case["k"][..., 0] = np.clip(case["k"][..., 0], -1.5, 1.5)      # logits in [-1.5, 1.5]
    phi, lo, hi = 1.0, -3.0, 1.0
    case["k"][0, 1, 300, 0] = 2.0            # x - phi == hi       -> flag, chunk 1 (chunk 256)
    case["k"][0, 2, 10, 0] = -2.0            # x - phi == lo       -> flag, chunk 0
    case["k"][0, 3, 511, 0] = 1.998046875    # one binary16 step inside hi -> no flag
    ocf, orf, _ = oracle.flags(case["q"], case["k"], case["seq_lens"], case["scale"], phi, lo, hi, 256)
    assert orf.reshape(-1).tolist() == [0, 1, 1, 0] and ocf[0, 1].tolist() == [0, 1] and ocf[0, 2].tolist() == [1, 0]
    dc = H.DeviceCase(case, chunk=256)
    for entry in UNIFIED:
        got = dc.run(entry, phi=phi, bounds=(lo, hi))
        cf, rf, n, rows = dc.flags()
        assert np.array_equal(cf, ocf) and np.array_equal(rf, orf) and rows.tolist() == [1, 2]
        H.assert_close(got, exact(oracle, case), entry + ", equality")


def test_invariance_to_phi_and_chunk(oracle, H):
    """Eq. 3 and Eq. 4 on the GPU: moving phi inside the safe range or changing the
    chunk size changes the output only by fp32 rounding noise."""
    case = synth.make_case(B=1, Hq=4, Hkv=4, D=128, Smax=3000, seed=330, seq_lens=[2900])
    ref = None
    for chunk in (256, 512, 1024):
        dc = H.DeviceCase(case, chunk=chunk)
        for phi in (1.0, 3.0, 5.0):
            got = dc.run("fd_decode_attn", phi=phi)
            assert dc.flags()[2] == 0
            ref = got if ref is None else ref
            assert np.abs(got - ref).max() <= 2.5e-4      # <= a couple of fp16 ulps at |out| < 0.25
    H.assert_close(ref, exact(oracle, case), "invariance")


@pytest.mark.parametrize("B,Hq,Hkv,Smax,entry", [
    (1, 32, 32, 9216, "fd_decode_attn"),          # 8 equal chunks of 1152 keys: 256 workgroups
    (2, 32, 32, 5000, "fd_decode_attn"),          # 4 x 1264
    (8, 64, 8, 5000, "fd_decode_attn_gqa"),       # grouped: 4 x 1264 keys, 256 workgroups
    (5, 40, 8, 4096, "fd_decode_attn_gqa"),       # grouped, 5 heads per group: 6 x 688 keys, one round of 240 workgroups
])
def test_the_picked_chunk_on_lengths_that_do_not_divide(oracle, H, B, Hq, Hkv, Smax, entry):
    """fd_pick_chunk's equal chunks (no power of two) end to end: output and flags against the oracle."""
    from paper_2311_01282_amd import fdattn
    case = synth.make_case(B=B, Hq=Hq, Hkv=Hkv, D=128, Smax=Smax, seed=300 + Smax + B, poison_padding=True)
    chunk = fdattn.fd_pick_chunk(fdattn.make_shape(B, Hq, Hkv, 128, Smax, 0, case["scale"]))
    assert chunk % 16 == 0 and chunk & (chunk - 1) != 0
    want = exact(oracle, case)
    ocf, orf, margin = oracle.flags(case["q"], case["k"], case["seq_lens"], case["scale"], synth.PHI, LO, HI, chunk, nthreads=8)
    dc = H.DeviceCase(case, chunk=chunk)
    got = dc.run(entry)
    H.assert_close(got, want, "%s, picked chunk %d" % (entry, chunk))
    cf, rf, n, rows = dc.flags()
    if margin.min() > 1e-2:
        assert np.array_equal(cf, ocf) and np.array_equal(rf, orf)


@pytest.mark.parametrize("B,Hq,Hkv,Smax,lens,chunk", [
    (2, 8, 8, 4096, [4096, 3001], 64),        # 64 chunks per row of a single block each: nothing to rotate
    (1, 32, 32, 8192, [8000], 128),           # 64 chunks per row, 2048 workgroups, two blocks per chunk
    (2, 16, 2, 4096, [4096, 2500], 64),       # grouped kernel, 64 chunks per head group, one block per wavefront
    (1, 64, 8, 16384, [16001], 256),          # grouped kernel, 64 chunks, four blocks per wavefront
    (1, 4, 4, 40000, [39999], 1024),          # 40 chunks of 1024 keys: eight blocks to rotate through
])
def test_rows_of_more_than_32_chunks(oracle, H, B, Hq, Hkv, Smax, lens, chunk):
    """Beyond 32 chunks per row every workgroup (grouped kernel: every wavefront) starts its chunk at a
    different key block and wraps around; the sums must not care, the flags must land on the right chunks."""
    case = synth.make_case(B=B, Hq=Hq, Hkv=Hkv, D=128, Smax=Smax, seed=3300 + Smax + chunk, seq_lens=lens,
                           poison_padding=True)
    planted = synth.plant_keys(case, 2, 36.0, seed=3301 + chunk, allow_shared_kv=Hq != Hkv)
    assert -(-Smax // chunk) > 32 and len(planted) == 2
    want = exact(oracle, case)
    ocf, orf, margin = oracle.flags(case["q"], case["k"], case["seq_lens"], case["scale"], synth.PHI, LO, HI, chunk, nthreads=8)
    assert margin.min() > 1e-2 and orf.sum() >= 2
    dc = H.DeviceCase(case, chunk=chunk)
    entries = ["fd_decode_attn"] + (["fd_decode_attn_gqa"] if 2 <= Hq // Hkv <= 16 else [])
    for entry in entries:
        for rep in range(2):
            got = dc.run(entry)
            H.assert_close(got, want, "%s, %d chunks per row" % (entry, -(-Smax // chunk)))
            cf, rf, n, rows = dc.flags()
            assert np.array_equal(cf, ocf) and np.array_equal(rf, orf)
            assert n == int(orf.sum()) and rows.tolist() == np.flatnonzero(orf.reshape(-1)).tolist()
