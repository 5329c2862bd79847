"""GPU parity at the benchmark's full sizes, through the entry points and launch
configurations bench.py times.  The fp64 oracle is fast enough (threads over
rows) to check every output element and every flag of all five workloads."""
import numpy as np
import pytest

from paper_2311_01282_amd import synth

pytestmark = pytest.mark.gpu
LO, HI = synth.BOUNDS


@pytest.fixture(scope="module")
def H():
    import fd_harness
    return fd_harness


def picked(name):
    """The chunk size bench.py times this workload with."""
    from paper_2311_01282_amd import fdattn
    c = synth.CONFIGS[name]
    return fdattn.fd_pick_chunk(fdattn.make_shape(c["B"], c["Hq"], c["Hkv"], c["D"], c["Smax"], 0, 1.0))


def check(oracle, H, name, entry, chunks, poison=False):
    chunks = sorted(set(chunks) | {picked(name)})
    case = synth.make_config(name, poison_padding=poison)
    want = oracle.attn_exact(case["q"], case["k"], case["v"], case["seq_lens"], case["scale"], nthreads=16)
    for chunk in chunks:
        ocf, orf, margin = oracle.flags(case["q"], case["k"], case["seq_lens"], case["scale"], synth.PHI, LO, HI,
                                        chunk, nthreads=16)
        assert margin.min() > 1e-2
        dc = H.DeviceCase(case, chunk=chunk)
        got = dc.run(entry)
        a, r = H.assert_close(got, want, "%s chunk %d" % (name, chunk))
        cf, rf, n, rows = dc.flags()
        assert np.array_equal(cf, ocf) and np.array_equal(rf, orf)
        assert n == int(orf.sum()) and rows.tolist() == np.flatnonzero(orf.reshape(-1)).tolist()
        # the literal chain (partial / flag reduction / atomic-free combine / whole-row recomputation of flagged
        # rows / synchronized merge): outputs, chunk and row flags, the ascending list and its count
        got_chain = dc.run("fd_decode_attn_multikernel")
        H.assert_close(got_chain, want, "%s chain chunk %d" % (name, chunk))
        ccf, crf, cn, crows = dc.flags()
        assert np.array_equal(ccf, ocf) and np.array_equal(crf, orf)
        assert cn == int(orf.sum()) and crows.tolist() == np.flatnonzero(orf.reshape(-1)).tolist()
        assert np.abs(got - got_chain)[orf == 0].max() <= 1e-3
        # the synchronized scheme on every row must agree with the unified path (unflagged rows)
        got_sync = dc.run("fd_decode_attn_sync")
        H.assert_close(got_sync, want, "%s sync chunk %d" % (name, chunk))
        keep = orf == 0
        assert np.abs(got - got_sync)[keep].max() <= 1e-3
        del dc
    return case, want, orf


def test_c0_llama7b_1k(oracle, H):
    _, _, orf = check(oracle, H, "c0_b1_h32_s1024", "fd_decode_attn", [256])
    assert not orf.any()


def test_c1_llama7b_8k_chunk_sweep(oracle, H):
    _, _, orf = check(oracle, H, "c1_b1_h32_s8192", "fd_decode_attn", [256, 512, 1024])
    assert not orf.any()


def test_c2_ragged_batch(oracle, H):
    case, _, orf = check(oracle, H, "c2_b16_h32_ragged4096", "fd_decode_attn", [256], poison=True)
    assert not orf.any()
    assert case["seq_lens"].min() >= 512 and case["seq_lens"].max() <= 4096


def test_c3_gqa_70b_shape(oracle, H):
    _, _, orf = check(oracle, H, "c3_b32_gqa64x8_s4096", "fd_decode_attn_gqa", [256])
    assert not orf.any()


def test_c4_overflow_stress(oracle, H):
    case, want, orf = check(oracle, H, "c4_b4_h32_s32768_overflow", "fd_decode_attn", [256])
    planted = case["planted"]
    assert len(planted) == 2 and int(orf.sum()) == 2
    for b, h, pos in planted:
        assert orf[b, h]
        np.testing.assert_allclose(want[b, h], case["v"][b, h, pos].astype(np.float64), atol=1e-6)
    # the literal planted magnitude gamma = 12 stays inside the bounds: nothing is flagged
    lit = synth.make_config("c4_b4_h32_s32768_overflow", plant_gamma=12.0)
    _, lrf, lmargin = oracle.flags(lit["q"], lit["k"], lit["seq_lens"], lit["scale"], synth.PHI, LO, HI, 256, nthreads=16)
    assert not lrf.any() and lmargin.min() > 1e-2
    dc = H.DeviceCase(lit, chunk=256)
    got = dc.run("fd_decode_attn")
    assert dc.flags()[2] == 0
    H.assert_close(got, oracle.attn_exact(lit["q"], lit["k"], lit["v"], lit["seq_lens"], lit["scale"], nthreads=16),
                   "c4, gamma 12")


@pytest.mark.parametrize("Smax,lens,chunk,mib", [(8192, [8192, 5000], 1024, 256), (8192, [8192, 8100], 512, 256),
                                                 (16384, [16384, 9000], 1024, 512), (12288, [12288, 700], 768, 384)])
def test_launches_of_257_to_1024_workgroups(oracle, H, Smax, lens, chunk, mib):
    """Between one and four workgroups per compute unit the per-row call picks its launch form by the
    size of the cache (row epilogue elected inside the kernel below 320 MiB, a second launch from
    there on): both forms, full and part-filled sequences, two planted out-of-range keys, checked
    on every output element, flag, list entry and count."""
    case = synth.make_case(B=2, Hq=32, Hkv=32, D=128, Smax=Smax, seed=7100 + chunk, seq_lens=lens, poison_padding=True)
    assert case["k"].nbytes + case["v"].nbytes == mib << 20
    planted = synth.plant_keys(case, 2, 36.0, seed=7200 + chunk)
    want = oracle.attn_exact(case["q"], case["k"], case["v"], case["seq_lens"], case["scale"], nthreads=16)
    ocf, orf, margin = oracle.flags(case["q"], case["k"], case["seq_lens"], case["scale"], synth.PHI, LO, HI, chunk, nthreads=16)
    assert margin.min() > 1e-2 and int(orf.sum()) == 2 and all(orf[b, h] for b, h, _ in planted)
    dc = H.DeviceCase(case, chunk=chunk)
    assert 256 < 64 * -(-Smax // chunk) <= 1024
    for entry in ("fd_decode_attn", "fd_decode_attn", "fd_decode_attn_multikernel"):
        got = dc.run(entry)
        H.assert_close(got, want, "%s, %d MiB" % (entry, mib))
        cf, rf, n, rows = dc.flags()
        assert np.array_equal(cf, ocf) and np.array_equal(rf, orf)
        assert n == 2 and rows.tolist() == np.flatnonzero(orf.reshape(-1)).tolist()
