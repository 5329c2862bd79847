"""fd_decode_attn_append on the GPU: the step's K/V rows are attended from the
step's own buffers and stored into the cache by the same launch.  The oracle
sees the cache with the rows already in place (the definition: concatenate,
then Eq. 1); the cache on the GPU must afterwards hold exactly those bits and
nothing else may have changed."""
import numpy as np
import pytest
import torch

from paper_2311_01282_amd import fdattn, synth

pytestmark = pytest.mark.gpu
LO, HI = synth.BOUNDS


@pytest.fixture(scope="module")
def H():
    import fd_harness
    return fd_harness


def appended(case, k_new, v_new):
    """The cache after the step, and the lengths that include the new token (host side)."""
    k2, v2 = case["k"].copy(), case["v"].copy()
    sl = np.clip(np.asarray(case["seq_lens"], dtype=np.int64), 0, case["Smax"])
    for b in range(case["B"]):
        if sl[b] < case["Smax"]:
            k2[b, :, sl[b], :] = k_new[b]
            v2[b, :, sl[b], :] = v_new[b]
    return k2, v2, np.minimum(sl + 1, case["Smax"]).astype(np.int32)


def run_append(H, case, k_new, v_new, chunk, phi=synth.PHI, bounds=synth.BOUNDS):
    dc = H.DeviceCase(case, chunk=chunk)
    kn = torch.from_numpy(k_new).to(dc.dev)
    vn = torch.from_numpy(v_new).to(dc.dev)
    dc.out.fill_(float("nan"))
    dc.last_entry = "fd_decode_attn_append"
    fdattn.fd_decode_attn_append(dc.shape, dc.q.data_ptr(), kn.data_ptr(), vn.data_ptr(), dc.k.data_ptr(), dc.v.data_ptr(),
                                 dc.seq_lens.data_ptr(), phi, bounds, dc.out.data_ptr(), *dc._ws(), dc._stream())
    torch.cuda.synchronize()
    return dc, dc.out.cpu().numpy().astype(np.float64)


def check(oracle, H, case, chunk, k_new=None, v_new=None, seed=1, expect_flagged=None):
    rng = np.random.default_rng(seed)
    B, Hkv, D = case["B"], case["Hkv"], case["D"]
    if k_new is None:
        k_new = rng.standard_normal((B, Hkv, D)).astype(np.float16)
    if v_new is None:
        v_new = rng.standard_normal((B, Hkv, D)).astype(np.float16)
    k2, v2, sl2 = appended(case, k_new, v_new)
    want = oracle.attn_exact(case["q"], k2, v2, sl2, case["scale"], nthreads=8)
    ocf, orf, margin = oracle.flags(case["q"], k2, sl2, case["scale"], synth.PHI, LO, HI, chunk, nthreads=8)
    assert margin.min() > 1e-2
    dc, got = run_append(H, case, k_new, v_new, chunk)
    H.assert_close(got, want, "append chunk %d" % chunk)
    # the cache: bit for bit the concatenation, nothing else touched (padding keeps its poison)
    assert np.array_equal(dc.k.cpu().numpy().view(np.uint16), k2.view(np.uint16))
    assert np.array_equal(dc.v.cpu().numpy().view(np.uint16), v2.view(np.uint16))
    # flags, with the lengths that include the new token
    dc.seq_lens.copy_(torch.from_numpy(sl2))
    cf, rf, n, rows = dc.flags()
    assert np.array_equal(cf, ocf) and np.array_equal(rf, orf)
    if expect_flagged is not None:
        assert int(orf.sum()) == expect_flagged
    return got, want


@pytest.mark.parametrize("B,Hq,Hkv,Smax,lens,chunk", [
    (1, 4, 4, 512, [300], 256),                       # new key inside the last chunk
    (1, 4, 4, 512, [256], 256),                       # new key opens a chunk of its own
    (2, 4, 4, 512, [511, 512], 256),                  # last free position; full cache (row dropped)
    (3, 8, 8, 1024, [0, 1, 1023], 128),               # empty sequence: the new key is the only one
    (4, 8, 8, 777, [776, 5, 64, 700], 64),            # odd maximum length, chunk edges
    (2, 32, 32, 2048, [2047, 1000], 1024),            # 8-wavefront workgroups
    (8, 32, 32, 2048, None, 256),                     # 2048 workgroups: row epilogue as a second launch
    (2, 16, 2, 600, [599, 256], 256),                 # grouped kernel, groups of 8
    (2, 12, 4, 515, [512, 0], 128),                   # groups of 3; new chunk; empty sequence
    (1, 64, 8, 4096, [4000], 1024),                   # grouped, long chunks
    (16, 64, 8, 1024, None, 256),                     # grouped, 512 workgroups: second launch
    (1, 34, 2, 300, [299], 64),                       # groups of 17: per-row kernel with shared KV heads
    (3, 16, 2, 512, [300, 510, 0], 512),              # grouped, one chunk per sequence: no epilogue; new key alone
    (2, 16, 2, 1024, [512, 511], 512),                # grouped: the new key opens a second chunk / completes the only one
    (3, 4, 4, 1200, [575, 576, 1151], 576),           # chunks of 576 keys: last key of a chunk, first of the next
    (3, 16, 2, 1200, [575, 576, 1151], 576),          # the same through the grouped kernel
])
def test_append_matches_concatenate_then_attend(oracle, H, B, Hq, Hkv, Smax, lens, chunk):
    if lens is None:
        lens = [Smax - 1 - 37 * b for b in range(B)]
    case = synth.make_case(B=B, Hq=Hq, Hkv=Hkv, D=128, Smax=Smax, seq_lens=lens, seed=4200 + Smax + B, poison_padding=True)
    check(oracle, H, case, chunk, seed=B + Smax)


def test_append_of_an_overflowing_key_is_flagged_and_recomputed(oracle, H):
    # the new key itself leaves the bounds (logit ~ +36): its chunk is redone with the
    # synchronized scheme, new key included; per-row and grouped kernels
    for (Hq, Hkv, lens, chunk) in ((4, 4, [700, 512], 256), (16, 2, [700, 512], 256), (16, 2, [700, 512], 1024)):
        case = synth.make_case(B=2, Hq=Hq, Hkv=Hkv, D=128, Smax=1024, seq_lens=lens, seed=91, poison_padding=True)
        G = Hq // Hkv
        k_new = np.random.default_rng(3).standard_normal((2, Hkv, 128)).astype(np.float16)
        qv = case["q"][1, 0].astype(np.float64)                 # aim at row (1, 0): KV head 0 of sequence 1
        k_new[1, 0] = (36.0 * qv / np.linalg.norm(qv)).astype(np.float16)
        check(oracle, H, case, chunk, k_new=k_new, seed=5, expect_flagged=1)


def test_append_then_plain_call_agree(oracle, H):
    # after the fused step the cache is complete: the plain call on it, with lengths + 1, gives the same output
    case = synth.make_case(B=2, Hq=8, Hkv=8, D=128, Smax=1024, seq_lens=[1000, 333], seed=17)
    rng = np.random.default_rng(8)
    k_new = rng.standard_normal((2, 8, 128)).astype(np.float16)
    v_new = rng.standard_normal((2, 8, 128)).astype(np.float16)
    dc, got = run_append(H, case, k_new, v_new, 256)
    dc.seq_lens.add_(1)
    again = dc.run("fd_decode_attn")
    assert np.abs(got - again).max() <= 2.5e-4


def test_append_rejects_missing_rows(H):
    case = synth.make_case(B=1, Hq=4, Hkv=4, D=128, Smax=256, seed=3)
    dc = H.DeviceCase(case, chunk=256)
    with pytest.raises(fdattn.FdError) as e:
        fdattn.fd_decode_attn_append(dc.shape, dc.q.data_ptr(), 0, dc.q.data_ptr(), dc.k.data_ptr(), dc.v.data_ptr(),
                                     dc.seq_lens.data_ptr(), synth.PHI, synth.BOUNDS, dc.out.data_ptr(), *dc._ws(), dc._stream())
    assert e.value.status == fdattn.FD_ERR_NULL
