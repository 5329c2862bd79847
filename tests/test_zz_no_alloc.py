"""fd_decode_attn_static, the entry point that allocates nothing: its workspace is a device array inside
the library.  Through the C ABI, against fd_decode_attn / fd_decode_attn_gqa on a caller-owned workspace
(same kernels: the outputs must agree bit for bit) and against the fp64 oracle at the usual tolerance, on
two calls in a row, the second with a smaller input; torch's allocator must see no allocation during the
calls."""
import numpy as np
import pytest
import torch

from paper_2311_01282_amd import fdattn, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import fd_harness
    return fd_harness


def run_static(dc):
    dc.out.fill_(float("nan"))
    before = torch.cuda.memory_stats(dc.dev).get("allocation.all.allocated", 0)
    fdattn.fd_decode_attn_static(*dc._args(), synth.PHI, synth.BOUNDS, dc.out.data_ptr(), dc._stream())
    after = torch.cuda.memory_stats(dc.dev).get("allocation.all.allocated", 0)
    assert after == before
    torch.cuda.synchronize(dc.dev)
    return dc.out.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("first,second,entry", [
    # (B, Hq, Hkv, Smax, lens, chunk): per-row kernel, one launch, then a smaller input
    ((2, 8, 8, 2048, [2048, 1100], 256), (1, 4, 4, 640, [601], 128), "fd_decode_attn"),
    # two-launch grid (2048 workgroups), then a single short row
    ((8, 32, 32, 2048, None, 256), (1, 1, 1, 64, [17], 64), "fd_decode_attn"),
    # grouped kernel
    ((4, 16, 2, 1024, [1024, 1000, 3, 0], 256), (2, 12, 4, 512, [512, 100], 128), "fd_decode_attn_gqa"),
])
def test_static_matches_workspace_entry_twice_in_a_row(oracle, H, first, second, entry):
    for i, (B, Hq, Hkv, Smax, lens, chunk) in enumerate((first, second, first)):
        case = synth.make_case(B=B, Hq=Hq, Hkv=Hkv, D=128, Smax=Smax, seed=9500 + i + Smax, seq_lens=lens, poison_padding=True)
        if i != 1:
            synth.plant_keys(case, 1, 36.0, seed=9600 + i, allow_shared_kv=Hq != Hkv)   # a flagged row goes through recomputation
        dc = H.DeviceCase(case, chunk=chunk)
        want = oracle.attn_exact(case["q"], case["k"], case["v"], case["seq_lens"], case["scale"], nthreads=8)
        ref = dc.run(entry)                       # caller-owned workspace
        H.assert_close(ref, want, "%s, call %d" % (entry, i))
        got = run_static(dc)
        H.assert_close(got, want, "fd_decode_attn_static, call %d" % i)
        assert np.array_equal(got, ref), "static and workspace forms differ on call %d" % i


def test_static_limit_is_an_error_and_leaves_out_alone(H):
    case = synth.make_case(B=1, Hq=2, Hkv=2, D=128, Smax=256, seed=9700)
    dc = H.DeviceCase(case, chunk=64)
    huge = fdattn.make_shape(64, 32, 32, 128, 32768, 64, case["scale"])
    assert fdattn.fd_workspace_bytes(huge) > fdattn.FD_STATIC_SCRATCH_BYTES
    with pytest.raises(fdattn.FdError) as e:
        fdattn.fd_decode_attn_static(huge, dc.q.data_ptr(), dc.k.data_ptr(), dc.v.data_ptr(), dc.seq_lens.data_ptr(),
                                     synth.PHI, synth.BOUNDS, dc.out.data_ptr(), dc._stream())
    assert e.value.status == fdattn.FD_ERR_STATIC_LIMIT
    torch.cuda.synchronize()
    assert torch.isnan(dc.out).all()             # nothing was enqueued


def test_static_entry_under_stream_capture(oracle, H):
    """What the entry point is for: a caller that records its step with a stream capture and may not allocate.
    After one eager call (the first call on a device looks the array's address up), the call is captured,
    replayed five times with eager calls of another shape in between (they share the one array), and every
    replay must reproduce the eager result bit for bit."""
    case = synth.make_case(B=2, Hq=8, Hkv=8, D=128, Smax=2048, seed=9800, seq_lens=[2048, 1500])
    synth.plant_keys(case, 1, 36.0, seed=9801)
    other = synth.make_case(B=1, Hq=16, Hkv=2, D=128, Smax=512, seed=9802, seq_lens=[400])
    dc, dco = H.DeviceCase(case, chunk=256), H.DeviceCase(other, chunk=128)
    want = oracle.attn_exact(case["q"], case["k"], case["v"], case["seq_lens"], case["scale"], nthreads=8)
    eager = run_static(dc)
    H.assert_close(eager, want, "eager")
    side = torch.cuda.Stream(device=dc.dev)
    graph = torch.cuda.CUDAGraph()
    out_g = torch.full_like(dc.out, float("nan"))
    side.wait_stream(torch.cuda.current_stream(dc.dev))
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            fdattn.fd_decode_attn_static(*dc._args(), synth.PHI, synth.BOUNDS, out_g.data_ptr(), side.cuda_stream)
    torch.cuda.synchronize(dc.dev)
    for i in range(5):
        out_g.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize(dc.dev)
        assert np.array_equal(out_g.cpu().numpy().astype(np.float64), eager), "replay %d differs from the eager call" % i
        run_static(dco)                                  # another shape through the same array between replays
    del graph
