"""Behaviour of the C ABI beyond the arithmetic: workspace reuse across shapes and
entry points, non-default streams, back-to-back calls without synchronisation,
the flag-list and read-probe calls."""
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


def test_one_workspace_many_calls_and_shapes(oracle, H):
    """One allocation, initialised ONCE (with the smallest shape it will see), serves different
    chunk sizes, entry points and problem shapes in turn, small after large and large after small:
    the arrival counters sit at the end of the workspace whatever the shape, every call leaves them
    zero, and no shape's data sections reach another shape's counters."""
    big = synth.make_case(B=2, Hq=4, Hkv=4, D=128, Smax=2048, seed=500, seq_lens=[2048, 900])
    small = synth.make_case(B=1, Hq=8, Hkv=2, D=128, Smax=640, seed=501, seq_lens=[600])
    synth.plant_keys(big, 2, 36.0, seed=502)
    dev = torch.device("cuda:0")
    nbytes = max(fdattn.fd_workspace_bytes(fdattn.make_shape(2, 4, 4, 128, 2048, 64, big["scale"])),
                 fdattn.fd_workspace_bytes(fdattn.make_shape(1, 8, 2, 128, 640, 64, small["scale"]))) + 100   # (no multiple of 256)
    ws = torch.full((nbytes,), 0x5A, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    fdattn.fd_workspace_init(fdattn.make_shape(1, 8, 2, 128, 640, 512, small["scale"]), ws.data_ptr(), nbytes, stream)
    want = {id(big): oracle.attn_exact(big["q"], big["k"], big["v"], big["seq_lens"], big["scale"]),
            id(small): oracle.attn_exact(small["q"], small["k"], small["v"], small["seq_lens"], small["scale"])}
    dev_t = {}
    for case in (big, small):
        dev_t[id(case)] = tuple(torch.from_numpy(np.ascontiguousarray(case[n])).to(dev) for n in ("q", "k", "v")) + (
            torch.from_numpy(case["seq_lens"]).to(dev),)
    plan = [(big, "fd_decode_attn", 256), (small, "fd_decode_attn_gqa", 128), (big, "fd_decode_attn", 64),
            (small, "fd_decode_attn", 64), (big, "fd_decode_attn_multikernel", 512), (small, "fd_decode_attn_gqa", 64),
            (big, "fd_decode_attn", 1024), (big, "fd_decode_attn", 1024), (big, "fd_decode_attn_multikernel", 1024),
            (big, "fd_decode_attn_sync", 128), (small, "fd_decode_attn_gqa", 320), (big, "fd_decode_attn", 64),
            (big, "fd_decode_attn", 1024)]
    for case, entry, chunk in plan:
        q, k, v, sl = dev_t[id(case)]
        shape = fdattn.make_shape(case["B"], case["Hq"], case["Hkv"], 128, case["Smax"], chunk, case["scale"])
        assert fdattn.fd_workspace_bytes(shape) <= nbytes
        out = torch.full((case["B"], case["Hq"], 128), float("nan"), dtype=torch.float16, device=dev)
        if entry == "fd_decode_attn_sync":
            fdattn.fd_decode_attn_sync(shape, q.data_ptr(), k.data_ptr(), v.data_ptr(), sl.data_ptr(), out.data_ptr(),
                                       ws.data_ptr(), nbytes, stream)
        else:
            getattr(fdattn, entry)(shape, q.data_ptr(), k.data_ptr(), v.data_ptr(), sl.data_ptr(), synth.PHI,
                                   synth.BOUNDS, out.data_ptr(), ws.data_ptr(), nbytes, stream)
        torch.cuda.synchronize()
        H.assert_close(out.cpu().numpy().astype(np.float64), want[id(case)], "%s chunk %d" % (entry, chunk))


def test_paged_caller_changes_max_seq_and_chunk_every_step(H):
    """What the header tells a paged caller to do: pass the longest current length, rounded up to a page, as
    max_seq and pick the chunk for it -- so the shape differs from step to step on one workspace that was
    initialised once.  Sequences grow, one shrinks back (a finished request replaced by a new one)."""
    from oracle import fd_paged_oracle as po
    page, B, Hq = 64, 3, 4
    cap = 4096
    case = synth.make_case(B=B, Hq=Hq, Hkv=Hq, D=128, Smax=cap, seed=540, seq_lens=[cap, cap, cap])
    k_pool, v_pool, table = synth.to_pages(case, page, seed=541)
    dev = torch.device("cuda:0")
    q, kp, vp = (torch.from_numpy(a).to(dev) for a in (case["q"], k_pool, v_pool))
    nbytes = fdattn.fd_workspace_bytes(fdattn.make_shape(B, Hq, Hq, 128, cap, 64, case["scale"]))
    ws = torch.full((nbytes,), 0xC3, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    fdattn.fd_workspace_init(fdattn.make_shape(B, Hq, Hq, 128, cap, 64, case["scale"]), ws.data_ptr(), nbytes, stream)
    steps = [([100, 70, 10], None), ([1000, 700, 300], None), ([4096, 3000, 2000], None), ([130, 3001, 2001], None),
             ([131, 64, 1], 64), ([2500, 65, 2], 1008), ([4096, 4096, 4096], None)]
    for lens, forced_chunk in steps:
        longest = -(-max(lens) // page) * page
        chunk = forced_chunk or fdattn.fd_pick_chunk(fdattn.make_shape(B, Hq, Hq, 128, longest, 0, case["scale"]))
        chunk = min(chunk, 64 * page)
        shape = fdattn.make_shape(B, Hq, Hq, 128, longest, chunk, case["scale"])
        assert fdattn.fd_workspace_bytes(shape) <= nbytes
        tb = torch.from_numpy(np.ascontiguousarray(table[:, :longest // page])).to(dev)
        sl_np = np.asarray(lens, dtype=np.int32)
        sl = torch.from_numpy(sl_np).to(dev)
        out = torch.full((B, Hq, 128), float("nan"), dtype=torch.float16, device=dev)
        fdattn.fd_decode_attn_paged(shape, q.data_ptr(), kp.data_ptr(), vp.data_ptr(), tb.data_ptr(), page, k_pool.shape[0],
                                    sl.data_ptr(), synth.PHI, synth.BOUNDS, out.data_ptr(), ws.data_ptr(), nbytes, stream)
        torch.cuda.synchronize()
        want = po.attn_exact(case["q"], k_pool, v_pool, table, page, sl_np, case["scale"], nthreads=8)
        H.assert_close(out.cpu().numpy().astype(np.float64), want, "lengths %s, max_seq %d, chunk %d" % (lens, longest, chunk))


def test_side_stream_and_back_to_back_calls(oracle, H):
    """Calls are enqueued on the stream they are given and need no synchronisation
    between them: 20 calls on a side stream into distinct outputs, one sync at the end."""
    case = synth.make_case(B=2, Hq=4, Hkv=4, D=128, Smax=1536, seed=510, seq_lens=[1536, 1000])
    want = oracle.attn_exact(case["q"], case["k"], case["v"], case["seq_lens"], case["scale"])
    dc = H.DeviceCase(case, chunk=256)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    outs = [torch.full_like(dc.out, float("nan")) for _ in range(20)]
    with torch.cuda.stream(side):
        for o in outs:
            fdattn.fd_decode_attn(dc.shape, dc.q.data_ptr(), dc.k.data_ptr(), dc.v.data_ptr(), dc.seq_lens.data_ptr(),
                                  synth.PHI, synth.BOUNDS, o.data_ptr(), dc.ws.data_ptr(), dc.ws_bytes, side.cuda_stream)
    side.synchronize()
    first = outs[0].cpu().numpy()
    H.assert_close(first.astype(np.float64), want, "side stream")
    for o in outs[1:]:
        assert np.array_equal(o.cpu().numpy(), first)      # fixed summation order: same bits every time


def test_flag_list_call_and_read_probe(oracle, H):
    case = synth.make_case(B=2, Hq=4, Hkv=4, D=128, Smax=1024, seed=520)
    planted = synth.plant_keys(case, 3, 36.0, seed=521)
    dc = H.DeviceCase(case, chunk=128)
    dc.run("fd_decode_attn")
    cf, rf, n, rows = dc.flags()                       # runs fd_list_flagged_rows
    assert n == 3 and rows.tolist() == sorted(b * 4 + h for b, h, _ in planted)
    assert rf.reshape(-1)[rows].all() and rf.sum() == 3
    # the probe only reads; it must accept the K and V buffers and reject odd sizes
    sink = torch.zeros(1, dtype=torch.int32, device=dc.dev)
    nbytes = dc.k.numel() * 2
    from paper_2311_01282_amd import fdprobe
    fdprobe.fd_probe_stream_read(dc.k.data_ptr(), dc.v.data_ptr(), nbytes, sink.data_ptr(), 0)
    torch.cuda.synchronize()
    with pytest.raises(RuntimeError):
        fdprobe.fd_probe_stream_read(dc.k.data_ptr(), dc.v.data_ptr(), nbytes - 2, sink.data_ptr(), 0)


@pytest.mark.parametrize("Smax,lens,chunk", [(100, [100], 256), (64, [1], 64), (300, [299], 1024), (4097, [4097], 512)])
def test_odd_sizes(oracle, H, Smax, lens, chunk):
    """Padded lengths that are no multiple of the chunk, a cache shorter than one chunk."""
    case = synth.make_case(B=1, Hq=3, Hkv=3, D=128, Smax=Smax, seed=530 + Smax, seq_lens=lens, poison_padding=True)
    want = oracle.attn_exact(case["q"], case["k"], case["v"], case["seq_lens"], case["scale"])
    dc = H.DeviceCase(case, chunk=chunk)
    for entry in ("fd_decode_attn", "fd_decode_attn_multikernel", "fd_decode_attn_sync"):
        H.assert_close(dc.run(entry), want, entry)


def test_hand_over_is_stable_over_many_calls(oracle, H):
    """The single-launch kernel hands partial results between workgroups of one launch.
    600 back-to-back calls on the 8K shape, alternating two KV caches, must reproduce
    the first results bit for bit (a stale read of a partial result would not)."""
    cases = [synth.make_config("c1_b1_h32_s8192", layer=l) for l in (0, 1)]
    dcs = [H.DeviceCase(c, chunk=1024) for c in cases]
    ref = [dc.run("fd_decode_attn") for dc in dcs]
    for c, r in zip(cases, ref):
        H.assert_close(r, oracle.attn_exact(c["q"], c["k"], c["v"], c["seq_lens"], c["scale"], nthreads=16), "c1")
    dev = dcs[0].dev
    stream = torch.cuda.current_stream(dev).cuda_stream
    n = 600
    outs = torch.empty((n,) + tuple(dcs[0].out.shape), dtype=torch.float16, device=dev)
    for i in range(n):
        dc = dcs[i % 2]
        fdattn.fd_decode_attn(dc.shape, dc.q.data_ptr(), dc.k.data_ptr(), dc.v.data_ptr(), dc.seq_lens.data_ptr(),
                              synth.PHI, synth.BOUNDS, outs[i].data_ptr(), dcs[0].ws.data_ptr(), dcs[0].ws_bytes, stream)
    torch.cuda.synchronize()
    got = outs.cpu().numpy().astype(np.float64)
    for i in range(n):
        assert np.array_equal(got[i], ref[i % 2]), "call %d differs from the first call on the same cache" % i


def test_calls_can_be_captured_in_a_graph_and_replayed(oracle, H):
    """The calls allocate nothing, synchronise nothing and leave their arrival counters at zero, so a
    stream capture of them replays: per-row and grouped entry points, single- and two-launch grids,
    each replayed five times with eager work in between and compared with the eager result."""
    import torch
    for (B, Hq, Hkv, Smax, chunk, entry) in ((1, 32, 32, 2048, 256, "fd_decode_attn"),        # 256 workgroups: one launch
                                             (8, 32, 32, 2048, 256, "fd_decode_attn"),        # 2048: two launches
                                             (4, 64, 8, 1024, 256, "fd_decode_attn_gqa")):
        case = synth.make_case(B=B, Hq=Hq, Hkv=Hkv, D=128, Smax=Smax, seed=8800 + B)
        dc = H.DeviceCase(case, chunk=chunk)
        want = oracle.attn_exact(case["q"], case["k"], case["v"], case["seq_lens"], case["scale"], nthreads=8)
        eager = dc.run(entry)
        H.assert_close(eager, want, "eager")
        side = torch.cuda.Stream(device=dc.dev)
        graph = torch.cuda.CUDAGraph()
        out_g = torch.full_like(dc.out, float("nan"))
        side.wait_stream(torch.cuda.current_stream(dc.dev))
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                getattr(fdattn, entry)(*dc._args(), synth.PHI, synth.BOUNDS, out_g.data_ptr(), *dc._ws(), side.cuda_stream)
        torch.cuda.synchronize(dc.dev)
        for i in range(5):
            out_g.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize(dc.dev)
            got = out_g.cpu().numpy().astype(np.float64)
            assert np.array_equal(got, eager), "replay %d differs from the eager call" % i
            again = dc.run(entry)                        # eager work on the same workspace between replays
            assert np.array_equal(again, eager)
        del graph


@pytest.mark.parametrize("chunk", [1024, 128])
def test_long_context(oracle, H, chunk):
    """128K keys per row: 128 chunks per row with the in-kernel hand-over (two levels of arrival
    counters), 1024 chunks per row with the epilogue launch (its double-buffered loop)."""
    case = synth.make_case(B=1, Hq=8, Hkv=8, D=128, Smax=131072, seq_lens=[131072 - 777], seed=9100)
    want = oracle.attn_exact(case["q"], case["k"], case["v"], case["seq_lens"], case["scale"], nthreads=8)
    ocf, orf, margin = oracle.flags(case["q"], case["k"], case["seq_lens"], case["scale"], synth.PHI, *synth.BOUNDS,
                                    chunk, nthreads=8)
    assert margin.min() > 1e-2
    dc = H.DeviceCase(case, chunk=chunk)
    got = dc.run("fd_decode_attn")
    H.assert_close(got, want, "128K context, chunk %d" % chunk)
    cf, rf, n, rows = dc.flags()
    assert np.array_equal(cf, ocf) and np.array_equal(rf, orf)
    got_sync = dc.run("fd_decode_attn_sync")
    H.assert_close(got_sync, want, "128K context, synchronized scheme")
