"""The hand-over between the workgroups of one fused launch must not depend on where the workgroups run.
The product library deals all chunks of a row to one XCD (one L2); the probe build of the library
(``libfdattn_phase.so``, -DFD_PHASE_PROBE) can deal them to eight different XCDs instead, so that every
partial result and every arrival crosses from one L2 to another.  Same inputs, both placements: the outputs
must agree bit for bit (fixed summation order) and with the oracle, over hundreds of back-to-back calls."""
import ctypes
import os

import numpy as np
import pytest
import torch

from paper_2311_01282_amd import fdattn, synth

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(fdattn.__file__))


@pytest.fixture(scope="module")
def probe_lib():
    path = os.path.join(HERE, "libfdattn_phase.so")
    if not os.path.exists(path):          # build only if nothing is built
        from paper_2311_01282_amd import build
        build.build_phase_probe()
    lib = fdattn._bind(ctypes.CDLL(path))
    lib.fd_phase_probe_scatter.restype = None
    lib.fd_phase_probe_scatter.argtypes = [ctypes.c_int]
    yield lib
    lib.fd_phase_probe_scatter(0)


@pytest.fixture(scope="module")
def H():
    import fd_harness
    return fd_harness


@pytest.mark.parametrize("B,Hq,Hkv,Smax,chunk,entry", [
    (1, 32, 32, 8192, 1024, "fd_decode_attn"),        # 8 chunks per row: one level of arrival counters, register epilogue
    (1, 32, 32, 8192, 256, "fd_decode_attn"),         # 32 chunks per row: two levels, sliced epilogue
    (2, 16, 16, 2048, 64, "fd_decode_attn"),          # 1024 workgroups, several per compute unit
    (4, 64, 8, 4096, 512, "fd_decode_attn_gqa"),      # grouped kernel, 8 chunks per head group
])
def test_outputs_do_not_depend_on_placement(oracle, H, probe_lib, B, Hq, Hkv, Smax, chunk, entry):
    cases = [synth.make_case(B=B, Hq=Hq, Hkv=Hkv, D=128, Smax=Smax, seed=9900 + l + Smax + chunk) for l in (0, 1)]
    synth.plant_keys(cases[1], 2, 36.0, seed=9950, allow_shared_kv=Hq != Hkv)      # recomputed chunks cross too
    dcs = [H.DeviceCase(c, chunk=chunk) for c in cases]
    want = [oracle.attn_exact(c["q"], c["k"], c["v"], c["seq_lens"], c["scale"], nthreads=16) for c in cases]
    fn = getattr(probe_lib, entry)
    dev = dcs[0].dev
    stream = torch.cuda.current_stream(dev).cuda_stream
    ws = fdattn.Workspace(dcs[0].ws.data_ptr(), dcs[0].ws_bytes)
    n = 300
    results = {}
    for scatter in (0, 1):
        probe_lib.fd_phase_probe_scatter(scatter)
        outs = torch.full((n,) + tuple(dcs[0].out.shape), float("nan"), dtype=torch.float16, device=dev)
        for i in range(n):
            dc = dcs[i % 2]
            st = fn(ctypes.byref(dc.shape), dc.q.data_ptr(), dc.k.data_ptr(), dc.v.data_ptr(), dc.seq_lens.data_ptr(),
                    synth.PHI, fdattn.Bounds(*synth.BOUNDS), outs[i].data_ptr(), ws, stream)
            assert st == 0
        torch.cuda.synchronize()
        results[scatter] = outs.cpu().numpy().astype(np.float64)
    probe_lib.fd_phase_probe_scatter(0)
    for i in range(2):
        H.assert_close(results[0][i], want[i], "one XCD per row, KV set %d" % i)
    for i in range(n):
        assert np.array_equal(results[0][i], results[0][i % 2]), "call %d (one XCD per row) differs from the first" % i
        assert np.array_equal(results[1][i], results[0][i % 2]), "call %d with rows spread over the XCDs differs" % i
