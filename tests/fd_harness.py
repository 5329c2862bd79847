"""Test-side plumbing: puts a seeded problem on the GPU and calls libfdattn
through its ctypes binding.  torch is used for device memory and the stream
only; no attention arithmetic happens here."""
import numpy as np
import torch

from paper_2311_01282_amd import fdattn, synth

ABS_TOL = 2e-3     # max |gpu - oracle| over all output elements
REL_TOL = 1e-2     # max |gpu - oracle| / max(|oracle|, REL_FLOOR)
REL_FLOOR = 1e-3   # fp16 outputs near zero cannot meet a pure ratio


class DeviceCase:
    def __init__(self, case, chunk=None, device="cuda:0"):
        self.case = case
        self.dev = torch.device(device)
        self.chunk = int(chunk or case.get("chunk", 256))
        self.q = torch.from_numpy(case["q"]).to(self.dev)
        self.k = torch.from_numpy(case["k"]).to(self.dev)
        self.v = torch.from_numpy(case["v"]).to(self.dev)
        self.seq_lens = torch.from_numpy(np.asarray(case["seq_lens"], dtype=np.int32)).to(self.dev)
        self.shape = fdattn.make_shape(case["B"], case["Hq"], case["Hkv"], case["D"], case["Smax"],
                                       self.chunk, case["scale"])
        self.rows = case["B"] * case["Hq"]
        self.nc = -(-case["Smax"] // self.chunk)
        self.ws_bytes = fdattn.fd_workspace_bytes(self.shape)
        assert self.ws_bytes > 0
        # garbage-filled so that nothing relies on a zeroed workspace
        self.ws = torch.full((self.ws_bytes,), 0xA5, dtype=torch.uint8, device=self.dev)
        fdattn.fd_workspace_init(self.shape, *self._ws(), self._stream())
        self.last_entry = None
        self.out = torch.full((case["B"], case["Hq"], case["D"]), float("nan"), dtype=torch.float16,
                              device=self.dev)

    def _stream(self):
        return torch.cuda.current_stream(self.dev).cuda_stream

    def _args(self):
        return (self.shape, self.q.data_ptr(), self.k.data_ptr(), self.v.data_ptr(), self.seq_lens.data_ptr())

    def _ws(self):
        return (self.ws.data_ptr(), self.ws_bytes)

    def run(self, entry="fd_decode_attn", phi=synth.PHI, bounds=synth.BOUNDS):
        self.out.fill_(float("nan"))
        self.last_entry = entry
        if entry == "fd_decode_attn_sync":
            fdattn.fd_decode_attn_sync(*self._args(), self.out.data_ptr(), *self._ws(), self._stream())
        else:
            getattr(fdattn, entry)(*self._args(), phi, bounds, self.out.data_ptr(), *self._ws(), self._stream())
        torch.cuda.synchronize(self.dev)
        return self.out.cpu().numpy().astype(np.float64)

    def run_partial(self, phi=synth.PHI, bounds=synth.BOUNDS):
        fdattn.fd_decode_attn_partial(*self._args(), phi, bounds, *self._ws(), self._stream())
        torch.cuda.synchronize(self.dev)

    def _view(self, addr, nbytes, dtype, shape):
        off = addr - self.ws.data_ptr()
        assert 0 <= off and off + nbytes <= self.ws_bytes
        return self.ws[off:off + nbytes].cpu().numpy().view(dtype).reshape(shape)

    def flags(self):
        """(chunk_flags [B,Hq,nc], row_flags [B,Hq], n_flagged, flagged_rows[:n_flagged])"""
        cf, rf, cnt, lst = fdattn.fd_get_flags(self.shape, *self._ws())
        B, Hq = self.case["B"], self.case["Hq"]
        chunk_flags = self._view(cf, self.rows * self.nc, np.uint8, (B, Hq, self.nc))
        row_flags = self._view(rf, self.rows, np.uint8, (B, Hq))
        if self.last_entry != "fd_decode_attn_multikernel":
            # the fused calls do not build the list themselves
            fdattn.fd_list_flagged_rows(self.shape, self.seq_lens.data_ptr(), *self._ws(), self._stream())
            torch.cuda.synchronize(self.dev)
            assert np.array_equal(row_flags, self._view(rf, self.rows, np.uint8, (B, Hq)))
        n = int(self._view(cnt, 4, np.int32, (1,))[0])
        rows = self._view(lst, 4 * self.rows, np.int32, (self.rows,))[:max(n, 0)]
        return chunk_flags, row_flags, n, rows

    def chunk_flags(self):
        cf, _, _, _ = fdattn.fd_get_flags(self.shape, *self._ws())
        return self._view(cf, self.rows * self.nc, np.uint8, (self.case["B"], self.case["Hq"], self.nc))

    def partials(self):
        num, den = fdattn.fd_get_partials(self.shape, *self._ws())
        B, Hq, D = self.case["B"], self.case["Hq"], self.case["D"]
        return (self._view(num, 4 * self.rows * self.nc * D, np.float32, (B, Hq, self.nc, D)),
                self._view(den, 4 * self.rows * self.nc, np.float32, (B, Hq, self.nc)))


def errors(got, want, rel_floor=REL_FLOOR):
    """(max abs error, max relative error with the denominator floor)"""
    diff = np.abs(got - want)
    return float(diff.max(initial=0.0)), float((diff / np.maximum(np.abs(want), rel_floor)).max(initial=0.0))


def assert_close(got, want, what="", rel_floor=REL_FLOOR):
    assert np.isfinite(got).all(), "%s: non-finite output" % what
    a, r = errors(got, want, rel_floor)
    assert a <= ABS_TOL and r <= REL_TOL, "%s: max-abs %.3e (tol %.0e), max-rel %.3e (tol %.0e)" % (
        what, a, ABS_TOL, r, REL_TOL)
    return a, r
