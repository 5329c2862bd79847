"""ctypes loader for the prefill oracle (``fd_prefill_oracle.c``).

TEST INFRASTRUCTURE ONLY.  ``prefill_rows`` computes causal attention (paper
Section 2.2, Eq. 1, for all tokens of a prompt; token i attends tokens 0..i) and
the range guard of Section 3 for the listed (b, head, i) rows, in fp64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fd_prefill_oracle.c")
_LIB = os.path.join(_HERE, "libfd_prefill_oracle.so")
_OVERRIDE = os.environ.get("FD_PREFILL_ORACLE_LIB")   # another build of the same interface (mutation test)
_lib = None


def build(force=False):
    if _OVERRIDE:
        return _OVERRIDE
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    tmp = _LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-pthread", "-ffp-contract=off",
                           "-o", tmp, _SRC, "-lm"])
    os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        c_i, c_f, c_p = ctypes.c_int, ctypes.c_float, ctypes.c_void_p
        L.fdp_prefill_rows.restype = c_i
        L.fdp_prefill_rows.argtypes = [c_p, c_p, c_p, c_p, c_i, c_i, c_i, c_i, c_i, c_f, c_p, c_i, c_p,
                                       c_f, c_f, c_f, c_p, c_p, c_i]
        _lib = L
    return _lib


def _f16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float16
    return a


def all_rows(B, Hq, Smax):
    """Every (b, head, i) triple, [B*Hq*Smax, 3] int32."""
    b, h, i = np.meshgrid(np.arange(B), np.arange(Hq), np.arange(Smax), indexing="ij")
    return np.stack([b.ravel(), h.ravel(), i.ravel()], axis=1).astype(np.int32)


def prefill_rows(q, k, v, seq_lens, scale, rows, phi=0.0, lo=-1e30, hi=1e30, nthreads=1):
    """q [B,Hq,Smax,D], k/v [B,Hkv,Smax,D] fp16.  Returns (out [n,D] f64, flag [n] u8, margin [n] f64)."""
    q, k, v = _f16(q), _f16(k), _f16(v)
    B, Hq, Smax, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (B, Hkv, Smax, D) and v.shape == k.shape
    sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
    n = rows.shape[0]
    out = np.zeros((n, D), dtype=np.float64)
    flag = np.zeros(n, dtype=np.uint8)
    margin = np.zeros(n, dtype=np.float64)
    rc = _load().fdp_prefill_rows(q.ctypes.data, k.ctypes.data, v.ctypes.data, sl.ctypes.data, B, Hq, Hkv, D, Smax,
                                  float(scale), rows.ctypes.data, n, out.ctypes.data, float(phi), float(lo), float(hi),
                                  flag.ctypes.data, margin.ctypes.data, int(nthreads))
    if rc != 0:
        raise ValueError("fdp_prefill_rows: bad argument (%d)" % rc)
    return out, flag, margin
