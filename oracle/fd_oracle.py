"""ctypes loader for the plain-C fp64 oracle (``fd_oracle.c``).

TEST INFRASTRUCTURE ONLY: the checker the GPU path is compared against.  It is
compiled with gcc, imports nothing from the GPU package, and is never used by
the product path.  Function names and what each computes follow the C file:

* ``attn_exact``      -- softmax(s q K^T) V  (paper Section 2.2, Eq. 1)
* ``flags``           -- range guard a < x - phi < b (Section 3, "Recomputation")
* ``attn_unified``    -- Eq. 4 written out (unified scaling factor phi)
* ``attn_syncsplit``  -- Eq. 2 written out (synchronized partial softmax)
* ``softmax`` / ``softmax_pv`` -- whole-vector softmax on given logits
* ``half_to_double``  -- binary16 decoding used by all of the above
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fd_oracle.c")
_LIB = os.path.join(_HERE, "libfd_oracle.so")
# FD_ORACLE_LIB points the loader at another build of the same interface: the mutation test
# uses it to show that the pins reject oracles with planted mistakes.
_OVERRIDE = os.environ.get("FD_ORACLE_LIB")
_lib = None


def build(force=False):
    """Compile fd_oracle.c with gcc into libfd_oracle.so next to it."""
    if _OVERRIDE:
        return _OVERRIDE
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-pthread",
                           "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
    os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        c_i, c_f, c_p = ctypes.c_int, ctypes.c_float, ctypes.c_void_p
        L.fdo_half_to_double.restype = ctypes.c_double
        L.fdo_half_to_double.argtypes = [ctypes.c_uint16]
        L.fdo_softmax.restype = None
        L.fdo_softmax.argtypes = [c_p, c_i, c_p]
        L.fdo_softmax_pv.restype = None
        L.fdo_softmax_pv.argtypes = [c_p, c_p, c_i, c_i, c_p]
        L.fdo_attn_exact.restype = c_i
        L.fdo_attn_exact.argtypes = [c_p, c_p, c_p, c_p, c_i, c_i, c_i, c_i, c_i, c_f, c_p, c_p, c_i]
        L.fdo_flags.restype = c_i
        L.fdo_flags.argtypes = [c_p, c_p, c_p, c_i, c_i, c_i, c_i, c_i, c_f, c_f, c_f, c_f, c_i,
                                c_p, c_p, c_p, c_i]
        L.fdo_attn_unified.restype = c_i
        L.fdo_attn_unified.argtypes = [c_p, c_p, c_p, c_p, c_i, c_i, c_i, c_i, c_i, c_f, c_f, c_i,
                                       c_p, c_p, c_p, c_i]
        L.fdo_attn_syncsplit.restype = c_i
        L.fdo_attn_syncsplit.argtypes = [c_p, c_p, c_p, c_p, c_i, c_i, c_i, c_i, c_i, c_f, c_i, c_p,
                                         c_p, c_i]
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _f16(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.float16:
        raise TypeError("expected float16, got %s" % a.dtype)
    return a


def _shapes(q, k, v):
    B, Hq, D = q.shape
    Bk, Hkv, Smax, Dk = k.shape
    if (Bk, Dk) != (B, D) or (v is not None and v.shape != k.shape):
        raise ValueError("inconsistent shapes q%s k%s" % (q.shape, k.shape))
    return B, Hq, Hkv, D, Smax


def _check(rc, name):
    if rc != 0:
        raise ValueError("%s rejected its arguments (code %d)" % (name, rc))


def half_to_double(bits):
    return _load().fdo_half_to_double(int(bits))


def softmax(x):
    x = np.ascontiguousarray(x, dtype=np.float64)
    w = np.empty_like(x)
    _load().fdo_softmax(_ptr(x), x.shape[0], _ptr(w))
    return w


def softmax_pv(x, v):
    x = np.ascontiguousarray(x, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    n, D = v.shape
    assert x.shape == (n,)
    out = np.empty(D, dtype=np.float64)
    _load().fdo_softmax_pv(_ptr(x), _ptr(v), n, D, _ptr(out))
    return out


def attn_exact(q, k, v, seq_lens, scale, nthreads=1, return_logits=False):
    q, k, v = _f16(q), _f16(k), _f16(v)
    B, Hq, Hkv, D, Smax = _shapes(q, k, v)
    sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    out = np.zeros((B, Hq, D), dtype=np.float64)
    x = np.full((B, Hq, Smax), np.nan, dtype=np.float64) if return_logits else None
    _check(_load().fdo_attn_exact(_ptr(q), _ptr(k), _ptr(v), _ptr(sl), B, Hq, Hkv, D, Smax,
                                  float(scale), _ptr(out), _ptr(x), int(nthreads)), "fdo_attn_exact")
    return (out, x) if return_logits else out


def flags(q, k, seq_lens, scale, phi, lo, hi, chunk, nthreads=1):
    """Returns (chunk_flags [B,Hq,nchunks] u8, row_flags [B,Hq] u8, row_margin [B,Hq] f64)."""
    q, k = _f16(q), _f16(k)
    B, Hq, Hkv, D, Smax = _shapes(q, k, None)
    sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    nc = (Smax + chunk - 1) // chunk
    cf = np.zeros((B, Hq, nc), dtype=np.uint8)
    rf = np.zeros((B, Hq), dtype=np.uint8)
    mg = np.zeros((B, Hq), dtype=np.float64)
    _check(_load().fdo_flags(_ptr(q), _ptr(k), _ptr(sl), B, Hq, Hkv, D, Smax, float(scale),
                             float(phi), float(lo), float(hi), int(chunk),
                             _ptr(cf), _ptr(rf), _ptr(mg), int(nthreads)), "fdo_flags")
    return cf, rf, mg


def attn_unified(q, k, v, seq_lens, scale, phi, chunk, nthreads=1, return_partials=False):
    q, k, v = _f16(q), _f16(k), _f16(v)
    B, Hq, Hkv, D, Smax = _shapes(q, k, v)
    sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    nc = (Smax + chunk - 1) // chunk
    out = np.zeros((B, Hq, D), dtype=np.float64)
    num = np.zeros((B, Hq, nc, D), dtype=np.float64) if return_partials else None
    den = np.zeros((B, Hq, nc), dtype=np.float64) if return_partials else None
    _check(_load().fdo_attn_unified(_ptr(q), _ptr(k), _ptr(v), _ptr(sl), B, Hq, Hkv, D, Smax,
                                    float(scale), float(phi), int(chunk),
                                    _ptr(out), _ptr(num), _ptr(den), int(nthreads)), "fdo_attn_unified")
    return (out, num, den) if return_partials else out


def attn_syncsplit(q, k, v, seq_lens, scale, chunk, merge_order=None, nthreads=1):
    q, k, v = _f16(q), _f16(k), _f16(v)
    B, Hq, Hkv, D, Smax = _shapes(q, k, v)
    sl = np.ascontiguousarray(seq_lens, dtype=np.int32)
    mo = None if merge_order is None else np.ascontiguousarray(merge_order, dtype=np.int32)
    out = np.zeros((B, Hq, D), dtype=np.float64)
    _check(_load().fdo_attn_syncsplit(_ptr(q), _ptr(k), _ptr(v), _ptr(sl), B, Hq, Hkv, D, Smax,
                                      float(scale), int(chunk), _ptr(mo), _ptr(out), int(nthreads)),
           "fdo_attn_syncsplit")
    return out
