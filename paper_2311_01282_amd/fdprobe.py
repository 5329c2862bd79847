"""ctypes binding of libfdprobe (the benchmark's plain streaming-read kernel).

Kept apart from ``fdattn``: it measures the device, it is no part of the method.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfdprobe.so")

if not os.path.exists(LIB_PATH):
    raise ImportError("libfdprobe.so is not built: run `python -m paper_2311_01282_amd.build` first")

_lib = ctypes.CDLL(LIB_PATH)
_lib.fd_probe_stream_read.restype = ctypes.c_int
_lib.fd_probe_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]


def fd_probe_stream_read(a, b, bytes_each, sink, stream=0):
    status = _lib.fd_probe_stream_read(a, b, bytes_each, sink, stream)
    if status != 0:
        raise RuntimeError("fd_probe_stream_read: status %d" % status)
