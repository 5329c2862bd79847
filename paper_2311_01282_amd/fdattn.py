"""ctypes binding of libfdattn: argument marshalling only.

Every function takes device pointers as Python ints (e.g. ``tensor.data_ptr()``)
and a ``Shape``; all arithmetic runs in the library's HIP kernels.  There is no
CPU fallback: if the compiled library is missing, importing this module raises.
Names mirror ``include/fdattn.h``.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfdattn.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libfdattn.so is not built: run `python -m paper_2311_01282_amd.build` "
        "(or __graft_entry__.build()) first; there is no fallback path")

_lib = ctypes.CDLL(LIB_PATH)

FD_OK, FD_ERR_NULL, FD_ERR_SHAPE, FD_ERR_BOUNDS, FD_ERR_WORKSPACE, FD_ERR_UNSUPPORTED, FD_ERR_HIP, FD_ERR_STATIC_LIMIT = range(8)
FD_STATIC_SCRATCH_BYTES = 8 << 20


class Shape(ctypes.Structure):
    """fd_shape"""
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("max_seq", ctypes.c_int32), ("chunk", ctypes.c_int32),
                ("scale", ctypes.c_float)]


class Bounds(ctypes.Structure):
    """fd_bounds"""
    _fields_ = [("lo", ctypes.c_float), ("hi", ctypes.c_float)]


class Workspace(ctypes.Structure):
    """fd_workspace"""
    _fields_ = [("ptr", ctypes.c_void_p), ("bytes", ctypes.c_size_t)]


class FdError(RuntimeError):
    def __init__(self, status):
        self.status = int(status)
        super().__init__(status_str(status))


_vp, _f = ctypes.c_void_p, ctypes.c_float
_sp = ctypes.POINTER(Shape)


class Calibration(ctypes.Structure):
    _fields_ = [("apply", ctypes.c_int32), ("phi", ctypes.c_float), ("bounds", Bounds),
                ("x_lo", ctypes.c_float), ("x_hi", ctypes.c_float), ("covered", ctypes.c_double)]


def _bind(lib):
    """Declare the argument and result types of every entry point on a loaded library."""
    lib.fd_workspace_bytes.restype = ctypes.c_size_t
    lib.fd_workspace_bytes.argtypes = [_sp]
    lib.fd_pick_chunk.restype = ctypes.c_int32
    lib.fd_pick_chunk.argtypes = [_sp]
    lib.fd_status_str.restype = ctypes.c_char_p
    lib.fd_status_str.argtypes = [ctypes.c_int]
    for _name in ("fd_decode_attn", "fd_decode_attn_gqa", "fd_decode_attn_multikernel"):
        getattr(lib, _name).restype = ctypes.c_int
        getattr(lib, _name).argtypes = [_sp, _vp, _vp, _vp, _vp, _f, Bounds, _vp, Workspace, _vp]
    lib.fd_decode_attn_static.restype = ctypes.c_int
    lib.fd_decode_attn_static.argtypes = [_sp, _vp, _vp, _vp, _vp, _f, Bounds, _vp, _vp]
    lib.fd_decode_attn_sync.restype = ctypes.c_int
    lib.fd_decode_attn_sync.argtypes = [_sp, _vp, _vp, _vp, _vp, _vp, Workspace, _vp]
    for _name in ("fd_decode_attn_partial", "fd_decode_attn_gqa_partial"):
        getattr(lib, _name).restype = ctypes.c_int
        getattr(lib, _name).argtypes = [_sp, _vp, _vp, _vp, _vp, _f, Bounds, Workspace, _vp]
    lib.fd_get_flags.restype = ctypes.c_int
    lib.fd_get_flags.argtypes = [_sp, Workspace] + [ctypes.POINTER(_vp)] * 4
    lib.fd_get_partials.restype = ctypes.c_int
    lib.fd_get_partials.argtypes = [_sp, Workspace] + [ctypes.POINTER(_vp)] * 2

    lib.fd_workspace_init.restype = ctypes.c_int
    lib.fd_workspace_init.argtypes = [_sp, Workspace, _vp]
    lib.fd_list_flagged_rows.restype = ctypes.c_int
    lib.fd_list_flagged_rows.argtypes = [_sp, _vp, Workspace, _vp]

    lib.fd_logit_histogram.restype = ctypes.c_int
    lib.fd_logit_histogram.argtypes = [_sp, _vp, _vp, _vp, _f, _f, ctypes.c_int32, _vp, _vp, _vp]
    lib.fd_calibrate.restype = ctypes.c_int
    lib.fd_calibrate.argtypes = [ctypes.POINTER(ctypes.c_uint64), ctypes.c_int32, _f, _f, ctypes.c_double, _f, _f,
                                  ctypes.c_int32, ctypes.POINTER(Calibration)]

    lib.fd_decode_attn_paged.restype = ctypes.c_int
    lib.fd_decode_attn_paged.argtypes = [_sp, _vp, _vp, _vp, _vp, ctypes.c_int32, ctypes.c_int32, _vp, _f, Bounds, _vp, Workspace, _vp]
    lib.fd_decode_attn_paged_append.restype = ctypes.c_int
    lib.fd_decode_attn_paged_append.argtypes = [_sp, _vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_int32, ctypes.c_int32, _vp, _f, Bounds, _vp,
                                                Workspace, _vp]
    lib.fd_decode_attn_append.restype = ctypes.c_int
    lib.fd_decode_attn_append.argtypes = [_sp, _vp, _vp, _vp, _vp, _vp, _vp, _f, Bounds, _vp, Workspace, _vp]

    lib.fd_prefill_workspace_bytes.restype = ctypes.c_size_t
    lib.fd_prefill_workspace_bytes.argtypes = [_sp]
    lib.fd_prefill_attn.restype = ctypes.c_int
    lib.fd_prefill_attn.argtypes = [_sp, _vp, _vp, _vp, _vp, _f, Bounds, _vp, Workspace, _vp]
    lib.fd_prefill_get_flags.restype = ctypes.c_int
    lib.fd_prefill_get_flags.argtypes = [_sp, Workspace, ctypes.POINTER(_vp)]
    return lib


_lib = _bind(_lib)

EXPORTS = ("fd_decode_attn_static", "fd_decode_attn_paged", "fd_decode_attn_paged_append", "fd_prefill_workspace_bytes", "fd_prefill_attn", "fd_prefill_get_flags", "fd_decode_attn_append", "fd_logit_histogram", "fd_calibrate", "fd_workspace_bytes", "fd_pick_chunk", "fd_workspace_init", "fd_decode_attn", "fd_decode_attn_gqa",
           "fd_decode_attn_multikernel", "fd_decode_attn_sync", "fd_list_flagged_rows",
           "fd_decode_attn_partial", "fd_decode_attn_gqa_partial", "fd_get_flags", "fd_get_partials",
           "fd_status_str")


def status_str(status):
    return _lib.fd_status_str(int(status)).decode()


def _check(status):
    if status != FD_OK:
        raise FdError(status)


def make_shape(batch, n_q_heads, n_kv_heads, head_dim, max_seq, chunk, scale):
    return Shape(int(batch), int(n_q_heads), int(n_kv_heads), int(head_dim), int(max_seq),
                 int(chunk), float(scale))


def fd_workspace_bytes(shape):
    return int(_lib.fd_workspace_bytes(ctypes.byref(shape)))


def fd_pick_chunk(shape):
    return int(_lib.fd_pick_chunk(ctypes.byref(shape)))


def fd_decode_attn(shape, q, k_cache, v_cache, seq_lens, phi, bounds, out, ws_ptr, ws_bytes, stream=0):
    _check(_lib.fd_decode_attn(ctypes.byref(shape), q, k_cache, v_cache, seq_lens, phi,
                               Bounds(*bounds), out, Workspace(ws_ptr, ws_bytes), stream))


def fd_decode_attn_gqa(shape, q, k_cache, v_cache, seq_lens, phi, bounds, out, ws_ptr, ws_bytes, stream=0):
    _check(_lib.fd_decode_attn_gqa(ctypes.byref(shape), q, k_cache, v_cache, seq_lens, phi,
                                   Bounds(*bounds), out, Workspace(ws_ptr, ws_bytes), stream))


def fd_decode_attn_static(shape, q, k_cache, v_cache, seq_lens, phi, bounds, out, stream=0):
    _check(_lib.fd_decode_attn_static(ctypes.byref(shape), q, k_cache, v_cache, seq_lens, phi,
                                      Bounds(*bounds), out, stream))


def fd_decode_attn_multikernel(shape, q, k_cache, v_cache, seq_lens, phi, bounds, out, ws_ptr, ws_bytes, stream=0):
    _check(_lib.fd_decode_attn_multikernel(ctypes.byref(shape), q, k_cache, v_cache, seq_lens, phi,
                                           Bounds(*bounds), out, Workspace(ws_ptr, ws_bytes), stream))


def fd_workspace_init(shape, ws_ptr, ws_bytes, stream=0):
    _check(_lib.fd_workspace_init(ctypes.byref(shape), Workspace(ws_ptr, ws_bytes), stream))


def fd_list_flagged_rows(shape, seq_lens, ws_ptr, ws_bytes, stream=0):
    _check(_lib.fd_list_flagged_rows(ctypes.byref(shape), seq_lens, Workspace(ws_ptr, ws_bytes), stream))


def fd_decode_attn_sync(shape, q, k_cache, v_cache, seq_lens, out, ws_ptr, ws_bytes, stream=0):
    _check(_lib.fd_decode_attn_sync(ctypes.byref(shape), q, k_cache, v_cache, seq_lens, out,
                                    Workspace(ws_ptr, ws_bytes), stream))


def fd_decode_attn_partial(shape, q, k_cache, v_cache, seq_lens, phi, bounds, ws_ptr, ws_bytes, stream=0):
    _check(_lib.fd_decode_attn_partial(ctypes.byref(shape), q, k_cache, v_cache, seq_lens, phi,
                                       Bounds(*bounds), Workspace(ws_ptr, ws_bytes), stream))


def fd_decode_attn_gqa_partial(shape, q, k_cache, v_cache, seq_lens, phi, bounds, ws_ptr, ws_bytes, stream=0):
    _check(_lib.fd_decode_attn_gqa_partial(ctypes.byref(shape), q, k_cache, v_cache, seq_lens, phi,
                                           Bounds(*bounds), Workspace(ws_ptr, ws_bytes), stream))


def fd_get_flags(shape, ws_ptr, ws_bytes):
    """Device addresses (ints) of chunk_flags, row_flags, n_flagged, flagged_rows."""
    outs = [ctypes.c_void_p() for _ in range(4)]
    _check(_lib.fd_get_flags(ctypes.byref(shape), Workspace(ws_ptr, ws_bytes),
                             *[ctypes.byref(o) for o in outs]))
    return tuple(o.value for o in outs)


def fd_get_partials(shape, ws_ptr, ws_bytes):
    """Device addresses (ints) of num and den."""
    outs = [ctypes.c_void_p() for _ in range(2)]
    _check(_lib.fd_get_partials(ctypes.byref(shape), Workspace(ws_ptr, ws_bytes),
                                *[ctypes.byref(o) for o in outs]))
    return tuple(o.value for o in outs)


def fd_logit_histogram(shape, q, k_cache, seq_lens, x_min, bin_width, n_bins, hist, min_max=None, stream=0):
    """hist / min_max: device pointers (n_bins + 2 uint64 / 2 floats or None)."""
    _check(_lib.fd_logit_histogram(ctypes.byref(shape), q, k_cache, seq_lens, x_min, bin_width, int(n_bins),
                                   hist, min_max, stream))


def fd_calibrate(hist, n_bins, x_min, bin_width, coverage, margin, phi_position, max_seq):
    """hist: host sequence of n_bins + 2 counts.  Returns the filled Calibration."""
    arr = (ctypes.c_uint64 * (n_bins + 2))(*[int(v) for v in hist])
    out = Calibration()
    _check(_lib.fd_calibrate(arr, int(n_bins), x_min, bin_width, coverage, margin, phi_position, int(max_seq),
                             ctypes.byref(out)))
    return out


def fd_decode_attn_append(shape, q, k_new, v_new, k_cache, v_cache, seq_lens, phi, bounds, out, ws_ptr, ws_bytes, stream=0):
    _check(_lib.fd_decode_attn_append(ctypes.byref(shape), q, k_new, v_new, k_cache, v_cache, seq_lens, phi,
                                      Bounds(*bounds), out, Workspace(ws_ptr, ws_bytes), stream))


def fd_decode_attn_paged(shape, q, k_pool, v_pool, block_table, page_size, n_pages, seq_lens, phi, bounds, out,
                         ws_ptr, ws_bytes, stream=0):
    _check(_lib.fd_decode_attn_paged(ctypes.byref(shape), q, k_pool, v_pool, block_table, page_size, n_pages, seq_lens, phi,
                                     Bounds(*bounds), out, Workspace(ws_ptr, ws_bytes), stream))


def fd_decode_attn_paged_append(shape, q, k_new, v_new, k_pool, v_pool, block_table, page_size, n_pages, seq_lens, phi, bounds,
                                out, ws_ptr, ws_bytes, stream=0):
    _check(_lib.fd_decode_attn_paged_append(ctypes.byref(shape), q, k_new, v_new, k_pool, v_pool, block_table, page_size, n_pages,
                                            seq_lens, phi, Bounds(*bounds), out, Workspace(ws_ptr, ws_bytes), stream))


def fd_prefill_workspace_bytes(shape):
    return int(_lib.fd_prefill_workspace_bytes(ctypes.byref(shape)))


def fd_prefill_attn(shape, q, k_cache, v_cache, seq_lens, phi, bounds, out, ws_ptr, ws_bytes, stream=0):
    _check(_lib.fd_prefill_attn(ctypes.byref(shape), q, k_cache, v_cache, seq_lens, phi, Bounds(*bounds), out,
                                Workspace(ws_ptr, ws_bytes), stream))


def fd_prefill_get_flags(shape, ws_ptr, ws_bytes):
    """Device address of tile_flags."""
    out = _vp()
    _check(_lib.fd_prefill_get_flags(ctypes.byref(shape), Workspace(ws_ptr, ws_bytes), ctypes.byref(out)))
    return out.value
