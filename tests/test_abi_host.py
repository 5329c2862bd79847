"""Host-only checks of the C-ABI library: it loads without a GPU, exports every
symbol the header declares, sizes workspaces as documented and rejects bad
arguments before touching the device.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fdattn.h")


@pytest.fixture(scope="module")
def fdattn():
    lib = os.path.join(ROOT, "paper_2311_01282_amd", "libfdattn.so")
    if not os.path.exists(lib):          # build only if nothing is built
        from paper_2311_01282_amd import build
        build.build()
    from paper_2311_01282_amd import fdattn as mod
    return mod


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fd_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(fdattn):
    names = declared_functions()
    assert len(names) >= 10 and "fd_decode_attn" in names and "fd_decode_attn_gqa" in names
    lib = ctypes.CDLL(fdattn.LIB_PATH)
    for name in names:
        assert hasattr(lib, name), "header declares %s but the library does not export it" % name
    assert sorted(fdattn.EXPORTS) == names, "binding and header disagree on the entry points"


def test_the_read_probe_is_a_library_of_its_own(fdattn):
    """The benchmark's streaming-read kernel is no entry point of the method: libfdattn does not export
    it, libfdprobe.so does, as its own header declares."""
    from paper_2311_01282_amd import fdprobe
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "fdprobe.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(fd_[a-z_]+)\s*\(", text)))
    assert names == ["fd_probe_stream_read"]
    assert hasattr(ctypes.CDLL(fdprobe.LIB_PATH), "fd_probe_stream_read")
    assert not hasattr(ctypes.CDLL(fdattn.LIB_PATH), "fd_probe_stream_read")
    # host-side checks come before any launch
    assert ctypes.CDLL(fdprobe.LIB_PATH).fd_probe_stream_read(None, None, 65536, None, None) == 1


def test_workspace_layout_depends_on_the_slot_count_alone(fdattn):
    """Shapes with the same number of (row, chunk) slots need the same bytes, and more slots never need fewer:
    that is what lets one workspace, initialised once, serve every shape it can hold."""
    a = fdattn.fd_workspace_bytes(fdattn.make_shape(4, 8, 8, 128, 1024, 256, 0.1))      # 32 rows x 4 chunks
    b = fdattn.fd_workspace_bytes(fdattn.make_shape(1, 128, 128, 128, 256, 256, 0.1))   # 128 rows x 1 chunk
    c = fdattn.fd_workspace_bytes(fdattn.make_shape(1, 1, 1, 128, 128 * 64, 64, 0.1))   # 1 row x 128 chunks
    assert a == b == c
    sizes = [fdattn.fd_workspace_bytes(fdattn.make_shape(1, 4, 4, 128, 256 * nc, 256, 0.1)) for nc in range(1, 40)]
    assert sizes == sorted(sizes)


def test_workspace_bytes(fdattn):
    sh = fdattn.make_shape(1, 32, 32, 128, 8192, 256, 0.0884)
    n = fdattn.fd_workspace_bytes(sh)
    rows, nc = 32, 32
    # per (row, chunk) slot: numerator, denominator, reference, chunk flag, slot record, arrival counter, and the
    # per-row flag and list entry sized by slots too (so that the layout depends on the slot count alone)
    need = rows * nc * (128 * 4 + 4 + 4 + 1 + 16 + 4 + 1 + 4) + 4
    assert need <= n <= need + 16 * 256 and n % 256 == 0
    # unsupported or invalid shapes give 0
    assert fdattn.fd_workspace_bytes(fdattn.make_shape(1, 32, 32, 64, 8192, 256, 0.1)) == 0     # head_dim
    for chunk in (100, 72, 48, 4112, 0, -64):                                                  # chunk: a multiple of 16 in [64, 4096]
        assert fdattn.fd_workspace_bytes(fdattn.make_shape(1, 32, 32, 128, 8192, chunk, 0.1)) == 0
    for chunk in (64, 80, 1152, 3008, 4096):
        nc = -(-8192 // chunk)
        n = fdattn.fd_workspace_bytes(fdattn.make_shape(1, 32, 32, 128, 8192, chunk, 0.1))
        assert n >= 32 * nc * (128 * 4 + 4 + 4 + 1 + 16 + 4 + 1 + 4)
    assert fdattn.fd_workspace_bytes(fdattn.make_shape(1, 32, 5, 128, 8192, 256, 0.1)) == 0     # heads
    assert fdattn.fd_workspace_bytes(fdattn.make_shape(1, 32, 32, 128, 0, 256, 0.1)) == 0       # max_seq
    # a ragged last chunk still gets a slot
    a = fdattn.fd_workspace_bytes(fdattn.make_shape(2, 4, 4, 128, 1024, 256, 0.1))
    b = fdattn.fd_workspace_bytes(fdattn.make_shape(2, 4, 4, 128, 1025, 256, 0.1))
    assert b > a


def call(fdattn, name, shape, ptrs, phi=3.0, bounds=(-60.0, 20.0), ws=(0x1000, 1 << 30)):
    q, k, v, sl, out = ptrs
    try:
        if name == "fd_decode_attn_sync":
            fdattn.fd_decode_attn_sync(shape, q, k, v, sl, out, *ws)
        elif name == "fd_decode_attn_partial":
            fdattn.fd_decode_attn_partial(shape, q, k, v, sl, phi, bounds, *ws)
        else:
            getattr(fdattn, name)(shape, q, k, v, sl, phi, bounds, out, *ws)
    except fdattn.FdError as e:
        return e.status
    return fdattn.FD_OK


@pytest.mark.parametrize("name", ["fd_decode_attn", "fd_decode_attn_gqa", "fd_decode_attn_multikernel",
                                  "fd_decode_attn_sync", "fd_decode_attn_partial"])
def test_bad_arguments_are_rejected_before_any_launch(fdattn, name):
    """Fake but well-aligned addresses: every call must fail in host-side
    validation (nothing is enqueued, so nothing can touch these addresses)."""
    grouped = name == "fd_decode_attn_gqa"
    good = fdattn.make_shape(1, 16 if grouped else 4, 2 if grouped else 4, 128, 1024, 256, 0.0884)
    ptrs = (0x10000, 0x20000, 0x30000, 0x40000, 0x50000)
    assert call(fdattn, name, good, (0,) + ptrs[1:]) == fdattn.FD_ERR_NULL
    assert call(fdattn, name, good, ptrs[:3] + (0,) + ptrs[4:]) == fdattn.FD_ERR_NULL
    assert call(fdattn, name, good, (0x10008,) + ptrs[1:]) == fdattn.FD_ERR_SHAPE          # misaligned q
    assert call(fdattn, name, good, ptrs, ws=(0, 1 << 30)) == fdattn.FD_ERR_WORKSPACE
    assert call(fdattn, name, good, ptrs, ws=(0x1010, 1 << 30)) == fdattn.FD_ERR_WORKSPACE  # 256-byte alignment
    assert call(fdattn, name, good, ptrs, ws=(0x1000, 1024)) == fdattn.FD_ERR_WORKSPACE     # too small
    bad_dim = fdattn.make_shape(1, 16 if grouped else 4, 2 if grouped else 4, 64, 1024, 256, 0.0884)
    assert call(fdattn, name, bad_dim, ptrs) == fdattn.FD_ERR_UNSUPPORTED
    bad_heads = fdattn.make_shape(1, 5, 2, 128, 1024, 256, 0.0884)
    assert call(fdattn, name, bad_heads, ptrs) == fdattn.FD_ERR_SHAPE
    if name not in ("fd_decode_attn_sync",):
        assert call(fdattn, name, good, ptrs, bounds=(5.0, 5.0)) == fdattn.FD_ERR_BOUNDS
        assert call(fdattn, name, good, ptrs, bounds=(float("nan"), 5.0)) == fdattn.FD_ERR_BOUNDS
        assert call(fdattn, name, good, ptrs, phi=float("inf")) == fdattn.FD_ERR_BOUNDS
    if name != "fd_decode_attn_partial" and name != "fd_decode_attn_sync":
        pass
    if name in ("fd_decode_attn", "fd_decode_attn_gqa", "fd_decode_attn_multikernel", "fd_decode_attn_sync"):
        assert call(fdattn, name, good, ptrs[:4] + (0,)) == fdattn.FD_ERR_NULL               # out


def test_static_entry_point_rejects_on_the_host(fdattn):
    """fd_decode_attn_static: every host-visible problem, its size limit included, is reported before the
    device is touched (there is none here)."""
    ptrs = (0x10000, 0x20000, 0x30000, 0x40000, 0x50000)
    def go(shape, p=ptrs, phi=3.0, bounds=(-60.0, 20.0)):
        try:
            fdattn.fd_decode_attn_static(shape, p[0], p[1], p[2], p[3], phi, bounds, p[4])
        except fdattn.FdError as e:
            return e.status
        return fdattn.FD_OK
    good = fdattn.make_shape(1, 4, 4, 128, 1024, 256, 0.0884)
    assert go(good, (0,) + ptrs[1:]) == fdattn.FD_ERR_NULL
    assert go(good, ptrs[:4] + (0,)) == fdattn.FD_ERR_NULL
    assert go(good, (0x10008,) + ptrs[1:]) == fdattn.FD_ERR_SHAPE
    assert go(good, bounds=(5.0, 5.0)) == fdattn.FD_ERR_BOUNDS
    assert go(good, phi=float("nan")) == fdattn.FD_ERR_BOUNDS
    assert go(fdattn.make_shape(1, 4, 4, 64, 1024, 256, 0.0884)) == fdattn.FD_ERR_UNSUPPORTED
    assert go(fdattn.make_shape(1, 5, 2, 128, 1024, 256, 0.0884)) == fdattn.FD_ERR_SHAPE
    # the limit: the shape's workspace must fit the library's static array
    too_big = fdattn.make_shape(64, 32, 32, 128, 32768, 64, 0.0884)
    assert fdattn.fd_workspace_bytes(too_big) > fdattn.FD_STATIC_SCRATCH_BYTES
    assert go(too_big) == fdattn.FD_ERR_STATIC_LIMIT
    assert "FD_STATIC_SCRATCH_BYTES" in fdattn.status_str(fdattn.FD_ERR_STATIC_LIMIT)
    text = open(HEADER).read()
    assert re.search(r"#define\s+FD_STATIC_SCRATCH_BYTES\s+\(8u << 20\)", text) and fdattn.FD_STATIC_SCRATCH_BYTES == 8 << 20
    # the benchmark workloads fit at their picked chunk sizes
    from paper_2311_01282_amd import synth
    for name, cfg in synth.CONFIGS.items():
        sh = fdattn.make_shape(cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["D"], cfg["Smax"], 0, 0.1)
        sh.chunk = cfg["chunk"] if name.startswith("c0") else fdattn.fd_pick_chunk(sh)
        assert 0 < fdattn.fd_workspace_bytes(sh) <= fdattn.FD_STATIC_SCRATCH_BYTES, name


def test_gqa_entry_point_needs_a_group(fdattn):
    ptrs = (0x10000, 0x20000, 0x30000, 0x40000, 0x50000)
    ungrouped = fdattn.make_shape(1, 4, 4, 128, 1024, 256, 0.0884)
    assert call(fdattn, "fd_decode_attn_gqa", ungrouped, ptrs) == fdattn.FD_ERR_UNSUPPORTED
    too_wide = fdattn.make_shape(1, 32, 1, 128, 1024, 256, 0.0884)
    assert call(fdattn, "fd_decode_attn_gqa", too_wide, ptrs) == fdattn.FD_ERR_UNSUPPORTED


def test_an_empty_batch_is_a_no_op(fdattn):
    ptrs = (0x10000, 0x20000, 0x30000, 0x40000, 0x50000)
    empty = fdattn.make_shape(0, 4, 4, 128, 1024, 256, 0.0884)
    assert fdattn.fd_workspace_bytes(empty) > 0
    for name in ("fd_decode_attn", "fd_decode_attn_multikernel", "fd_decode_attn_sync", "fd_decode_attn_partial"):
        assert call(fdattn, name, empty, ptrs) == fdattn.FD_OK


def test_status_strings_and_getters(fdattn):
    for code in range(8):
        assert fdattn.status_str(code).startswith("FD_")
    assert "unknown" in fdattn.status_str(99)
    sh = fdattn.make_shape(1, 4, 4, 128, 1024, 256, 0.0884)
    n = fdattn.fd_workspace_bytes(sh)
    base = 0x7000000000
    cf, rf, cnt, lst = fdattn.fd_get_flags(sh, base, n)
    num, den = fdattn.fd_get_partials(sh, base, n)
    addrs = [num, den, cf, rf, lst, cnt]
    assert all(base <= a < base + n for a in addrs) and len(set(addrs)) == 6
    assert num == base and all(a % 256 == 0 for a in addrs)
    with pytest.raises(fdattn.FdError):
        fdattn.fd_get_flags(sh, base, 16)


def test_pick_chunk_on_the_benchmark_shapes_ignores_the_chunk_field(fdattn):
    from paper_2311_01282_amd import synth
    for name, cfg in synth.CONFIGS.items():
        picks = set()
        for chunk in (0, 64, 256, 1000):
            sh = fdattn.make_shape(cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["D"], cfg["Smax"], chunk, 0.1)
            picks.add(fdattn.fd_pick_chunk(sh))
        assert len(picks) == 1, name
        c = picks.pop()
        assert c in (64, 128, 256, 512, 1024, 2048, 4096), name     # (the benchmark shapes are powers of two)
        assert c <= 1024 or cfg["Hq"] != cfg["Hkv"], name          # long chunks are for grouped heads only
        # the picked size is accepted by the sizing call
        assert fdattn.fd_workspace_bytes(fdattn.make_shape(cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["D"], cfg["Smax"], c, 0.1)) > 0


def test_pick_chunk_fills_the_chip_when_the_shape_allows_it(fdattn):
    # one workgroup per (row or head group, chunk): at least 256 of them when any supported length gives that many
    fill = lambda w: w / (256.0 * -(-w // 256))
    for (B, Hq, Hkv, Smax) in [(1, 32, 32, 1024), (1, 32, 32, 8192), (16, 32, 32, 4096), (32, 64, 8, 4096),
                               (4, 32, 32, 32768), (1, 8, 8, 300), (1, 1, 1, 64), (3, 40, 40, 5000), (8, 64, 8, 4096),
                               (64, 64, 8, 4096), (1, 64, 8, 32768), (2, 32, 8, 8192), (48, 64, 8, 4096), (5, 40, 8, 4096),
                               (1, 32, 32, 9216), (1, 32, 32, 10000), (2, 32, 32, 5000), (8, 64, 8, 5000), (1, 64, 8, 40000),
                               (32, 64, 8, 4112), (3, 64, 8, 777)]:
        c = fdattn.fd_pick_chunk(fdattn.make_shape(B, Hq, Hkv, 128, Smax, 0, 0.1))
        units = B * (Hkv if Hq != Hkv else Hq)
        wgs = lambda cc: units * (-(-Smax // cc))
        assert 64 <= c <= 4096 and c % 16 == 0
        assert fdattn.fd_workspace_bytes(fdattn.make_shape(B, Hq, Hkv, 128, Smax, c, 0.1)) > 0
        if Hq != Hkv and wgs(c) >= 256 and c < 4096:
            # grouped: the fewest equal chunks that fill whole rounds of the chip -- one chunk fewer does not
            nb = -(-Smax // c)
            if nb > 1:
                longer = -(-(-(-Smax // (nb - 1))) // 16) * 16
                assert longer > 4096 or wgs(longer) < 256 or fill(wgs(longer)) < 0.9, (B, Hq, Hkv, Smax, c)
        if wgs(64) >= 256:
            assert wgs(c) >= 0.9 * 256, (B, Hq, Hkv, Smax, c)
            # a launch of up to four rounds of the chip fills its last round
            if wgs(c) <= 1024:
                assert fill(wgs(c)) >= 0.9, (B, Hq, Hkv, Smax, c, wgs(c))
        else:
            assert c == 64
    # the shapes the sweeps were fitted on keep their power-of-two picks; lengths between them get equal chunks
    for shape, want in (((1, 32, 32, 8192), 1024), ((32, 64, 8, 4096), 4096), ((16, 64, 8, 4096), 2048), ((8, 64, 8, 4096), 1024),
                        ((16, 32, 32, 4096), 512), ((4, 32, 32, 32768), 1024), ((1, 32, 32, 9216), 1152), ((1, 32, 32, 12288), 1536),
                        ((8, 64, 8, 5000), 1264), ((32, 64, 8, 4112), 2064),
                        # one round of the chip that is 90 % full beats two rounds when it needs at most 2/3 of the chunks
                        ((5, 64, 8, 3000), 512), ((30, 64, 8, 4096), 4096), ((1, 64, 8, 32768), 1024)):
        assert fdattn.fd_pick_chunk(fdattn.make_shape(*shape[:3], 128, shape[3], 0, 0.1)) == want, shape
    # groups of more than 16 heads run on the per-row kernel (one workgroup per query head and chunk): the pick is
    # the per-row one, not the grouped kernel's long chunks
    for (B, Hq, Hkv, Smax) in [(1, 34, 2, 8192), (4, 40, 2, 4096), (1, 64, 1, 32768), (16, 32, 1, 4096)]:
        assert Hq // Hkv > 16
        assert (fdattn.fd_pick_chunk(fdattn.make_shape(B, Hq, Hkv, 128, Smax, 0, 0.1)) ==
                fdattn.fd_pick_chunk(fdattn.make_shape(B, Hq, Hq, 128, Smax, 0, 0.1))), (B, Hq, Hkv, Smax)
    # invalid shapes give 0
    assert fdattn.fd_pick_chunk(fdattn.make_shape(1, 32, 32, 64, 8192, 256, 0.1)) == 0
    assert fdattn.fd_pick_chunk(fdattn.make_shape(1, 32, 5, 128, 8192, 256, 0.1)) == 0
