"""Where the time of one fused per-row decode call goes, from inside the kernel.

    python -m paper_2311_01282_amd.phase_probe [--workload c1_b1_h32_s8192] [--chunk 0] [--rounds 12]

Runs ``libfdattn_phase.so`` -- the library built with ``-DFD_PHASE_PROBE``
(``python -m paper_2311_01282_amd.build --phase-probe``; ``__graft_entry__.build()`` builds it
too) -- in which thread 0 of every workgroup of ``decode_fused_kernel`` stamps the device's
constant-rate clock (100 MHz, one tick = 10 ns) at eight points.  Each round enqueues 40
back-to-back calls over rotating KV sets (the benchmark's cold-cache protocol) and reads the
stamps of the LAST call; times are relative to the first workgroup's entry in that call.  Prints
a markdown table: per phase the earliest, median and latest workgroup (median over rounds), and
the critical path of the call.  The stamps cost a few scalar memory operations per workgroup;
the product library contains none of this.
"""
import argparse
import ctypes
import os
import statistics
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PHASES = ["kernel entered", "first block's data used", "chunk loop done", "sums reduced, stores issued",
          "stores performed", "arrival counted", "finisher: partials merged", "finisher: output performed"]
SLOTS = 8
TICK_US = 0.01


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c1_b1_h32_s8192")
    ap.add_argument("--chunk", type=int, default=0)
    ap.add_argument("--rounds", type=int, default=12)
    ap.add_argument("--calls", type=int, default=40)
    ap.add_argument("--scatter", action="store_true", help="deal the chunks of a row to eight different XCDs (every hand-over then crosses L2s)")
    ap.add_argument("--detail", action="store_true", help="also: when the workgroups finish their chunk loop, by XCD and by chunk index")
    args = ap.parse_args()

    import numpy as np
    import torch
    from paper_2311_01282_amd import fdattn, synth

    path = os.path.join(HERE, "libfdattn_phase.so")
    if not os.path.exists(path):
        raise SystemExit("libfdattn_phase.so is not built: python -m paper_2311_01282_amd.build --phase-probe")
    lib = fdattn._bind(ctypes.CDLL(path))
    lib.fd_phase_probe_read.restype = ctypes.c_int
    lib.fd_phase_probe_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
    lib.fd_phase_probe_scatter.restype = None
    lib.fd_phase_probe_scatter.argtypes = [ctypes.c_int]
    lib.fd_phase_probe_scatter(1 if args.scatter else 0)

    cfg = synth.CONFIGS[args.workload]
    B, Hq, Hkv, D, Smax = cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["D"], cfg["Smax"]
    if Hq != Hkv:
        raise SystemExit("the probe instruments the per-row kernel (n_q_heads == n_kv_heads)")
    scale = synth.default_scale(D)
    chunk = args.chunk or (cfg["chunk"] if args.workload.startswith("c0") else
                           fdattn.fd_pick_chunk(fdattn.make_shape(B, Hq, Hkv, D, Smax, 0, scale)))
    nc = -(-Smax // chunk)
    grid = 8 * ((B * Hq + 7) // 8) * nc
    if grid > 1024:
        raise SystemExit("the launch has %d workgroups: beyond 1024 the row epilogue is a launch of its own" % grid)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    layers = max(2, min(64, -(-(1 << 30) // (B * Hkv * Smax * D * 4))))
    if args.workload.startswith("c1"):
        layers = 32
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg["seed"])
    qs = [torch.randn((B, Hq, D), generator=gen, device=dev, dtype=torch.float32).half() for _ in range(layers)]
    ks = [torch.randn((B, Hkv, Smax, D), generator=gen, device=dev, dtype=torch.float32).half() for _ in range(layers)]
    vs = [torch.randn((B, Hkv, Smax, D), generator=gen, device=dev, dtype=torch.float32).half() for _ in range(layers)]
    sl = torch.full((B,), Smax, dtype=torch.int32, device=dev)
    out = torch.empty((B, Hq, D), dtype=torch.float16, device=dev)
    shape = fdattn.make_shape(B, Hq, Hkv, D, Smax, chunk, scale)
    nws = fdattn.fd_workspace_bytes(shape)
    ws = torch.empty(nws, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    W = fdattn.Workspace(ws.data_ptr(), nws)
    assert lib.fd_workspace_init(ctypes.byref(shape), W, stream) == 0

    def call(i):
        l = i % layers
        st = lib.fd_decode_attn(ctypes.byref(shape), qs[l].data_ptr(), ks[l].data_ptr(), vs[l].data_ptr(), sl.data_ptr(),
                                synth.PHI, fdattn.Bounds(*synth.BOUNDS), out.data_ptr(), W, stream)
        assert st == 0, st

    host = np.zeros(grid * SLOTS, dtype=np.uint64)
    details = []
    per_round = []          # [round][phase] -> (min, median, max) in us; plus the event time of the loop
    ev_us = []
    for r in range(args.rounds):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(args.calls):
            call(r * args.calls + i)
        e1.record()
        torch.cuda.synchronize()
        ev_us.append(e0.elapsed_time(e1) * 1e3 / args.calls)
        assert lib.fd_phase_probe_read(host.ctypes.data, host.size) == 0
        t = host.reshape(grid, SLOTS).astype(np.int64)
        t0 = t[:, 0].min()
        rel = (t - t0) * TICK_US
        finisher = t[:, 7] >= t[:, 0]          # stamps 6 and 7 are written by the finishers of this call only
        rows = []
        for ph in range(SLOTS):
            x = rel[finisher, ph] if ph >= 6 else rel[:, ph]
            rows.append((float(x.min()), float(np.median(x)), float(x.max())))
        # per-workgroup durations between consecutive phases
        d = [float(np.median(rel[:, ph] - rel[:, ph - 1])) for ph in range(1, 6)]
        df = [float(np.median(rel[finisher, 6] - rel[finisher, 5])), float(np.median(rel[finisher, 7] - rel[finisher, 6]))]
        per_round.append((rows, d + df))
        if args.detail:
            # workgroup index -> (XCD, chunk): blockIdx & 7 is the XCD, blockIdx >> 3 = chunk * groups8 + row group
            groups8 = (B * Hq + 7) // 8
            wg = np.arange(grid)
            details.append((np.array([np.median(rel[(wg & 7) == x, 3]) for x in range(8)]),
                            np.array([np.median(rel[(wg >> 3) // groups8 == c, 3]) for c in range(nc)]),
                            np.array([np.median(rel[(wg & 7) == x, 1]) for x in range(8)])))
    med = lambda xs: statistics.median(xs)
    print("workload %s, chunk %d, %d workgroups, %d rounds of %d back-to-back calls (last call of each round)%s"
          % (args.workload, chunk, grid, args.rounds, args.calls, "; chunks of a row on 8 different XCDs" if args.scatter else ""))
    print("event-timed call in the same loops: %.2f us (median of rounds)" % med(ev_us))
    print()
    print("| phase (thread 0 of each workgroup) | earliest wg, us | median wg, us | latest wg, us | median step from previous phase, us |")
    print("|---|---|---|---|---|")
    for ph in range(SLOTS):
        lo = med([pr[0][ph][0] for pr in per_round])
        mid = med([pr[0][ph][1] for pr in per_round])
        hi = med([pr[0][ph][2] for pr in per_round])
        step = "" if ph == 0 else "%.2f" % med([pr[1][ph - 1] for pr in per_round])
        print("| %d %s | %.2f | %.2f | %.2f | %s |" % (ph, PHASES[ph], lo, mid, hi, step))
    if args.detail:
        fmt = lambda a: " ".join("%.2f" % x for x in a)
        print()
        print("phase 3 (sums reduced), median over the workgroups of each XCD 0..7, us: " + fmt(np.median([d[0] for d in details], axis=0)))
        print("phase 3, median over the workgroups of each chunk index 0..%d, us: " % (nc - 1) + fmt(np.median([d[1] for d in details], axis=0)))
        print("phase 1 (first block used), median per XCD, us: " + fmt(np.median([d[2] for d in details], axis=0)))
    last = med([pr[0][7][2] for pr in per_round])
    print()
    print("in-kernel span (first entry to last output performed): %.2f us; the event-timed call adds the launch "
          "itself (dispatch before the first workgroup runs, completion after the last): %.2f us"
          % (last, med(ev_us) - last))
    return 0


if __name__ == "__main__":
    sys.exit(main())
