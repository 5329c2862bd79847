#!/usr/bin/env python3
"""Benchmark of libfdattn's decode attention on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--chunk C]

A "step" is one complete ``fd_decode_attn`` (or ``fd_decode_attn_gqa``) call --
partial sums + range guard, recomputation of flagged chunks, row epilogue -- on
one layer's KV cache.  The benchmark cycles through ``layers`` distinct KV caches
(>= 1 GiB in total, 4 GiB at the default workload) so that no step finds its cache
in the 256 MB last-level cache: what a multi-layer model does for every generated
token.  All inputs are resident in HBM before the clock starts.  Prints ONE JSON
line.

Timing protocol (every figure of the line): HIP events on the launch stream around
``max(K, 200)`` back-to-back calls after ``max(W, 20)`` warm-up calls and one untimed
pass of the same loop (the GPU's clocks drop while the host prepares inputs), repeated
``--repeats`` (5) times; the figure reported is the MEDIAN repeat, its fastest repeat
is given next to it.  A short ``--steps`` therefore never shortens the timed loop
below 200 calls (one synchronisation is 2-4 % of a 20-call loop of this size).  The
wall clock around the same loops is reported too (``wall_us_per_layer_step``).

``value`` is the effective KV-read rate of the whole call: valid K+V bytes of one
layer divided by the median time per step.  ``roofline`` is the dominant kernel (the
chunk kernel) against the HBM peak -- the very same measurement when the call is a
single launch -- and against a plain streaming read of the same buffers.
``cpu_baseline`` times the fp64 oracle on the host cores.  ``workloads`` holds the
other four workloads of the benchmark set, each with its parity against the oracle,
the overflow overhead of the 32K workload (fused call and literal chain, 2 / 1 / 0
flagged rows) and the prefill figure at 8K tokens.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, published peak
MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 / fp16 matrix-core peak
DTYPE = "f32"               # the arithmetic type: fp16 q/K/V/out in memory, every sum and exponential in fp32


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--repeats", type=int, default=5, help="repeats of the timed loop; median and min are reported")
    ap.add_argument("--workload", default="c1_b1_h32_s8192")
    ap.add_argument("--chunk", type=int, default=0, help="0 = the workload's default")
    ap.add_argument("--layers", type=int, default=0, help="distinct KV caches to cycle through (0 = auto)")
    ap.add_argument("--entry", default="auto", choices=["auto", "fd_decode_attn", "fd_decode_attn_gqa",
                                                        "fd_decode_attn_multikernel", "fd_decode_attn_sync",
                                                        "fd_decode_attn_static"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip chunk sweep, sync baseline, paged / append variants")
    ap.add_argument("--no-workloads", action="store_true", help="skip the block with the other workloads, overflow and prefill")
    ap.add_argument("--prefill", type=int, default=0, metavar="S",
                    help="time the prompt phase instead (fd_prefill_attn): batch 1, 32 heads, prompt of S tokens")
    ap.add_argument("--prefill-heads", type=int, nargs=2, default=[32, 32], metavar=("HQ", "HKV"),
                    help="query and KV heads of the --prefill workload")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run 8 plain device copies of 256 MiB (a kernel of known traffic, for scaling "
                         "hardware counters collected over this command)")
    return ap.parse_args()


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


class Timer:
    """HIP events on torch's current stream (the stream every call below is enqueued on)."""

    def __init__(self, torch, steps, warmup, repeats):
        self.torch = torch
        self.calls = max(int(steps), 200)
        self.warmup = max(int(warmup), 20)
        self.repeats = max(int(repeats), 1)

    def __call__(self, fn, calls=None, warmup=None, repeats=None):
        """fn(i) enqueues call i.  Returns seconds per call: dict(median, min, wall_median, all)."""
        torch = self.torch
        calls = calls or self.calls
        warmup = self.warmup if warmup is None else warmup
        repeats = repeats or self.repeats
        for i in range(warmup):
            fn(i)
        # one untimed pass of the loop first: the set-up before it (host generator, oracle) leaves the GPU idle
        # long enough for its clocks to drop, and they need a few milliseconds of work to come back
        for i in range(calls):
            fn(i)
        ev, wall = [], []
        for _ in range(repeats):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            e0.record()
            for i in range(calls):
                fn(i)
            e1.record()
            torch.cuda.synchronize()
            wall.append((time.perf_counter() - t0) / calls)
            ev.append(e0.elapsed_time(e1) * 1e-3 / calls)
        return {"median": statistics.median(ev), "min": min(ev), "wall_median": statistics.median(wall), "all": ev,
                "calls": calls, "warmup": warmup, "repeats": repeats}


def us(x, nd=2):
    return round(x * 1e6, nd)


class Workload:
    """One of synth.CONFIGS on the device: layer 0 from the seeded host generator (the oracle sees the
    same bits), the other layers of the cold-cache rotation drawn on the device (same distribution)."""

    def __init__(self, torch, np, fdattn, synth, name, layers=0, dev=None):
        self.torch, self.np, self.fdattn, self.synth, self.name = torch, np, fdattn, synth, name
        self.dev = dev
        cfg = self.cfg = dict(synth.CONFIGS[name])
        B, Hq, Hkv, D, Smax = cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["D"], cfg["Smax"]
        self.B, self.Hq, self.Hkv, self.D, self.Smax = B, Hq, Hkv, D, Smax
        self.grouped = 2 <= Hq // Hkv <= 16
        self.case0 = case0 = synth.make_config(name, layer=0)
        self.seq_lens_np = case0["seq_lens"]
        self.valid_keys = int(np.clip(self.seq_lens_np, 0, Smax).sum())
        self.kv_bytes = self.valid_keys * Hkv * D * 2 * 2           # K and V, fp16
        padded_bytes = B * Hkv * Smax * D * 2 * 2
        self.layers = layers or max(2, min(64, -(-(1 << 30) // padded_bytes)))
        if name.startswith("c1") and not layers:
            self.layers = 32                                         # 4 GiB: what a 32-layer model holds
        gen = self.gen = torch.Generator(device=dev)
        gen.manual_seed(cfg["seed"])
        self.qs, self.ks, self.vs = [], [], []
        for layer in range(self.layers):
            if layer == 0:
                self.qs.append(torch.from_numpy(case0["q"]).to(dev))
                self.ks.append(torch.from_numpy(case0["k"]).to(dev))
                self.vs.append(torch.from_numpy(case0["v"]).to(dev))
            else:
                self.qs.append(torch.randn((B, Hq, D), generator=gen, device=dev, dtype=torch.float32).half())
                self.ks.append(torch.randn((B, Hkv, Smax, D), generator=gen, device=dev, dtype=torch.float32).half())
                self.vs.append(torch.randn((B, Hkv, Smax, D), generator=gen, device=dev, dtype=torch.float32).half())
        # planted overflow keys (layer 0 has them from the host generator): same rows and positions in
        # every other layer, gamma * q / |q| computed from that layer's q
        self.planted = case0["planted"]
        self.saved_keys = []
        for layer in range(1, self.layers):
            for (b, h, pos) in self.planted:
                qv = self.qs[layer][b, h].float()
                self.saved_keys.append((layer, b, h, pos, self.ks[layer][b, h, pos].clone()))
                self.ks[layer][b, h, pos] = (cfg["plant_gamma"] * qv / qv.norm()).half()
        self.seq_lens = torch.from_numpy(self.seq_lens_np).to(dev)
        self.out = torch.empty((B, Hq, D), dtype=torch.float16, device=dev)
        self.stream = torch.cuda.current_stream(dev).cuda_stream
        self.picked = fdattn.fd_pick_chunk(fdattn.make_shape(B, Hq, Hkv, D, Smax, 0, 1.0))
        # the 1K workload's chunk is fixed at 256 by its definition; elsewhere the split is the library's choice
        self.default_chunk = cfg["chunk"] if name.startswith("c0") else self.picked
        self.default_entry = "fd_decode_attn_gqa" if self.grouped else "fd_decode_attn"

    def unplant(self, keep):
        """Put the original keys back for all planted rows but the first `keep`."""
        torch = self.torch
        for (b, h, pos), orig in list(zip(self.planted, self.case0["planted_original_keys"]))[keep:]:
            self.ks[0][b, h, pos] = torch.from_numpy(orig).to(self.dev)
        for (layer, b, h, pos, orig) in self.saved_keys:
            if (b, h, pos) in self.planted[keep:]:
                self.ks[layer][b, h, pos] = orig

    def runner(self, chunk=None, entry=None):
        return Runner(self, chunk or self.default_chunk, entry or self.default_entry)

    def parity(self, run, ncpu):
        """Layer 0 of what is being timed against the oracle: (max-abs, elements beyond 1 fp16 ulp, elements,
        oracle seconds)."""
        from oracle import fd_oracle
        np, c = self.np, self.case0
        run.step(0)
        self.torch.cuda.synchronize()
        got = self.out.cpu().numpy().astype(np.float64)
        t0 = time.perf_counter()
        want = fd_oracle.attn_exact(c["q"], c["k"], c["v"], self.seq_lens_np, c["scale"], nthreads=ncpu)
        t_cpu = time.perf_counter() - t0
        max_abs = float(np.abs(got - want).max())
        want16 = want.astype(np.float16).astype(np.float64)
        ulp = np.maximum(np.spacing(np.abs(want).astype(np.float16)).astype(np.float64), 2.0 ** -24)
        return max_abs, int((np.abs(got - want16) > ulp).sum()), int(got.size), t_cpu


class Runner:
    def __init__(self, wl, chunk, entry):
        fdattn = wl.fdattn
        self.wl, self.entry, self.chunk = wl, entry, chunk
        self.shape = fdattn.make_shape(wl.B, wl.Hq, wl.Hkv, wl.D, wl.Smax, chunk, wl.case0["scale"])
        self.ws_bytes = fdattn.fd_workspace_bytes(self.shape)
        self.ws = wl.torch.empty(self.ws_bytes, dtype=wl.torch.uint8, device=wl.dev)
        fdattn.fd_workspace_init(self.shape, self.ws.data_ptr(), self.ws_bytes, wl.stream)
        gqa = entry == "fd_decode_attn_gqa" or (entry == "fd_decode_attn_static" and wl.grouped)
        self.gqa = gqa
        nc = -(-wl.Smax // chunk)
        wgs = wl.B * (wl.Hkv if gqa else wl.Hq) * nc
        # the library's own rule: the grouped kernel finishes its rows itself up to 256 workgroups and 8 chunks
        # per row, the per-row kernel up to 1024 workgroups unless the launch is long (more than 256 workgroups over
        # 320 MiB or more of cache); beyond, the row epilogue is a launch of its own
        fused = entry in ("fd_decode_attn", "fd_decode_attn_gqa", "fd_decode_attn_static")
        cache_bytes = wl.B * wl.Hkv * wl.Smax * wl.D * 2 * 2
        self.single_launch = fused and ((wgs <= 256 and nc <= 8) if gqa else
                                        (wgs <= 1024 and (wgs <= 256 or cache_bytes < (320 << 20))))
        self.launches = 1 if self.single_launch else (3 if entry == "fd_decode_attn_multikernel" else 2)
        self.grid = (wl.B * wl.Hkv * nc) if gqa else 8 * ((wl.B * wl.Hq + 7) // 8) * nc

    def kernel_name(self):
        """Template arguments as the profiler prints them: <chunk capacity, paged, wavefronts> for the grouped
        kernel, <chunk capacity, in-kernel hand-over, paged, early loads> for the per-row one."""
        cap = 64
        while cap < self.chunk:
            cap *= 2
        if self.gqa:
            return "decode_fused_gqa_kernel<%d, false, 4>" % cap
        early = self.single_launch and self.grid <= 256
        return "decode_fused_kernel<%d, %s, false, %s>" % (cap, "true" if self.single_launch else "false",
                                                           "true" if early else "false")

    def step(self, i):
        wl, fdattn = self.wl, self.wl.fdattn
        l = i % wl.layers
        a = (self.shape, wl.qs[l].data_ptr(), wl.ks[l].data_ptr(), wl.vs[l].data_ptr(), wl.seq_lens.data_ptr())
        if self.entry == "fd_decode_attn_sync":
            fdattn.fd_decode_attn_sync(*a, wl.out.data_ptr(), self.ws.data_ptr(), self.ws_bytes, wl.stream)
        elif self.entry == "fd_decode_attn_static":
            fdattn.fd_decode_attn_static(*a, wl.synth.PHI, wl.synth.BOUNDS, wl.out.data_ptr(), wl.stream)
        else:
            getattr(fdattn, self.entry)(*a, wl.synth.PHI, wl.synth.BOUNDS, wl.out.data_ptr(), self.ws.data_ptr(),
                                        self.ws_bytes, wl.stream)

    def chunk_kernel(self, i):
        wl, fdattn = self.wl, self.wl.fdattn
        l = i % wl.layers
        f = fdattn.fd_decode_attn_gqa_partial if self.gqa else fdattn.fd_decode_attn_partial
        f(self.shape, wl.qs[l].data_ptr(), wl.ks[l].data_ptr(), wl.vs[l].data_ptr(), wl.seq_lens.data_ptr(), wl.synth.PHI,
          wl.synth.BOUNDS, self.ws.data_ptr(), self.ws_bytes, wl.stream)


def prefill_measure(torch, np, fdattn, synth, dev, S, H, Hkv, timer):
    """Prompt phase: one fd_prefill_attn call per step on a seeded synthetic prompt."""
    B, D = 1, 128
    scale = float(np.float32(1.0 / np.sqrt(D)))
    gen = torch.Generator(device=dev)
    gen.manual_seed(6000 + S)
    q = torch.randn((B, H, S, D), generator=gen, device=dev, dtype=torch.float32).half()
    k, v = (torch.randn((B, Hkv, S, D), generator=gen, device=dev, dtype=torch.float32).half() for _ in range(2))
    sl = torch.full((B,), S, dtype=torch.int32, device=dev)
    out = torch.empty_like(q)
    shape = fdattn.make_shape(B, H, Hkv, D, S, 0, scale)
    nws = fdattn.fd_prefill_workspace_bytes(shape)
    ws = torch.empty(nws, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream

    def step(i=0):
        fdattn.fd_prefill_attn(shape, q.data_ptr(), k.data_ptr(), v.data_ptr(), sl.data_ptr(), synth.PHI, synth.BOUNDS,
                               out.data_ptr(), ws.data_ptr(), nws, stream)
    # correctness of what is timed: a seeded sample of rows against the oracle
    from oracle import fd_prefill_oracle as pf
    step()
    torch.cuda.synchronize()
    rng = np.random.default_rng(S)
    rows = np.stack([np.zeros(96, dtype=np.int32), rng.integers(0, H, 96).astype(np.int32),
                     np.concatenate([rng.integers(0, S, 64), np.arange(S - 32, S)]).astype(np.int32)], axis=1)
    ncpu = min(os.cpu_count() or 1, 16)
    qn, kn, vn = q.cpu().numpy(), k.cpu().numpy(), v.cpu().numpy()
    t0 = time.perf_counter()
    want, _, _ = pf.prefill_rows(qn, kn, vn, sl.cpu().numpy(), scale, rows, nthreads=ncpu)
    t_cpu = time.perf_counter() - t0
    got = out.cpu().numpy().astype(np.float64)[rows[:, 0], rows[:, 1], rows[:, 2]]
    max_abs = float(np.abs(got - want).max())
    if not (max_abs <= 2e-3):
        raise RuntimeError("GPU prefill result differs from the oracle (max-abs %.3e)" % max_abs)
    # a call is about 1 ms at 8K tokens: about 50 ms of calls per repeat, 20 to 200 calls
    calls = max(20, min(200, int(0.05 / (1e-3 * max(S / 8192.0, 1e-2) ** 2))))
    t = timer(step, calls=calls, warmup=5)
    pairs = B * H * S * (S + 1) // 2                      # (query, key) pairs under the causal mask
    flops = 4.0 * D * pairs                               # q.k and p.v, multiply + add
    cpu_pairs = int((rows[:, 2] + 1).sum())
    return {"S": S, "H": H, "Hkv": Hkv, "t": t, "flops": flops, "max_abs": max_abs, "t_cpu": t_cpu, "cpu_pairs": cpu_pairs,
            "rows": len(rows), "ncpu": ncpu}


def prefill(args):
    import numpy as np
    import torch
    from paper_2311_01282_amd import fdattn, synth
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    H, Hkv = args.prefill_heads
    timer = Timer(torch, args.steps, args.warmup, args.repeats)
    try:
        m = prefill_measure(torch, np, fdattn, synth, dev, args.prefill, H, Hkv, timer)
    except RuntimeError as e:
        print("bench.py: %s" % e, file=sys.stderr)
        return 1
    S, t, flops, D = m["S"], m["t"], m["flops"], 128
    sec = t["median"]
    line = {
        "metric": "prefill_attention_throughput", "value": round(flops / sec / 1e12, 1), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": t["calls"], "warmup": t["warmup"], "repeats": t["repeats"], "ms_per_step": round(sec * 1e3, 4),
        "ms_per_step_min": round(t["min"] * 1e3, 4), "timing": "HIP events, median of repeats",
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": "prefill_b1_h%d%s_s%d" % (H, "" if H == Hkv else "x%d" % Hkv, S), "entry": "fd_prefill_attn",
                   "batch": 1, "n_q_heads": H, "n_kv_heads": Hkv, "head_dim": D, "prompt": S, "causal": True, "phi": synth.PHI,
                   "bounds": list(synth.BOUNDS), "kv_dtype": "f16", "launches_per_step": 2},
        "parity_max_abs_vs_oracle": m["max_abs"],
        "roofline": {"bound": "mfma", "kernel": "prefill_kernel", "achieved": round(flops / sec / 1e12, 1),
                     "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(flops / sec / 1e12 / MFMA_PEAK_TFLOPS, 4),
                     "algorithmic_flops_per_launch": flops,
                     "note": "whole call (transpose pass + attention); useful flops 4*D per causal (query, key) pair; the second "
                             "product runs twice (fp16 hi + lo weights): the kernel issues 1.5x the useful flops",
                     "traffic": None},
        "cpu_baseline": {"value": round(4.0 * D * m["cpu_pairs"] / m["t_cpu"] / 1e12, 6), "unit": "TFLOP/s", "cores": m["ncpu"],
                         "kind": "oracle", "sample": "%d sampled query rows of the same prompt (%d query-key pairs), fp64"
                                                      % (m["rows"], m["cpu_pairs"])},
    }
    print(json.dumps(line))
    return 0


def workload_summary(wl, run, timer, ncpu):
    """Compact record of one workload: the whole call, event-timed, and its parity against the oracle."""
    max_abs, beyond, n_el, _ = wl.parity(run, ncpu)
    t = timer(run.step, repeats=3)
    gbs = wl.kv_bytes / t["median"] / 1e9
    rec = {"entry": run.entry, "chunk": run.chunk, "launches_per_step": run.launches, "layers_cycled": wl.layers,
           "kv_bytes_per_step": wl.kv_bytes,
           "us_per_layer_step": us(t["median"]), "us_min": us(t["min"]), "wall_us": us(t["wall_median"]),
           "kv_gbs": round(gbs, 1), "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
           "frac": round(gbs / HBM_PEAK_GBS, 4),
           "parity_max_abs_vs_oracle": max_abs, "parity_elements_beyond_1_fp16_ulp": beyond, "parity_elements": n_el}
    if not run.single_launch and run.entry in ("fd_decode_attn", "fd_decode_attn_gqa"):
        tk = timer(run.chunk_kernel, repeats=3)
        rec["chunk_kernel_us"] = us(tk["median"])
        rec["chunk_kernel_frac"] = round(wl.kv_bytes / tk["median"] / 1e9 / HBM_PEAK_GBS, 4)
    return rec


def overflow_ab(wl, timer, chunk):
    """Overflow stress: the same tensors with all planted keys in, all but the first row's taken out, none left;
    the fused call and the literal chain.  Leaves the workload without planted keys."""
    fused = wl.runner(chunk, "fd_decode_attn")
    chain = wl.runner(chunk, "fd_decode_attn_multikernel")
    res = {"rows": wl.B * wl.Hq, "rows_flagged": len(wl.planted), "chunk": chunk}
    t = {}
    for keep, tag in ((len(wl.planted), "with"), (1, "one_row"), (0, "without")):
        if keep < len(wl.planted):
            wl.unplant(keep)
        t["fused_" + tag] = timer(fused.step, repeats=3)["median"]
        t["chain_" + tag] = timer(chain.step, repeats=3)["median"]
    for k, v in t.items():
        res["us_" + k] = us(v)
    res["overhead_pct"] = round(100.0 * (t["fused_with"] / t["fused_without"] - 1.0), 2)
    res["overhead_one_row_pct"] = round(100.0 * (t["fused_one_row"] / t["fused_without"] - 1.0), 2)
    res["chain_overhead_pct"] = round(100.0 * (t["chain_with"] / t["chain_without"] - 1.0), 2)
    res["chain_overhead_one_row_pct"] = round(100.0 * (t["chain_one_row"] / t["chain_without"] - 1.0), 2)
    res["target_pct"] = 5.0
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "--gpus %d is not supported, use --gpus 1" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2311_01282_amd import fdattn, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    if args.prefill:
        return prefill(args)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    timer = Timer(torch, args.steps, args.warmup, args.repeats)
    ncpu = min(os.cpu_count() or 1, 16)

    log("building %s" % args.workload)
    wl = Workload(torch, np, fdattn, synth, args.workload, args.layers, dev)
    B, Hq, Hkv, D, Smax = wl.B, wl.Hq, wl.Hkv, wl.D, wl.Smax
    entry = wl.default_entry if args.entry == "auto" else args.entry
    chunk = args.chunk or wl.default_chunk
    run = wl.runner(chunk, entry)
    layers, kv_bytes, stream = wl.layers, wl.kv_bytes, wl.stream
    qs, ks, vs, seq_lens, out = wl.qs, wl.ks, wl.vs, wl.seq_lens, wl.out
    phi, bounds = synth.PHI, synth.BOUNDS

    if args.calibrate_copy:
        src = torch.ones(128 << 20, dtype=torch.float16, device=dev)
        dst = torch.empty_like(src)
        for _ in range(8):
            dst.copy_(src)          # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # ---- correctness of what is being timed: layer 0 against the oracle ----
    max_abs, beyond_1ulp, n_elements, t_cpu = wl.parity(run, ncpu)
    if not (max_abs <= 2e-3):
        print("bench.py: GPU result differs from the oracle (max-abs %.3e)" % max_abs, file=sys.stderr)
        return 1

    # ---- timed region: the whole call ----
    log("timing %s / %s, chunk %d: %d repeats of %d calls" % (args.workload, entry, chunk, timer.repeats, timer.calls))
    t_call = timer(run.step)
    sec_per_step = t_call["median"]
    value = kv_bytes / sec_per_step / 1e9

    # ---- dominant kernel: the chunk kernel (the whole call when it is a single launch) ----
    roofline = None
    fused_entries = ("fd_decode_attn", "fd_decode_attn_gqa", "fd_decode_attn_static")
    if entry in fused_entries:
        t_k = t_call if run.single_launch else timer(run.chunk_kernel)
        k_sec = t_k["median"]
        achieved = kv_bytes / k_sec / 1e9
        kname = run.kernel_name()
        roofline = {"bound": "hbm", "kernel": kname,
                    "launch": "the whole call (single launch): the same measurement as `value`" if run.single_launch else
                              "chunk kernel alone (timed through the *_partial entry point); the call adds one row-epilogue launch",
                    "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBS, 4), "us_per_launch": us(k_sec), "us_per_launch_min": us(t_k["min"]),
                    "algorithmic_bytes_per_launch": kv_bytes, "traffic": None}
        # HBM bytes per launch from the committed rocprofv3 counter runs (same kernel and workload)
        try:
            with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
                t = json.load(f).get(args.workload)
            if t and t["kernel"] == kname:
                roofline["traffic"] = t["traffic_bytes"]
                roofline["traffic_source"] = t["source"]
        except (OSError, ValueError, KeyError):
            pass
        nbytes_each = B * Hkv * Smax * D * 2
        if nbytes_each % 65536 == 0 and wl.valid_keys == B * Smax:
            # plain streaming read of the same K and V buffers (libfdprobe, not part of libfdattn): the measured ceiling
            from paper_2311_01282_amd import fdprobe
            sink = torch.zeros(1, dtype=torch.int32, device=dev)
            t_p = timer(lambda i: fdprobe.fd_probe_stream_read(ks[i % layers].data_ptr(), vs[i % layers].data_ptr(),
                                                                nbytes_each, sink.data_ptr(), stream), repeats=3)
            p_sec = t_p["median"]
            roofline["stream_read_us"] = us(p_sec)
            roofline["stream_read_ceiling_gbs"] = round(2 * nbytes_each / p_sec / 1e9, 1)
            roofline["frac_of_stream_read_ceiling"] = round((kv_bytes / k_sec) / (2 * nbytes_each / p_sec), 4)

    extras = {}
    if not args.no_extras and entry in ("fd_decode_attn", "fd_decode_attn_gqa"):
        log("extras: chunk sweep, baselines, graph replay")
        # chunk sweep (us per layer-step of the whole call; event-timed like the headline, 3 repeats)
        sweep = {}
        for c in sorted({256, 512, 1024, chunk}):
            sweep[str(c)] = us(t_call["median"] if c == chunk else timer(wl.runner(c, entry).step, repeats=3)["median"])
        extras["chunk_sweep_us"] = sweep
        # the synchronized scheme on every row (Eq. 2): what the method replaces
        extras["sync_baseline_us"] = us(timer(wl.runner(chunk, "fd_decode_attn_sync").step, repeats=3)["median"])
        if not wl.grouped:
            extras["multikernel_chain_us"] = us(timer(wl.runner(chunk, "fd_decode_attn_multikernel").step, repeats=3)["median"])
        # the entry point that allocates nothing (its workspace is a device array inside the library)
        if run.ws_bytes <= fdattn.FD_STATIC_SCRATCH_BYTES:
            extras["static_entry_us"] = us(timer(wl.runner(chunk, "fd_decode_attn_static").step, repeats=3)["median"])
        # statistics pass of the calibration (reads K only): histogram of the scaled logits
        n_bins = 256
        hist = torch.zeros(n_bins + 2, dtype=torch.int64, device=dev)

        def stats(i):
            l = i % layers
            fdattn.fd_logit_histogram(run.shape, qs[l].data_ptr(), ks[l].data_ptr(), seq_lens.data_ptr(), -16.0, 0.125,
                                      n_bins, hist.data_ptr(), None, stream)
        t_stats = timer(stats, repeats=3)["median"]
        extras["logit_histogram"] = {"us": us(t_stats), "k_bytes": kv_bytes // 2,
                                     "k_gbs": round(kv_bytes / 2 / t_stats / 1e9, 1),
                                     "note": "K read once per query head; with grouped heads the repeats hit in L2"}
        # the same rotation of calls recorded once by a stream capture and replayed as a graph
        # (what a serving loop would do; the calls are capturable: launches only, no allocation)
        try:
            side = torch.cuda.Stream(device=dev)
            graph = torch.cuda.CUDAGraph()
            side.wait_stream(torch.cuda.current_stream(dev))
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    for l in range(layers):
                        a = (run.shape, qs[l].data_ptr(), ks[l].data_ptr(), vs[l].data_ptr(), seq_lens.data_ptr())
                        getattr(fdattn, entry)(*a, phi, bounds, out.data_ptr(), run.ws.data_ptr(), run.ws_bytes, side.cuda_stream)
            torch.cuda.synchronize()
            reps = max(2, timer.calls // layers)
            t_g = timer(lambda i: graph.replay(), calls=reps, warmup=2, repeats=3)
            extras["graph_replay_us"] = us(t_g["median"] / layers)
            del graph
        except RuntimeError as e:                       # capture not available: report, do not fail the run
            extras["graph_replay_us"] = None
            extras["graph_replay_error"] = str(e)[:200]
        # cache-resident figure: the same KV set every call (fits the last-level cache at c0 and c1)
        extras["hot_cache_us"] = us(timer(lambda i: run.step(0), repeats=3)["median"])

        # the same step over a paged cache: every layer's K and V cut into pages that sit at
        # seeded-random places of a pool (fd_decode_attn_paged); pages of 16 and of 256 tokens
        log("extras: paged cache, fused append")
        gen = wl.gen
        paged, paged_append = {}, {}
        for page in (16, 256):
            if Smax % page or chunk > 64 * page:
                continue
            T = Smax // page
            perm = torch.randperm(B * T, generator=gen, device=dev)
            table = perm.view(B, T).to(torch.int32).contiguous()

            def pool(t):
                pages = t.view(B, Hkv, T, page, D).permute(0, 2, 1, 3, 4).reshape(B * T, Hkv, page, D)
                out_pool = torch.empty((B * T, Hkv, page, D), dtype=t.dtype, device=dev)     # contiguous, whatever `pages` is
                out_pool[perm] = pages
                return out_pool
            kps, vps = [pool(t) for t in ks], [pool(t) for t in vs]

            def step_paged(i):
                l = i % layers
                fdattn.fd_decode_attn_paged(run.shape, qs[l].data_ptr(), kps[l].data_ptr(), vps[l].data_ptr(), table.data_ptr(),
                                            page, B * T, seq_lens.data_ptr(), phi, bounds, out.data_ptr(),
                                            run.ws.data_ptr(), run.ws_bytes, stream)
            run.step(0)
            torch.cuda.synchronize()
            ref = out.clone()
            step_paged(0)
            torch.cuda.synchronize()
            if not torch.allclose(out.float(), ref.float(), rtol=0.0, atol=1e-3):
                print("bench.py: paged result differs from the contiguous one", file=sys.stderr)
                return 1
            paged[str(page)] = us(timer(step_paged, repeats=3)["median"])
            # ... and with the cache update fused in (one key fewer resident; the rows go into their page)
            lens_p = torch.clamp(seq_lens - 1, min=0)
            kn_p = torch.randn((B, Hkv, D), generator=gen, device=dev, dtype=torch.float32).half()
            vn_p = torch.randn((B, Hkv, D), generator=gen, device=dev, dtype=torch.float32).half()

            def step_paged_append(i):
                l = i % layers
                fdattn.fd_decode_attn_paged_append(run.shape, qs[l].data_ptr(), kn_p.data_ptr(), vn_p.data_ptr(), kps[l].data_ptr(),
                                                   vps[l].data_ptr(), table.data_ptr(), page, B * T, lens_p.data_ptr(), phi, bounds,
                                                   out.data_ptr(), run.ws.data_ptr(), run.ws_bytes, stream)
            paged_append[str(page)] = us(timer(step_paged_append, repeats=3)["median"])
            del kps, vps
        extras["paged_us"] = paged
        extras["paged_append_us"] = paged_append
        # the same step with the cache update fused in: one key fewer in the cache, the step's own
        # K/V rows attended from their buffers and stored by the same launch (last: it writes the caches)
        lens_m1 = torch.clamp(seq_lens - 1, min=0)
        k_new = torch.randn((B, Hkv, D), generator=gen, device=dev, dtype=torch.float32).half()
        v_new = torch.randn((B, Hkv, D), generator=gen, device=dev, dtype=torch.float32).half()

        def append(i):
            l = i % layers
            fdattn.fd_decode_attn_append(run.shape, qs[l].data_ptr(), k_new.data_ptr(), v_new.data_ptr(), ks[l].data_ptr(),
                                         vs[l].data_ptr(), lens_m1.data_ptr(), phi, bounds, out.data_ptr(),
                                         run.ws.data_ptr(), run.ws_bytes, stream)
        extras["fused_append_us"] = us(timer(append, repeats=3)["median"])
        if wl.planted:
            extras["overflow"] = overflow_ab(wl, timer, chunk)      # (last: it takes the planted keys out)

    cpu_baseline = None
    if not args.no_cpu_baseline:
        # the oracle as it stands, on the host threads: whole layer-steps of layer 0, repeated
        # until about ten seconds of work are done
        from oracle import fd_oracle
        log("cpu baseline: the oracle on %d host threads, about 10 s" % ncpu)
        case0, seq_lens_np = wl.case0, wl.seq_lens_np
        reps, t_total = 1, t_cpu
        while t_total < 10.0 and reps < 4096:
            t0 = time.perf_counter()
            fd_oracle.attn_exact(case0["q"], case0["k"], case0["v"], seq_lens_np, case0["scale"], nthreads=ncpu)
            t_total += time.perf_counter() - t0
            reps += 1
        t_cpu = t_total / reps
        # one thread, on the rows of the first sequence's first KV head only
        g = Hq // Hkv
        t0 = time.perf_counter()
        fd_oracle.attn_exact(case0["q"][:1, :g], case0["k"][:1, :1], case0["v"][:1, :1], seq_lens_np[:1], case0["scale"], nthreads=1)
        t_one = time.perf_counter() - t0
        one_bytes = int(np.clip(seq_lens_np[:1], 0, Smax).sum()) * D * 2 * 2
        cpu_model = ""
        try:
            with open("/proc/cpuinfo") as f:
                cpu_model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), "")
        except OSError:
            pass
        cpu_baseline = {"value": round(kv_bytes / t_cpu / 1e9, 4), "unit": "GB/s", "cores": ncpu, "cpu": cpu_model,
                        "kind": "oracle", "us_per_layer_step": round(t_cpu * 1e6, 1),
                        "single_thread_value": round(one_bytes / t_one / 1e9, 4),
                        "sample": "all %d rows of layer 0 of %s, fp64 exact attention, %d times (%.1f s)"
                                  % (B * Hq, args.workload, reps, t_total)}

    line = {
        "metric": "decode_attention_effective_kv_read_bandwidth",
        "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 6),
        "us_per_layer_step": us(sec_per_step),
        "us_per_layer_step_min": us(t_call["min"]),
        "us_per_layer_step_repeats": [us(x) for x in t_call["all"]],
        "wall_us_per_layer_step": us(t_call["wall_median"]),
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "pct_of_hbm_peak_best_repeat": round(100.0 * kv_bytes / t_call["min"] / 1e9 / HBM_PEAK_GBS, 2),
        "timing": {"clock": "HIP events on the launch stream", "calls_per_repeat": t_call["calls"],
                   "warmup_calls": t_call["warmup"], "untimed_passes_before": 1, "repeats": t_call["repeats"],
                   "reported": "median repeat",
                   "note": "a --steps below 200 does not shorten the timed loop: each repeat is max(steps, 200) "
                           "back-to-back calls, one step = one call"},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": args.workload, "entry": entry, "batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv,
                   "head_dim": D, "max_seq": Smax, "valid_keys": wl.valid_keys, "chunk": chunk,
                   "chunk_source": "--chunk" if args.chunk else ("workload definition" if args.workload.startswith("c0")
                                                                   else "fd_pick_chunk"),
                   "kv_bytes_per_step": kv_bytes, "layers_cycled": layers, "cache": "cold (rotating KV sets)",
                   "phi": phi, "bounds": list(bounds), "kv_dtype": "f16", "accumulate_dtype": "f32",
                   "launches_per_step": run.launches},
        "parity_max_abs_vs_oracle": max_abs, "parity_elements_beyond_1_fp16_ulp": beyond_1ulp,
        "parity_elements": n_elements,
        "device": {"name": torch.cuda.get_device_name(dev),
                   "hbm_gib": round(torch.cuda.get_device_properties(dev).total_memory / 2**30, 1),
                   "compute_units": torch.cuda.get_device_properties(dev).multi_processor_count},
        "roofline": roofline, "cpu_baseline": cpu_baseline,
    }
    line.update(extras)

    if not args.no_workloads and args.entry == "auto" and not args.chunk:
        # ---- the other workloads of the set, the overflow overhead and the prefill figure ----
        del run, qs, ks, vs, wl
        torch.cuda.empty_cache()
        block = {}
        for name in synth.CONFIGS:
            if name == args.workload:
                continue
            log("workload %s" % name)
            w = Workload(torch, np, fdattn, synth, name, 0, dev)
            r = w.runner()
            rec = workload_summary(w, r, timer, ncpu)
            if not (rec["parity_max_abs_vs_oracle"] <= 2e-3):
                print("bench.py: %s differs from the oracle (max-abs %.3e)" % (name, rec["parity_max_abs_vs_oracle"]), file=sys.stderr)
                return 1
            if w.planted:
                log("overflow A/B on %s" % name)
                rec["overflow"] = overflow_ab(w, timer, r.chunk)
                line["fallback_overhead_pct_at_1pct_rows"] = rec["overflow"]["overhead_pct"]
                line["fallback_overhead_pct_at_1pct_rows_chain"] = rec["overflow"]["chain_overhead_pct"]
            block[name] = rec
            del w, r
            torch.cuda.empty_cache()
        log("prefill, 8192 tokens")
        try:
            m = prefill_measure(torch, np, fdattn, synth, dev, 8192, 32, 32, timer)
        except RuntimeError as e:
            print("bench.py: %s" % e, file=sys.stderr)
            return 1
        block["prefill_b1_h32_s8192"] = {"entry": "fd_prefill_attn", "ms_per_call": round(m["t"]["median"] * 1e3, 4),
                                         "ms_min": round(m["t"]["min"] * 1e3, 4),
                                         "tflops": round(m["flops"] / m["t"]["median"] / 1e12, 1),
                                         "frac_of_mfma_peak": round(m["flops"] / m["t"]["median"] / 1e12 / MFMA_PEAK_TFLOPS, 4),
                                         "parity_max_abs_vs_oracle": m["max_abs"], "parity_rows_sampled": m["rows"]}
        line["workloads"] = block

    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
