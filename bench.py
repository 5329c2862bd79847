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

``value`` is the effective KV-read rate of the whole call: valid K+V bytes of one
layer divided by the mean time per step (``us_per_layer_step``).  ``roofline``
times the dominant kernel (the chunk kernel) alone with HIP events on the launch
stream and sets it against the HBM peak and against a plain streaming read of the
same buffers.  ``cpu_baseline`` times the fp64 oracle on the host cores.
Secondary measurements (``chunk_sweep``, ``sync_baseline``, ``overflow``) use
shorter loops of their own after the timed region.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="c1_b1_h32_s8192")
    ap.add_argument("--chunk", type=int, default=0, help="0 = the workload's default")
    ap.add_argument("--layers", type=int, default=0, help="distinct KV caches to cycle through (0 = auto)")
    ap.add_argument("--entry", default="auto", choices=["auto", "fd_decode_attn", "fd_decode_attn_gqa",
                                                        "fd_decode_attn_multikernel", "fd_decode_attn_sync"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip chunk sweep, sync baseline and overflow A/B")
    ap.add_argument("--prefill", type=int, default=0, metavar="S",
                    help="time the prompt phase instead (fd_prefill_attn): batch 1, 32 heads, prompt of S tokens")
    ap.add_argument("--prefill-heads", type=int, nargs=2, default=[32, 32], metavar=("HQ", "HKV"),
                    help="query and KV heads of the --prefill workload")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run 8 plain device copies of 256 MiB (a kernel of known traffic, for scaling "
                         "hardware counters collected over this command)")
    return ap.parse_args()


MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 / fp16 matrix-core peak


def prefill(args):
    """Prompt phase: one fd_prefill_attn call per step on a seeded synthetic prompt."""
    import numpy as np
    import torch
    from paper_2311_01282_amd import fdattn, synth
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    B, D, S = 1, 128, args.prefill
    H, Hkv = args.prefill_heads
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

    def step():
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
        print("bench.py: GPU prefill result differs from the oracle (max-abs %.3e)" % max_abs, file=sys.stderr)
        return 1
    steps, warmup = max(5, args.steps // 32), max(2, args.warmup // 16)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    pairs = B * H * S * (S + 1) // 2                      # (query, key) pairs under the causal mask
    flops = 4.0 * D * pairs                               # q.k and p.v, multiply + add
    cpu_pairs = int((rows[:, 2] + 1).sum())
    line = {
        "metric": "prefill_attention_throughput", "value": round(flops / sec / 1e12, 1), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(sec * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "prefill_b1_h%d%s_s%d" % (H, "" if H == Hkv else "x%d" % Hkv, S), "entry": "fd_prefill_attn",
                   "batch": B, "n_q_heads": H, "n_kv_heads": Hkv, "head_dim": D, "prompt": S, "causal": True, "phi": synth.PHI,
                   "bounds": list(synth.BOUNDS), "kv_dtype": "f16", "launches_per_step": 2},
        "parity_max_abs_vs_oracle": max_abs,
        "roofline": {"bound": "mfma", "kernel": "prefill_kernel", "achieved": round(flops / sec / 1e12, 1),
                     "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(flops / sec / 1e12 / MFMA_PEAK_TFLOPS, 4),
                     "algorithmic_flops_per_launch": flops,
                     "note": "whole call (transpose pass + attention); useful flops 4*D per causal (query, key) pair; "
                             "the kernel issues 2x that on the matrix cores (bf16 hi+lo operands)", "traffic": None},
        "cpu_baseline": {"value": round(4.0 * D * cpu_pairs / t_cpu / 1e12, 6), "unit": "TFLOP/s", "cores": ncpu,
                         "kind": "oracle", "sample": "%d sampled query rows of the same prompt (%d query-key pairs), fp64"
                                                      % (len(rows), cpu_pairs)},
    }
    print(json.dumps(line))
    return 0


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

    cfg = dict(synth.CONFIGS[args.workload])
    B, Hq, Hkv, D, Smax = cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["D"], cfg["Smax"]
    grouped = Hq != Hkv
    entry = args.entry
    if entry == "auto":
        entry = "fd_decode_attn_gqa" if grouped else "fd_decode_attn"
    # the 1K workload's chunk is fixed at 256; elsewhere the split is the library's to choose
    # (for the 8K workload, swept over {256, 512, 1024}, that is the best of the three)
    picked = fdattn.fd_pick_chunk(fdattn.make_shape(B, Hq, Hkv, D, Smax, 0, 1.0))
    default_chunk = cfg["chunk"] if args.workload.startswith("c0") else picked
    chunk = args.chunk or default_chunk

    # ---- layer 0 from the seeded host generator (the oracle sees the same bits) ----
    case0 = synth.make_config(args.workload, layer=0)
    seq_lens_np = case0["seq_lens"]
    valid_keys = int(np.clip(seq_lens_np, 0, Smax).sum())
    kv_bytes = valid_keys * Hkv * D * 2 * 2           # K and V, fp16
    padded_bytes = B * Hkv * Smax * D * 2 * 2
    layers = args.layers or max(2, min(64, -(-(1 << 30) // padded_bytes)))
    if args.workload.startswith("c1") and not args.layers:
        layers = 32

    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg["seed"])
    qs, ks, vs = [], [], []
    for layer in range(layers):
        if layer == 0:
            qs.append(torch.from_numpy(case0["q"]).to(dev))
            ks.append(torch.from_numpy(case0["k"]).to(dev))
            vs.append(torch.from_numpy(case0["v"]).to(dev))
        else:   # same distribution, drawn on the device to keep set-up short
            qs.append(torch.randn((B, Hq, D), generator=gen, device=dev, dtype=torch.float32).half())
            ks.append(torch.randn((B, Hkv, Smax, D), generator=gen, device=dev, dtype=torch.float32).half())
            vs.append(torch.randn((B, Hkv, Smax, D), generator=gen, device=dev, dtype=torch.float32).half())
    # planted overflow keys (layer 0 has them from the host generator): same rows and
    # positions in every other layer, gamma * q / |q| computed from that layer's q
    planted = case0["planted"]
    saved_keys = []
    for layer in range(layers):
        for (b, h, pos) in planted:
            if layer > 0:
                qv = qs[layer][b, h].float()
                saved_keys.append((layer, b, h, pos, ks[layer][b, h, pos].clone()))
                ks[layer][b, h, pos] = (cfg["plant_gamma"] * qv / qv.norm()).half()
    seq_lens = torch.from_numpy(seq_lens_np).to(dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    phi, bounds = synth.PHI, synth.BOUNDS
    out = torch.empty((B, Hq, D), dtype=torch.float16, device=dev)

    class Runner:
        def __init__(self, chunk, entry):
            self.entry = entry
            self.shape = fdattn.make_shape(B, Hq, Hkv, D, Smax, chunk, case0["scale"])
            self.ws_bytes = fdattn.fd_workspace_bytes(self.shape)
            self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=dev)
            fdattn.fd_workspace_init(self.shape, self.ws.data_ptr(), self.ws_bytes, stream)
            gqa = entry == "fd_decode_attn_gqa"
            nc = -(-Smax // chunk)
            wgs = B * (Hkv if gqa else Hq) * nc
            # the library's own rule: the grouped kernel finishes its rows itself up to 256 workgroups and 8 chunks
            # per row, the per-row kernel up to 1024 workgroups; beyond, the row epilogue is a launch of its own
            self.single_launch = ((wgs <= 256 and nc <= 8) if gqa else wgs <= 1024) and entry in ("fd_decode_attn", "fd_decode_attn_gqa")

        def step(self, i):
            l = i % layers
            a = (self.shape, qs[l].data_ptr(), ks[l].data_ptr(), vs[l].data_ptr(), seq_lens.data_ptr())
            if self.entry == "fd_decode_attn_sync":
                fdattn.fd_decode_attn_sync(*a, out.data_ptr(), self.ws.data_ptr(), self.ws_bytes, stream)
            else:
                getattr(fdattn, self.entry)(*a, phi, bounds, out.data_ptr(), self.ws.data_ptr(), self.ws_bytes, stream)

        def chunk_kernel(self, i):
            l = i % layers
            f = fdattn.fd_decode_attn_gqa_partial if self.entry == "fd_decode_attn_gqa" else fdattn.fd_decode_attn_partial
            f(self.shape, qs[l].data_ptr(), ks[l].data_ptr(), vs[l].data_ptr(), seq_lens.data_ptr(), phi, bounds,
              self.ws.data_ptr(), self.ws_bytes, stream)

    def wall(fn, steps, warmup):
        for i in range(warmup):
            fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def events(fn, steps, warmup):
        for i in range(warmup):
            fn(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(steps):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / steps

    run = Runner(chunk, entry)
    if args.calibrate_copy:
        src = torch.ones(128 << 20, dtype=torch.float16, device=dev)
        dst = torch.empty_like(src)
        for _ in range(8):
            dst.copy_(src)          # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # ---- correctness of what is being timed: layer 0 against the oracle ----
    from oracle import fd_oracle
    ncpu = min(os.cpu_count() or 1, 16)
    run.step(0)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    t0 = time.perf_counter()
    want = fd_oracle.attn_exact(case0["q"], case0["k"], case0["v"], seq_lens_np, case0["scale"], nthreads=ncpu)
    t_cpu = time.perf_counter() - t0
    max_abs = float(np.abs(got - want).max())
    if not (max_abs <= 2e-3):
        print("bench.py: GPU result differs from the oracle (max-abs %.3e)" % max_abs, file=sys.stderr)
        return 1
    # diagnostic: output elements more than one fp16 unit in the last place away from the rounded oracle value
    want16 = want.astype(np.float16).astype(np.float64)
    ulp = np.maximum(np.spacing(np.abs(want).astype(np.float16)).astype(np.float64), 2.0 ** -24)
    beyond_1ulp = int((np.abs(got - want16) > ulp).sum())

    # ---- timed region: the whole call ----
    sec_per_step = wall(run.step, args.steps, args.warmup)
    value = kv_bytes / sec_per_step / 1e9

    short = max(50, args.steps // 4)
    # ---- dominant kernel alone, HIP events on the launch stream ----
    roofline = None
    if entry in ("fd_decode_attn", "fd_decode_attn_gqa"):
        # template arguments as the profiler prints them: <chunk, paged, wavefronts> for the grouped kernel,
        # <chunk, in-kernel hand-over, paged, early loads (launches of at most 256 workgroups)> for the per-row one
        grid = 8 * ((B * Hq + 7) // 8) * ((Smax + chunk - 1) // chunk)
        early = run.single_launch and grid <= 256
        kname = ("decode_fused_gqa_kernel<%d, false, 4>" % chunk if entry == "fd_decode_attn_gqa" else
                 "decode_fused_kernel<%d, %s, false, %s>" % (chunk, "true" if run.single_launch else "false",
                                                             "true" if early else "false"))
        k_sec = events(run.step if run.single_launch else run.chunk_kernel, args.steps, args.warmup)
        achieved = kv_bytes / k_sec / 1e9
        roofline = {"bound": "hbm", "kernel": kname,
                    "launch": "the whole call (single launch)" if run.single_launch else
                              "chunk kernel alone; the call adds one row-epilogue launch",
                    "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBS, 4), "us_per_launch": round(k_sec * 1e6, 2),
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
        if nbytes_each % 65536 == 0 and valid_keys == B * Smax:
            # plain streaming read of the same K and V buffers: the measured ceiling
            sink = torch.zeros(1, dtype=torch.int32, device=dev)
            from paper_2311_01282_amd import fdprobe
            p_sec = events(lambda i: fdprobe.fd_probe_stream_read(ks[i % layers].data_ptr(), vs[i % layers].data_ptr(),
                                                                  nbytes_each, sink.data_ptr(), stream),
                           short, 10)
            roofline["stream_read_ceiling_gbs"] = round(2 * nbytes_each / p_sec / 1e9, 1)
            roofline["frac_of_stream_read_ceiling"] = round((kv_bytes / k_sec) / (2 * nbytes_each / p_sec), 4)

    extras = {}
    if not args.no_extras and entry in ("fd_decode_attn", "fd_decode_attn_gqa"):
        # chunk sweep (us per layer-step of the whole call)
        sweep = {}
        for c in sorted({256, 512, 1024, chunk}):
            r = run if c == chunk else Runner(c, entry)
            sweep[str(c)] = round(wall(r.step, short, 10) * 1e6, 2)
        extras["chunk_sweep_us"] = sweep
        # the synchronized scheme on every row (Eq. 2): what the method replaces
        rs = Runner(chunk, "fd_decode_attn_sync")
        extras["sync_baseline_us"] = round(wall(rs.step, short, 10) * 1e6, 2)
        if not grouped:
            rm = Runner(chunk, "fd_decode_attn_multikernel")
            extras["multikernel_chain_us"] = round(wall(rm.step, short, 10) * 1e6, 2)
        # statistics pass of the calibration (reads K only): histogram of the scaled logits
        n_bins = 256
        hist = torch.zeros(n_bins + 2, dtype=torch.int64, device=dev)
        def stats(i):
            l = i % layers
            fdattn.fd_logit_histogram(run.shape, qs[l].data_ptr(), ks[l].data_ptr(), seq_lens.data_ptr(), -16.0, 0.125,
                                      n_bins, hist.data_ptr(), None, stream)
        t_stats = wall(stats, short, 10)
        extras["logit_histogram"] = {"us": round(t_stats * 1e6, 2), "k_bytes": kv_bytes // 2,
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
            reps = max(2, short // layers)
            for _ in range(2):
                graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                graph.replay()
            torch.cuda.synchronize()
            extras["graph_replay_us"] = round((time.perf_counter() - t0) / (reps * layers) * 1e6, 2)
            del graph
        except RuntimeError as e:                       # capture not available: report, do not fail the run
            extras["graph_replay_us"] = None
            extras["graph_replay_error"] = str(e)[:200]
        # cache-resident figure: the same KV set every call (fits the last-level cache at c0 and c1)
        extras["hot_cache_us"] = round(wall(lambda i: run.step(0), short, 10) * 1e6, 2)
        if planted:
            # overflow A/B on the same tensors: all planted keys in, then all but the first
            # row's taken out, then none left
            def unplant(keep):
                for (b, h, pos), orig in list(zip(planted, case0["planted_original_keys"]))[keep:]:
                    ks[0][b, h, pos] = torch.from_numpy(orig).to(dev)
                for (layer, b, h, pos, orig) in saved_keys:
                    if (b, h, pos) in planted[keep:]:
                        ks[layer][b, h, pos] = orig
            t_with = wall(run.step, short, 10)
            unplant(1)
            t_one = wall(run.step, short, 10)
            unplant(0)
            t_without = wall(run.step, short, 10)
            chain = None
            if not grouped:
                # the five-kernel chain with nothing flagged still enqueues its flag reduction and its
                # (empty) recomputation launches: the fixed cost of the flag machinery
                chain = round(wall(rm.step, short, 10) * 1e6, 2)
            extras["overflow"] = {"rows_flagged": len(planted), "rows": B * Hq,
                                  "chain_us_with": extras.get("multikernel_chain_us"), "chain_us_without": chain,
                                  "us_with": round(t_with * 1e6, 2), "us_with_one_row": round(t_one * 1e6, 2),
                                  "us_without": round(t_without * 1e6, 2),
                                  "overhead_pct": round(100.0 * (t_with / t_without - 1.0), 2),
                                  "overhead_one_row_pct": round(100.0 * (t_one / t_without - 1.0), 2)}

    if not args.no_extras and entry in ("fd_decode_attn", "fd_decode_attn_gqa"):
        # the same step over a paged cache: every layer's K and V cut into pages that sit at
        # seeded-random places of a pool (fd_decode_attn_paged); pages of 16 and of 256 tokens
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
            paged[str(page)] = round(wall(step_paged, short, 10) * 1e6, 2)
            # ... and with the cache update fused in (one key fewer resident; the rows go into their page)
            lens_p = torch.clamp(seq_lens - 1, min=0)
            kn_p = torch.randn((B, Hkv, D), generator=gen, device=dev, dtype=torch.float32).half()
            vn_p = torch.randn((B, Hkv, D), generator=gen, device=dev, dtype=torch.float32).half()
            def step_paged_append(i):
                l = i % layers
                fdattn.fd_decode_attn_paged_append(run.shape, qs[l].data_ptr(), kn_p.data_ptr(), vn_p.data_ptr(), kps[l].data_ptr(),
                                                   vps[l].data_ptr(), table.data_ptr(), page, B * T, lens_p.data_ptr(), phi, bounds,
                                                   out.data_ptr(), run.ws.data_ptr(), run.ws_bytes, stream)
            paged_append[str(page)] = round(wall(step_paged_append, short, 10) * 1e6, 2)
            del kps, vps
        extras["paged_us"] = paged
        extras["paged_append_us"] = paged_append

    if not args.no_extras and entry in ("fd_decode_attn", "fd_decode_attn_gqa"):
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
        extras["fused_append_us"] = round(wall(append, short, 10) * 1e6, 2)

    cpu_baseline = None
    if not args.no_cpu_baseline:
        # the oracle as it stands, on the host threads: whole layer-steps of layer 0, repeated
        # until about ten seconds of work are done
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
        "us_per_layer_step": round(sec_per_step * 1e6, 2),
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "entry": entry, "batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv,
                   "head_dim": D, "max_seq": Smax, "valid_keys": valid_keys, "chunk": chunk,
                   "chunk_source": "--chunk" if args.chunk else ("workload definition" if chunk != picked or args.workload.startswith("c0")
                                                                   else "fd_pick_chunk"),
                   "kv_bytes_per_step": kv_bytes, "layers_cycled": layers, "cache": "cold (rotating KV sets)",
                   "phi": phi, "bounds": list(bounds), "kv_dtype": "f16",
                   "launches_per_step": 1 if run.single_launch else (5 if entry == "fd_decode_attn_multikernel" else 2)},
        "parity_max_abs_vs_oracle": max_abs, "parity_elements_beyond_1_fp16_ulp": beyond_1ulp,
        "parity_elements": int(got.size),
        "device": {"name": torch.cuda.get_device_name(dev),
                   "hbm_gib": round(torch.cuda.get_device_properties(dev).total_memory / 2**30, 1),
                   "compute_units": torch.cuda.get_device_properties(dev).multi_processor_count},
        "roofline": roofline, "cpu_baseline": cpu_baseline,
    }
    line.update(extras)
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
