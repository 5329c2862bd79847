#!/usr/bin/env python3
"""Benchmark of libfdattn's decode attention on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--chunk C]

A "step" is one complete ``fd_decode_attn`` call (partial sums + range guard,
flag reduction, combine, fallback for flagged rows) on one layer's KV cache.
The benchmark cycles through ``layers`` distinct KV caches (>= 1 GiB in total)
so that no step finds its cache in the 256 MB last-level cache -- what a
multi-layer model does for every generated token.  All inputs are resident in
HBM before the clock starts.  Prints ONE JSON line.

``value`` is the effective KV-read rate of the whole call chain: valid K+V bytes
of one layer divided by the mean time per step.  ``roofline`` times the dominant
kernel (the unified-phi chunk kernel) alone with HIP events on the launch stream.
``cpu_baseline`` times the fp64 oracle on the host cores for the same layer.
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
    ap.add_argument("--steps", type=int, default=640)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--workload", default="c1_b1_h32_s8192")
    ap.add_argument("--chunk", type=int, default=0, help="0 = the workload's default")
    ap.add_argument("--layers", type=int, default=0, help="distinct KV caches to cycle through (0 = auto)")
    ap.add_argument("--entry", default="auto", choices=["auto", "fd_decode_attn", "fd_decode_attn_gqa",
                                                        "fd_decode_attn_multikernel", "fd_decode_attn_sync"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    return ap.parse_args()


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
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    cfg = dict(synth.CONFIGS[args.workload])
    chunk = args.chunk or cfg["chunk"]
    B, Hq, Hkv, D, Smax = cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["D"], cfg["Smax"]
    entry = args.entry
    if entry == "auto":
        entry = "fd_decode_attn_gqa" if Hq != Hkv else "fd_decode_attn"

    # ---- layer 0 from the seeded host generator (the oracle sees the same bits) ----
    case0 = synth.make_config(args.workload, layer=0)
    seq_lens_np = case0["seq_lens"]
    valid_keys = int(np.clip(seq_lens_np, 0, Smax).sum())
    kv_bytes = valid_keys * Hkv * D * 2 * 2           # K and V, fp16
    padded_bytes = B * Hkv * Smax * D * 2 * 2
    layers = args.layers or max(2, min(64, -(-(1 << 30) // padded_bytes)))
    if args.workload.startswith("c1"):
        layers = args.layers or 32

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
    seq_lens = torch.from_numpy(seq_lens_np).to(dev)
    shape = fdattn.make_shape(B, Hq, Hkv, D, Smax, chunk, case0["scale"])
    ws_bytes = fdattn.fd_workspace_bytes(shape)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    out = torch.empty((B, Hq, D), dtype=torch.float16, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    phi, bounds = synth.PHI, synth.BOUNDS
    fdattn.fd_workspace_init(shape, ws.data_ptr(), ws_bytes, stream)

    def step(i):
        l = i % layers
        if entry == "fd_decode_attn_sync":
            fdattn.fd_decode_attn_sync(shape, qs[l].data_ptr(), ks[l].data_ptr(), vs[l].data_ptr(),
                                       seq_lens.data_ptr(), out.data_ptr(), ws.data_ptr(), ws_bytes, stream)
        else:
            getattr(fdattn, entry)(shape, qs[l].data_ptr(), ks[l].data_ptr(), vs[l].data_ptr(),
                                   seq_lens.data_ptr(), phi, bounds, out.data_ptr(), ws.data_ptr(),
                                   ws_bytes, stream)

    def kernel_only(i):
        l = i % layers
        fdattn.fd_decode_attn_partial(shape, qs[l].data_ptr(), ks[l].data_ptr(), vs[l].data_ptr(),
                                      seq_lens.data_ptr(), phi, bounds, ws.data_ptr(), ws_bytes, stream)

    # ---- correctness of what is being timed: layer 0 against the oracle ----
    from oracle import fd_oracle
    ncpu = min(os.cpu_count() or 1, 16)
    step(0)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    t0 = time.perf_counter()
    want = fd_oracle.attn_exact(case0["q"], case0["k"], case0["v"], seq_lens_np, case0["scale"], nthreads=ncpu)
    t_cpu = time.perf_counter() - t0
    max_abs = float(np.abs(got - want).max())
    if not (max_abs <= 2e-3):
        print("bench.py: GPU result differs from the oracle (max-abs %.3e)" % max_abs, file=sys.stderr)
        return 1

    # ---- timed region: the whole call chain ----
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    sec_per_step = dt / args.steps
    value = kv_bytes / sec_per_step / 1e9

    # ---- dominant kernel alone, HIP events on the launch stream ----
    roofline = None
    if entry == "fd_decode_attn":
        kernel_only = step        # the whole method is one launch of decode_fused_kernel
        for i in range(args.warmup):
            kernel_only(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(args.steps):
            kernel_only(i)
        e1.record()
        torch.cuda.synchronize()
        k_sec = e0.elapsed_time(e1) * 1e-3 / args.steps
        achieved = kv_bytes / k_sec / 1e9
        roofline = {"bound": "hbm", "kernel": "decode_fused_kernel<%d>" % chunk,
                    "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBS, 4), "us_per_launch": round(k_sec * 1e6, 2),
                    "algorithmic_bytes_per_launch": kv_bytes, "traffic": None}

    # ---- plain streaming read of the same K and V buffers: the measured ceiling ----
    if roofline is not None and (B * Hkv * Smax * D * 2) % 65536 == 0:
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        nbytes_each = B * Hkv * Smax * D * 2

        def probe(i):
            l = i % layers
            fdattn.fd_probe_stream_read(ks[l].data_ptr(), vs[l].data_ptr(), nbytes_each, sink.data_ptr(), stream)
        for i in range(args.warmup):
            probe(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(args.steps):
            probe(i)
        e1.record()
        torch.cuda.synchronize()
        p_sec = e0.elapsed_time(e1) * 1e-3 / args.steps
        roofline["stream_read_ceiling_gbs"] = round(2 * nbytes_each / p_sec / 1e9, 1)
        roofline["frac_of_stream_read_ceiling"] = round(
            (kv_bytes / k_sec) / (2 * nbytes_each / p_sec), 4)

    cpu_baseline = None
    if not args.no_cpu_baseline:
        cpu_baseline = {"value": round(kv_bytes / t_cpu / 1e9, 4), "unit": "GB/s", "cores": ncpu,
                        "kind": "oracle", "us_per_layer_step": round(t_cpu * 1e6, 1),
                        "sample": "all %d rows of layer 0 of %s, fp64 exact attention, once" % (B * Hq, args.workload)}

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
                   "kv_bytes_per_step": kv_bytes, "layers_cycled": layers, "cache": "cold (rotating KV sets)",
                   "phi": phi, "bounds": list(bounds), "kv_dtype": "f16"},
        "parity_max_abs_vs_oracle": max_abs,
        "roofline": roofline, "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
