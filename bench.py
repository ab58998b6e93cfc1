#!/usr/bin/env python3
"""Benchmark of the MI355X decayed causal linear attention library (one GPU).

A step is one pass of the whole prefill hot path -- stage, scores, mask, intra and inter
outputs, store, state update; one column-split chunk-walk kernel where the library's automatic
choice takes it (the headline shape), else segment pre-pass, segment scan and chunk walk -- over one batch
of the headline workload: B=4, H=16, N=4096, d=128, bf16 inputs, fp32 accumulate and output,
per-head gamma_h = 1 - 2^-(5 + 3h/15), seeded synthetic q, k, v ~ N(0,1)/sqrt(d).  Inputs
are resident in HBM before the timed region.  The decode step (config 5) and the
long-context prefill (config 4) are timed in the same run and reported under "extra".

Prints ONE JSON line.  ``value`` is tokens/s (B*N per step) of the headline workload over
exactly --steps steps of plain library calls; ``ms_per_step_graph`` is the same step captured
once into a HIP graph and replayed (reported for comparison, it measured no faster).
``roofline`` is for the dominant kernel (the chunk walk), whose per-launch duration is measured
with HIP events on the launch stream; ``cpu_baseline`` is the fp64 oracle (recurrent form)
timed on this host's cores on the same workload.

The device's clocks take on the order of 100 ms of continuous work to settle (kernel durations in
a profiler trace fall steadily over the first several hundred launches), so short runs from an
idle device read 10-25 % slower.  Two things keep that out of the figures: before each timed
section the device is kept busy for --settle-ms (default 250 ms) with a plain copy kernel on
buffers of its own -- conditioning, not workload, and outside every timed region -- and the
defaults are long (1000 warm-up and 1000 timed steps).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published
FP32_VECTOR_PEAK_TFLOPS = 157.3  # MI355X fp32 vector ALUs, published (256 CUs x 4 SIMDs x 2.4 GHz x 64 flop/clk with packed fp32)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=1000)
    ap.add_argument("--settle-ms", type=float, default=250.0,
                    help="keep the device busy this long with a plain copy kernel before each timed section, "
                         "so that its clocks have settled whatever --warmup is (0 disables)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-extra", action="store_true", help="skip the config-4 and decode legs")
    ap.add_argument("--no-graph", action="store_true", help="time plain calls only (no HIP graph replay)")
    ap.add_argument("--segments", type=int, default=0, help="0 = library's choice (the shipped configuration)")
    ap.add_argument("--kernel", choices=["auto", "wide", "column-split"], default="auto",
                    help="bf16 prefill kernel (auto, the library default, picks per shape)")
    ap.add_argument("--calibrate", action="store_true",
                    help="also launch the plain 1 GiB copy kernel once (known traffic, for scaling profiler byte counters)")
    return ap.parse_args()


def alg_bytes_forward(cfg, in_bytes):
    # per token-head: q, k, v read once + fp32 output written once
    return cfg.B * cfg.H * cfg.N * cfg.d * (3 * in_bytes + 4)


def alg_flops_forward(cfg):
    # causal-exact count at chunk 64: 4 d^2 (inter + state) + 2*64*d (intra), per token-head
    return cfg.B * cfg.H * cfg.N * (4 * cfg.d * cfg.d + 2 * 64 * cfg.d)


_SETTLE = {"ms": 0.0, "fn": None}


def settle(torch):
    """Device conditioning, outside every timed region and not part of the workload: a plain copy
    kernel (64 MiB buffers, not the workload's) keeps the GPU busy until its clocks have settled."""
    if _SETTLE["ms"] <= 0 or _SETTLE["fn"] is None:
        return
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < _SETTLE["ms"]:
        for _ in range(50):
            _SETTLE["fn"]()
        torch.cuda.synchronize()


def time_eager(torch, step, steps, warmup):
    """(host-clock ms per step, HIP-event ms per step) over exactly `steps` plain calls."""
    settle(torch)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()   # on the stream the library launches on (torch's current stream)
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps


def time_graph(torch, step, steps, warmup):
    """One step captured into a HIP graph, replayed `steps` times; None if capture fails."""
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(3):
                step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        settle(torch)
        for _ in range(warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps
    except Exception as exc:  # noqa: BLE001  (fall back to the eager figure, say why)
        print(f"bench.py: HIP graph capture unavailable ({exc}); reporting eager timing", file=sys.stderr)
        return None


def kernel_times(binding, q, k, v, gamma, out, reps, segments):
    acc = [0.0, 0.0, 0.0]
    for _ in range(reps):
        _, ms = binding.leet_attn_forward_profile(q, k, v, gamma, out=out, segments=segments)
        acc = [a + m for a, m in zip(acc, ms)]
    return [a / reps for a in acc]


def load_traffic(workload, kernel):
    """HBM bytes per launch of the dominant kernel from the committed profiler summary, or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            rec = json.load(f)
        ent = rec.get(f"{workload}/{kernel}")
        return None if ent is None else ent.get("hbm_bytes_per_launch")
    except (OSError, ValueError):
        return None


def prefill_leg(torch, binding, W, cfg, dev, steps, warmup, segments, use_graph):
    q, k, v, gamma = (t.to(dev) for t in W.make_forward_inputs(cfg))
    out = torch.empty((cfg.B, cfg.H, cfg.N, cfg.d), dtype=torch.float32, device=dev)

    def step():
        binding.leet_attn_forward_ex(q, k, v, gamma, out=out, segments=segments)

    ms_eager, ms_events = time_eager(torch, step, steps, warmup)
    ms_graph = time_graph(torch, step, steps, warmup) if use_graph else None
    kms = kernel_times(binding, q, k, v, gamma, out, max(3, min(steps, 20)), segments)
    del q, k, v, out
    return ms_eager, ms_graph, kms, ms_events


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}); "
              "the path would shard over (batch, head) without communication", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2501_02573_amd import binding, workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    binding.set_bf16_kernel({"auto": binding.KERNEL_AUTO, "wide": binding.KERNEL_WIDE,
                             "column-split": binding.KERNEL_COLUMN_SPLIT}[args.kernel])

    _SETTLE["ms"] = args.settle_ms
    if args.settle_ms > 0:
        sa = torch.zeros(16 << 20, dtype=torch.float32, device=dev)
        sb = torch.empty_like(sa)
        _SETTLE["fn"] = lambda: binding.calibration_stream("copy", sa, sb, sa.numel() * 4, 4096)

    # ---------------- headline: config 3
    cfg = W.CONFIG3
    nseg3, kern3 = binding.query_plan(cfg.B, cfg.H, cfg.N, cfg.d, binding.LEET_BF16, args.segments)
    kernel_ran = "column-split" if kern3 == binding.KERNEL_COLUMN_SPLIT else "wide"
    walk_name = {"wide": "fwd_16bit_kernel<128,128,true,bf16>", "column-split": "fwd_16bit_coop_kernel<128,128,true,bf16>"}[kernel_ran]
    ms_eager, ms_graph, kms, ms_events = prefill_leg(torch, binding, W, cfg, dev, args.steps, args.warmup,
                                                     args.segments, not args.no_graph)
    ms = ms_eager
    tokens = cfg.B * cfg.N
    nbytes = alg_bytes_forward(cfg, 2)
    nflops = alg_flops_forward(cfg)
    # Duration of the dominant kernel.  With one segment the step is that one kernel, and the HIP
    # events around the timed steps give its average launch-to-launch time in the timed region
    # itself (an upper bound on its duration).  With segments the step is three kernels and the
    # walk's share comes from events around repeated launches of it, taken after the timed loops.
    single_kernel = nseg3 == 1
    walk_ms = ms_events if single_kernel else kms[2]
    result = {
        "metric": "tokens/s, chunked decayed causal linear attention forward (B4 H16 N4096 d128 bf16)",
        "value": tokens / (ms * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_ms": args.settle_ms,
        "ms_per_step": ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "H": cfg.H, "N": cfg.N, "d": cfg.d,
                   "chunk": 64, "segments": nseg3, "kernel": kernel_ran, "kernel_choice": args.kernel,
                   "launch": "eager",
                   "gamma": "1-2^-(5+3h/15)", "seed": cfg.seed, "out_dtype": "f32"},
        "ms_per_step_graph": ms_graph,
        "tflops_algorithmic": nflops / (ms * 1e-3) / 1e12,
        "mfma_peak_frac": nflops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "hbm_frac_whole_step": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "kernel_ms": {"segment_state_prepass": kms[0], "segment_scan": kms[1], "chunk_walk": walk_ms},
        "roofline": {
            "kernel": f"{walk_name} (chunk walk)",
            "bound": "hbm",
            "achieved": nbytes / (walk_ms * 1e-3) / 1e9,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": nbytes / (walk_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "traffic": load_traffic(cfg.name, kernel_ran),
            "algorithmic_bytes_per_launch": nbytes,
            "avg_launch_ms": walk_ms,
            "timed_by": ("HIP events around the timed steps (one kernel per step)" if single_kernel else
                         "HIP events around 5 back-to-back launches, 20 times, after the timed loops"),
        },
        "kernel_ms_isolated": {"note": "event-timed repeated launches after the timed loops",
                               "segment_state_prepass": kms[0], "segment_scan": kms[1], "chunk_walk": kms[2]},
    }

    if args.calibrate:
        nb = 1 << 30
        a = torch.zeros(nb // 4, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        binding.calibration_stream("copy", a, b, nb, 65536)
        torch.cuda.synchronize()
        del a, b

    # ---------------- extra legs: long context (config 4) and decode (config 5)
    if not args.no_extra:
        extra = {}
        cfg4 = W.CONFIG4
        e4, g4, kms4, _ = prefill_leg(torch, binding, W, cfg4, dev, max(5, args.steps // 2), max(2, args.warmup // 2), 0,
                                   not args.no_graph)
        ms4 = e4
        b4, f4 = alg_bytes_forward(cfg4, 2), alg_flops_forward(cfg4)
        extra["long_context"] = {
            "workload": cfg4.name, "ms_per_step": ms4, "ms_per_step_graph": g4,
            "tokens_per_s": cfg4.B * cfg4.N / (ms4 * 1e-3),
            "tflops_algorithmic": f4 / (ms4 * 1e-3) / 1e12,
            "hbm_frac_whole_step": b4 / (ms4 * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "kernel_ms": {"segment_state_prepass": kms4[0], "segment_scan": kms4[1], "chunk_walk": kms4[2]},
            "walk_hbm_frac": b4 / (kms4[2] * 1e-3) / 1e9 / HBM_PEAK_GBS,
        }

        c5 = W.CONFIG5
        state0, gamma5, steps_it = W.decode_stream(c5)
        S = state0.to(dev)
        gamma5 = gamma5.to(dev)
        qkv = [tuple(t.to(dev) for t in next(steps_it)) for _ in range(4)]
        o = torch.empty((c5.B, c5.H, c5.d), dtype=torch.float32, device=dev)
        settle(torch)
        for i in range(16):
            binding.leet_attn_decode_step(*qkv[i % 4], gamma5, S, o)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(c5.steps):
            binding.leet_attn_decode_step(*qkv[i % 4], gamma5, S, o)
        e1.record()
        torch.cuda.synchronize()
        ms5 = e0.elapsed_time(e1) / c5.steps
        b5 = c5.B * c5.H * (2 * c5.d * c5.d * 4 + 3 * c5.d * 2 + c5.d * 4)
        extra["decode"] = {
            "workload": c5.name, "us_per_step": ms5 * 1e3, "tokens_per_s": c5.B / (ms5 * 1e-3),
            "roofline": {"kernel": "decode_kernel<128,128,bf16>", "bound": "hbm",
                         "achieved": b5 / (ms5 * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": b5 / (ms5 * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "traffic": load_traffic(c5.name, "decode"),
                         "algorithmic_bytes_per_launch": b5,
                         "note": "256 back-to-back steps; the 128 MiB state fits the 256 MB Infinity Cache"},
        }
        # the same step over three distinct 128 MiB state buffers in turn (384 MiB > the 256 MB
        # Infinity Cache), so that every step streams its state from and to HBM
        cold = [S, S.clone(), S.clone()]
        for i in range(12):
            binding.leet_attn_decode_step(*qkv[i % 4], gamma5, cold[i % 3], o)
        torch.cuda.synchronize()
        e0.record()
        for i in range(c5.steps):
            binding.leet_attn_decode_step(*qkv[i % 4], gamma5, cold[i % 3], o)
        e1.record()
        torch.cuda.synchronize()
        ms5c = e0.elapsed_time(e1) / c5.steps
        binding.set_decode_store(binding.DECODE_STORE_STREAM)
        for i in range(12):
            binding.leet_attn_decode_step(*qkv[i % 4], gamma5, cold[i % 3], o)
        torch.cuda.synchronize()
        e0.record()
        for i in range(c5.steps):
            binding.leet_attn_decode_step(*qkv[i % 4], gamma5, cold[i % 3], o)
        e1.record()
        torch.cuda.synchronize()
        binding.set_decode_store(binding.DECODE_STORE_AUTO)
        ms5s = e0.elapsed_time(e1) / c5.steps
        extra["decode_cold"] = {
            "workload": c5.name + ", three state buffers in rotation (every step streams from and to HBM)",
            "default_store_policy": {"us_per_step": ms5c * 1e3, "achieved_GBps": b5 / (ms5c * 1e-3) / 1e9,
                                     "hbm_frac": b5 / (ms5c * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "streaming_stores": {"us_per_step": ms5s * 1e3, "achieved_GBps": b5 / (ms5s * 1e-3) / 1e9,
                                 "hbm_frac": b5 / (ms5s * 1e-3) / 1e9 / HBM_PEAK_GBS},
        }
        del S, qkv, o, cold

        # the two element-wise comparison kernels on the headline workload (vector ALUs only):
        # 3 multiply-adds = 5 flops per (token, rank index, value column)
        q3, k3, v3, g3 = (t.to(dev) for t in W.make_forward_inputs(cfg))
        o3 = torch.empty((cfg.B, cfg.H, cfg.N, cfg.d), dtype=torch.float32, device=dev)
        alu_flops = 5.0 * cfg.B * cfg.H * cfg.N * cfg.d * cfg.d
        extra["elementwise_methods"] = {"workload": cfg.name, "flops_per_call": alu_flops}
        for name, fn in (("row_based", binding.leet_attn_forward_recurrent), ("fleet_attention", binding.leet_attn_forward_fleet)):
            settle(torch)
            for _ in range(5):
                fn(q3, k3, v3, g3, out=o3)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(20):
                fn(q3, k3, v3, g3, out=o3)
            e1.record()
            torch.cuda.synchronize()
            ms_e = e0.elapsed_time(e1) / 20
            extra["elementwise_methods"][name] = {
                "ms_per_call": ms_e, "tokens_per_s": tokens / (ms_e * 1e-3),
                "roofline": {"kernel": "elementwise_kernel<128,128,bf16,16,%s>" % ("rank-major" if name == "fleet_attention" else "token-major"),
                             "bound": "alu", "achieved": alu_flops / (ms_e * 1e-3) / 1e12, "peak": FP32_VECTOR_PEAK_TFLOPS,
                             "unit": "TFLOP/s", "frac": alu_flops / (ms_e * 1e-3) / 1e12 / FP32_VECTOR_PEAK_TFLOPS, "traffic": None},
            }
        del q3, k3, v3, o3
        result["extra"] = extra

    # ---------------- CPU baseline: the oracle as it stands, on this host's cores
    if not args.no_cpu_baseline:
        import oracle
        qc, kc, vc, gc = W.make_forward_inputs(cfg)
        q64, k64, v64, g64 = (W.to_f64(t) for t in (qc, kc, vc, gc))
        best = None
        for _ in range(3):
            t0 = time.perf_counter()
            oracle.recurrent(q64, k64, v64, g64)
            dt = time.perf_counter() - t0
            best = dt if best is None else min(best, dt)
        result["cpu_baseline"] = {
            "value": tokens / best, "unit": "tokens/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": f"whole {cfg.name} workload, fp64 recurrent form (Alg. 1 with decay), best of 3, {best:.2f} s",
        }
        # the decode oracle on a bounded sample of config 5: 8 of its 256 steps
        import numpy as np
        c5 = W.CONFIG5
        state0, g5, it5 = W.decode_stream(c5)
        S64 = np.ascontiguousarray(W.to_f64(state0))
        g5 = W.to_f64(g5)
        sample = [tuple(W.to_f64(t) for t in next(it5)) for _ in range(8)]
        t0 = time.perf_counter()
        for q5, k5, v5 in sample:
            oracle.decode_step(q5, k5, v5, g5, S64)
        dt5 = time.perf_counter() - t0
        result["cpu_baseline"]["decode"] = {
            "value": c5.B * len(sample) / dt5, "unit": "tokens/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": f"8 of the 256 steps of {c5.name}, fp64 decode step, {dt5:.2f} s",
        }

    print(json.dumps(result))


if __name__ == "__main__":
    main()
