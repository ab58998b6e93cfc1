"""Latency versus sequence length, in the layout of the paper's single-layer tables.

``python -m paper_2501_02573_amd.latency_table [--out FILE]`` times one attention layer on
random tensors for N in {128, 512, 2048, 8192, 12800, 25600, 100000} and batch sizes 1 and 16,
with and without the decaying mask, following the protocol of Section 5.1: 15 repetitions,
mean and standard deviation, seconds.  The paper does not state heads, dimensions or dtype for
those tables; this harness uses heads = 32 and rank = dim = 128 (its usage example has
heads = 32, rank = 128) and says so in the output.

Rows are this library's methods:
  chunked bf16 / fp16 / fp32   the chunked path (block-based with decay; the role the paper's
                               lightningAttention-2 rows play), fp32 output
  chunked bf16, bf16 out       the same with 16-bit output
  row-based bf16               the token-by-token recursion (the role of causal-dot-product)
  FleetAttention bf16          the rank-sum of discounted cumulative sums (Alg. 5), element-wise
  chunked bf16, dim 256        rank 128 with value width 256, the shape of the paper's usage example
The paper's own lightningAttention-2 row (Section 5.1, decaying mask) and FleetAttention row
(Appendix E; both masks) are printed underneath: one A6000, other hardware, so context only.

PyTorch is used for device memory, random inputs and events; all arithmetic of the operator
runs in the library's kernels.
"""
from __future__ import annotations

import argparse
import math
import sys

N_LIST = (128, 512, 2048, 8192, 12800, 25600, 100000)
HEADS, DIM = 32, 128
REPS = 15

# Section 5.1, tables for batch 1 and batch 16 (seconds, one A6000, heads/dim/dtype unstated):
# row "LA" (lightningAttention-2, Triton).  None = out of memory there.
# Appendix E, runtime table of FleetAttention: row "FA" (Triton, atomic rank sum).
PAPER_ROWS = {
    # (batch, decay): {row: values over N_LIST}
    (1, True): {"LA (paper, A6000)": (1.27e-4, 1.96e-4, 7.49e-4, 2.9e-3, 4.51e-3, 9.08e-3, 4.14e-2),
                "FA (paper, A6000)": (1.26e-3, 5.49e-3, 2.71e-2, 1.14e-1, 1.78e-1, 3.59e-1, 1.42)},
    (1, False): {"FA (paper, A6000)": (1.26e-3, 5.46e-3, 2.72e-2, 1.13e-1, 1.77e-1, 3.58e-1, 1.41)},
    (16, True): {"LA (paper, A6000)": (6.52e-4, 2.57e-3, 1.05e-2, 4.28e-2, 6.49e-2, 1.34e-1, None),
                 "FA (paper, A6000)": (1.85e-2, 7.49e-2, 3.90e-1, 1.48, 2.32, 4.65, None)},
    (16, False): {"FA (paper, A6000)": (1.85e-2, 7.42e-2, 3.92e-1, 1.48, 2.31, 4.63, None)},
}


def _methods(torch, binding):
    bf16, f16, f32 = torch.bfloat16, torch.float16, torch.float32
    fwd = binding.leet_attn_forward_v2
    rec = binding.leet_attn_forward_recurrent
    flt = binding.leet_attn_forward_fleet
    frd = binding.leet_attn_forward_rd
    # (name, input dtype, output dtype, value width, call)
    return (
        ("chunked bf16", bf16, f32, DIM, lambda q, k, v, g, o, m: fwd(q, k, v, g, out=o, mask=m)),
        ("chunked fp16", f16, f32, DIM, lambda q, k, v, g, o, m: fwd(q, k, v, g, out=o, mask=m)),
        ("chunked fp32", f32, f32, DIM, lambda q, k, v, g, o, m: fwd(q, k, v, g, out=o, mask=m)),
        ("chunked bf16, bf16 out", bf16, bf16, DIM, lambda q, k, v, g, o, m: fwd(q, k, v, g, out=o, mask=m)),
        ("row-based bf16", bf16, f32, DIM, lambda q, k, v, g, o, m: rec(q, k, v, g, out=o, mask=m)),
        ("FleetAttention bf16", bf16, f32, DIM, lambda q, k, v, g, o, m: flt(q, k, v, g, out=o, mask=m)),
        ("chunked bf16, dim 256", bf16, f32, 2 * DIM, lambda q, k, v, g, o, m: frd(q, k, v, g, out=o, mask=m)),
    )


def _time_one(torch, call, reps):
    """mean and std over `reps` timed calls (HIP events on the current stream), seconds."""
    for _ in range(2):
        call()
    torch.cuda.synchronize()
    times = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        call()
        e1.record()
        e1.synchronize()
        times.append(e0.elapsed_time(e1) * 1e-3)
    mean = sum(times) / len(times)
    std = math.sqrt(sum((t - mean) ** 2 for t in times) / len(times))
    return mean, std


def run(out_path=None, n_list=N_LIST, batches=(1, 16), reps=REPS, max_bytes=200e9):
    import torch
    from . import binding, workloads as W

    if not torch.cuda.is_available():
        raise SystemExit("latency_table needs a GPU")
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev).manual_seed(0)
    gamma = W.make_gamma("pow2:5:10", HEADS).to(dev)
    lines = [
        "# Single-layer latency versus sequence length (seconds, mean ± std of %d runs)" % reps,
        "",
        "MI355X, one GPU; shape [batch, %d, N, %d], rank = dim = %d (last row: dim 256); synthetic q, k, v ~ N(0,1)/sqrt(d);"
        % (HEADS, DIM, DIM),
        "per-head gamma = 1 - 2^-(5 + 5h/31).  Layout and protocol follow the paper's single-layer tables",
        "(Section 5.1), whose heads, dimensions and dtype are not stated.",
        "",
    ]
    for batch in batches:
        for decay in (True, False):
            mask = binding.LEET_MASK_DECAY if decay else binding.LEET_MASK_CAUSAL
            title = "batch %d, %s" % (batch, "decaying mask" if decay else "0/1 causal mask (no decay)")
            print("== " + title, flush=True)
            lines += ["## " + title, "", "| method | " + " | ".join("N=%d" % n for n in n_list) + " |",
                      "|---|" + "---|" * len(n_list)]
            rows = {name: [] for name, *_ in _methods(torch, binding)}
            for n in n_list:
                shape = (batch, HEADS, n, DIM)
                rows_n = batch * HEADS * n
                cache = {}
                for name, in_dt, out_dt, dv, fn in _methods(torch, binding):
                    isz, osz = torch.empty((), dtype=in_dt).element_size(), torch.empty((), dtype=out_dt).element_size()
                    need = rows_n * ((2 * DIM + dv) * isz + dv * osz)
                    if need > max_bytes:
                        rows[name].append("too large")
                        continue
                    if (in_dt, dv) not in cache:
                        cache.clear()
                        cache[(in_dt, dv)] = tuple(
                            torch.randn(shape[:3] + (w,), device=dev, generator=gen, dtype=in_dt).mul_(w ** -0.5)
                            for w in (DIM, DIM, dv))
                    q, k, v = cache[(in_dt, dv)]
                    out = torch.empty(v.shape, dtype=out_dt, device=dev)
                    mean, std = _time_one(torch, lambda: fn(q, k, v, gamma, out, mask), reps)
                    rows[name].append("%.3g ± %.1g" % (mean, std))
                    print("  N=%d %s: %.3g s" % (n, name, mean), flush=True)
                    del out
                cache.clear()
                torch.cuda.empty_cache()
            for name, vals in rows.items():
                lines.append("| " + name + " | " + " | ".join(vals) + " |")
            for name, vals in PAPER_ROWS.get((batch, decay), {}).items():
                if tuple(n_list) == N_LIST:
                    lines.append("| " + name + " | " + " | ".join("%.3g" % x if x is not None else "OOM" for x in vals) + " |")
            lines.append("")
    text = "\n".join(lines) + "\n"
    if out_path:
        with open(out_path, "w") as f:
            f.write(text)
    else:
        sys.stdout.write(text)
    return text


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--out", default=None, help="write the markdown tables here instead of stdout")
    ap.add_argument("--quick", action="store_true", help="N up to 8192 and 5 repetitions")
    args = ap.parse_args()
    if args.quick:
        run(args.out, n_list=N_LIST[:4], reps=5)
    else:
        run(args.out)


if __name__ == "__main__":
    main()
