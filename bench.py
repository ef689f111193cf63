#!/usr/bin/env python3
"""Benchmark of the op-preemptible prefill path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass of the whole hot path -- fp_prefill_begin, all n_layers*9 operators through
fp_prefill_advance (preemption checks enabled at every operator boundary, none fired),
fp_prefill_end -- over one batch of synthetic input already resident in HBM.  The workload is
cfg2: Llama-3-8B-shaped 4-layer stack, bf16, one 8192-token prompt.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 MFMA peak (vendor, no sparsity)


def op_flops(spec, lengths):
    """Algorithmic FLOPs of each of the 9 operators of one layer (causal half only for attn)."""
    t = sum(lengths)
    d, f, hq, dh = spec.hidden, spec.ffn, spec.n_q_heads, spec.head_dim
    attn = sum(2.0 * hq * dh * n * (n + 1) for n in lengths)
    return [0.0, 2.0 * t * d * spec.qkv_width, 0.0, attn, 2.0 * t * hq * dh * d, 0.0,
            2.0 * t * d * 2 * f, 0.0, 2.0 * t * f * d]


def cpu_baseline(spec, seed, sample_tokens, sample_layers):
    """The oracle, as it stands, timed on this host on a bounded sample of the same workload."""
    import torch
    from oracle import prefill_oracle as O
    from paper_2602_16603_amd import inputs as I
    sub = spec.with_layers(sample_layers)
    weights = I.make_weights(sub, seed, torch.bfloat16, "cpu")
    hidden = I.make_hidden(sample_tokens, spec.hidden, seed, torch.bfloat16, "cpu")
    shape = O.Shape(sub.n_layers, sub.hidden, sub.n_q_heads, sub.n_kv_heads, sub.head_dim, sub.ffn,
                    sub.rms_eps, sub.rope_theta)
    layers = [O.LayerWeights(**w) for w in weights]
    t0 = time.perf_counter()
    O.prefill(shape, layers, hidden, [0, sample_tokens])
    dt = time.perf_counter() - t0
    scale = spec.n_layers / sample_layers
    return {"value": sample_tokens / (dt * scale), "unit": "tokens/s", "cores": torch.get_num_threads(),
            "kind": "oracle", "seconds": dt,
            "sample": f"first {sample_tokens} tokens of the prompt through {sample_layers} of "
                      f"{spec.n_layers} layers (fp64 oracle); time scaled by {scale:g} to the full stack"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--config", default="cfg2", help="cfg2 (default); other names are for exploration")
    ap.add_argument("--layers", type=int, default=0, help="override layer count (exploration only)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a 1 GiB device-to-device copy (known HBM traffic) for scaling "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import torch
    from paper_2602_16603_amd import binding as B, inputs as I, runner as R

    if args.calibrate_copy:
        n = 1 << 30
        src = torch.full((n,), 3, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": n, "calibrate_copy_bytes_written": n, "launches": 5}))
        return 0

    cfg = I.CONFIGS[args.config]
    spec, seed = cfg["shape"], cfg["seed"]
    lengths = cfg["lengths"] if cfg["lengths"] is not None else I.lognormal_lengths(16, seed)
    if args.layers:
        spec = spec.with_layers(args.layers)
    total = sum(lengths)
    torch.cuda.set_device(0)
    weights = I.make_weights(spec, seed, torch.bfloat16, "cuda")
    hidden = I.make_hidden(total, spec.hidden, seed, torch.bfloat16, "cuda")
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, kv_num_blocks=total // 16 + len(lengths) + 64,
                           max_position=max(lengths))

    n_ops = spec.n_layers * B.FP_OPS_PER_LAYER
    op_ms = [[] for _ in range(B.FP_OPS_PER_LAYER)]

    def step(timed: bool):
        task = model.begin(hidden, lengths, boundary_mask=B.FP_BOUNDARY_EVERY_OP)
        if timed:
            B.fp_prefill_set_timing(task.handle, True)
        task.run_to_completion()
        if timed:
            for i, ms in enumerate(B.fp_prefill_op_times(task.handle, n_ops)):
                op_ms[i % B.FP_OPS_PER_LAYER].append(ms)
        task.end()

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    ms_per_step = elapsed / args.steps * 1e3
    tokens_per_s = total * args.steps / elapsed
    per_layer = op_flops(spec, lengths)
    step_flops = sum(per_layer) * spec.n_layers
    tflops = step_flops / (elapsed / args.steps) / 1e12

    # Dominant kernel: gemm_bf16_pp_kernel<false>, the ping-pong 256x256 bf16 MFMA GEMM with bf16
    # output (the qkv_proj and gate_up_proj launches; gate_up alone is 47% of a layer's FLOPs).
    dom_ops = (1, 6)
    dom_ms = [ms for o in dom_ops for ms in op_ms[o]]
    dom_flops = sum(per_layer[o] for o in dom_ops) / len(dom_ops)      # mean per launch
    dom_avg_ms = statistics.fmean(dom_ms)
    achieved = dom_flops / (dom_avg_ms * 1e-3) / 1e12
    per_op = {}
    for o, name in enumerate(B.OP_NAMES):
        avg = statistics.fmean(op_ms[o])
        per_op[name] = {"ms": round(avg, 4)}
        if per_layer[o] > 0:
            per_op[name]["tflops"] = round(per_layer[o] / (avg * 1e-3) / 1e12, 1)

    # HBM-side bytes per launch of the dominant kernel come from the committed rocprofv3 --pmc
    # summary (FETCH_SIZE and WRITE_SIZE, scaled by a plain copy); null when that file is absent
    # or describes another workload.
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "gemm_bf16_pp_cfg2_traffic.json")
    if args.config == "cfg2" and not args.layers and os.path.exists(tpath):
        with open(tpath) as fh:
            traffic = json.load(fh).get("hbm_bytes_per_launch")

    out = {
        "metric": "prefill tokens/s, Llama-3-8B-shaped 4-layer stack, bf16, 1 GPU",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.config}: {spec.n_layers}-layer hidden {spec.hidden} "
                               f"{spec.n_q_heads}q/{spec.n_kv_heads}kv x{spec.head_dim} ffn {spec.ffn}, "
                               f"{len(lengths)} prompt(s), {total} tokens, 9 ops/layer with a preemption "
                               f"check at every boundary", "seed": seed},
        "tflops": round(tflops, 1), "mfma_frac": round(tflops / BF16_MFMA_PEAK_TFLOPS, 4),
        "per_op": per_op,
        "roofline": {"bound": "mfma", "kernel": "gemm_bf16_pp_kernel<false> (qkv_proj, gate_up_proj)",
                     "achieved": round(achieved, 1), "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / BF16_MFMA_PEAK_TFLOPS, 4), "traffic": traffic,
                     "avg_launch_ms": round(dom_avg_ms, 4), "flops_per_launch": dom_flops},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(spec, seed, sample_tokens=min(2048, max(lengths)),
                                           sample_layers=min(2, spec.n_layers))
        out["cpu_baseline"]["value"] = round(out["cpu_baseline"]["value"], 2)
        out["cpu_baseline"]["seconds"] = round(out["cpu_baseline"]["seconds"], 2)
    model.close()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
