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
HBM_PEAK_GBPS = 8000.0             # MI355X HBM3E peak (vendor)


def op_flops(spec, lengths):
    """Algorithmic FLOPs of each of the 9 operators of one layer (causal half only for attn)."""
    t = sum(lengths)
    d, f, hq, dh = spec.hidden, spec.ffn, spec.n_q_heads, spec.head_dim
    attn = sum(2.0 * hq * dh * n * (n + 1) for n in lengths)
    if getattr(spec, "n_experts", 0):      # gate (router) | experts: gate/up | experts: down, top_k experts per token
        ffn = [2.0 * t * d * spec.n_experts, 2.0 * t * spec.top_k * d * 2 * f, 2.0 * t * spec.top_k * f * d]
    else:
        ffn = [2.0 * t * d * 2 * f, 0.0, 2.0 * t * f * d]
    return [0.0, 2.0 * t * d * spec.qkv_width, 0.0, attn, 2.0 * t * hq * dh * d, 0.0] + ffn


def host_cpu():
    """(model name, physical cores, logical CPUs) of this host from /proc/cpuinfo."""
    model, phys, logical = "unknown", set(), 0
    try:
        pkg = core = None
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                key, _, val = line.partition(":")
                key, val = key.strip(), val.strip()
                if key == "model name":
                    model = val
                elif key == "processor":
                    logical += 1
                elif key == "physical id":
                    pkg = val
                elif key == "core id":
                    core = val
                elif not key and pkg is not None and core is not None:
                    phys.add((pkg, core))
                    pkg = core = None
    except OSError:
        pass
    return model, len(phys) or None, logical or os.cpu_count()


def cpu_baseline(spec, seed, lengths, sample_layers):
    """The oracle, as it stands, timed on this host on the WHOLE prompt set of the workload through
    `sample_layers` of its layers (every layer costs the same: same shapes, same lengths), scaled
    to the full depth."""
    import torch
    from oracle import prefill_oracle as O
    from paper_2602_16603_amd import inputs as I
    sub = spec.with_layers(sample_layers)
    total = sum(lengths)
    weights = I.make_weights(sub, seed, torch.bfloat16, "cpu")
    hidden = I.make_hidden(total, spec.hidden, seed, torch.bfloat16, "cpu")
    shape = O.Shape(sub.n_layers, sub.hidden, sub.n_q_heads, sub.n_kv_heads, sub.head_dim, sub.ffn,
                    sub.rms_eps, sub.rope_theta)
    layers = [O.LayerWeights(**w) for w in weights]
    t0 = time.perf_counter()
    O.prefill(shape, layers, hidden, I.cu_seqlens_of(lengths))
    dt = time.perf_counter() - t0
    scale = spec.n_layers / sample_layers
    model, phys, logical = host_cpu()
    # The larger configurations at the FLOP rate this sample measured (not run: hours of CPU time).
    cpu_flops = sum(op_flops(sub, lengths)) * sample_layers / dt
    extrapolated = {}
    for name in ("cfg3", "cfg4", "cfg5"):
        c = I.CONFIGS[name]
        lens = c["lengths"] if c["lengths"] is not None else I.lognormal_lengths(16, c["seed"])
        extrapolated[name] = {"seconds": round(sum(op_flops(c["shape"], lens)) * c["shape"].n_layers / cpu_flops, 1),
                              "label": "extrapolated from this sample's FLOP rate, not measured"}
    return {"value": total / (dt * scale), "unit": "tokens/s", "cores": torch.get_num_threads(),
            "tflops": round(cpu_flops / 1e12, 4), "extrapolated": extrapolated,
            "kind": "oracle", "seconds": dt, "cpu_model": model, "physical_cores": phys, "logical_cpus": logical,
            "sample": f"all {total} tokens of the prompt through {sample_layers} of {spec.n_layers} layers "
                      f"(fp64 oracle, {torch.get_num_threads()} threads); layers cost the same, time scaled by "
                      f"{scale:g} to the full stack"}


def percentile(values, q):
    if not values:
        return None
    v = sorted(values)
    return v[min(len(v) - 1, int(round(q * (len(v) - 1))))]


def preemption_workload(seconds: float, seed: int = 4, short_seconds: float = 3.0):
    """cfg4: a 32768-token prompt always in flight on the 32-layer 8B shape while 128..1024-token
    prompts arrive as a seeded Poisson process (20 req/s); every arrival preempts the long prompt
    at the next boundary, runs, and the long prompt resumes.  Blocking time = signal ->
    acknowledgement (paper Section 6.4).  Modes: checks after every operator (launch-ahead 2 and
    1), after the paper's five core operators only, after every layer only (the layer-level
    comparison of Section 6.4), fixed chunked prefill with chunk 512 / 2048 / 8192 (boundary =
    chunk end only), and operator-level checks inside chunks of 4096 / 8192 / 16384 tokens (the
    combination of Section 6.5).  The modes the headline compares -- every operator (launch-ahead 2
    and 1), layer level, fixed chunks of 512 / 2048 / 8192 -- run the full `seconds` window (cfg4:
    10 s, about 200 arrivals); the remaining modes run its first `short_seconds`."""
    import torch
    from paper_2602_16603_amd import binding as B, eventloop as E, inputs as I, runner as R

    spec = I.CONFIGS["cfg4"]["shape"]
    long_n = I.CONFIGS["cfg4"]["lengths"][0]
    weights = I.make_weights(spec, seed, torch.bfloat16, "cuda")
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, kv_num_blocks=long_n // 16 + 8 * 70 + 64,
                           max_position=long_n)
    long_hidden = I.make_hidden(long_n, spec.hidden, seed, torch.bfloat16, "cuda")
    short_hidden = I.make_hidden(1024, spec.hidden, seed + 1, torch.bfloat16, "cuda")
    arrivals = I.poisson_arrivals(20.0, seconds, seed)

    # One uninterrupted long prefill with per-op timing: the layer time the latency is judged by.
    task = model.begin(long_hidden, [long_n])
    task.run_to_completion()
    task.end()
    task = model.begin(long_hidden, [long_n])
    B.fp_prefill_set_timing(task.handle, True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    task.run_to_completion()
    long_s = time.perf_counter() - t0
    ops = B.fp_prefill_op_times(task.handle, spec.n_layers * 9)
    task.end()
    per_op = [statistics.fmean(ops[i::9]) for i in range(9)]
    long_flops = sum(op_flops(spec, [long_n])) * spec.n_layers
    result = {"workload": f"cfg4: {spec.n_layers}-layer 8B shape, {long_n}-token prompt in flight, "
                          f"{len(arrivals)} Poisson arrivals (20/s, 128-1024 tokens) over {seconds:g} s",
              "long_prefill_uninterrupted_s": round(long_s, 4),
              "long_prefill_tokens_per_s": round(long_n / long_s, 1),
              "long_prefill_tflops": round(long_flops / long_s / 1e12, 1),
              "long_prefill_mfma_frac": round(long_flops / long_s / 1e12 / BF16_MFMA_PEAK_TFLOPS, 4),
              "op_roof_frac": {n: round(f / (v * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS, 3)
                               for n, v, f in zip(B.OP_NAMES, per_op, op_flops(spec, [long_n])) if f > 0},
              "layer_ms": round(sum(per_op), 3), "slowest_op_ms": round(max(per_op), 3),
              "op_ms": {n: round(v, 3) for n, v in zip(B.OP_NAMES, per_op)}, "modes": {}}

    short_s = min(seconds, short_seconds)
    modes = [("op_level_ahead2", 0, 2, B.FP_BOUNDARY_EVERY_OP, seconds), ("op_level_ahead1", 0, 1, B.FP_BOUNDARY_EVERY_OP, seconds),
             ("paper_five_ops", 0, 2, B.FP_BOUNDARY_PAPER_OPS, short_s), ("layer_level", 0, 2, B.FP_BOUNDARY_LAYER, seconds),
             ("chunk_512", 512, 2, 0, seconds), ("chunk_2048", 2048, 2, 0, seconds), ("chunk_8192", 8192, 2, 0, seconds),
             ("op_level_in_chunk_4096", 4096, 2, B.FP_BOUNDARY_EVERY_OP, short_s),
             ("op_level_in_chunk_8192", 8192, 2, B.FP_BOUNDARY_EVERY_OP, short_s),
             ("op_level_in_chunk_16384", 16384, 2, B.FP_BOUNDARY_EVERY_OP, short_s)]
    all_arrivals = arrivals
    for name, chunk, ahead, mask, seconds in modes:
        arrivals = [a for a in all_arrivals if a[0] < seconds]
        pool = E.MixedPool(model, mask or B.FP_BOUNDARY_EVERY_OP, launch_ahead=ahead,
                           chunk_op_mask=mask if chunk else 0)
        state = {"longs": 0, "stop": False}

        def reissue(req, state=state):
            if req.name.startswith("L") and not state["stop"]:
                state["longs"] += 1
                loop.post_arrival(E.Request(f"L{state['longs']}", long_n, (long_hidden, chunk)))

        # Fixed rule: a short request overtakes the long prompt; shorts run in arrival order.
        loop = E.EventLoop(pool, priority=lambda r: (r.name.startswith("L"), r.order), on_complete=reissue)
        shorts = [E.Request(f"s{i}", n, (short_hidden[:n], 0), arrival=t) for i, (t, n) in enumerate(arrivals)]
        loop.post_arrival(E.Request("L0", long_n, (long_hidden, chunk)))
        loop.step(5.0)
        t_start = time.perf_counter()
        E.feed_arrivals(loop, shorts)
        while True:
            loop.step(0.05)
            n_short_done = sum(1 for r in loop.finished if r.name.startswith("s"))
            if n_short_done == len(shorts) and time.perf_counter() - t_start >= seconds:
                break
            if time.perf_counter() - t_start > seconds + 60:
                raise TimeoutError(f"preemption workload {name} did not drain")
        state["stop"] = True
        elapsed = time.perf_counter() - t_start
        last = loop.running
        if last is not None:                            # stop the background long prompt
            pool.preempt(last.handle)
        loop.close()                                    # joins the executor thread
        if last is not None:
            pool.finish(last.handle)
        lat_us = [x * 1e6 for x, who in zip(loop.preempt_latency_s, loop.preempt_victims) if who.startswith("L")]
        ttft_ms = [(r.t_finished - r.t_arrived) * 1e3 for r in loop.finished if r.name.startswith("s")]
        result["modes"][name] = {
            "window_s": seconds, "arrivals": len(arrivals), "preemptions": len(lat_us),
            # with fewer than 100 samples the 99th percentile IS the largest sample
            "p99_is": "p99" if len(lat_us) >= 100 else f"max of {len(lat_us)}",
            "blocking_us": {"p50": round(percentile(lat_us, 0.5) or 0, 1), "p99": round(percentile(lat_us, 0.99) or 0, 1),
                            "max": round(max(lat_us) if lat_us else 0, 1)},
            "short_ttft_ms": {"p50": round(percentile(ttft_ms, 0.5) or 0, 2), "p99": round(percentile(ttft_ms, 0.99) or 0, 2)},
            "long_prompts_completed": state["longs"], "elapsed_s": round(elapsed, 3)}
    model.close()
    return result


def slo_workload(seconds: float, points, seed: int = 6, token_budget: int = 4096, model_name: str = "8b"):
    """Multi-SLO serving on the 32-layer 8B shape (Section 6.2's experiment on a synthetic stand-in
    for its trace): Poisson arrivals of the four request classes of Table 1 with the TTFT SLOs of
    Table 2, scheduled by the native event-driven scheduler.  Systems compared: S-EDF + SLO-aware
    batching + operator-level preemption (the paper's system), the same without batching, EDF over
    fixed chunked prefill with chunk 2048 / 8192 (the CP2K / CP8K baselines) and FCFS without
    preemption.  TTFT = arrival -> end of the request's prefill; SLO attainment = share of the
    requests that arrived in the window whose TTFT met their SLO (unfinished ones count as missed)."""
    import numpy as np
    import torch
    from paper_2602_16603_amd import binding as B, eventloop as E, inputs as I, runner as R

    # "8b": the dense 32-layer 8B shape of Section 6.2; "moe": the 48-layer 30B-A3B shape of Section 7.
    spec = I.CONFIGS["cfg4"]["shape"] if model_name == "8b" else I.QWEN3_30B_A3B
    max_n = 32768
    weights = I.make_weights(spec, seed, torch.bfloat16, "cuda")
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, kv_num_blocks=(1 << 20) // 16, max_position=max_n)
    buf = I.make_hidden(max_n, spec.hidden, seed, torch.bfloat16, "cuda")

    # Offline TTFT profile -> polynomial (Section 6.3): second-order fit of prefill time over token count.
    prof_n, prof_t = [256, 1024, 4096, 8192, 16384], []
    for n in prof_n:
        best = None
        for _ in range(2):
            task = model.begin(buf[:n], [n])
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            task.run_to_completion()
            dt = time.perf_counter() - t0
            task.end()
            best = dt if best is None else min(best, dt)
        prof_t.append(best)
    coef = [float(c) for c in np.polyfit(np.asarray(prof_n, dtype=np.float64), np.asarray(prof_t), 2)[::-1]]
    result = {"workload": f"{spec.n_layers}-layer {'8B' if model_name == '8b' else '30B-A3B mixture-of-experts'} shape; request classes and shares of Table 1, TTFT SLOs of "
                          f"Table 2 (Llama3-8B row); Poisson arrivals for {seconds:g} s per point; token budget G = {token_budget}",
              "ttft_fit_seconds": {"coef_c0_c1_c2": coef, "profile_tokens": prof_n,
                                   "profile_seconds": [round(t, 5) for t in prof_t]},
              "rates": {}}
    systems = [("s_edf_batching_op_level", B.FP_SCHED_SEDF, True, 0), ("s_edf_op_level", B.FP_SCHED_SEDF, False, 0),
               ("edf_chunk_2048", B.FP_SCHED_EDF, False, 2048), ("edf_chunk_8192", B.FP_SCHED_EDF, False, 8192),
               ("fcfs", B.FP_SCHED_FCFS, False, 0)]
    for rate, slo_scale in points:
        trace = I.multi_slo_trace(rate, seconds, seed + int(rate * 100), slo_scale=slo_scale)
        point = {"requests": len(trace), "tokens": sum(t[1] for t in trace)}
        for name, policy, batching, chunk in systems:
            pool = E.BatchPool(model, B.FP_BOUNDARY_EVERY_OP, chunk=chunk)
            loop = E.SloEventLoop(pool, token_budget, coef, policy, batching)
            reqs = [E.SloRequest(i, n, slo, t, buf[:n], kind) for i, n, t, slo, kind in trace]
            t_start = time.perf_counter()
            E.feed_slo_arrivals(loop, reqs)
            while len(loop.finished) < len(reqs) and time.perf_counter() - t_start < seconds + 20.0:
                loop.step(0.05)
            elapsed = time.perf_counter() - t_start
            met = {r.id for r in loop.finished if r.t_finished - r.t_arrived <= r.slo}
            per_class = {}
            for kind in sorted({t[4] for t in trace}):
                ids = [t[0] for t in trace if t[4] == kind]
                per_class[kind] = round(sum(1 for i in ids if i in met) / len(ids), 4)
            text_ttft = [(r.t_finished - r.t_arrived) * 1e3 for r in loop.finished if r.kind == "text"]
            lat = [x * 1e3 for x in loop.preempt_latency_s]
            point[name] = {"slo_attainment": round(len(met) / max(1, len(trace)), 4), "per_class": per_class,
                           "finished": len(loop.finished), "elapsed_s": round(elapsed, 2),
                           "text_ttft_ms": {"p50": round(percentile(text_ttft, 0.5) or 0, 1),
                                            "p99": round(percentile(text_ttft, 0.99) or 0, 1)},
                           "rounds": loop.rounds, "commands": dict(loop.commands),
                           "mean_batch": round(statistics.fmean(loop.batch_sizes), 2) if loop.batch_sizes else 0,
                           "blocking_ms_p99": round(percentile(lat, 0.99) or 0, 2)}
            loop.close()
            torch.cuda.synchronize()
            print(f"[slo] {rate:g}/s x{slo_scale:g} {name}: attainment {point[name]['slo_attainment']}, "
                  f"{elapsed:.1f} s", file=sys.stderr, flush=True)
        result["rates"][f"{rate:g}/s, SLO x{slo_scale:g}"] = point
    model.close()
    return result


def other_configs(seed_short: int = 9):
    """Throughput at the other single-GPU 8B-shape workloads: cfg3 (the full 32-layer stack on 16
    log-normal prompts, paged KV with a permuted block table) and one short request of the kind
    cfg4's arrivals are (256 tokens through 32 layers, no launch-ahead bound), the latter against
    the time HBM needs to stream the stack's weights once."""
    import torch
    from paper_2602_16603_amd import binding as B, inputs as I, runner as R

    cfg = I.CONFIGS["cfg3"]
    spec, seed = cfg["shape"], cfg["seed"]
    lengths = I.lognormal_lengths(16, seed)
    total = sum(lengths)
    pool = total // 16 + 64
    table, _ = I.permuted_block_tables(lengths, None, 16, pool, seed=seed)
    weights = I.make_weights(spec, seed, torch.bfloat16, "cuda")
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, pool + 64, max(lengths))
    hidden = I.make_hidden(total, spec.hidden, seed, torch.bfloat16, "cuda")
    times = []
    for i in range(3):
        task = model.begin(hidden, lengths, cached=[0] * len(lengths), block_tables=table)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        task.run_to_completion()
        times.append(time.perf_counter() - t0)
        task.end()
    dt = min(times[1:])
    flops = sum(op_flops(spec, lengths)) * spec.n_layers
    out = {"cfg3": {"workload": f"{spec.n_layers}-layer 8B shape, 16 prompts (log-normal lengths, {min(lengths)}..{max(lengths)}), "
                                f"{total} tokens packed, paged KV with a permuted block table",
                    "seconds_per_step": round(dt, 4), "tokens_per_s": round(total / dt, 1),
                    "tflops": round(flops / dt / 1e12, 1),
                    "mfma_frac": round(flops / dt / 1e12 / BF16_MFMA_PEAK_TFLOPS, 4)}}

    n_short = 256
    short = I.make_hidden(n_short, spec.hidden, seed_short, torch.bfloat16, "cuda")
    times = []
    for i in range(6):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        task = model.begin(short, [n_short])
        B.fp_prefill_set_launch_ahead(task.handle, 0)
        task.run_to_completion()
        task.end()
        times.append(time.perf_counter() - t0)
    dt = statistics.median(times[2:])
    weight_bytes = spec.params_per_layer() * spec.n_layers * 2.0
    out["short_request"] = {"workload": f"one {n_short}-token prompt through {spec.n_layers} layers of the 8B shape "
                                        f"(begin + advance + end, launch_ahead 0)",
                            "ms": round(dt * 1e3, 3), "tokens_per_s": round(n_short / dt, 1),
                            "weight_bytes": weight_bytes,
                            "hbm_floor_ms": round(weight_bytes / (HBM_PEAK_GBPS * 1e9) * 1e3, 3),
                            "hbm_frac": round(weight_bytes / dt / 1e9 / HBM_PEAK_GBPS, 4)}
    model.close()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--config", default="cfg2", help="cfg2 (default); other names are for exploration")
    ap.add_argument("--layers", type=int, default=0, help="override layer count (exploration only)")
    ap.add_argument("--slo-seconds", type=float, default=4.0,
                    help="arrival window of each (system, rate) point of the multi-SLO scheduling workload; 0 skips it")
    ap.add_argument("--slo-model", default="8b", choices=["8b", "moe"],
                    help="model of the scheduling workload: the dense 8B shape or the 30B-A3B mixture-of-experts shape")
    ap.add_argument("--slo-points", default="32:1,24:0.2",
                    help="rate:slo_scale points of that workload (requests per second : factor on Table 2's SLOs)")
    ap.add_argument("--preempt-seconds", type=float, default=10.0,
                    help="arrival window of the headline modes of the preemption-latency workload (cfg4 states "
                         "10 s at 20 requests/s); the extra modes run its first 3 s; 0 skips the workload")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the cfg3 batch and the short-request measurement")
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
    # What the matrix pipes sustain on this chip with nothing else in the way (register-only MFMA
    # loop, random operands, ~0.3 s so the clock settles): the second yardstick next to the vendor peak.
    mfma_ceiling = B.fp_diag_mfma_ceiling(300)

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

    # Dominant kernel: gemm_bf16_w4_kernel<3>, the one-wave-per-SIMD bf16 MFMA GEMM with the SwiGLU
    # epilogue (the gate_up_proj launch, one per layer: 47% of a layer's FLOPs, 39% of its time).
    dom_ops = (6,)
    dom_ms = [ms for o in dom_ops for ms in op_ms[o]]
    dom_flops = sum(per_layer[o] for o in dom_ops) / len(dom_ops)      # mean per launch
    dom_avg_ms = statistics.fmean(dom_ms)
    achieved = dom_flops / (dom_avg_ms * 1e-3) / 1e12
    # Algorithmic HBM bytes of the bandwidth-bound operators (fp32 residual in, bf16 out for the
    # norms; RoPE reads q,k,v and writes q,k back plus k,v into the cache).
    kvw = spec.n_kv_heads * spec.head_dim
    hbm_bytes = {0: total * spec.hidden * 6.0, 5: total * spec.hidden * 6.0,
                 2: total * 2.0 * (spec.qkv_width + (spec.n_q_heads * spec.head_dim + kvw) + 2 * kvw)}
    per_op = {}
    for o, name in enumerate(B.MOE_OP_NAMES if getattr(spec, "n_experts", 0) else B.OP_NAMES):
        avg = statistics.fmean(op_ms[o])
        per_op[name] = {"ms": round(avg, 4)}
        if avg <= 0:
            per_op[name]["note"] = "launches nothing here: carried out by the neighbouring operator's kernel"
        elif per_layer[o] > 0:
            per_op[name]["tflops"] = round(per_layer[o] / (avg * 1e-3) / 1e12, 1)
            per_op[name]["roof_frac"] = round(per_layer[o] / (avg * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS, 3)
        elif o in hbm_bytes:
            per_op[name]["gbps"] = round(hbm_bytes[o] / (avg * 1e-3) / 1e9, 1)
            per_op[name]["roof_frac"] = round(hbm_bytes[o] / (avg * 1e-3) / 1e9 / HBM_PEAK_GBPS, 3)

    # What the preemption checks cost when no signal ever fires (Section 6.5): the same steps with
    # a check after every operator (bounded launch-ahead) and with no checks at all, untimed per op.
    check_overhead = None
    if args.config == "cfg2" and not args.layers:
        def plain(mask):
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.steps):
                task = model.begin(hidden, lengths, boundary_mask=mask)
                task.run_to_completion()
                task.end()
            torch.cuda.synchronize()
            return (time.perf_counter() - t1) / args.steps * 1e3
        ms_none, ms_every = plain(B.FP_BOUNDARY_NONE), plain(B.FP_BOUNDARY_EVERY_OP)
        check_overhead = {"ms_per_step_no_checks": round(ms_none, 4), "ms_per_step_check_every_op": round(ms_every, 4),
                          "ratio": round(ms_every / ms_none, 4)}

    # HBM-side bytes per launch of the dominant kernel come from the committed rocprofv3 --pmc
    # summary (FETCH_SIZE and WRITE_SIZE, scaled by a plain copy); null when that file is absent
    # or describes another workload.
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "gemm_bf16_w4_cfg2_traffic.json")
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
        # The headline: whole-path FLOPs over wall time against the bf16 MFMA peak (target >= 0.60).
        # `roofline` below is the dominant kernel alone and reads higher.
        "end_to_end_frac": round(tflops / BF16_MFMA_PEAK_TFLOPS, 4),
        "mfma_ceiling_tflops": round(mfma_ceiling, 1), "measured_peak_frac": round(tflops / mfma_ceiling, 4),
        "per_op": per_op, "check_overhead": check_overhead,
        "roofline": {"bound": "mfma", "kernel": "gemm_bf16_w4_kernel<3> (gate_up_proj with fused SiLU*up)",
                     "achieved": round(achieved, 1), "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / BF16_MFMA_PEAK_TFLOPS, 4), "traffic": traffic,
                     "scope": "dominant kernel only; the whole path is end_to_end_frac",
                     "avg_launch_ms": round(dom_avg_ms, 4), "flops_per_launch": dom_flops},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(spec, seed, lengths, sample_layers=1)
        out["cpu_baseline"]["value"] = round(out["cpu_baseline"]["value"], 2)
        out["cpu_baseline"]["seconds"] = round(out["cpu_baseline"]["seconds"], 2)
    model.close()
    del model, weights, hidden
    torch.cuda.empty_cache()
    if not args.no_other_configs and args.config == "cfg2" and not args.layers:
        out["configs"] = other_configs()
        torch.cuda.empty_cache()
    if args.preempt_seconds > 0 and args.config == "cfg2" and not args.layers:
        out["preemption"] = preemption_workload(args.preempt_seconds)
        out["configs"] = dict(out.get("configs", {}), cfg4_long_prompt={
            "workload": "one 32768-token prompt through the 32-layer 8B shape, uninterrupted",
            "seconds_per_step": out["preemption"]["long_prefill_uninterrupted_s"],
            "tokens_per_s": out["preemption"]["long_prefill_tokens_per_s"],
            "tflops": out["preemption"]["long_prefill_tflops"],
            "mfma_frac": out["preemption"]["long_prefill_mfma_frac"]})
    if args.slo_seconds > 0 and args.config == "cfg2" and not args.layers:
        out["slo_scheduling"] = slo_workload(
            args.slo_seconds, [tuple(float(v) for v in x.split(":")) for x in args.slo_points.split(",")],
            model_name=args.slo_model)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
