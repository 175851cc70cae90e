#!/usr/bin/env python3
"""Benchmark of the SSSD verification step on one MI355X.

One "step" is one whole verify pass (embed -> L decoder layers -> LM head ->
greedy acceptance) over one batch of synthetic input that is already resident in
HBM.  Default workload: the Llama-3-8B-shaped decoder, B = 1, KV context 2048,
k = 8 drafts (the benchmark's second configuration, at the k its latency target is stated on),
plus the latency curve over k = 0..16.  Prints ONE JSON line.

Timing: `ms_per_step` / `value` come from EXACTLY --steps steps between two device synchronisations
(wall clock); `step_ms_events` repeats the same steps with one HIP event pair per step (median, p10,
p90).  `roofline.achieved` is the weight bytes of one GEMM launch over the launch's own duration (HIP
events stamped by the dispatch itself); `stream_read_gbps` / `stream_copy_gbps` are what a plain
read-only pass and a device copy reach in the same run, and `frac_of_achievable` rates the kernel
against the former.  `roofline.traffic` is null unless --traffic-bytes passes in what rocprofv3's
FETCH_SIZE + WRITE_SIZE counted for this command (profiles/ holds those runs).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0     # MI355X published HBM3E bandwidth


WORKLOADS = {
    # name: (shape, B, ctx spec, k, k sweep)
    "cfg2": dict(shape="8b", B=1, ctx=2048, k=8, sweep=list(range(17)), seed=3),
    "cfg3": dict(shape="8b", B=32, ctx=(1024, 4096), k=4, sweep=[0, 4], seed=3),
    "cfg4": dict(shape="8b", B=4, ctx=32768, k=8, sweep=[0, 8], seed=3),
    "cfg5": dict(shape="70b", B=16, ctx=2048, k=8, sweep=[0, 2, 4, 8], seed=6),
    "tiny": dict(shape="tiny", B=1, ctx=128, k=4, sweep=[0, 4], seed=1),
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2", choices=sorted(WORKLOADS))
    ap.add_argument("--k", type=int, default=None, help="drafts per sequence of the timed workload")
    ap.add_argument("--sweep-steps", type=int, default=20)
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies (known traffic) to calibrate rocprofv3 byte counters")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per launch of the dominant kernel measured by rocprofv3 --pmc runs of THIS command "
                         "(FETCH_SIZE + WRITE_SIZE, calibrated); reported as roofline.traffic, which is null without it")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    from paper_2411_05894_amd import binding as sv
    from paper_2411_05894_amd import cost_model as cm
    from sssd_synth import (MODEL_SHAPES, TensorId, global_weight_specs, layer_weight_specs, make_kv_prefill,
                            make_weight, uniform_int)

    wl = WORKLOADS[args.workload]
    shape = MODEL_SHAPES[wl["shape"]]
    B, k = wl["B"], (wl["k"] if args.k is None else args.k)
    sweep = [] if args.no_sweep else sorted(set(wl["sweep"]) | {k})
    max_k = max(sweep + [k])
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    seed = wl["seed"]

    if isinstance(wl["ctx"], tuple):
        lens_cpu = uniform_int(5, TensorId.LENS, (B,), wl["ctx"][0], wl["ctx"][1])
    else:
        lens_cpu = torch.full((B,), wl["ctx"], dtype=torch.int32)
    max_seq = int(lens_cpu.max()) + max_k + 1

    # ---- synthetic model and cache, generated on the device ----
    in_place = wl["shape"] == "70b"          # two copies of 141 GB do not fit
    t0 = time.time()
    layers = [{n: make_weight(seed, n, TensorId.layer(l, slot), shp, device=dev)
               for n, slot, shp in layer_weight_specs(shape)} for l in range(shape.n_layers)]
    g = {n: make_weight(seed, n, tid, shp, device=dev) for n, tid, shp in global_weight_specs(shape)}
    host_sample = None
    # oracle sample sized for 10-30 s of host work: every layer of the 8B shape, 8 layers of the 70B shape
    n_cpu_layers = min(shape.n_layers, 32 if shape.hidden <= 4096 else 8)
    if not args.no_cpu_baseline:
        host_sample = ([{n: t.cpu() for n, t in layers[l].items()} for l in range(n_cpu_layers)],
                       {n: t.cpu() for n, t in g.items()})
    cfg = sv.make_config(shape, B, max_k, max_seq)
    ctx = sv.VerifyContext(cfg, layers, g, in_place=in_place)
    if not in_place:
        for l in layers:
            for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
                del l[n]
        del g["lm_head"]
        torch.cuda.empty_cache()
    kv_sample = []
    for b in range(B):
        n_rows = int(lens_cpu[b])
        for l in range(shape.n_layers):
            K, V = make_kv_prefill(seed * 1000 + b, l, (shape.n_kv_heads, n_rows, shape.head_dim), device=dev)
            ctx.sssd_kv_import(l, b, 0, K, V)
            if host_sample is not None and b == 0 and l < n_cpu_layers:
                kv_sample.append((K.cpu(), V.cpu()))
        torch.cuda.synchronize()
    setup_s = time.time() - t0

    lens = lens_cpu.to(dev)
    acc = torch.zeros(B, dtype=torch.int32, device=dev)
    nxt = torch.zeros(B, dtype=torch.int32, device=dev)
    dims = cm.Dims.of(shape)

    def tokens_for(kk: int):
        return uniform_int(4, TensorId.TOKENS + 100 * kk, (B, kk + 1), 0, shape.vocab - 1, device=dev)

    def time_steps(kk: int, n_warm: int, n_steps: int) -> float:
        tok = tokens_for(kk)
        for _ in range(n_warm):
            ctx.sssd_verify_step(tok, lens, acc, nxt)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(n_steps):
            ctx.sssd_verify_step(tok, lens, acc, nxt)     # lens is not advanced: context stays fixed
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / n_steps

    def quantiles(xs):
        xs = sorted(xs)
        pick = lambda q: xs[min(len(xs) - 1, int(round(q * (len(xs) - 1))))]
        return {"median": round(pick(0.5), 4), "p10": round(pick(0.1), 4), "p90": round(pick(0.9), 4), "n": len(xs)}

    def step_quantiles(kk: int, n_steps: int):
        """One HIP event pair per step, on the stream the step is launched on (torch's current stream)."""
        tok = tokens_for(kk)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_steps)]
        for a, b in ev:
            a.record()
            ctx.sssd_verify_step(tok, lens, acc, nxt)
            b.record()
        torch.cuda.synchronize()
        return quantiles([a.elapsed_time(b) for a, b in ev])

    def stream_figures():
        """What plain kernels reach on this device in this run: a read-only pass (the library's own
        yardstick kernel) and a device-to-device copy, over 2 GiB each, median of 10."""
        n = 1 << 31
        src = torch.zeros(n, dtype=torch.uint8, device=dev)
        sink = torch.zeros(4096, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        rd, cp = [], []
        for i in range(13):
            a, b, c = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            a.record()
            sv.sssd_op_stream_read(src, sink)
            b.record()
            dst.copy_(src)
            c.record()
            torch.cuda.synchronize()
            if i >= 3:
                rd.append(a.elapsed_time(b))
                cp.append(b.elapsed_time(c))
        rd.sort(), cp.sort()
        del src, dst
        torch.cuda.empty_cache()
        return n / (rd[len(rd) // 2] * 1e-3) / 1e9, 2 * n / (cp[len(cp) // 2] * 1e-3) / 1e9

    if args.pmc_calibration:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)     # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # Part of set-up: a second of steps so that the clocks have settled before the W warm-up steps
    # (the first launches after the idle set-up phase measured 3-5 % slower than steady state).
    settle = tokens_for(k)
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < 1.0:
        for _ in range(10):
            ctx.sssd_verify_step(settle, lens, acc, nxt)
        torch.cuda.synchronize()

    # ---- the timed region ----
    ms = time_steps(k, args.warmup, args.steps)
    assert ctx.sssd_verify_sync() == 0
    step_q = step_quantiles(k, args.steps)
    read_gbps, copy_gbps = stream_figures()
    M = B * (k + 1)
    value = M / (ms * 1e-3)
    bytes_alg = cm.algorithmic_bytes(dims, lens_cpu.tolist(), k)

    # ---- per-kernel-class durations (HIP events on the launch stream, inside the library) ----
    ctx.sssd_profile_enable(True)
    prof_steps = max(3, min(10, args.steps))
    tok = tokens_for(k)
    for _ in range(prof_steps):
        ctx.sssd_verify_step(tok, lens, acc, nxt)
    prof = ctx.sssd_profile_read()
    ctx.sssd_profile_enable(False)
    # dominant kernel: the weight streamer (one launch per GEMM; every weight byte is read once)
    kname, launches = sv.sssd_op_gemm_kernel_name(M), prof["gemm"]["launches"] / prof_steps
    ms_per_launch = prof["gemm"]["ms"] / prof["gemm"]["launches"]
    bytes_per_launch = bytes_alg["weights"] / launches
    achieved = bytes_per_launch / (ms_per_launch * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": kname, "achieved": round(achieved, 1),
                "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBPS, 4),
                "traffic": args.traffic_bytes,
                "stream_read_gbps": round(read_gbps, 1), "stream_copy_gbps": round(copy_gbps, 1),
                "frac_of_achievable": round(achieved / read_gbps, 4),
                "bytes_per_launch": round(bytes_per_launch), "launches_per_step": launches,
                "avg_launch_us": round(ms_per_launch * 1e3, 2)}
    classes_ms = {n: round(v["ms"] / prof_steps, 4) for n, v in prof.items()}

    # ---- the same step over draft trees (seeded random trees of k+1 nodes) and the host drafter's cost ----
    tree_ms = sampled_ms = None
    if k >= 1:
        raw = uniform_int(4, TensorId.LENS + 7, (B, k + 1), 0, 1 << 20).tolist()
        par = torch.tensor([[0] + [raw[b][i] % i for i in range(1, k + 1)] for b in range(B)], dtype=torch.int32, device=dev)
        path = torch.zeros(B, k + 1, dtype=torch.int32, device=dev)
        for _ in range(3):
            ctx.sssd_verify_step_tree(tok, par, lens, acc, nxt, path)
        torch.cuda.synchronize()
        t = time.perf_counter()
        n_tree = max(3, args.sweep_steps)
        for _ in range(n_tree):
            ctx.sssd_verify_step_tree(tok, par, lens, acc, nxt, path)
        torch.cuda.synchronize()
        tree_ms = (time.perf_counter() - t) * 1e3 / n_tree
        # ... and with target-only speculative sampling on those trees (Sec. 4.4's setting: T 0.6, top-p 0.95)
        uni = (uniform_int(4, TensorId.LENS + 9, (B, k + 1), 0, (1 << 24) - 1, device=dev).float() / float(1 << 24)).contiguous()
        lscratch = torch.empty(B * (k + 1), shape.vocab, dtype=torch.float32, device=dev)
        sp = sv.SamplingParams(0.6, 0, 0.95)
        for _ in range(3):
            ctx.sssd_verify_step_tree_sampled(tok, par, lens, sp, uni, lscratch, acc, nxt, path)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(n_tree):
            ctx.sssd_verify_step_tree_sampled(tok, par, lens, sp, uni, lscratch, acc, nxt, path)
        torch.cuda.synchronize()
        sampled_ms = (time.perf_counter() - t) * 1e3 / n_tree
        del lscratch
    from paper_2411_05894_amd import drafter as dr
    from sssd_synth import repetitive_stream
    d = dr.Drafter(n_sequences=1)
    d.sssd_draft_datastore_add(repetitive_stream(9, 1, 200_000, vocab=shape.vocab, n_templates=64))
    d.sssd_draft_input_append(0, repetitive_stream(9, 2, 1024, vocab=shape.vocab, n_templates=64))
    t = time.perf_counter()
    n_prop = 200
    for _ in range(n_prop):
        d.sssd_draft_propose(0, k + 1)
    draft_us = (time.perf_counter() - t) * 1e6 / n_prop

    # ---- latency curve over k ----
    curve, curve_q = {}, {}
    for kk in sweep:
        curve[kk] = ms if kk == k else time_steps(kk, 3, args.sweep_steps)
        curve_q[str(kk)] = step_q if kk == k else step_quantiles(kk, args.sweep_steps)
    ratio = {str(kk): round(v / curve[0], 4) for kk, v in curve.items()} if 0 in curve else None

    # ---- the oracle, timed on this machine's host cores on a bounded sample ----
    cpu = None
    if host_sample is not None:
        import oracle
        hl, hg = host_sample
        om = oracle.OracleModel(shape, hl, hg, 1, max_seq)
        for l, (K, V) in enumerate(kv_sample):
            om.K[l, 0, :, : K.shape[1]] = K
            om.V[l, 0, :, : V.shape[1]] = V
        tok0 = tokens_for(k)[:1].cpu()
        t = time.perf_counter()
        x = om.embed(tok0)
        for l in range(n_cpu_layers):
            om.layer_verify(l, x, lens_cpu[:1], 1, k)
        t_layers = time.perf_counter() - t
        t = time.perf_counter()
        om.lm_head(x)
        t_head = time.perf_counter() - t
        est = t_layers * shape.n_layers / n_cpu_layers + t_head       # seconds per sequence-step
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cpu = {"value": round((k + 1) / est, 3), "unit": "verified tokens/s", "cores": cores, "kind": "oracle",
               "sample": f"sequence 0 of the workload, k={k}: {n_cpu_layers} of {shape.n_layers} layers "
                         f"({t_layers:.2f} s) scaled to all layers + the LM head ({t_head:.2f} s)"}

    out = {
        "metric": "verified tokens/s of the verify step (B*(k+1) positions per step)",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "step_ms_events": step_q, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {wl['shape']}-shaped decoder, B={B}, KV context {wl['ctx']}, k={k}",
                   "B": B, "k": k, "M": M, "in_place_weights": in_place},
        "algorithmic_bytes": bytes_alg,
        "hbm_gbps_whole_step": round(bytes_alg["total"] / (ms * 1e-3) / 1e9, 1),
        "hbm_frac_whole_step": round(bytes_alg["total"] / (ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4),
        "latency_ms_vs_k": {str(kk): round(v, 4) for kk, v in curve.items()},
        "latency_ratio_vs_k0": ratio,
        "latency_ms_vs_k_events": curve_q,
        "kernel_class_ms_per_step": classes_ms,
        "tree_step_ms": None if tree_ms is None else round(tree_ms, 4),
        "sampled_tree_step_ms": None if sampled_ms is None else round(sampled_ms, 4),
        "host_draft_us_per_proposal": round(draft_us, 1),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "setup_s": round(setup_s, 1),
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
