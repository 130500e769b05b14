#!/usr/bin/env python3
"""Benchmark of the MoE hot path on one MI355X.

A step is one pass of the whole path (moe_route_dispatch [= moe_route, moe_dispatch] -> moe_ffn_input
-> moe_ffn_output -> moe_combine) over one batch of seeded synthetic input that is already resident in HBM. The
default workload is the Mixtral-8x22B-shaped decode micro-batch (d=6144, f=16384, E=8, top-2,
bf16, T=256), the configuration the headline metric is quoted on.

Prints ONE JSON line. `value`, `ms_per_step` and `roofline` belong to `config.workload`. `roofline`
is for the dominant kernel (the fused gate|up "FFN Input" GEMM): algorithmic bytes or flops per
launch over its average duration, measured with events on the launch stream inside the timed
region. `cpu_baseline` is the CPU oracle, as it stands, timed on this machine's host cores on a
bounded sample.

The metric is a curve over the per-expert batch, so the default run (no --workload) also times the
same layer at T = 32 ... 4096 on the same weights, each point with the same W warm-up and K timed
steps, and carries them in `sweep` (`roofline_large_batch` repeats the FFN-input roofline of the
largest point, the matrix-core-bound end), and it times the fine-grained many-expert layer cut into
m = 1 ... 4 micro-batches on two alternating streams (`micro_batch_study`).

    python bench.py [--gpus 1] [--steps K] [--warmup W]            # headline + sweep + micro-batch study
    python bench.py --workload NAME [--sweep] [--no-cpu-baseline]  # one workload (profiles are taken this way)
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

import numpy as np  # noqa: E402


def dev(a, torch):
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def upload_and_pack(cfg, seed, path, torch, synth, keep=True):
    """Generate the expert weights on the host, upload, pre-pack once (outside any timed region).
    keep=False drops the host copy (it is only needed where the CPU oracle runs on the same weights)."""
    t0 = time.time()
    W = synth.make_all_expert_weights(cfg, seed, workers=min(16, os.cpu_count() or 8))
    gen_s = time.time() - t0
    wg, wu, wd = (dev(w, torch) for w in W)
    path.pack_weights(wg, wu, wd)
    torch.cuda.synchronize()
    del wg, wu, wd
    torch.cuda.empty_cache()
    return (W if keep else None), gen_s


def make_inputs(cfg, seed, synth):
    """Activations and router logits. The gating GEMM is not part of the timed path, so for the
    layer whose tests route through a gating matrix the logits are simply drawn here."""
    return synth.make_activations(cfg, seed), synth.make_logits(cfg, seed)


kSettleSeconds = 0.3


def time_workload(cfg, paths, x_d, logits_d, steps, warmup, torch, R, synth, breakdown=True, w_router_d=None):
    """W warm-up steps, then exactly K timed steps between device synchronisations.

    A step runs the whole path over the batch. With cfg.micro_batches = m > 1 the batch is cut
    into m contiguous micro-batches issued on two alternating streams (each stream has its own
    buffer set; the packed weights are shared), the single-GPU echo of the paper's ping-pong
    micro-batching (Section 4.1). With w_router_d the step starts at the gating GEMM (moe_gate_route_dispatch on
    x and the gating matrix) instead of at given logits."""
    ranges = synth.microbatch_ranges(cfg.T, cfg.micro_batches)
    if cfg.micro_batches > 1:
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    else:
        streams = [torch.cuda.current_stream()]

    def step(ev=None, serial=False):
        for i, (a, b) in enumerate(ranges):
            j = 0 if serial else i % len(streams)
            path, stream = paths[j], streams[j]
            T = b - a
            if w_router_d is not None:
                path.gate_route_dispatch(x_d[a:b], w_router_d, None, T, stream)   # gating GEMM + routing + dispatch pack
            else:
                path.route_dispatch(x_d[a:b], logits_d[a:b], T, stream)   # = moe_route then moe_dispatch
            if ev is not None:
                ev[i][0].record(stream)
            path.ffn_input(T, stream)
            if ev is not None:
                ev[i][1].record(stream)
            path.ffn_output(T, stream)
            path.combine(T, stream)

    def sync():
        torch.cuda.synchronize()

    # Warm-up: the W steps asked for, then on until the device has been busy for kSettleSeconds. The
    # memory-bound workloads run ~3 % slower for their first ~0.15 s (clocks still ramping); a serving
    # loop lives in the settled state, so that is the state timed.
    t_warm = time.perf_counter()
    warm_steps = 0
    while warm_steps < warmup or (time.perf_counter() - t_warm < kSettleSeconds and warm_steps < 5000):
        step()
        warm_steps += 1
        if warm_steps >= warmup and warm_steps % 10 == 0:
            sync()
    m = len(ranges)
    events = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(m)]
              for _ in range(steps)]
    sync()
    t0 = time.perf_counter()
    for i in range(steps):
        step(events[i])
    sync()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    ffn_in_all = [a.elapsed_time(b) for evs in events for a, b in evs]
    ffn_in_ms = float(np.mean(ffn_in_all))
    ffn_in_pct = [float(np.percentile(ffn_in_all, q)) for q in (10, 50, 90)]

    serial_ms = None
    if m > 1:   # the same micro-batches back to back on one stream, for comparison
        for _ in range(2):
            step(serial=True)
        sync()
        t0 = time.perf_counter()
        for _ in range(steps):
            step(serial=True)
        sync()
        serial_ms = (time.perf_counter() - t0) * 1e3 / steps

    # per-call breakdown on the first micro-batch (separate, untimed pass)
    a, b = ranges[0]
    T, path, stream = b - a, paths[0], streams[0]
    names = ["route", "dispatch", "route_dispatch", "ffn_input", "ffn_output", "combine"]
    calls = [lambda: path.route(logits_d[a:b], T, stream), lambda: path.dispatch(x_d[a:b], T, stream),
             lambda: path.route_dispatch(x_d[a:b], logits_d[a:b], T, stream),
             lambda: path.ffn_input(T, stream), lambda: path.ffn_output(T, stream), lambda: path.combine(T, stream)]
    if w_router_d is not None:     # the gated forms come first, so that the FFN calls below see the gated routing
        names = ["gate_route", "gate_route_dispatch"] + names[3:]
        calls = [lambda: path.gate_route(x_d[a:b], w_router_d, None, T, stream),
                 lambda: path.gate_route_dispatch(x_d[a:b], w_router_d, None, T, stream)] + calls[3:]
    reps = max(5, min(steps, 20)) if breakdown else 0
    acc = {n: [] for n in names}
    for _ in range(reps):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)]
        calls[-1]()                    # the first timed call must not pay for a device that just went idle
        evs[0].record(stream)
        for i, c in enumerate(calls):
            c()
            evs[i + 1].record(stream)
        sync()
        for i, n in enumerate(names):
            acc[n].append(evs[i].elapsed_time(evs[i + 1]))
    calls_ms = {n: float(np.median(v)) if v else None for n, v in acc.items()}

    counts = path.counts.cpu().numpy()          # of the first micro-batch
    active = int((counts > 0).sum())
    s = 2 if cfg.dtype == "bf16" else 4
    # cost of one launch of the dominant kernel (one micro-batch) and of the whole step
    launch_cost = R.layer_cost(T, cfg.d, cfg.f, cfg.E, cfg.k, s, active_experts=active)
    step_flops = sum(R.layer_cost(q - p, cfg.d, cfg.f, cfg.E, cfg.k, s, active_experts=active).flops for p, q in ranges)
    step_min_bytes = sum(R.layer_cost(q - p, cfg.d, cfg.f, cfg.E, cfg.k, s, active_experts=active).layer_min_bytes
                         for p, q in ranges)
    kernels = {"ffn_input": paths[0].ffn_kernel_name(T, 0), "ffn_output": paths[0].ffn_kernel_name(T, 1)}
    return dict(kernels=kernels, warm_steps=warm_steps, ms_per_step=ms_per_step, ffn_in_ms=ffn_in_ms, ffn_in_pct=ffn_in_pct, calls_ms=calls_ms, counts=counts, cost=launch_cost,
                step_flops=step_flops, step_min_bytes=step_min_bytes, serial_ms=serial_ms)


def expert_plan_experiment(cfg, path, x_d, logits_d, N, S, B, torch, reps=10):
    """Hot-expert redundancy on this workload (the paper's "Load balance" paragraph): every expert
    node is one GPU, so each node's share of the expert FFN is timed alone on this GPU, for the
    plain deployment (E / N consecutive experts per node, no copies) and for the greedy plan with
    S slots per node. The per-expert loads are this batch's own counts (the paper plans from the
    traffic of a previous period). Costs a_i and the cold floor K come from two timed single-expert
    runs on this GPU: a small one (weight streaming) and a large one (per-row slope)."""
    T, E, k = cfg.T, cfg.E, cfg.k
    A = T * k
    path.route(logits_d, T)
    path.dispatch(x_d, T)
    torch.cuda.synchronize()
    counts = path.counts.cpu().tolist()
    i32 = torch.int32

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def one_expert(rows):
        b = torch.zeros(1, dtype=i32, device="cuda")
        e = torch.full((1,), rows, dtype=i32, device="cuda")
        ex = torch.zeros(1, dtype=i32, device="cuda")
        return timed(lambda: B.moe_expert_ffn_segments(path.ctx, T, 1, rows, path.xp, b, e, ex, path.packed, path.h, path.y))

    big = min(A, 2048)
    K_ms = one_expert(min(A, 16))
    per_row_ms = (one_expert(big) - one_expert(big // 2)) / (big - big // 2)   # slope where rows, not weights, cost time
    a = [c * per_row_ms for c in counts]

    def measure(replicas, slots):
        times, rows = [], []
        for node in slots:
            share = path.node_share(node, replicas)
            hint = int(sum(counts[e] / replicas[e] for e, _ in node))
            times.append(timed(lambda: path.expert_ffn_node(T, share, rows_hint=hint)))
            rows.append(hint)
        return times, rows

    per = E // N
    plain_slots = [[(e, 0) for e in range(j * per, (j + 1) * per if j < N - 1 else E)] for j in range(N)]
    plain_cost = [sum(max(a[e], K_ms) for e, _ in node) for node in plain_slots]
    plain_t, plain_rows = measure([1] * E, plain_slots)
    replicas, slots, cost = B.moe_plan_experts(a, K_ms, N, S)
    plan_t, plan_rows = measure(replicas, slots)
    r3 = lambda v: [round(x, 4) for x in v]
    return {"expert_plan": f"{cfg.name}: {E} experts on {N} nodes", "counts": counts,
            "cost_model_ms": {"K_cold_floor": round(K_ms, 4), "per_row": round(per_row_ms, 6)},
            "plain": {"slots_per_node": per, "rows": plain_rows, "predicted_ms": r3(plain_cost), "measured_ms": r3(plain_t),
                      "max_ms": round(max(plain_t), 4), "max_over_mean": round(max(plain_t) / (sum(plain_t) / N), 3)},
            "greedy": {"slots_per_node": S, "replicas": replicas, "slots": slots, "rows": plan_rows,
                       "predicted_ms": r3(cost), "measured_ms": r3(plan_t), "max_ms": round(max(plan_t), 4),
                       "max_over_mean": round(max(plan_t) / (sum(plan_t) / N), 3)},
            "max_node_time_ratio_greedy_over_plain": round(max(plan_t) / max(plain_t), 3)}


def per_expert_breakdown(cfg, path, x_d, logits_d, B, R, torch, reps=10):
    """Every expert's own rows through both FFN GEMMs, timed alone (one segment per call): rows, time,
    rates, and which roof of the paper's model (Section 2.3) the expert sits under on this chip. The
    sum over experts exceeds the fused launch, where experts overlap and share the chip."""
    T, E = cfg.T, cfg.E
    path.route(logits_d, T)
    path.dispatch(x_d, T)
    torch.cuda.synchronize()
    counts = path.counts.cpu().tolist()
    offsets = path.offsets.cpu().tolist()
    s = 2 if cfg.dtype == "bf16" else 4
    ridge = R.ridge_batch(R.MI355X_BF16_DENSE_FLOPS, R.MI355X_HBM_BYTES_PER_S)
    i32 = torch.int32
    rows_out = []
    for e in range(E):
        c = counts[e]
        if c == 0:
            rows_out.append({"expert": e, "rows": 0})
            continue
        b = torch.full((1,), offsets[e], dtype=i32, device="cuda")
        en = torch.full((1,), offsets[e + 1], dtype=i32, device="cuda")
        ex = torch.full((1,), e, dtype=i32, device="cuda")
        call = lambda: B.moe_expert_ffn_segments(path.ctx, T, 1, c, path.xp, b, en, ex, path.packed, path.h, path.y)
        call()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            call()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        flops = 6.0 * c * cfg.d * cfg.f
        nbytes = 3.0 * cfg.d * cfg.f * s + c * (2 * cfg.d + 2 * cfg.f) * s
        rows_out.append({"expert": e, "rows": c, "ms": round(ms, 4), "TFLOP/s": round(flops / ms / 1e9, 1),
                         "GB/s": round(nbytes / ms / 1e6, 1), "roof": "hbm" if c < ridge else "mfma"})
    alone = sum(r.get("ms", 0.0) for r in rows_out)
    return {"per_expert": cfg.name, "ridge_rows": round(ridge, 1), "experts": rows_out,
            "sum_of_experts_alone_ms": round(alone, 4)}


def measure_ceilings(path, B, torch, reps=5):
    """What this chip reaches for the roofline's two denominators, measured beside the layer: a plain
    streaming read of the packed weights, and matrix-core issue from registers with real weight bits as
    operands (bf16 layers only)."""
    sink = torch.zeros(16, dtype=torch.float32, device="cuda")

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3

    nbytes = path.packed.numel()
    got = B.moe_probe_stream_read(path.ctx, path.packed, nbytes, sink)
    out = {"stream_read_GB/s": round(got / timed(lambda: B.moe_probe_stream_read(path.ctx, path.packed, nbytes, sink)) / 1e9, 1),
           "stream_read_bytes": got}
    if path.dtype == "bf16":
        flops = B.moe_probe_mfma(path.ctx, path.packed, 2048, 1024, sink)
        out["mfma_loop_TFLOP/s"] = round(flops / timed(lambda: B.moe_probe_mfma(path.ctx, path.packed, 2048, 1024, sink)) / 1e12, 1)
        out["mfma_loop"] = "v_mfma_f32_32x32x16_bf16 from registers, 1 wave per SIMD, operands = packed weight bits"
    return out


def roofline_entry(cfg, cost, ffn_in_ms, R):
    t = ffn_in_ms * 1e-3
    if cfg.dtype == "bf16":
        peak_flops, unit_f = R.MI355X_BF16_DENSE_FLOPS, "TFLOP/s"
    else:
        peak_flops, unit_f = R.MI355X_FP32_VECTOR_FLOPS, "TFLOP/s"
    t_mem = cost.ffn_in_bytes / R.MI355X_HBM_BYTES_PER_S
    t_cmp = cost.ffn_in_flops / peak_flops
    if t_mem >= t_cmp:
        achieved, peak, unit, bound = cost.ffn_in_bytes / t / 1e9, R.MI355X_HBM_BYTES_PER_S / 1e9, "GB/s", "hbm"
    else:
        achieved, peak, unit = cost.ffn_in_flops / t / 1e12, peak_flops / 1e12, unit_f
        bound = "mfma" if cfg.dtype == "bf16" else "alu"
    # `traffic` cannot be measured inside this process (it needs the profiler's counters): it is the
    # stored result of the rocprofv3 --pmc runs of this workload, and is labelled as such.
    traffic, source = None, None
    rel = f"profiles/traffic_{cfg.name}.json"
    if os.path.exists(os.path.join(ROOT, rel)):
        try:
            traffic = json.load(open(os.path.join(ROOT, rel))).get("ffn_input_hbm_bytes_per_launch")
            source = f"{rel} (stored from earlier rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs; not measured in this run)"
        except Exception:
            traffic = None
    return {"kernel": "ffn_input (fused gate|up GEMM + SiLU*up)", "bound": bound, "achieved": round(achieved, 2),
            "peak": peak, "unit": unit, "frac": round(achieved / peak, 4), "traffic": traffic,
            "traffic_source": source,
            "algorithmic_bytes": cost.ffn_in_bytes, "algorithmic_flops": cost.ffn_in_flops,
            "avg_launch_ms": round(ffn_in_ms, 5)}


def cpu_baseline(cfg, seed, W, x, logits, oracle_mod, sample_tokens):
    """The oracle's whole layer on the first `sample_tokens` tokens of the same batch."""
    n = min(sample_tokens, cfg.T)
    affinity = len(os.sched_getaffinity(0))
    try:
        from threadpoolctl import threadpool_info
        pools = [p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"]
        threads, source = max(pools), "threadpoolctl: threads of the BLAS pool numpy's matmul runs on"
    except Exception:
        threads, source = affinity, "sched_getaffinity (the BLAS pool could not be queried)"
    t0 = time.perf_counter()
    oracle_mod.moe_layer(x[:n], logits[:n], cfg.k, lambda e: (W[0][e], W[1][e], W[2][e]))
    dt = time.perf_counter() - t0
    return {"value": round(n / dt, 3), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"whole layer (route, dispatch, expert FFN, combine) on the first {n} of {cfg.T} tokens, "
                      f"float64 numpy, {dt:.1f} s",
            "gflops": round(6.0 * n * cfg.k * cfg.d * cfg.f / dt / 1e9, 1),
            "cores_source": source, "sched_getaffinity_cpus": affinity, "host_cpus": os.cpu_count()}


def per_call_rates(cfg, r, R):
    """Algorithmic GB/s (and TFLOP/s for the GEMMs) of every call of the first micro-batch, from the per-call times."""
    c, ms = r["cost"], r["calls_ms"]
    gate = cfg.T // cfg.micro_batches * cfg.d * (2 if cfg.dtype == "bf16" else 4) + cfg.E * cfg.d * 4   # x and the gating matrix
    by = {"route": c.route_bytes, "dispatch": c.dispatch_bytes, "route_dispatch": c.route_bytes + c.dispatch_bytes,
          "gate_route": gate + c.route_bytes, "gate_route_dispatch": gate + c.route_bytes + c.dispatch_bytes,
          "ffn_input": c.ffn_in_bytes, "ffn_output": c.ffn_out_bytes, "combine": c.combine_bytes}
    fl = {"ffn_input": c.ffn_in_flops, "ffn_output": c.ffn_out_flops}
    out = {}
    for n, t in ms.items():
        out[n] = {"GB/s": round(by[n] / (t * 1e-3) / 1e9, 1)}
        if n in fl:
            out[n]["TFLOP/s"] = round(fl[n] / (t * 1e-3) / 1e12, 1)
    return out


def synth_skew(cfg):
    from workloads import synth
    return synth.expected_load_skew(cfg)


def result_line(cfg, steps, warmup, r, R, cpu, ceilings=None, router="logits"):
    ms_per_step, counts, cost = r["ms_per_step"], r["counts"], r["cost"]
    sec = ms_per_step * 1e-3
    line = {
        "metric": "MoE-layer tokens/sec (route+dispatch+expert FFN+combine), 1 MI355X",
        "value": round(cfg.T / sec, 1), "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "warmup_steps_run": r.get("warm_steps", warmup),
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "T": cfg.T, "d": cfg.d, "f": cfg.f, "E": cfg.E, "k": cfg.k,
                   "router": "gating GEMM x*W_r inside the timed step (moe_gate_route_dispatch)" if router == "gate"
                   else "logits given (moe_route_dispatch)",
                   "ffn_kernel": r.get("kernels"),
                   "micro_batches": cfg.micro_batches, "load_skew_hint": round(synth_skew(cfg), 3),
                   "tokens_per_expert_mean": cfg.T * cfg.k / cfg.E / cfg.micro_batches,
                   "tokens_per_expert_max": int(counts.max()), "tokens_per_expert_min": int(counts.min()),
                   "tokens_per_expert": [int(c) for c in counts]},
        "roofline": roofline_entry(cfg, cost, r["ffn_in_ms"], R),
        "cpu_baseline": cpu,
        "layer": {"tflops": round(r["step_flops"] / sec / 1e12, 2),
                  "min_bytes": r["step_min_bytes"],
                  "hbm_frac_of_min_bytes": round(r["step_min_bytes"] / sec / R.MI355X_HBM_BYTES_PER_S, 4),
                  "mfma_frac": round(r["step_flops"] / sec / R.MI355X_BF16_DENSE_FLOPS, 4)
                  if cfg.dtype == "bf16" else None,
                  "calls_ms": {k: round(v, 5) for k, v in r["calls_ms"].items()},
                  "calls_rates": per_call_rates(cfg, r, R)},
    }
    line["roofline"]["launch_ms_p10_p50_p90"] = [round(v, 5) for v in r["ffn_in_pct"]]
    if ceilings:
        line["ceilings"] = ceilings
        rf = line["roofline"]
        key = "stream_read_GB/s" if rf["bound"] == "hbm" else "mfma_loop_TFLOP/s"
        if ceilings.get(key):
            rf["frac_of_measured_ceiling"] = round(rf["achieved"] / ceilings[key], 4)
    if r["serial_ms"] is not None:
        line["layer"]["one_stream_ms_per_step"] = round(r["serial_ms"], 5)
    return line


def sweep_entry(line):
    """One point of the curve `sweep` carries: what the per-expert batch was, what the step cost, and
    where the FFN-input GEMM sits against its roofline."""
    c, rf, lay = line["config"], line["roofline"], line["layer"]
    return {"workload": c["workload"], "T": c["T"], "tokens_per_expert_mean": c["tokens_per_expert_mean"],
            "tokens_per_expert_min": c["tokens_per_expert_min"], "tokens_per_expert_max": c["tokens_per_expert_max"],
            "ms_per_step": line["ms_per_step"], "tokens_per_s": line["value"], "layer_tflops": lay["tflops"],
            "ffn_kernel": c.get("ffn_kernel"),
            "ffn_input": {k: rf[k] for k in ("bound", "achieved", "peak", "unit", "frac", "avg_launch_ms")},
            "ffn_output_ms": lay["calls_ms"]["ffn_output"],
            "layer_hbm_frac_of_min_bytes": lay["hbm_frac_of_min_bytes"], "layer_mfma_frac": lay["mfma_frac"]}


def resolve_workload(name, synth):
    if name in synth.CONFIGS:
        return synth.CONFIGS[name]
    if "_T" in name and any(n.startswith(name.split("_T")[0] + "_T") for n in synth.CONFIGS):
        base, T = name.split("_T")          # a named shape at another token count, e.g. mixtral_T1024
        return next(c for n, c in synth.CONFIGS.items() if n.startswith(base + "_T")).with_T(int(T))
    raise SystemExit(f"unknown workload {name!r}; known: {sorted(synth.CONFIGS)}, or one of these shapes at "
                     f"another token count (<shape>_T<N>)")


def micro_batch_study(args, torch, B, R, synth, ms=(1, 2, 3, 4)):
    """The fine-grained many-expert layer (8192 tokens) cut into m micro-batches on two alternating streams
    (the single-GPU echo of the paper's ping-pong micro-batching, Section 4.1, whose m is capped at 4 because
    smaller micro-batches lower GEMM efficiency, Section 4.2): ms per step on two streams and on one."""
    from dataclasses import replace
    base = synth.CONFIGS["finegrained_T8192"]
    paths = [B.MoEPath(base.T, base.d, base.f, base.E, base.k, base.dtype) for _ in range(2)]
    _, gen_s = upload_and_pack(base, args.seed, paths[0], torch, synth, keep=False)
    paths[1].packed = paths[0].packed
    x, logits = make_inputs(base, args.seed, synth)
    x_d, l_d = dev(x, torch), dev(logits, torch)
    rows = []
    for m in ms:
        c = replace(base, micro_batches=m, name=f"{base.name}_m{m}")
        r = time_workload(c, paths, x_d, l_d, args.steps, args.warmup, torch, R, synth, breakdown=False)
        rows.append({"m": m, "tokens_per_expert_mean": round(c.T * c.k / c.E / m, 1),
                     "two_stream_ms_per_step": round(r["ms_per_step"], 5),
                     "one_stream_ms_per_step": round(r["serial_ms"], 5) if r["serial_ms"] is not None else None,
                     "tokens_per_s": round(c.T / (r["ms_per_step"] * 1e-3), 1),
                     "ffn_input_avg_launch_ms": round(r["ffn_in_ms"], 5)})
    for p in paths:
        p.close()
    del paths, x_d, l_d
    torch.cuda.empty_cache()
    return {"workload": base.name, "T": base.T, "d": base.d, "f": base.f, "E": base.E, "k": base.k,
            "streams": 2, "steps": args.steps, "warmup": args.warmup, "rows": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=None,
                    help="time this workload only (default: mixtral_T256 as the headline, plus the Mixtral-shaped "
                         "T sweep and the micro-batch study)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--sweep", action="store_true", help="with --workload mixtral_*: also run the T sweep")
    ap.add_argument("--sweep-lines", action="store_true", help="print one JSON line per sweep point as well")
    ap.add_argument("--no-sweep", action="store_true", help="default run without the T sweep")
    ap.add_argument("--no-micro-batch-study", action="store_true", help="default run without the micro-batch study")
    ap.add_argument("--micro-batches", type=int, default=0,
                    help="override the workload's micro-batch count m (m > 1: two alternating streams)")
    ap.add_argument("--fit", action="store_true",
                    help="with the sweep: fit the paper's expert-time model T_e = k3*b_e + k4 to the measured FFN times")
    ap.add_argument("--expert-plan", default="", metavar="N,S",
                    help="also time every node's share of the expert FFN for N expert nodes, plain deployment "
                         "against the greedy plan with S slots per node (hot experts get copies)")
    ap.add_argument("--per-expert", action="store_true",
                    help="also time every expert's own rows alone (both FFN GEMMs) and print rows, time, rates and roof")
    ap.add_argument("--router", choices=("logits", "gate"), default="logits",
                    help="logits: the step starts at given router logits, as the workloads define; gate: it starts at "
                         "the gating GEMM on x and a seeded gating matrix (moe_gate_route_dispatch)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--ceilings", action="store_true",
                    help="time the streaming-read and register-only MFMA probes even with --no-cpu-baseline")
    ap.add_argument("--cpu-sample-tokens", type=int, default=256)
    ap.add_argument("--calibrate", action="store_true",
                    help="only run a plain device copy of known size (1 GiB) a few times and print its rate; "
                         "under rocprofv3 --pmc this gives the scale of the FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2504_02263_amd import binding as B
    from paper_2504_02263_amd import roofline as R
    from workloads import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    if args.calibrate:
        n = 1 << 30
        src = torch.full((n,), 3, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 10
        print(json.dumps({"calibration": "device copy", "bytes_read": n, "bytes_written": n, "launches": 13,
                          "ms": round(dt * 1e3, 4), "GB/s_read_plus_write": round(2 * n / dt / 1e9, 1)}))
        return

    full = args.workload is None          # the default run: headline + sweep + micro-batch study
    cfg = resolve_workload(args.workload or "mixtral_T256", synth)
    if args.micro_batches > 0:
        from dataclasses import replace
        cfg = replace(cfg, micro_batches=args.micro_batches, name=f"{cfg.name}_m{args.micro_batches}")
    do_sweep = cfg.name.startswith("mixtral") and cfg.micro_batches == 1 and ((full and not args.no_sweep) or args.sweep)
    sweep_T = list(synth.MIXTRAL_SWEEP_T) if do_sweep else []
    T_max = max([cfg.T] + sweep_T)
    if cfg.micro_batches > 1:
        T_max = max(b - a for a, b in synth.microbatch_ranges(cfg.T, cfg.micro_batches))
    # the one thing a serving engine knows about the load that the kernels cannot see from the host: how skewed
    # the router is (1 for the near-uniform workloads; the Zipf workload states its own skew)
    skew = synth.expected_load_skew(cfg)
    paths = [B.MoEPath(T_max, cfg.d, cfg.f, cfg.E, cfg.k, cfg.dtype, load_skew=skew)
             for _ in range(2 if cfg.micro_batches > 1 else 1)]
    W, gen_s = upload_and_pack(cfg, args.seed, paths[0], torch, synth)
    for p in paths[1:]:
        p.packed = paths[0].packed          # one packed weight set serves every stream
    print(f"[bench] weights generated in {gen_s:.1f} s and packed", file=sys.stderr, flush=True)

    w_router = synth.make_router_weight(cfg, args.seed) if args.router == "gate" else None
    w_router_d = dev(w_router, torch) if w_router is not None else None

    def run(c, want_cpu):
        x, logits = make_inputs(c, args.seed, synth)
        x_d, l_d = dev(x, torch), dev(logits, torch)
        r = time_workload(c, paths, x_d, l_d, args.steps, args.warmup, torch, R, synth, w_router_d=w_router_d)
        cpu = None
        if want_cpu:
            print("[bench] timing the CPU oracle on a sample ...", file=sys.stderr, flush=True)
            from oracle import moe_oracle  # the cpu_baseline leg is the only user of the oracle here
            if w_router is not None:       # the oracle computes its own gate scores from the same gating matrix
                logits = moe_oracle.gate_logits(x, w_router)
            cpu = cpu_baseline(c, args.seed, W, x, logits, moe_oracle, args.cpu_sample_tokens)
        return result_line(c, args.steps, args.warmup, r, R, cpu,
                           measure_ceilings(paths[0], B, torch) if want_cpu or args.ceilings else None, router=args.router)

    head = run(cfg, not args.no_cpu_baseline)
    lines = []
    for T in sweep_T:
        if T == cfg.T:
            lines.append(head)
            continue
        print(f"[bench] sweep point T = {T} ...", file=sys.stderr, flush=True)
        lines.append(run(cfg.with_T(T), False))
        if args.sweep_lines:
            print(json.dumps(lines[-1]), flush=True)
    if lines:
        head["sweep"] = [sweep_entry(l) for l in lines]
        big = lines[-1]
        head["roofline_large_batch"] = dict(big["roofline"], workload=big["config"]["workload"],
                                            tokens_per_expert_mean=big["config"]["tokens_per_expert_mean"])
        if head.get("ceilings", {}).get("mfma_loop_TFLOP/s") and big["roofline"]["bound"] == "mfma":
            head["roofline_large_batch"]["frac_of_measured_ceiling"] = round(
                big["roofline"]["achieved"] / head["ceilings"]["mfma_loop_TFLOP/s"], 4)
    if args.fit and len(lines) >= 4:
        # expert time of one layer call = the two FFN GEMMs; b_e = mean tokens per expert
        pts = sorted((l["config"]["tokens_per_expert_mean"],
                      l["layer"]["calls_ms"]["ffn_input"] + l["layer"]["calls_ms"]["ffn_output"]) for l in lines)
        fit = R.fit_expert_time([p[0] for p in pts], [p[1] for p in pts], split=128)
        fit["roofline_ridge_b"] = R.ridge_batch(R.MI355X_BF16_DENSE_FLOPS, R.MI355X_HBM_BYTES_PER_S)
        head["expert_time_model"] = {"model": "T_e[ms] = k3*b_e + k4", "points": pts, "fit": fit}
    if args.per_expert:
        x, logits = make_inputs(cfg, args.seed, synth)
        a0, b0 = synth.microbatch_ranges(cfg.T, cfg.micro_batches)[0]     # the first micro-batch stands for the others
        from dataclasses import replace as _replace
        pe = per_expert_breakdown(_replace(cfg, T=b0 - a0), paths[0], dev(x[a0:b0], torch), dev(logits[a0:b0], torch),
                                  B, R, torch)
        pe["fused_launches_ms"] = round(head["layer"]["calls_ms"]["ffn_input"] + head["layer"]["calls_ms"]["ffn_output"], 4)
        print(json.dumps(pe), flush=True)
    if args.expert_plan:
        N, S = (int(v) for v in args.expert_plan.split(","))
        if cfg.E % N or N * S < cfg.E:
            raise SystemExit("--expert-plan N,S needs E divisible by N and N*S >= E")
        x, logits = make_inputs(cfg, args.seed, synth)
        print(json.dumps(expert_plan_experiment(cfg, paths[0], dev(x, torch), dev(logits, torch), N, S, B, torch)),
              flush=True)
    for p in paths:
        p.close()
    del paths, W
    torch.cuda.empty_cache()
    if full and not args.no_micro_batch_study:
        print("[bench] micro-batch study on finegrained_T8192 ...", file=sys.stderr, flush=True)
        head["micro_batch_study"] = micro_batch_study(args, torch, B, R, synth)
    head["library_source_hash"] = B.library_source_hash()
    print(json.dumps(head), flush=True)


if __name__ == "__main__":
    main()
