#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

Throughput (default).  A step is one pass of the whole path over one batch: moe_route ->
moe_permute -> moe_expert_run (to completion) -> moe_combine, inputs already resident in HBM.  The
default workload is the Mixtral-shaped bf16 prefill batch (512 tokens, 128 LS + 384 BE, 8 experts
top-2, H 4096, F 14336), seeded synthetic data.  Prints ONE JSON line with the throughput, the
roofline figure of the dominant kernel (timed with HIP events on the launch stream, inside the
timed region), the CPU oracle timed on a bounded sample of the same workload and, for the Mixtral
weights, the LS completion latency when a 3584-token BE prompt is in flight (--latency-trials).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg4|cfg5|cfg3_be|cfg3_ls]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published

# HBM bytes per launch of the gate-up kernel measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
# scaled by what the same counters read for a 1 GiB device copy (profiles/bench_<workload>.md).
MEASURED_TRAFFIC_BYTES = {"cfg2": 2032283507, "cfg4": 1919675526, "cfg3_be": 3263265902, "cfg5": 2658861615,
                          "cfg4_mxfp4": 515344980, "cfg3_be_mxfp4": 1775656828}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def gate_up_bytes(cfg, counts, es, ws):
    """Algorithmic HBM bytes of the gate-up launch of a run-to-completion call: W1 and W3 of every
    expert that has rows, once (the launch merges an expert's LS and BE rows into one pass over
    its weights; ws bytes per weight element), the gathered x rows once, the activation written once."""
    touched = int((counts.sum(1) > 0).sum())
    return int(touched * 2 * cfg.F * cfg.H * ws) + cfg.A * cfg.H * es + cfg.A * cfg.F * es


def down_bytes(cfg, counts, es, ws, ksplit):
    touched = int((counts.sum(1) > 0).sum())
    planes = ksplit * cfg.A * cfg.H * 4 * 2 if ksplit > 1 else 0     # partial planes written, then read
    return int(touched * cfg.H * cfg.F * ws) + cfg.A * cfg.F * es + cfg.A * cfg.H * 4 + planes


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def layer_bytes(cfg, counts, es, ws, passes="once"):
    """Algorithmic HBM bytes of one pass of the whole layer: the three weight matrices of every expert
    that has rows (once; or, passes="per_class", once per priority class in which it has rows: the
    strict LS-phase-then-BE-phase order), x read by the router and gathered by the experts, the
    activation written and read, the fp32 expert outputs written and read, y written."""
    if passes == "per_class":
        touched = int((counts[:, 0] > 0).sum()) + int((counts[:, 1] > 0).sum())
    else:
        touched = int((counts.sum(1) > 0).sum())
    return (int(touched * 3 * cfg.F * cfg.H * ws) + cfg.N * cfg.H * es + cfg.A * cfg.H * es + 2 * cfg.A * cfg.F * es +
            2 * cfg.A * cfg.H * 4 + cfg.N * cfg.H * es)


def expert_boundaries(units):
    return [i for i in range(1, len(units)) if units[i][0] != units[i - 1][0] or units[i][1] != units[i - 1][1]]


def measure(cfg, inp, dw, steps, warmup, mx, rowmajor, cuts=0, down_ksplit=0):
    """Times one workload.  Order: W warm-up steps; K steps with HIP events around the gate-up launches and
    K with events around the down launches (per-kernel times); then the timed region, K steps between
    two synchronisations with nothing else on the stream (the figure of record); then per-stage and
    per-step event timings."""
    import numpy as np
    import torch

    import workloads as wl
    from paper_2503_09304_amd.layer import GpuLayer

    es = wl.elem_bytes(cfg)
    ws = 0.5 + 1.0 / 32 if mx else es      # bytes per expert-weight element (4-bit code + its share of a scale byte)
    # 4-bit weights on a decode-sized batch: a workgroup's K-iteration is bound by its conversions, two
    # workgroups share a CU, and four K ranges (512 workgroups, one round) beat the two the
    # configuration default would take (0.057-0.066 against 0.073 ms for the down projection).
    force_ks = down_ksplit or (4 if (mx and cfg.A <= 32 * cfg.E and cfg.F % 256 == 0) else 0)
    g = GpuLayer(inp, dw, down_ksplit=force_ks)
    g.ctx.stream_handle = int(torch.cuda.current_stream().cuda_stream)     # one stream throughout: skip the per-call lookup
    torch.cuda.synchronize()

    def step():
        g.route_permute()
        g.run()
        g.combine()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    counts = g.ctx.get("counts").cpu().numpy()
    # ---- per-kernel times first: the same K steps with the gate-up launches bracketed by events on the launch
    # stream, then with the down launches bracketed (these loops also bring the chip to its steady clocks, which a
    # few warm-up steps of half a millisecond do not: the gate-up loop is therefore run twice, before and after the
    # down loop, and both averages are reported)
    prof = {}
    for tag, kinds in (("gate_up_first_loop", ["gate_up"]), ("down", ["down"]), ("gate_up", ["gate_up"])):
        g.ctx.profile(kinds)
        g.ctx.profile_read()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        prof[tag] = g.ctx.profile_read()[kinds[0]]
    g.ctx.profile(False)

    # ---- timed region (the figure of record): K steps, no event on the stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / steps
    tokens_per_s = cfg.N / (ms_per_step * 1e-3)
    # ---- per-stage times
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
    acc = [0.0] * 4
    for _ in range(5):
        ev[0].record(); g.ctx.route(g.x, g.dw.struct, g.bias, n_tokens=cfg.N)
        ev[1].record(); g.ctx.permute(g.prio)
        ev[2].record(); g.run()
        ev[3].record(); g.combine()
        ev[4].record(); torch.cuda.synchronize()
        for i in range(4):
            acc[i] += ev[i].elapsed_time(ev[i + 1]) / 5
    stages = dict(zip(("route_ms", "permute_ms", "experts_ms", "combine_ms"), (round(v, 4) for v in acc)))
    # ---- spread of single steps
    n_each = max(1, min(steps, 100))
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_each)]
    for a, b in pairs:
        a.record(); step(); b.record()
    torch.cuda.synchronize()
    each = np.array([a.elapsed_time(b) for a, b in pairs])
    step_ms = {"median": round(float(np.median(each)), 4), "min": round(float(each.min()), 4),
               "max": round(float(each.max()), 4), "n": n_each}

    # ---- the same layer stopped and resumed at `cuts` seeded expert boundaries (throughput with the cuts)
    with_cuts = None
    if cuts:
        units = g.ctx.units()
        cps = wl.cut_points(cfg.seed, expert_boundaries(units), cuts)

        def step_cut():
            g.route_permute()
            prev = 0
            for c in cps:
                g.run(c - prev)
                prev = c
            g.run()
            g.combine()
        for _ in range(3):
            step_cut()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step_cut()
        torch.cuda.synchronize()
        ms_cut = (time.perf_counter() - t0) * 1e3 / steps
        with_cuts = {"cuts_at_units": cps, "ms_per_step": round(ms_cut, 4), "tokens_per_s": round(cfg.N / (ms_cut * 1e-3), 1),
                     "slowdown": round(ms_cut / ms_per_step, 4)}

    # what down_ksplit = 0 picks (include/qmoe.h): the fewest K ranges that give every CU a workgroup
    ksplit = 1
    if cfg.N * cfg.k <= 256 * cfg.E:
        wgs = cfg.E * ((cfg.H + 255) // 256)
        if wgs >= 256:
            ksplit = 1
        elif 2 * wgs >= 256 and cfg.F % 128 == 0:
            ksplit = 2
        else:
            ksplit = 4 if cfg.F % 256 == 0 else (2 if cfg.F % 128 == 0 else 1)
    ksplit = force_ks or ksplit
    gu_ms, gu_n = prof["gate_up"]
    dn_ms, dn_n = prof["down"]
    gu_avg_ms = gu_ms / max(gu_n, 1)
    dn_avg_ms = dn_ms / max(dn_n, 1)
    gub = gate_up_bytes(cfg, counts, es, ws)
    dnb = down_bytes(cfg, counts, es, ws, ksplit)
    flops = wl.flops(cfg)
    gu_flops = 4.0 * cfg.A * cfg.H * cfg.F
    hbm_bound = (gub / (HBM_PEAK_GBS * 1e9)) >= (gu_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12))
    if hbm_bound:
        achieved = gub / (gu_avg_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4)}
    else:
        achieved = gu_flops / (gu_avg_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": round(achieved, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4)}
    roof["traffic"] = MEASURED_TRAFFIC_BYTES.get(cfg.name + ("_mxfp4" if mx else "")) if not rowmajor else None
    roof.update({"kernel": "expert_bf16 gate-up (W1,W3 GEMM + SwiGLU)", "avg_launch_ms": round(gu_avg_ms, 4),
                 "launches": gu_n, "timed_by": "HIP events on the launch stream around every gate-up launch, in a loop "
                                               "of the same K steps run right before the timed region (the third such loop; "
                                               "the first, run straight after the W warm-up steps while the clocks still "
                                               "settle, is avg_launch_ms_first_loop)",
                 "avg_launch_ms_first_loop": round(prof["gate_up_first_loop"][0] / max(prof["gate_up_first_loop"][1], 1), 4),
                 "algorithmic_bytes_per_launch": int(gub),
                 "algorithmic_flops_per_launch": gu_flops,
                 "down_avg_launch_ms": round(dn_avg_ms, 4),
                 "down_algorithmic_bytes_per_launch": int(dnb),
                 "down_achieved_GBps": round(dnb / (dn_avg_ms * 1e-3) / 1e9, 1) if dn_ms > 0 else None,
                 "down_achieved_TFLOPs": round(2.0 * cfg.A * cfg.H * cfg.F / (dn_avg_ms * 1e-3) / 1e12, 1) if dn_ms > 0 else None})
    lb = layer_bytes(cfg, counts, es, ws)
    if hbm_bound:
        la = lb / (ms_per_step * 1e-3) / 1e9
        layer = {"bound": "hbm", "algorithmic_bytes": int(lb), "achieved": round(la, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                 "frac": round(la / HBM_PEAK_GBS, 4)}
    else:
        la = flops / (ms_per_step * 1e-3) / 1e12
        layer = {"bound": "mfma", "algorithmic_flops": flops, "achieved": round(la, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                 "unit": "TFLOP/s", "frac": round(la / MFMA_BF16_PEAK_TFLOPS, 4)}
    return {"workload": cfg.name, "ms_per_step": ms_per_step, "tokens_per_s": round(tokens_per_s, 1),
            "layer_tflops": round(flops / (ms_per_step * 1e-3) / 1e12, 2), "layer": layer, "stages_ms": stages,
            "step_ms": step_ms, "roofline": roof, "with_cuts": with_cuts, "_layer": g, "_ws": ws}


def compact(r):
    """The sub-record of a workload other than the headline one."""
    ro = r["roofline"]
    out = {"ms_per_step": round(r["ms_per_step"], 4), "tokens_per_s": r["tokens_per_s"], "layer_tflops": r["layer_tflops"],
           "layer": r["layer"],
           "gate_up": {k: ro[k] for k in ("bound", "achieved", "peak", "unit", "frac", "avg_launch_ms", "traffic",
                                          "algorithmic_bytes_per_launch")},
           "down": {"avg_launch_ms": ro["down_avg_launch_ms"], "GBps": ro["down_achieved_GBps"], "TFLOPs": ro["down_achieved_TFLOPs"]}}
    if r["with_cuts"]:
        out["with_4_preempt_resume_cuts"] = r["with_cuts"]
    return out


def pct(v, p):
    import numpy as np
    return float(np.percentile(np.asarray(v), p))


def ls_latency(wl, q, torch, GpuLayer, dw, trials, units_per_call, lookahead, be_ksplit=0, seed=77, ls_own_stream=False,
               units_per_launch=None):
    """LS completion latency when a BE prompt is in flight (cfg3): the BE context is fed
    `units_per_call` work units per moe_expert_run with at most `lookahead` calls outstanding; at a
    seeded offset into the BE layer an LS batch arrives, the host stops feeding BE, runs the LS
    context to completion and resumes BE from its cursor.  Latency = arrival -> the host sees the
    LS combine finished."""
    import numpy as np
    upl = units_per_launch or q.UINT32_MAX         # launch size of the enqueued (device-stopped) sequence: default the whole layer
    cbe, cls_ = wl.CONFIGS["cfg3_be"], wl.CONFIGS["cfg3_ls"]
    be = GpuLayer(wl.make_inputs(cbe, weights={}), dw, down_ksplit=be_ksplit)
    ls = GpuLayer(wl.make_inputs(cls_, weights={}), dw)

    def run_ls():
        ls.route_permute(); ls.run(); ls.combine(q.MOE_CLASS_LS)

    # With --ls-own-stream the arriving LS batch goes to a stream of its own (default priority): its
    # kernels need not wait for the BE launch in flight to drain, they take the CUs that launch's
    # last workgroups leave free.
    side = torch.cuda.Stream() if ls_own_stream else None

    def run_ls_arrived():
        """LS batch at its arrival under BE load; returns when the host sees its combine done."""
        if side is None:
            run_ls()
            ev = torch.cuda.Event(); ev.record()
        else:
            with torch.cuda.stream(side):
                run_ls()
                ev = torch.cuda.Event(); ev.record()
        ev.synchronize()

    def run_be_all():
        be.route_permute(); be.run(); be.combine()

    for _ in range(3):
        run_be_all(); run_ls()
    torch.cuda.synchronize()
    if side is not None:                      # first use of the stream stays out of the measurement
        with torch.cuda.stream(side):
            run_ls()
        torch.cuda.synchronize()
    # references: BE alone, LS alone on an idle GPU
    t = []
    for _ in range(5):
        torch.cuda.synchronize(); t0 = time.perf_counter(); run_be_all(); torch.cuda.synchronize()
        t.append(time.perf_counter() - t0)
    be_ms = 1e3 * min(t)
    y_ref = be.y.clone()
    t = []
    for _ in range(10):
        torch.cuda.synchronize(); t0 = time.perf_counter(); run_ls(); torch.cuda.synchronize()
        t.append(time.perf_counter() - t0)
    ls_alone_ms = 1e3 * float(np.median(t))

    # the BE layer fed the preemptible way (bounded look-ahead), nothing arriving: what being
    # stoppable at every chunk costs in BE throughput
    def feed_be():
        be.route_permute()
        pending, done = [], False
        while not done:
            while pending and pending[0].query():
                pending.pop(0)
            if len(pending) < lookahead:
                done = be.run(units_per_call) == q.MOE_DONE
                ev = torch.cuda.Event(); ev.record(); pending.append(ev)
        be.combine()
    t = []
    for _ in range(5):
        torch.cuda.synchronize(); t0 = time.perf_counter(); feed_be(); torch.cuda.synchronize()
        t.append(time.perf_counter() - t0)
    be_fed_ms = 1e3 * min(t)

    # the BE layer enqueued whole as gated launches (moe_expert_enqueue), nothing arriving
    def enqueue_be():
        be.route_permute()
        while be.ctx.expert_enqueue(be.x, be.dw.struct, upl) != q.MOE_DONE:
            if be.ctx.expert_collect() == q.MOE_DONE:
                break
        be.combine()
    t = []
    for _ in range(5):
        torch.cuda.synchronize(); t0 = time.perf_counter(); enqueue_be(); torch.cuda.synchronize()
        t.append(time.perf_counter() - t0)
    be_enq_ms = 1e3 * min(t)

    rng = np.random.default_rng(seed)
    fractions = rng.uniform(0.02, 0.95, size=trials)     # arrival point as a fraction of the BE layer's duration
    lat_dev, identical_dev = [], True
    lat, lat_nopre, waited_units, identical = [], [], [], True
    for i, frac in enumerate(fractions):
        # --- run-to-completion baseline: the BE layer is enqueued whole; LS waits behind it
        off = frac * be_ms * 1e-3
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_be_all()
        while time.perf_counter() - t0 < off:
            pass
        run_ls()
        torch.cuda.synchronize()
        lat_nopre.append(time.perf_counter() - (t0 + off))
        # --- preemptive: bounded look-ahead, stop at the next expert-chunk boundary
        off = frac * be_fed_ms * 1e-3
        be.y.fill_(float("nan"))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        cur = be.route_permute()
        pending, done, arrived, t_done = [], False, False, None
        while not done or pending:
            now = time.perf_counter() - t0
            if not arrived and now >= off:
                arrived = True
                waited_units.append(len(pending) * units_per_call)
                run_ls_arrived()
                t_done = time.perf_counter() - t0
                continue
            while pending and pending[0].query():
                pending.pop(0)
            if not done and len(pending) < lookahead:
                rc = be.run(units_per_call)
                ev = torch.cuda.Event(); ev.record(); pending.append(ev)
                done = rc == q.MOE_DONE
        if not arrived:                       # BE finished before the arrival time: LS runs on an idle GPU
            while time.perf_counter() - t0 < off:
                pass
            run_ls(); torch.cuda.synchronize()
            t_done = time.perf_counter() - t0
        be.combine()
        torch.cuda.synchronize()
        lat.append(t_done - off)
        if i < 8:
            identical = identical and bool(torch.equal(be.y.view(torch.int16), y_ref.view(torch.int16)))
        # --- device-side stop: the whole BE layer is on the stream as gated launches; at the arrival the
        # host sets the stop word and enqueues the LS batch behind whatever still runs
        off = frac * be_enq_ms * 1e-3
        be.y.fill_(float("nan"))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        be.route_permute()
        rc = be.ctx.expert_enqueue(be.x, be.dw.struct, upl)
        while time.perf_counter() - t0 < off:
            pass
        be.ctx.expert_stop()
        run_ls_arrived()
        lat_dev.append(time.perf_counter() - t0 - off)
        while rc != q.MOE_DONE:
            rc = be.ctx.expert_collect()
            if rc != q.MOE_DONE:
                rc = be.ctx.expert_enqueue(be.x, be.dw.struct, upl)
        be.combine()
        torch.cuda.synchronize()
        if i < 8:
            identical_dev = identical_dev and bool(torch.equal(be.y.view(torch.int16), y_ref.view(torch.int16)))
    ms = lambda v: round(1e3 * v, 4)
    return {
        "workload": "cfg3: 3584-token BE prompt in flight (28 units of <=256 rows), 512-token LS batch arrives",
        "trials": trials, "units_per_call": units_per_call, "lookahead_calls": lookahead,
        "ls_stream": "own" if ls_own_stream else "shared with BE",
        "ls_latency_ms": {"p50": ms(pct(lat, 50)), "p99": ms(pct(lat, 99)), "max": ms(max(lat))},
        "ls_alone_idle_gpu_ms": round(ls_alone_ms, 4),
        "ls_latency_no_preemption_ms": {"p50": ms(pct(lat_nopre, 50)), "p99": ms(pct(lat_nopre, 99))},
        "be_layer_uninterrupted_ms": round(be_ms, 4),
        "be_layer_fed_with_lookahead_ms": round(be_fed_ms, 4),
        "be_down_ksplit": be_ksplit,
        "device_stop": {"ls_latency_ms": {"p50": ms(pct(lat_dev, 50)), "p99": ms(pct(lat_dev, 99)), "max": ms(max(lat_dev))},
                        "be_layer_enqueued_ms": round(be_enq_ms, 4),
                        "units_per_launch": "all remaining units (the whole layer in one launch pair)" if upl == q.UINT32_MAX else upl,
                        "be_output_bit_identical_after_resume": identical_dev},
        "be_units_enqueued_at_arrival_mean": round(float(np.mean(waited_units)), 2) if waited_units else 0.0,
        "be_output_bit_identical_after_resume": identical,
    }


def serve_bench(args) -> int:
    """Serving comparison above the layer path: a stack of Mixtral-shaped MoE layers, a seeded
    synthetic request stream (Poisson arrivals, 20 % LS, log-normal lengths), batches of at most 32
    jobs formed by the C++ scheduler; the preemptive priority-aware policy against the
    priority-oblivious run-to-completion baseline, at several arrival rates."""
    import torch

    import paper_2503_09304_amd as q
    import workloads as wl
    import serve_glue
    from paper_2503_09304_amd import serve

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 3
    from paper_2503_09304_amd.build import ensure_built
    ensure_built()
    q.lib()
    c = wl.CONFIGS["cfg2"]
    w, keep = serve_glue.synthetic_weights(c.E, c.H, c.F, seed=c.weight_seed or c.seed)
    glue = serve_glue.SyntheticGlue(c.H, c.k)
    rates = [float(r) for r in args.serve_rates.split(",")]
    rows = []
    for rate in rates:
        d = wl.make_jobs(args.serve_jobs, rate, 0.2, seed=9000 + int(rate), max_prompt=args.serve_max_prompt,
                         max_out=args.serve_max_out)
        row = {"rate_jobs_per_s": rate}
        for pre in (False, True):
            jobs = [serve.Job(i, float(d["arrival_s"][i]), q.SCHED_LS if d["is_ls"][i] else q.SCHED_BE,
                              int(d["prompt_len"][i]), int(d["out_len"][i])) for i in range(args.serve_jobs)]
            eng = serve.Engine(w, glue, c.E, c.k, c.H, c.F, layers=args.serve_layers, batch_size=32,
                               max_prompt=args.serve_max_prompt, preemptive=pre, units_per_call=args.units_per_call,
                               lookahead=args.lookahead, chunk_rows=c.chunk_rows)
            warm = [serve.Job(i, 0.0, q.SCHED_BE, args.serve_max_prompt, 2) for i in range(4)]
            eng.run(warm)                      # first-use costs stay out of the measurement
            eng.trace.clear()
            st = eng.run(jobs)
            log(json.dumps(st))
            row[st["policy"]] = st
            del eng
        a, b = row["fcfs_run_to_completion"], row["preemptive"]
        row["ls_ttft_mean_speedup"] = round(a["ls"]["ttft_ms"]["mean"] / b["ls"]["ttft_ms"]["mean"], 2)
        row["ls_turnaround_mean_speedup"] = round(a["ls"]["turnaround_ms"]["mean"] / b["ls"]["turnaround_ms"]["mean"], 2)
        row["be_turnaround_mean_ratio"] = round(b["be"]["turnaround_ms"]["mean"] / a["be"]["turnaround_ms"]["mean"], 2)
        row["jobs_per_s_ratio"] = round(b["jobs_per_s"] / a["jobs_per_s"], 3)
        rows.append(row)
    out = {"metric": "LS time-to-first-token, preemptive vs run-to-completion, layer-stack level",
           "unit": "ms", "n_gpus": 1, "data": "synthetic", "dtype": "bf16",
           "config": {"workload": f"{args.serve_layers} MoE layers of the Mixtral shape (H={c.H} F={c.F} E={c.E} top-{c.k}), "
                                  f"{args.serve_jobs} jobs per rate, 20% LS, prompts 16..{args.serve_max_prompt} tokens, "
                                  f"outputs 4..{args.serve_max_out} tokens, batch size 32",
                      "units_per_call": args.units_per_call, "lookahead_calls": args.lookahead},
           "rates": rows}
    print(json.dumps(out), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--serve", action="store_true",
                    help="run the serving comparison (scheduler + layer stack) instead of the layer benchmark")
    ap.add_argument("--serve-rates", default="40,80,120")
    ap.add_argument("--serve-jobs", type=int, default=200)
    ap.add_argument("--serve-layers", type=int, default=8)
    ap.add_argument("--serve-max-prompt", type=int, default=512)
    ap.add_argument("--serve-max-out", type=int, default=32)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--cpu-sample-tokens", type=int, default=512)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--down-ksplit", type=int, default=0, choices=[0, 1, 2, 4],
                    help="down_ksplit of the benchmarked context (0 = chosen from the configuration)")
    ap.add_argument("--no-ls-first", action="store_true", help="skip the LS-phase-first measurement (profiling runs)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the sub-records of cfg4, cfg3_be and cfg5 that the default (cfg2) run adds")
    ap.add_argument("--rowmajor", action="store_true", help="keep the weights row-major (default: packed at load)")
    ap.add_argument("--weights", default="bf16", choices=["bf16", "mxfp4"],
                    help="expert weight format: bf16 (the headline workload) or 4-bit microscaling FP4")
    ap.add_argument("--latency-trials", type=int, default=100,
                    help="LS-under-BE-load latency trials (Mixtral weights only; 0 = skip)")
    ap.add_argument("--units-per-call", type=int, default=4)
    ap.add_argument("--lookahead", type=int, default=1)
    ap.add_argument("--units-per-launch", type=int, default=0,
                    help="launch size of the enqueued, device-stopped BE sequence (0 = the whole layer at once)")
    ap.add_argument("--be-ksplit", type=int, default=4, choices=[0, 1, 2, 4],
                    help="down_ksplit of the BE context in the latency scenario (0 = from the configuration)")
    ap.add_argument("--calib-gemm", action="store_true",
                    help="also time torch.matmul (the vendor GEMM library) on dense GEMMs of the gate-up shape: a yardstick")
    ap.add_argument("--calib-mfma", action="store_true",
                    help="also launch the register-only MFMA loop, the yardstick for MFMA-busy and clock counters")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy, the yardstick for HBM byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (no sharding, no collectives); --gpus must be 1")
        return 2
    if args.serve:
        return serve_bench(args)

    import numpy as np
    import torch

    import paper_2503_09304_amd as q
    import workloads as wl
    from paper_2503_09304_amd.layer import DevWeights, GpuLayer

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 3
    from paper_2503_09304_amd.build import ensure_built
    ensure_built()  # what is built is what runs; built here only if there is nothing
    q.lib()  # fail loudly if the HIP library is missing
    cfg = wl.CONFIGS[args.workload]
    log("workload", wl.describe(cfg))
    t0 = time.time()
    mx = args.weights == "mxfp4"
    if mx:
        from paper_2503_09304_amd.layer import DevWeightsMX
        w4 = wl.make_weights_mxfp4(cfg)
        inp = wl.make_inputs(cfg, weights={})
    else:
        inp = wl.make_inputs(cfg)
    log(f"inputs drawn in {time.time() - t0:.1f}s")
    if mx:
        dw = DevWeightsMX(w4).packed()
    else:
        dw = DevWeights(inp.w)
        if not args.rowmajor:
            dw = dw.packed()      # one-time re-layout at model load, outside the timed region
    torch.cuda.synchronize()
    if args.calib_copy:
        src = torch.ones(1 << 29, dtype=torch.bfloat16, device="cuda:0")      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.calib_mfma and cfg.dtype == "bf16" and not mx:
        # yardstick for the MFMA counters: the register-only MFMA loop on the workload's own x and W1 bits,
        # one workgroup (4 waves, one per SIMD) per compute unit
        xs = torch.from_numpy(inp.x.view(np.int16)).to("cuda:0")
        sink = torch.zeros(1, dtype=torch.float32, device="cuda:0")
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        # the clock settles over the first tens of milliseconds of load: three launches to warm up, then
        # one wave per SIMD, two waves per SIMD, and one wave per SIMD again
        for label, wgs in (("warm-up", cus), ("1 wave/SIMD", cus), ("2 waves/SIMD", 2 * cus), ("1 wave/SIMD again", cus)):
            for rep in range(3):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                q.moe_probe_mfma(xs, dw.W1, 20000, wgs, sink)
                b.record()
                torch.cuda.synchronize()
                ms = a.elapsed_time(b)
                log(f"mfma probe ({label}): {wgs} workgroups x 4 waves x 20000 x 8 MFMAs in {ms:.3f} ms = "
                    f"{wgs * 4 * 20000 * 8 * 32768 / ms / 1e9:.1f} TFLOP/s")
        del xs, sink

    if args.calib_gemm and cfg.dtype == "bf16":
        # yardstick: the vendor library (whatever torch.matmul dispatches to) on dense GEMMs of the gate-up shape,
        # random operands of the workload's distributions; no gather, no SwiGLU, no ragged segments
        rows = cfg.A // cfg.E // 32 * 32
        for name, a_shape, b_shape in (("one dense GEMM [A,H] x [H,2F]", (cfg.A, cfg.H), (cfg.H, 2 * cfg.F)),
                                        ("batched over experts [E,A/E,H] x [E,H,2F]", (cfg.E, rows, cfg.H), (cfg.E, cfg.H, 2 * cfg.F))):
            ta = torch.randn(a_shape, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
            tb = (torch.randn(b_shape, device="cuda:0", dtype=torch.float32) * 0.02).to(torch.bfloat16)
            flop = 2.0 * ta.numel() * b_shape[-1]
            for _ in range(5):
                torch.matmul(ta, tb)
            torch.cuda.synchronize()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
            for e0, e1 in ev:
                e0.record(); torch.matmul(ta, tb); e1.record()
            torch.cuda.synchronize()
            ts = sorted(e0.elapsed_time(e1) for e0, e1 in ev)
            log(f"vendor GEMM yardstick, {name}: median {ts[10]:.3f} ms = {flop / ts[10] / 1e9:.0f} TFLOP/s, best {flop / ts[0] / 1e9:.0f}")
            del ta, tb

    m = measure(cfg, inp, dw, args.steps, args.warmup, mx, args.rowmajor, down_ksplit=args.down_ksplit)
    g = m.pop("_layer")
    ms_per_step = m["ms_per_step"]

    # ---- LS tokens first inside a mixed batch (the strict priority-major order: every LS unit, the LS
    # rows combined, then every BE unit): two passes over the weights of experts that hold both classes
    ls_first = None
    n_ls_units = sum(1 for u in g.ctx.units() if u[1] == 0)
    if 0 < n_ls_units < g.ctx.cursor.n_units and not args.no_ls_first:
        counts = g.ctx.get("counts").cpu().numpy()
        t_ls, t_all = [], []
        for _ in range(10):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            g.route_permute()
            g.run(n_ls_units)
            g.combine(q.MOE_CLASS_LS)
            e_ls = torch.cuda.Event(); e_ls.record()
            g.run()
            g.combine(q.MOE_CLASS_BE)
            e_ls.synchronize()
            t_ls.append(time.perf_counter() - t0)
            torch.cuda.synchronize()
            t_all.append(time.perf_counter() - t0)
        two_pass_bytes = layer_bytes(cfg, counts, wl.elem_bytes(cfg), m["_ws"], passes="per_class")
        whole = float(np.median(t_all))
        ls_first = {"ls_rows_ready_ms": round(1e3 * float(np.median(t_ls)), 4), "whole_batch_ms": round(1e3 * whole, 4),
                    "tokens_per_s": round(cfg.N / whole, 1),
                    "algorithmic_bytes": int(two_pass_bytes),
                    "layer_GBps": round(two_pass_bytes / whole / 1e9, 1),
                    "layer_frac_of_hbm_peak": round(two_pass_bytes / whole / 1e9 / HBM_PEAK_GBS, 4),
                    "single_call_ms": round(ms_per_step, 4), "ls_units": n_ls_units, "units": int(g.ctx.cursor.n_units)}
        log("LS-first inside the mixed batch:", json.dumps(ls_first))

    # ---- LS latency while a long BE batch is in flight (Mixtral weights)
    lat = None
    mixtral = cfg.weight_seed == wl.CONFIGS["cfg2"].weight_seed and cfg.dtype == "bf16" and not mx and not args.rowmajor
    if args.latency_trials > 0 and mixtral:
        lat = ls_latency(wl, q, torch, GpuLayer, dw, args.latency_trials, args.units_per_call, args.lookahead,
                         be_ksplit=args.be_ksplit, units_per_launch=args.units_per_launch)
        own = ls_latency(wl, q, torch, GpuLayer, dw, args.latency_trials, args.units_per_call, args.lookahead,
                         be_ksplit=args.be_ksplit, ls_own_stream=True, units_per_launch=args.units_per_launch)
        lat["ls_on_own_stream"] = {"ls_latency_ms": own["ls_latency_ms"], "device_stop": own["device_stop"],
                                   "be_output_bit_identical_after_resume": own["be_output_bit_identical_after_resume"]}
        log("LS latency under BE load:", json.dumps(lat))

    # ---- the other workloads the targets are stated on, as compact sub-records of the same run
    others = {}
    if not args.no_other_workloads and args.workload == "cfg2" and mixtral:
        for name in ("cfg4", "cfg3_be"):
            c = wl.CONFIGS[name]
            r = measure(c, wl.make_inputs(c, weights={}), dw, args.steps, max(3, args.warmup // 2), False, False)
            r.pop("_layer")
            others[name] = compact(r)
            log(name, json.dumps(others[name]))
        c = wl.CONFIGS["cfg5"]
        i5 = wl.make_inputs(c)
        dw5 = DevWeights(i5.w).packed()
        r = measure(c, i5, dw5, args.steps, max(3, args.warmup // 2), False, False, cuts=4)
        r.pop("_layer")
        others["cfg5"] = compact(r)
        log("cfg5", json.dumps(others["cfg5"]))
        del dw5, i5

    # ---- the oracle, as it stands, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        ns = min(args.cpu_sample_tokens, cfg.N)
        xs, ps = inp.x[:ns], inp.prio[:ns]
        t0 = time.perf_counter()
        w_or = oracle.mxfp4_weights_as_bf16(w4) if mx else inp.w
        lay = oracle.OracleLayer(xs, w_or, ps, inp.bias, cfg.k, cfg.chunk_rows)
        lay.run()
        y_ref, _ = lay.y()
        t_cpu = time.perf_counter() - t0
        nthreads = oracle.threads()
        # one thread, the tiny fp32 layer (cfg1): the oracle's per-core speed
        c1 = wl.CONFIGS["cfg1"]
        i1 = wl.make_inputs(c1)
        oracle.set_threads(1)
        t0 = time.perf_counter()
        l1 = oracle.OracleLayer(i1.x, i1.w, i1.prio, i1.bias, c1.k, c1.chunk_rows)
        l1.run(); l1.y()
        t_one = time.perf_counter() - t0
        oracle.set_threads(nthreads)
        cpu = {"value": round(ns / t_cpu, 3), "unit": "tokens/s", "cores": nthreads, "kind": "oracle",
               "sample": f"first {ns} tokens of the {cfg.name} batch through the whole layer (fp64, {t_cpu:.1f} s)",
               "cpu_model": cpu_model(), "cfg1_single_thread_ms": round(1e3 * t_one, 3)}
        log(f"oracle: {ns} tokens in {t_cpu:.1f}s on {nthreads} threads ({cpu_model()}); cfg1 on one thread {1e3 * t_one:.2f} ms")

    out = {
        "metric": "MoE-layer tokens/s + % MFMA/HBM roofline (Mixtral shape); LS latency under BE load",
        "value": m["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: N={cfg.N} ({cfg.n_ls} LS) H={cfg.H} F={cfg.F} E={cfg.E} top-{cfg.k} "
                               f"chunk_rows={cfg.chunk_rows} seed={cfg.seed}",
                   "call": "one run-to-completion moe_expert_run (LS units first in the unit list; an expert's "
                           "LS and BE rows share one pass over its weights)",
                   "weights": ("4-bit microscaling FP4 (e2m1 + e8m0 per 32), packed at load" if mx else
                               "row-major" if args.rowmajor else "packed at load (moe_pack_weights)"),
                   "units": int(g.ctx.cursor.n_units)},
        "layer_tflops": m["layer_tflops"],
        "layer_roofline": m["layer"],
        "stages_ms": m["stages_ms"],
        "step_ms": m["step_ms"],
        "roofline": m["roofline"],
        "execution_order": {
            "value_is": "merged_single_call",
            "merged_single_call": {"ms": round(ms_per_step, 4), "tokens_per_s": m["tokens_per_s"],
                                   "what": "one call spans both phases; an expert's LS and BE rows share one pass over its weights"},
            "priority_major_two_phase": ls_first,
        },
        "other_workloads": others or None,
        "ls_latency_under_be_load": lat,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
