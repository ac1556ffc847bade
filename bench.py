#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

A step is one pass of the whole path over one batch: moe_route -> moe_permute -> moe_expert_run
(to completion) -> moe_combine, inputs already resident in HBM.  The default workload is the
Mixtral-shaped bf16 prefill batch (512 tokens, 128 LS + 384 BE, 8 experts top-2, H 4096, F 14336),
seeded synthetic data.  Prints ONE JSON line with the throughput, the roofline figure of the
dominant kernel (timed with HIP events on the launch stream, inside the timed region) and the CPU
oracle timed on a bounded sample of the same workload.

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
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def gate_up_bytes(cfg, counts, es):
    """Algorithmic HBM bytes of the gate-up launch of a run-to-completion call: W1 and W3 of every
    expert once per priority phase in which it has rows, the gathered x rows once, the activation
    written once."""
    touched = int((counts > 0).sum())          # (expert, phase) pairs with work
    w = touched * 2 * cfg.F * cfg.H * es
    return w + cfg.A * cfg.H * es + cfg.A * cfg.F * es


def down_bytes(cfg, counts, es):
    touched = int((counts > 0).sum())
    return touched * cfg.H * cfg.F * es + cfg.A * cfg.F * es + cfg.A * cfg.H * 4


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--cpu-sample-tokens", type=int, default=512)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--rowmajor", action="store_true", help="keep the weights row-major (default: packed at load)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy, the yardstick for HBM byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (no sharding, no collectives); --gpus must be 1")
        return 2

    import numpy as np
    import torch

    import paper_2503_09304_amd as q
    import workloads as wl
    from gpu_util import DevWeights, GpuLayer

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 3
    q.lib()  # fail loudly if the HIP library is missing
    cfg = wl.CONFIGS[args.workload]
    es = wl.elem_bytes(cfg)
    log("workload", wl.describe(cfg))
    t0 = time.time()
    inp = wl.make_inputs(cfg)
    log(f"inputs drawn in {time.time() - t0:.1f}s")
    dw = DevWeights(inp.w)
    if not args.rowmajor:
        dw = dw.packed()          # one-time re-layout at model load, outside the timed region
    g = GpuLayer(inp, dw)
    torch.cuda.synchronize()

    def step():
        g.route_permute()
        g.run()
        g.combine()

    if args.calib_copy:
        src = torch.ones(1 << 29, dtype=torch.bfloat16, device="cuda:0")      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    counts = g.ctx.get("counts").cpu().numpy()
    g.ctx.profile(True)
    g.ctx.profile_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = g.ctx.profile_read()
    g.ctx.profile(False)
    ms_per_step = dt * 1e3 / args.steps
    tokens_per_s = cfg.N / (ms_per_step * 1e-3)

    # ---- per-stage times (separate, untimed-region loop; for the log only)
    stages = {}
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

    gu_ms, gu_n = prof["gate_up"]
    dn_ms = prof["down"][0] + prof["down_reduce"][0]
    gu_avg_ms = gu_ms / max(gu_n, 1)
    gub = gate_up_bytes(cfg, counts, es)
    dnb = down_bytes(cfg, counts, es)
    flops = wl.flops(cfg)
    gu_flops = 4.0 * cfg.A * cfg.H * cfg.F
    hbm_bound = (gub / (HBM_PEAK_GBS * 1e9)) >= (gu_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12))
    if hbm_bound:
        achieved = gub / (gu_avg_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None}
    else:
        achieved = gu_flops / (gu_avg_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": round(achieved, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None}
    roof.update({"kernel": "expert_bf16 gate-up (W1,W3 GEMM + SwiGLU)", "avg_launch_ms": round(gu_avg_ms, 4),
                 "launches": gu_n, "algorithmic_bytes_per_launch": int(gub),
                 "algorithmic_flops_per_launch": gu_flops,
                 "down_kernel_ms_per_step": round(dn_ms / max(args.steps, 1), 4),
                 "down_algorithmic_bytes_per_step": int(dnb)})

    # ---- the oracle, as it stands, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        ns = min(args.cpu_sample_tokens, cfg.N)
        xs, ps = inp.x[:ns], inp.prio[:ns]
        t0 = time.perf_counter()
        lay = oracle.OracleLayer(xs, inp.w, ps, inp.bias, cfg.k, cfg.chunk_rows)
        lay.run()
        y_ref, _ = lay.y()
        t_cpu = time.perf_counter() - t0
        cpu = {"value": round(ns / t_cpu, 3), "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
               "sample": f"first {ns} tokens of the {cfg.name} batch through the whole layer (fp64, {t_cpu:.1f} s)"}
        log(f"oracle: {ns} tokens in {t_cpu:.1f}s on {oracle.threads()} threads")

    out = {
        "metric": "MoE-layer tokens/s",
        "value": round(tokens_per_s, 1),
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
                   "order": "priority-major (LS units, then BE units)",
                   "weights": "row-major" if args.rowmajor else "packed at load (moe_pack_weights)", "units": int(g.ctx.cursor.n_units)},
        "layer_tflops": round(flops / (ms_per_step * 1e-3) / 1e12, 2),
        "stages_ms": stages,
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
