"""Expert work enqueued ahead and stopped from the device side (moe_expert_enqueue / moe_expert_stop /
moe_expert_collect): with or without a stop, wherever the stop lands, and with another context run
in between, the final output equals the uninterrupted run bit for bit and the oracle within
tolerance; a stop takes effect inside a launch (units are booked one by one, not launch by launch);
the context refuses other calls while pending."""
from __future__ import annotations

import time

import numpy as np
import pytest
import torch

import oracle
import paper_2503_09304_amd as q
import workloads as wl
from gpu_util import GpuLayer, as_f64, rel_err, to_host

pytestmark = pytest.mark.gpu


def bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


def cases():
    yield "bf16", wl.LayerConfig("e1", dtype="bf16", seed=950, E=8, k=2, H=1024, F=2048, N=3000, n_ls=0, chunk_rows=128)
    yield "bf16_mixed", wl.LayerConfig("e2", dtype="bf16", seed=951, E=16, k=4, H=256, F=512, N=900, n_ls=200, chunk_rows=32)
    yield "f32", wl.LayerConfig("e3", dtype="f32", seed=952, E=5, k=3, H=100, F=72, N=400, n_ls=100, chunk_rows=16)


@pytest.mark.parametrize("name,cfg", list(cases()), ids=[n for n, _ in cases()])
def test_enqueue_stop_collect_resume(name, cfg):
    inp = wl.make_inputs(cfg)
    ref = GpuLayer(inp).full()
    dw = ref.dw.packed() if cfg.dtype == "bf16" else ref.dw
    other = GpuLayer(wl.make_inputs(wl.scaled(cfg, N=64, n_ls=64, seed=cfg.seed + 7), weights=inp.w), dw)
    other_ref = GpuLayer(other.inp, dw).full()
    g = GpuLayer(inp, dw)

    # no stop at all: one enqueue, one collect
    cur = g.route_permute()
    nu = cur.n_units
    assert g.ctx.expert_enqueue(g.x, g.dw.struct, 3) == q.MOE_OK
    with pytest.raises(q.MoeError) as e:
        g.combine()
    assert e.value.code == q.MOE_E_STATE                         # pending: collect first
    with pytest.raises(q.MoeError) as e:
        g.run(1)
    assert e.value.code == q.MOE_E_STATE
    assert g.ctx.expert_collect() == q.MOE_DONE and g.ctx.cursor.next_unit == nu
    g.combine()
    torch.cuda.synchronize()
    assert torch.equal(bits(g.y), bits(ref.y))

    # stops at different points of the sequence; another context runs while this one is parked
    seen = set()
    for trial, delay_us in enumerate([0, 0, 30, 80, 150, 300, 600, 1200, 2500]):
        g.y.fill_(float("nan"))
        cur = g.route_permute()
        per = (1, 2, 3, q.UINT32_MAX)[trial % 4]         # launches of 1-3 units, or the whole remainder at once
        rounds = 0
        while True:
            rc = g.ctx.expert_enqueue(g.x, g.dw.struct, per)
            if rc == q.MOE_DONE:
                break
            if rounds == 0:
                t0 = time.perf_counter()
                while (time.perf_counter() - t0) * 1e6 < delay_us:
                    pass
                g.ctx.expert_stop()
                other.full()                                       # enqueued behind whatever still runs
                assert torch.equal(bits(other.y), bits(other_ref.y))
            rc = g.ctx.expert_collect()
            if rounds == 0:
                # units that had run when the stop took effect: any subset of the list, booked one by one
                complete = torch.zeros(cfg.N, dtype=torch.uint8, device=g.y.device)
                g.ctx.combine_complete(g.y, complete)
                torch.cuda.synchronize()
                m = complete.bool()
                assert torch.equal(bits(g.y[m]), bits(ref.y[m]))   # what is booked is final
                seen.add(int(m.sum().item()))
            rounds += 1
            if rc == q.MOE_DONE:
                break
            if rounds == 1 and trial % 2:
                g.run(2)                                           # the cursor call carries on just as well
        assert g.ctx.cursor.next_unit == nu
        g.combine()
        torch.cuda.synchronize()
        assert torch.equal(bits(g.y), bits(ref.y)), (trial, delay_us)
        assert torch.equal(g.ctx.get("expert_out").view(torch.int32), ref.ctx.get("expert_out").view(torch.int32))
    print(f"  {name}: {nu} units, {cfg.N} tokens; tokens complete when the stop took effect, per trial: {sorted(seen)}", flush=True)

    # and the result is the oracle's
    r = g.fetch("logits", "y")
    lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows, logits=r["logits"].astype(np.float64))
    lay.run()
    y_or, _ = lay.y()
    assert rel_err(as_f64(r["y"]), y_or) <= (2e-2 if cfg.dtype == "bf16" else 1e-4)
