"""Policy-chosen unit order on the GPU (moe_expert_run_units, moe_combine_complete) against the
oracle: the completion mask is exact, complete tokens' rows equal the uninterrupted run bit for bit,
incomplete rows stay untouched, and finishing the layer in any order reproduces the uninterrupted
output bit for bit."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import paper_2503_09304_amd as q
import workloads as wl
from gpu_util import DEV, GpuLayer, as_f64, rel_err, to_host

pytestmark = pytest.mark.gpu


def cases():
    base = dict(dtype="bf16", seed=930, E=8, k=2, H=256, F=512, N=300, n_ls=75, chunk_rows=32)
    yield "bf16", wl.LayerConfig("p1", **base)
    yield "bf16_top4_skew", wl.LayerConfig("p2", **{**base, "E": 16, "k": 4, "N": 500, "n_ls": 100, "chunk_rows": 48,
                                                    "bias_kind": "zipf", "bias_arg": 1.1, "seed": 931})
    yield "f32", wl.LayerConfig("p3", dtype="f32", seed=932, E=5, k=3, H=100, F=72, N=150, n_ls=40, chunk_rows=17)
    # enough segments that one call needs several launches
    yield "bf16_many_units", wl.LayerConfig("p4", dtype="bf16", seed=933, E=256, k=4, H=128, F=128, N=1500, n_ls=400,
                                            chunk_rows=4)


@pytest.mark.parametrize("name,cfg", list(cases()), ids=[n for n, _ in cases()])
def test_any_unit_order_matches_oracle_and_the_uninterrupted_run(name, cfg):
    inp = wl.make_inputs(cfg)
    ref = GpuLayer(inp).full()                                   # uninterrupted, list order
    y_ref = ref.y.clone()
    o_ref = ref.ctx.get("expert_out").clone()
    pk = ref.dw.packed() if cfg.dtype == "bf16" else ref.dw

    lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows,
                             logits=to_host(ref.ctx.get("logits")).astype(np.float64))
    g = GpuLayer(inp, pk)
    cur = g.route_permute()
    nu = cur.n_units
    assert nu == lay.n_units and nu > 8
    rng = np.random.default_rng(cfg.seed)
    order = [int(u) for u in rng.permutation(nu)]
    a, b = order[: nu // 3], order[nu // 3: 2 * nu // 3]

    # a policy's first pick: a third of the units, arbitrary order
    rc = g.ctx.expert_run_units(g.x, g.dw.struct, a)
    assert rc == q.MOE_OK
    lay.run_units(a)
    assert g.ctx.cursor.next_unit == lay.next_unit
    comp = torch.full((cfg.N,), 7, dtype=torch.uint8, device=DEV)
    g.combine_complete = lambda c=None: g.ctx.combine_complete(g.y, c)
    g.combine_complete(comp)
    torch.cuda.synchronize()
    y_or, comp_or = lay.y()
    comp_h = comp.cpu().numpy().astype(bool)
    assert np.array_equal(comp_h, comp_or)                       # completion mask: exact
    print(f"  {name}: {nu} units, after {len(a)}: {int(comp_h.sum())}/{cfg.N} tokens complete", flush=True)
    if name == "bf16_many_units":
        assert len(a) > 384          # more row segments than one launch takes: the call loops
    y_mid = g.y.clone()
    same = y_mid.view(torch.int16 if cfg.dtype == "bf16" else torch.int32) == y_ref.view(torch.int16 if cfg.dtype == "bf16" else torch.int32)
    done_rows = torch.from_numpy(comp_h).to(DEV)
    assert bool(same[done_rows].all())                           # complete rows: final value already
    assert bool(torch.isnan(y_mid[~done_rows].float()).all())    # the others untouched (NaN sentinel)
    if comp_h.any():
        tol = 2e-2 if cfg.dtype == "bf16" else 1e-4
        got = as_f64(to_host(y_mid))[comp_h]
        assert rel_err(got, y_or[comp_h]) <= tol

    # the cursor path carries on from the first unit that has not run, skipping what already ran
    rc = g.run(3)
    lay.run(3)
    assert g.ctx.cursor.next_unit == lay.next_unit
    # class-wise combine is refused while a class has unexecuted units
    if lay.executed[lay.units[:, 1] == 0].min() == 0:
        with pytest.raises(q.MoeError) as e:
            g.combine(q.MOE_CLASS_LS)
        assert e.value.code == q.MOE_E_INCOMPLETE
    # second pick, then everything that is left in reverse list order
    b = [u for u in b if not lay.executed[u]]
    g.ctx.expert_run_units(g.x, g.dw.struct, b)
    lay.run_units(b)
    g.combine_complete(comp)
    torch.cuda.synchronize()
    assert np.array_equal(comp.cpu().numpy().astype(bool), lay.y()[1])
    rest = [u for u in range(nu) if not lay.executed[u]][::-1]
    rc = g.ctx.expert_run_units(g.x, g.dw.struct, rest)
    assert rc == q.MOE_DONE and g.ctx.cursor.next_unit == nu
    lay.run_units(rest)
    g.y.fill_(float("nan"))
    g.combine()                                                  # every class is finished now
    torch.cuda.synchronize()
    it = torch.int16 if cfg.dtype == "bf16" else torch.int32
    assert torch.equal(g.y.view(it), y_ref.view(it))             # any order == list order, bit for bit
    assert torch.equal(g.ctx.get("expert_out").view(torch.int32), o_ref.view(torch.int32))
    g.y.fill_(float("nan"))
    g.combine_complete(comp)
    torch.cuda.synchronize()
    assert bool(comp.all()) and torch.equal(g.y.view(it), y_ref.view(it))


def test_bad_unit_lists_run_nothing():
    cfg = wl.LayerConfig("p5", dtype="bf16", seed=934, E=8, k=2, H=128, F=128, N=100, n_ls=30, chunk_rows=16)
    inp = wl.make_inputs(cfg)
    g = GpuLayer(inp)
    cur = g.route_permute()
    nu = cur.n_units
    for bad in ([0, 1, 1], [nu], [2, 0, nu + 5]):
        with pytest.raises(q.MoeError) as e:
            g.ctx.expert_run_units(g.x, g.dw.struct, bad)
        assert e.value.code == q.MOE_E_ARG
    assert g.ctx.cursor.next_unit == 0
    g.ctx.expert_run_units(g.x, g.dw.struct, [1])
    assert g.ctx.cursor.next_unit == 0                           # unit 0 has not run
    with pytest.raises(q.MoeError):
        g.ctx.expert_run_units(g.x, g.dw.struct, [1])            # already executed
    g.ctx.expert_run_units(g.x, g.dw.struct, [])                 # an empty pick is fine
    g.ctx.expert_run_units(g.x, g.dw.struct, [0])
    assert g.ctx.cursor.next_unit == 2
    assert g.run() == q.MOE_DONE
    ref = GpuLayer(inp).full()
    g.combine()
    torch.cuda.synchronize()
    assert torch.equal(g.y.view(torch.int16), ref.y.view(torch.int16))


def test_example_policies():
    from paper_2503_09304_amd import policies
    cfg = wl.LayerConfig("p6", dtype="bf16", seed=935, E=8, k=2, H=128, F=256, N=400, n_ls=90, chunk_rows=32,
                         bias_kind="zipf", bias_arg=1.1)
    inp = wl.make_inputs(cfg)
    ref = GpuLayer(inp).full()
    it = torch.int16
    # busiest expert first: same bits as the list order
    g = GpuLayer(inp, ref.dw)
    g.route_permute()
    units = g.ctx.units()
    order = policies.busiest_expert_first(units)
    assert sorted(order) == policies.list_order(units)
    assert [units[i][1] for i in order] == sorted(u[1] for u in units)         # LS chunks still first
    assert g.ctx.expert_run_units(g.x, g.dw.struct, order) == q.MOE_DONE
    g.combine()
    torch.cuda.synchronize()
    assert torch.equal(g.y.view(it), ref.y.view(it))
    # hold one expert back: exactly the tokens that did not choose it are complete
    g = GpuLayer(inp, ref.dw)
    g.route_permute()
    held = 2
    now, later = policies.without_experts(units, [held])
    g.ctx.expert_run_units(g.x, g.dw.struct, now)
    comp = torch.zeros(cfg.N, dtype=torch.uint8, device=DEV)
    g.ctx.combine_complete(g.y, comp)
    torch.cuda.synchronize()
    idx = to_host(g.ctx.get("topk_idx"))
    assert np.array_equal(comp.cpu().numpy().astype(bool), ~(idx == held).any(axis=1))
    assert g.ctx.expert_run_units(g.x, g.dw.struct, later) == q.MOE_DONE
    g.combine()
    torch.cuda.synchronize()
    assert torch.equal(g.y.view(it), ref.y.view(it))
