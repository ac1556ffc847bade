"""Parity at the full workload sizes, in the launch configuration the benchmark times: the oracle
runs every token of every named workload (seconds each on the host's cores) and expert outputs and y
are compared element by element; integer artefacts are compared in full.  Needs an MI355X (-m gpu)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_09304_amd as q
import workloads as wl
from gpu_util import DevWeights, GpuLayer, rel_err, to_host
from test_gpu_parity import assert_bit_identical, bits, check_layer, check_values, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mixtral():
    w = wl.make_weights(wl.CONFIGS["cfg2"])
    return w, DevWeights(w).packed()       # the layout the benchmark times


def sample(cfg, n, seed=0):
    rng = np.random.default_rng([cfg.seed, 555, seed])
    return np.sort(rng.choice(cfg.N, size=min(n, cfg.N), replace=False))


def expert_boundaries(units):
    """Cursor positions where the expert or the phase changes between consecutive units."""
    return [i for i in range(1, len(units)) if units[i][0] != units[i - 1][0] or units[i][1] != units[i - 1][1]]


def test_cfg2_mixtral_prefill(mixtral):
    w, dw = mixtral
    cfg = wl.CONFIGS["cfg2"]
    inp = wl.make_inputs(cfg, weights=w)
    g, r = check_layer(inp, dev_w=dw)
    say("  counts [E][LS,BE]:", r["counts"].tolist())
    units = g.ctx.units()
    assert_bit_identical(inp, wl.cut_points(cfg.seed, expert_boundaries(units), 4), dev_w=dw, base=g)


def test_cfg4_mixtral_decode_hot_expert(mixtral):
    w, dw = mixtral
    cfg = wl.CONFIGS["cfg4"]
    inp = wl.make_inputs(cfg, weights=w)
    g, r = check_layer(inp, dev_w=dw)
    share0 = r["counts"][0].sum() / cfg.A
    say(f"  expert 0 holds {share0:.1%} of the assignments; counts {r['counts'].tolist()}")
    assert share0 > 0.2
    units = g.ctx.units()
    assert_bit_identical(inp, tuple(range(1, len(units))), dev_w=dw, base=g)


def test_cfg3_ls_batch_preempts_a_be_prompt(mixtral):
    w, dw = mixtral
    cbe, cls_ = wl.CONFIGS["cfg3_be"], wl.CONFIGS["cfg3_ls"]
    ibe, ils = wl.make_inputs(cbe, weights=w), wl.make_inputs(cls_, weights=w)
    base, _ = check_layer(ibe, dev_w=dw)
    units = base.ctx.units()
    assert all(u[1] == 1 for u in units) and max(u[3] for u in units) == 256
    # BE in flight, one unit per call; after a third of the units the LS batch arrives, runs to
    # completion on its own context, then BE resumes from its cursor.
    be = GpuLayer(ibe, dw)
    cur = be.route_permute()
    stop = cur.n_units // 3
    for _ in range(stop):
        be.run(1)
    ls = GpuLayer(ils, dw).full()
    assert be.ctx.cursor.next_unit == stop
    while be.run(2) != q.MOE_DONE:
        pass
    be.combine()
    torch.cuda.synchronize()
    assert torch.equal(bits(be.y), bits(base.y))
    assert torch.equal(bits(be.ctx.get("expert_out")), bits(base.ctx.get("expert_out")))
    # the LS batch itself is right, every token of it
    lay = oracle.OracleLayer(ils.x, ils.w, ils.prio, ils.bias, cls_.k, cls_.chunk_rows)
    assert np.array_equal(lay.idx, to_host(ls.ctx.get("topk_idx")))
    assert np.array_equal(lay.perm, to_host(ls.ctx.get("perm")))
    say("  LS batch (cfg3_ls):")
    check_values(cls_, lay, ls, to_host(ls.y))


def test_cfg5_fine_grained_skewed_with_four_preemptions():
    cfg = wl.CONFIGS["cfg5"]
    inp = wl.make_inputs(cfg)
    g, r = check_layer(inp, dev_w=DevWeights(inp.w).packed())
    tot = r["counts"].sum(1)
    say(f"  rows per expert: max {tot.max()} min {tot.min()}; units {len(g.ctx.units())}")
    units = g.ctx.units()
    cuts = wl.cut_points(cfg.seed, expert_boundaries(units), 4)
    assert len(cuts) == 4
    assert_bit_identical(inp, cuts, base=g)


def test_cfg4_decode_with_4bit_weights_full_size():
    """The decode workload with 4-bit expert weights at the Mixtral shape, as bench.py --weights mxfp4
    times it: every token against the oracle's reading of the same codes, and one unit per call."""
    from gpu_util import DevWeightsMX
    cfg = wl.CONFIGS["cfg4"]
    w4 = wl.make_weights_mxfp4(cfg)
    inp = wl.make_inputs(cfg, weights=oracle.mxfp4_weights_as_bf16(w4))
    mx = DevWeightsMX(w4).packed()
    g = GpuLayer(inp, mx, down_ksplit=4).full()         # four K ranges, as the benchmark sets for this case
    r = g.fetch("logits", "topk_idx", "counts", "perm", "y")
    lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows, logits=r["logits"].astype(np.float64))
    assert np.array_equal(r["topk_idx"], lay.idx) and np.array_equal(r["counts"], lay.cnt) and np.array_equal(r["perm"], lay.perm)
    check_values(cfg, lay, g, r["y"], label="cfg4, 4-bit weights")
    nu = g.ctx.cursor.n_units
    h = GpuLayer(inp, mx, down_ksplit=4).full(tuple(range(1, nu)))
    assert torch.equal(bits(h.y), bits(g.y))


def test_activation_larger_than_4_gib():
    """Rows of the SwiGLU activation beyond the first 4 GiB: the down projection addresses its token
    rows with 32-bit offsets counted in 16-byte units, so the last experts' rows lie past what a
    32-bit byte offset reaches.  Every sampled token passes through all eight experts."""
    cfg = wl.scaled(wl.CONFIGS["cfg5"], name="act_5gib", N=80000, n_ls=10000, H=128, F=4096, E=8, k=8,
                    seed=7711, bias_kind="none", bias_arg=0.0)
    assert cfg.A * cfg.F * 2 > 1 << 32
    inp = wl.make_inputs(cfg)
    say("case", wl.describe(cfg))
    g = GpuLayer(inp, DevWeights(inp.w).packed()).full()
    r = g.fetch("logits", "topk_idx", "counts", "perm", "y")
    lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows, logits=r["logits"].astype(np.float64))
    assert np.array_equal(r["topk_idx"], lay.idx) and np.array_equal(r["counts"], lay.cnt) and np.array_equal(r["perm"], lay.perm)
    toks = sample(cfg, 24)
    e = rel_err(wl.as_f64(r["y"])[toks], lay.y_tokens_direct(toks))
    say(f"  y rel err on {len(toks)} tokens {e:.3e}")
    assert e <= 2e-2
    units = g.ctx.units()
    high = [i for i, u in enumerate(units) if u[2] * cfg.F * 2 >= 1 << 32]
    assert len(high) > 100
    assert_bit_identical(inp, (high[0], high[len(high) // 2]), base=g)
