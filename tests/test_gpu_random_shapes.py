"""Seeded random layer shapes within the documented limits (expert counts 1..256, top-k 1..9, ragged
H/F/N, every chunk size class, all-LS / all-BE / mixed batches, skewed routers; weights fp32, bf16
row-major, bf16 packed or 4-bit; every down-projection K split): integer artefacts bit-exact against
the oracle, values element by element, and the same bits whether the expert work runs in one call,
with cursor cuts, or enqueued ahead with a stop landing somewhere.

The global 2e-2 bar is asserted with bf16 and fp32 weights and only reported with 4-bit weights: it
is stated for the named workloads, and with reductions as short as 64-192 and the heavy-tailed 4-bit
values a single output's own error bar can lie above 2e-2 of the tensor's RMS.  The per-element bars
and the RMS gates, which follow from the arithmetic at any shape, are asserted everywhere."""
import time

import numpy as np
import pytest
import torch

import oracle
import paper_2503_09304_amd as q
import workloads as wl
from gpu_util import DevWeights, DevWeightsMX, GpuLayer, rel_err
from test_gpu_parity import check_values

pytestmark = pytest.mark.gpu

N_CASES = 48


def random_case(i: int):
    rng = np.random.default_rng([950, i])
    dtype = "bf16" if rng.random() < 0.85 else "f32"
    E = int(rng.choice([1, 2, 3, 5, 8, 16, 17, 33, 64, 72, 130, 256]))
    k = int(rng.integers(1, min(E, 9) + 1))
    if dtype == "bf16":
        H = int(rng.choice([64, 128, 192, 320, 512]))
        F = int(rng.choice([64, 128, 192, 256, 448, 512, 1024]))
    else:
        H = int(rng.choice([7, 64, 100, 130]))
        F = int(rng.choice([5, 72, 128, 200]))
    N = int(rng.choice([1, 2, 15, 16, 17, 63, 100, 333, 700, 1500, 2600]))
    C = int(rng.choice([1, 16, 32, 64, 100, 256]))
    if N * k / C > 2500:
        C = 256
    n_ls = int(rng.choice([0, N, rng.integers(0, N + 1)]))
    ks = int(rng.choice([0, 1, 2, 4])) if dtype == "bf16" else 0
    if ks > 1 and F % (64 * ks):
        ks = 0
    wfmt = str(rng.choice(["rowmajor", "packed", "mxfp4"])) if dtype == "bf16" else "f32"
    cfg = wl.LayerConfig(f"rnd{i}", dtype=dtype, seed=9500000 + i, E=E, k=k, H=H, F=F, N=N, n_ls=n_ls, chunk_rows=C,
                         bias_kind=str(rng.choice(["none", "zipf", "expert0"])), bias_arg=1.0)
    return cfg, ks, wfmt, rng


def bits(t):
    return t.contiguous().view(torch.uint8)


@pytest.mark.parametrize("i", range(N_CASES))
def test_random_shape(i):
    cfg, ks, wfmt, rng = random_case(i)
    print("case", wl.describe(cfg), "down_ksplit", ks, "weights", wfmt, flush=True)
    if wfmt == "mxfp4":
        inp = wl.make_inputs(cfg, weights={})
        w4 = wl.make_weights_mxfp4(cfg)
        inp.w = oracle.mxfp4_weights_as_bf16(w4)          # the oracle's own reading of the codes
        dw = DevWeightsMX(w4).packed()
    else:
        inp = wl.make_inputs(cfg)
        dw = DevWeights(inp.w).packed() if wfmt == "packed" else DevWeights(inp.w)
    g = GpuLayer(inp, dw, down_ksplit=ks).full()
    r = g.fetch("logits", "topk_idx", "topk_w", "counts", "offsets", "perm", "inv", "units", "y")
    # integer artefacts: the oracle's selection replayed on the kernel's fp32 logits
    assert rel_err(r["logits"], oracle.gate_logits(inp.x, inp.w["Wg"], inp.bias)) <= 2e-5
    lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows, logits=r["logits"].astype(np.float64))
    assert np.array_equal(r["topk_idx"], lay.idx) and np.array_equal(r["counts"], lay.cnt)
    assert np.array_equal(r["offsets"], lay.off)
    assert np.array_equal(r["perm"], lay.perm) and np.array_equal(r["inv"], lay.inv)
    units = oracle.units(lay.cnt, cfg.chunk_rows)
    assert [tuple(int(v) for v in u) for u in units] == g.ctx.units()
    np.testing.assert_allclose(r["topk_w"], lay.wt, rtol=0, atol=2e-6)
    # values, every element
    check_values(cfg, lay, g, r["y"], need_global=wfmt != "mxfp4")
    # preempted == uninterrupted
    nu = g.ctx.cursor.n_units
    ref_out = g.ctx.get("expert_out").clone()
    if nu > 1:
        cuts = tuple(sorted(set(int(c) for c in rng.integers(1, nu, size=min(4, nu - 1)))))
        h = GpuLayer(inp, dw, down_ksplit=ks).full(cuts)
        assert torch.equal(bits(h.y), bits(g.y)), cuts
        assert torch.equal(bits(h.ctx.get("expert_out")), bits(ref_out)), cuts
    # enqueued ahead, stopped somewhere (or not at all), collected, carried on
    h = GpuLayer(inp, dw, down_ksplit=ks)
    h.route_permute()
    per = int(rng.choice([1, 2, 3, 7, q.UINT32_MAX]))
    stop_first = rng.random() < 0.7
    delay_s = float(rng.choice([0, 20, 100, 400])) * 1e-6
    rounds = 0
    while True:
        if h.ctx.expert_enqueue(h.x, h.dw.struct, per) == q.MOE_DONE:
            break
        if rounds == 0 and stop_first:
            t1 = time.perf_counter()
            while time.perf_counter() - t1 < delay_s:
                pass
            h.ctx.expert_stop()
        rc = h.ctx.expert_collect()
        rounds += 1
        if rc == q.MOE_DONE:
            break
        if rounds == 1 and rng.random() < 0.5:
            if h.run(1) == q.MOE_DONE:
                break
        assert rounds <= nu + 2, "every enqueue after the stopped one must finish at least one unit"
    assert h.ctx.cursor.next_unit == nu
    h.combine()
    torch.cuda.synchronize()
    assert torch.equal(bits(h.y), bits(g.y))
    assert torch.equal(bits(h.ctx.get("expert_out")), bits(ref_out))
