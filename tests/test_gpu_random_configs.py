"""Seeded sweep over small valid configurations (expert counts around the 16- and 64-boundaries,
top-k up to 9, ragged token counts, every chunk size class, both dtypes, both weight layouts, every
K-split): integer artefacts bit-exact against the oracle, values within the configuration's bar, a
run cut at seeded cursor positions bit-identical to the uninterrupted one.  Needs an MI355X (-m gpu)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_09304_amd as q
import workloads as wl
from gpu_util import DevWeights, GpuLayer, rel_err
from test_gpu_parity import check_values

pytestmark = pytest.mark.gpu


def draw(case):
    rng = np.random.default_rng([4242, case])
    dtype = "bf16" if rng.random() < 0.8 else "f32"
    E = int(rng.choice([1, 2, 3, 5, 8, 16, 17, 33, 64, 72, 130]))
    k = int(rng.integers(1, min(E, 9) + 1))
    H = int(rng.choice([64, 128, 192, 320]))
    F = int(rng.choice([64, 128, 192, 256, 448, 512]))
    N = int(rng.choice([1, 2, 15, 16, 17, 63, 100, 333, 700, 1500]))
    C = int(rng.choice([1, 16, 64, 256]))
    if N * k / C > 3000:
        C = 256
    ks = int(rng.choice([0, 1, 2, 4])) if dtype == "bf16" else 0
    if ks > 1 and F % (64 * ks):
        ks = 0
    cfg = wl.LayerConfig(f"rc{case}", dtype=dtype, seed=71000 + case, E=E, k=k, H=H, F=F, N=N,
                         n_ls=int(rng.integers(0, N + 1)), chunk_rows=C,
                         bias_kind=str(rng.choice(["none", "zipf"])), bias_arg=1.0)
    return cfg, ks, bool(dtype == "bf16" and rng.random() < 0.5), rng


@pytest.mark.parametrize("case", range(24))
def test_random_configuration(case):
    cfg, ks, packed, rng = draw(case)
    print(f"  {wl.describe(cfg)} down_ksplit {ks} packed {packed}", flush=True)
    inp = wl.make_inputs(cfg)
    dw = DevWeights(inp.w).packed() if packed else DevWeights(inp.w)
    g = GpuLayer(inp, dw, down_ksplit=ks).full()
    r = g.fetch("logits", "topk_idx", "counts", "perm", "inv", "y")
    assert rel_err(r["logits"], oracle.gate_logits(inp.x, inp.w["Wg"], inp.bias)) <= 2e-5
    # the oracle's selection replayed on the kernel's fp32 logits, and everything downstream of it
    lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows, logits=r["logits"].astype(np.float64))
    assert np.array_equal(r["topk_idx"], lay.idx) and np.array_equal(r["counts"], lay.cnt)
    assert np.array_equal(r["perm"], lay.perm) and np.array_equal(r["inv"], lay.inv)
    assert [tuple(int(v) for v in u) for u in oracle.units(lay.cnt, cfg.chunk_rows)] == g.ctx.units()
    check_values(cfg, lay, g, r["y"])
    bf = cfg.dtype == "bf16"
    nu = g.ctx.cursor.n_units
    if nu > 1:
        cuts = tuple(sorted(set(int(c) for c in rng.integers(1, nu, size=min(4, nu - 1)))))
        h = GpuLayer(inp, dw, down_ksplit=ks).full(cuts)
        view = torch.int16 if bf else torch.int32
        assert torch.equal(h.y.view(view), g.y.view(view)), cuts
        assert torch.equal(h.ctx.get("expert_out").view(torch.int32), g.ctx.get("expert_out").view(torch.int32)), cuts
