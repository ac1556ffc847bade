"""4-bit (microscaling FP4) expert weights on the GPU against the oracle, which reads the same codes
and scales with its own table and computes in fp64: routing artefacts bit-exact, outputs within the
bf16 tolerance, preempted == uninterrupted bit for bit, the packed block order equal to the formula
in the header, and bit-identical to the bf16 kernels run on the dequantised weights."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import paper_2503_09304_amd as q
import workloads as wl
from gpu_util import DevWeights, DevWeightsMX, GpuLayer, to_host
from test_gpu_parity import check_values

pytestmark = pytest.mark.gpu


def cases():
    base = dict(dtype="bf16", seed=940, E=8, k=2, H=256, F=512, N=300, n_ls=75, chunk_rows=64)
    yield "prefill_small", wl.LayerConfig("q1", **base)
    yield "decode_hot_expert", wl.LayerConfig("q2", **{**base, "N": 64, "n_ls": 16, "bias_kind": "expert0", "bias_arg": 1.5,
                                                       "seed": 941})
    yield "large_units", wl.LayerConfig("q3", **{**base, "N": 1300, "n_ls": 200, "chunk_rows": 256, "seed": 942})
    yield "skew_top8_no_ksplit", wl.LayerConfig("q4", dtype="bf16", seed=943, E=64, k=8, H=128, F=192, N=600, n_ls=100,
                                                chunk_rows=256, bias_kind="zipf", bias_arg=1.1)
    yield "one_token", wl.LayerConfig("q5", **{**base, "N": 1, "n_ls": 1, "seed": 944})


@pytest.mark.parametrize("name,cfg", list(cases()), ids=[n for n, _ in cases()])
def test_4bit_weights_match_oracle_and_survive_preemption(name, cfg):
    inp = wl.make_inputs(cfg, weights={})
    w4 = wl.make_weights_mxfp4(cfg)
    wb = oracle.mxfp4_weights_as_bf16(w4)                       # the oracle's own reading of the codes
    mx = DevWeightsMX(w4).packed()
    g = GpuLayer(inp, mx).full()
    r = g.fetch("logits", "topk_idx", "counts", "perm", "inv", "y")
    lay = oracle.OracleLayer(inp.x, wb, inp.prio, inp.bias, cfg.k, cfg.chunk_rows,
                             logits=r["logits"].astype(np.float64))
    assert np.array_equal(r["topk_idx"], lay.idx) and np.array_equal(r["counts"], lay.cnt)
    assert np.array_equal(r["perm"], lay.perm) and np.array_equal(r["inv"], lay.inv)
    # every element of the expert outputs and of y (bars: tests/gpu_util.py)
    print(f"  {name}:", flush=True)
    check_values(cfg, lay, g, r["y"])
    # the bf16 kernels on the dequantised weights compute the same bits: dequantisation is exact
    gb = GpuLayer(inp, DevWeights(wb).packed()).full()
    assert torch.equal(gb.y.view(torch.int16), g.y.view(torch.int16))
    assert torch.equal(gb.ctx.get("expert_out").view(torch.int32), g.ctx.get("expert_out").view(torch.int32))
    # preempted == uninterrupted
    nu = g.ctx.cursor.n_units
    if nu > 1:
        for cuts in (wl.cut_points(cfg.seed, range(1, nu), 4), tuple(range(1, nu))):
            h = GpuLayer(inp, mx).full(cuts)
            assert torch.equal(h.y.view(torch.int16), g.y.view(torch.int16))
            assert torch.equal(h.ctx.get("expert_out").view(torch.int32), g.ctx.get("expert_out").view(torch.int32))


def test_packed_4bit_layout_is_the_documented_one():
    cfg = wl.LayerConfig("q6", dtype="bf16", seed=945, E=3, k=2, H=128, F=192, N=4, n_ls=1, chunk_rows=4)
    w4 = wl.make_weights_mxfp4(cfg)
    pk = DevWeightsMX(w4).packed()
    for n, sn in (("W1", "S1"), ("W3", "S3"), ("W2", "S2")):
        codes, scales = w4[n + "q"], w4[n + "s"]
        E, R, K2 = codes.shape
        K = 2 * K2
        got_c = to_host(getattr(pk, n)).reshape(E, -1)
        got_s = to_host(getattr(pk, sn)).reshape(E, -1)
        want_c = np.empty_like(got_c)
        want_s = np.empty_like(got_s)
        for r in range(R):
            for k0 in range(0, K, 8):                     # 8 elements = 4 bytes = one word of one lane
                blk = (r // 32) * (K // 64) + k0 // 64
                lane = r % 32 + 32 * ((k0 % 16) // 8)
                word = (k0 % 64) // 16
                dst = blk * 1024 + lane * 16 + word * 4
                want_c[:, dst:dst + 4] = codes[:, r, k0 // 2:k0 // 2 + 4]
            for b in range(K // 32):
                blk = (r // 32) * (K // 64) + b // 2
                want_s[:, blk * 64 + (r % 32) * 2 + b % 2] = scales[:, r, b]
        assert np.array_equal(got_c, want_c), n
        assert np.array_equal(got_s, want_s), sn


def test_4bit_argument_checks():
    cfg = wl.LayerConfig("q7", dtype="bf16", seed=946, E=4, k=2, H=128, F=128, N=16, n_ls=4, chunk_rows=8)
    inp = wl.make_inputs(cfg, weights={})
    raw = DevWeightsMX(wl.make_weights_mxfp4(cfg))
    g = GpuLayer(inp, raw)
    with pytest.raises(q.MoeError) as e:
        g.route_permute()                                  # row-major 4-bit weights must be packed first
    assert e.value.code == q.MOE_E_ARG
    pk = raw.packed()
    bad = q.Context.weights(pk.Wg, pk.W1, pk.W3, pk.W2, q.MOE_W_MXFP4, None, pk.S3, pk.S2)
    with pytest.raises(q.MoeError) as e:
        g.ctx.route(g.x, bad, None, n_tokens=cfg.N)        # a scale pointer is missing
    assert e.value.code == q.MOE_E_ARG


def test_4bit_weights_with_narrow_gate_up_waves(monkeypatch):
    """The launch policy keeps 32-column waves for 4-bit weights, but the kernels take any width: a
    forced width of 20 gives the bits of the default."""
    cfg = wl.LayerConfig("q6", dtype="bf16", seed=947, E=6, k=2, H=192, F=448, N=333, n_ls=77, chunk_rows=64)
    inp = wl.make_inputs(cfg, weights={})
    mx = DevWeightsMX(wl.make_weights_mxfp4(cfg)).packed()
    ref = GpuLayer(inp, mx).full()
    monkeypatch.setenv("QMOE_GATE_UP_WAVE_COLUMNS", "20")
    g = GpuLayer(inp, mx)                          # the variable is read when the context is created
    monkeypatch.delenv("QMOE_GATE_UP_WAVE_COLUMNS")
    g.full((2, 5))
    assert torch.equal(g.ctx.get("act").view(torch.int16), ref.ctx.get("act").view(torch.int16))
    assert torch.equal(g.y.view(torch.int16), ref.y.view(torch.int16))
