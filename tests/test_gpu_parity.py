"""GPU path vs CPU oracle, element by element, through the C ABI.  Needs an MI355X (-m gpu).

Integer results (expert indices, counts, offsets, permutation, unit list) are compared
bit-exactly; floating point within max|err|/RMS(ref) <= 1e-4 (fp32 configs) / 2e-2 (bf16 configs).
The top-k decision is taken on fp32 logits by the kernel; the oracle's selection code is replayed
on those logits (must agree everywhere) and the pure-fp64 decision must agree for every token whose
logit gaps exceed TAU."""
import numpy as np
import pytest
import torch

import gpu_util
import oracle
import paper_2503_09304_amd as q
import workloads as wl
from gpu_util import (DevWeights, GpuLayer, check_bf16_expert_out, check_bf16_y, fmt, rel_err, sigma_out_layer,
                      sigma_y, to_host)

pytestmark = pytest.mark.gpu

TAU = 1e-4
TOL = {"f32": 1e-4, "bf16": 2e-2}


def say(*a):
    print(*a, flush=True)


def check_values(cfg, lay, g, y_bits, label=None, need_global=True):
    """Expert outputs and y of the device against the oracle layer `lay` (run here in full), every
    element.  fp32: max|err|/RMS <= 1e-4.  bf16 (bars: gpu_util): global 2e-2 (need_global), per-element
    bar and RMS gate on the expert outputs and on the unrounded fp32 y; the bf16 y must be exactly that
    fp32 y rounded to nearest-even, and is held to its per-element bar and RMS gate against the oracle."""
    lay.keep_act = cfg.dtype == "bf16"       # the activations give the per-element sigma of the bf16 bars
    lay.run()
    y_ref, comp = lay.y()
    assert comp.all()
    O = to_host(g.ctx.get("expert_out"))
    y_got = wl.as_f64(y_bits)
    assert np.isfinite(y_got).all() and np.isfinite(O).all()
    if cfg.dtype != "bf16":
        e_o, e_y = rel_err(O, lay.O), rel_err(y_got, y_ref)
        say(f"  rel err: expert_out {e_o:.2e}  y {e_y:.2e}  (tol {TOL[cfg.dtype]})")
        if cfg.name in wl.CONFIGS:
            gpu_util.REPORT.append(f"{cfg.name} (fp32) max|err|/RMS: expert_out {e_o:.2e}  y {e_y:.2e}")
        assert e_o <= TOL[cfg.dtype] and e_y <= TOL[cfg.dtype]
        return
    sigma = sigma_out_layer(lay, lambda e: wl.as_f64(lay.w["W2"][e]))
    sig_y = sigma_y(lay.wt, lay.inv, sigma)
    y32 = torch.empty((cfg.N, cfg.H), dtype=torch.float32, device=g.y.device)
    g.ctx.combine(y32, q.MOE_CLASS_ALL | q.MOE_Y_F32)
    torch.cuda.synchronize()
    y32 = y32.cpu().numpy()
    ro = check_bf16_expert_out(O, lay.O, sigma, need_global)
    r32 = check_bf16_expert_out(y32, y_ref, sig_y, need_global)
    ry = check_bf16_y(y_got, y_ref, sig_y)
    y_rounded = wl.as_f64(wl.f32_to_bf16_bits(np.asarray(y_ref, dtype=np.float32)))
    name = label or cfg.name
    lines = [f"{name} expert_out: {fmt(ro)}", f"{name} y (fp32):   {fmt(r32)}",
             f"{name} y (bf16):   {fmt(ry)}  [rounding the exact y to bf16 alone: {rel_err(y_rounded, y_ref):.2e}]"]
    for ln in lines:
        say("  " + ln)
    if cfg.name in wl.CONFIGS:
        gpu_util.REPORT.extend(lines)
    assert ro["ok"], ro
    assert r32["ok"], r32
    assert np.array_equal(wl.f32_to_bf16_bits(y32), np.asarray(y_bits)), "bf16 y is not the fp32 y rounded once"
    assert ry["ok"], ry


def check_layer(inp, cuts=(), sample_tokens=None, dev_w=None):
    """Full comparison of one layer-batch: integer artefacts bit-exact, values element by element
    (sample_tokens: y only, and only for these tokens, each computed on its own by the oracle)."""
    cfg = inp.cfg
    say("case", wl.describe(cfg), "cuts", list(cuts))
    g = GpuLayer(inp, dev_w).full(cuts)
    r = g.fetch("logits", "topk_idx", "topk_w", "counts", "offsets", "perm", "inv", "units", "y")
    # ---- oracle on the same bits
    L64 = oracle.gate_logits(inp.x, inp.w["Wg"], inp.bias)
    e_logit = rel_err(r["logits"], L64)
    assert e_logit <= 2e-5, e_logit
    # (i) replay: the oracle's selection applied to the kernel's fp32 logits
    idx_rep, wt_rep = oracle.topk(r["logits"].astype(np.float64), cfg.k)
    assert np.array_equal(idx_rep, r["topk_idx"])
    np.testing.assert_allclose(r["topk_w"], wt_rep, rtol=0, atol=2e-6)
    np.testing.assert_allclose(r["topk_w"].astype(np.float64).sum(1), 1.0, atol=1e-6)
    cnt, off, perm, inv = oracle.queues(r["topk_idx"], inp.prio, cfg.E)
    assert np.array_equal(cnt, r["counts"]) and np.array_equal(off, r["offsets"])
    assert np.array_equal(perm, r["perm"]) and np.array_equal(inv, r["inv"])
    units = oracle.units(cnt, cfg.chunk_rows)
    assert [tuple(int(v) for v in u) for u in units] == g.ctx.units()
    assert np.array_equal(units.reshape(-1, 4), r["units"].reshape(-1, 4))
    assert cnt.sum() == cfg.A
    # (ii) direct: pure fp64 decision, wherever it is not within TAU of a tie
    idx64, wt64 = oracle.topk(L64, cfg.k)
    margin = oracle.topk_margin(L64, cfg.k)
    clear = margin >= TAU
    mism = np.any(idx64 != r["topk_idx"], axis=1)
    say(f"  tokens within {TAU} of a tie: {int((~clear).sum())}; index mismatches vs fp64: {int(mism.sum())}")
    assert not np.any(mism & clear)
    assert not mism.any(), "seed chosen so that the fp64 decision matches everywhere"
    np.testing.assert_allclose(r["topk_w"], wt64, rtol=0, atol=1e-5)
    # ---- values
    lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows)
    if sample_tokens is None:
        say(f"  rel err: logits {e_logit:.2e}")
        check_values(cfg, lay, g, r["y"])
    else:
        toks = np.asarray(sample_tokens)
        y_ref = lay.y_tokens_direct(toks)
        y_got = wl.as_f64(r["y"])[toks]
        e_y = rel_err(y_got, y_ref)
        say(f"  rel err: logits {e_logit:.2e}  y on {len(toks)} sampled tokens {e_y:.2e}  (tol {TOL[cfg.dtype]})")
        assert np.isfinite(y_got).all()
        assert e_y <= TOL[cfg.dtype]
    return g, r


def bits(t: torch.Tensor) -> torch.Tensor:
    return t.contiguous().view(torch.uint8)


def assert_bit_identical(inp, cuts, dev_w=None, base=None):
    a = base if base is not None else GpuLayer(inp, dev_w).full(())
    b = GpuLayer(inp, dev_w or a.dw).full(cuts)
    assert torch.equal(bits(a.y), bits(b.y)), f"y differs after cuts {cuts}"
    assert torch.equal(bits(a.ctx.get("expert_out")), bits(b.ctx.get("expert_out"))), f"expert_out differs {cuts}"
    assert torch.equal(bits(a.ctx.get("act")), bits(b.ctx.get("act")))
    return a


# ------------------------------------------------------------------------------------------------
def test_cfg1_tiny_fp32_with_preemption_after_expert_1():
    cfg = wl.CONFIGS["cfg1"]
    inp = wl.make_inputs(cfg)
    g, r = check_layer(inp)
    units = g.ctx.units()
    # preempt after the last LS-phase unit of expert 1, and (second variant) after its last BE unit
    for cls in (0, 1):
        last = max(i for i, u in enumerate(units) if u[0] == 1 and u[1] == cls)
        assert_bit_identical(inp, (last + 1,), base=g)
    # every possible single cut, and one multi-cut
    for c in range(0, len(units) + 1):
        assert_bit_identical(inp, (c,), base=g)
    assert_bit_identical(inp, wl.cut_points(11, range(1, len(units)), 4), base=g)


def small_cases():
    base = dict(dtype="bf16", seed=910, E=8, k=2, H=256, F=512, N=300, n_ls=75, chunk_rows=64)
    yield "bf16_small_units", wl.LayerConfig("s1", **base)
    yield "bf16_large_units", wl.LayerConfig("s2", **{**base, "N": 1300, "n_ls": 200, "chunk_rows": 256, "seed": 911})
    yield "bf16_chunk_100", wl.LayerConfig("s3", **{**base, "N": 777, "n_ls": 333, "chunk_rows": 100, "seed": 912})
    yield "bf16_skew_no_ksplit", wl.LayerConfig("s4", dtype="bf16", seed=913, E=64, k=8, H=128, F=192, N=600,
                                                n_ls=100, chunk_rows=256, bias_kind="zipf", bias_arg=1.1)
    yield "bf16_hot_expert0", wl.LayerConfig("s5", **{**base, "N": 64, "n_ls": 16, "bias_kind": "expert0",
                                                      "bias_arg": 1.5, "seed": 914})
    yield "f32_ragged", wl.LayerConfig("s6", dtype="f32", seed=915, E=5, k=3, H=100, F=72, N=150, n_ls=40,
                                       chunk_rows=37)
    yield "bf16_k1", wl.LayerConfig("s7", **{**base, "k": 1, "seed": 916})
    yield "bf16_k_equals_E", wl.LayerConfig("s8", **{**base, "E": 4, "k": 4, "N": 90, "n_ls": 30, "seed": 917})
    yield "bf16_all_ls", wl.LayerConfig("s9", **{**base, "n_ls": 300, "seed": 918})
    yield "bf16_all_be", wl.LayerConfig("s10", **{**base, "n_ls": 0, "seed": 919})
    yield "bf16_one_token", wl.LayerConfig("s11", **{**base, "N": 1, "n_ls": 1, "seed": 920})
    yield "bf16_many_experts", wl.LayerConfig("s12", dtype="bf16", seed=921, E=256, k=6, H=128, F=128, N=257,
                                              n_ls=64, chunk_rows=32)
    # the limits of the configuration: top-32 routing, one row per unit, the smallest bf16 dimensions
    yield "bf16_top32", wl.LayerConfig("s15", dtype="bf16", seed=924, E=64, k=32, H=128, F=128, N=40, n_ls=10,
                                       chunk_rows=64)
    yield "bf16_one_row_units", wl.LayerConfig("s16", dtype="bf16", seed=925, E=4, k=2, H=128, F=128, N=20, n_ls=5,
                                               chunk_rows=1)
    yield "bf16_min_dims", wl.LayerConfig("s17", dtype="bf16", seed=926, E=3, k=2, H=64, F=64, N=70, n_ls=20,
                                          chunk_rows=16)
    # more row segments than fit the kernel arguments: the launch reads the device unit list instead
    yield "bf16_many_segments", wl.LayerConfig("s13", dtype="bf16", seed=922, E=64, k=8, H=128, F=128, N=16384,
                                               n_ls=4000, chunk_rows=256)


@pytest.mark.parametrize("name,cfg", list(small_cases()), ids=[n for n, _ in small_cases()])
def test_reduced_size_cases_match_oracle_and_survive_preemption(name, cfg):
    inp = wl.make_inputs(cfg)
    g, r = check_layer(inp)
    nu = len(g.ctx.units())
    if nu > 1:
        assert_bit_identical(inp, wl.cut_points(cfg.seed, range(1, nu), 4), base=g)
        assert_bit_identical(inp, tuple(range(1, nu)), base=g)          # one unit per call
    if cfg.dtype == "bf16":
        # the packed weight layout computes the same bits, preempted or not
        pk = g.dw.packed()
        assert pk.struct.layout == q.MOE_W_PACKED
        gp, _ = check_layer(inp, dev_w=pk)
        assert torch.equal(bits(gp.y), bits(g.y))
        assert torch.equal(bits(gp.ctx.get("expert_out")), bits(g.ctx.get("expert_out")))
        assert torch.equal(bits(gp.ctx.get("logits")), bits(g.ctx.get("logits")))
        if nu > 1:
            assert_bit_identical(inp, wl.cut_points(cfg.seed + 1, range(1, nu), 3), dev_w=pk, base=gp)


@pytest.mark.parametrize("ks", [1, 2, 4])
def test_down_projection_k_split_is_a_configuration_choice(ks):
    """Every setting matches the oracle and is bit-stable under preemption; auto picks per config."""
    cfg = wl.LayerConfig("ks", dtype="bf16", seed=930 + ks, E=8, k=2, H=256, F=512, N=700, n_ls=150, chunk_rows=128)
    inp = wl.make_inputs(cfg)
    lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows)
    base = GpuLayer(inp, down_ksplit=ks).full()
    assert np.array_equal(lay.idx, to_host(base.ctx.get("topk_idx")))
    check_values(cfg, lay, base, to_host(base.y))
    nu = len(base.ctx.units())
    for cuts in (wl.cut_points(ks, range(1, nu), 5), tuple(range(1, nu))):
        other = GpuLayer(inp, base.dw, down_ksplit=ks).full(cuts)
        assert torch.equal(bits(base.y), bits(other.y))
        assert torch.equal(bits(base.ctx.get("expert_out")), bits(other.ctx.get("expert_out")))
    with pytest.raises(q.MoeError):
        q.moe_workspace_bytes(q.MoeConfig(8, 2, 256, 512, q.MOE_BF16, 64, 16, 3))
    with pytest.raises(q.MoeError):
        q.moe_workspace_bytes(q.MoeConfig(8, 2, 256, 192, q.MOE_BF16, 64, 16, 4))     # F not a multiple of 256
    with pytest.raises(q.MoeError):
        q.moe_workspace_bytes(q.MoeConfig(8, 2, 256, 192, q.MOE_BF16, 64, 16, 2))     # nor of 128
    q.moe_workspace_bytes(q.MoeConfig(8, 2, 256, 384, q.MOE_BF16, 64, 16, 2))
    with pytest.raises(q.MoeError):
        q.moe_workspace_bytes(q.MoeConfig(8, 2, 256, 512, q.MOE_F32, 64, 16, 4))


def test_packed_layout_is_the_documented_permutation():
    """moe_pack_weights against the index formula of qmoe.h, written out in numpy: byte-exact."""
    E, F, H = 3, 128, 192
    rng = np.random.default_rng(5)
    w = {"Wg": rng.integers(0, 65536, size=(H, E), dtype=np.uint16),
         "W1": rng.integers(0, 65536, size=(E, F, H), dtype=np.uint16),
         "W3": rng.integers(0, 65536, size=(E, F, H), dtype=np.uint16),
         "W2": rng.integers(0, 65536, size=(E, H, F), dtype=np.uint16)}
    pk = DevWeights(w).packed()

    def ref(m):                                   # m [E,R,K] -> packed order
        e_, R, K = m.shape
        out = np.empty(e_ * R * K, dtype=np.uint16)
        r, k = np.meshgrid(np.arange(R), np.arange(K), indexing="ij")
        dst = (((r // 32) * (K // 16) + k // 16) * 64 + (r % 32) + 32 * ((k % 16) // 8)) * 8 + k % 8
        for e in range(e_):
            out[e * R * K + dst.reshape(-1)] = m[e].reshape(-1)
        return out

    for name in ("W1", "W3", "W2"):
        got = to_host(getattr(pk, name)).reshape(-1)
        assert np.array_equal(got, ref(w[name])), name
    wgt = to_host(pk.Wg)
    assert wgt.shape == (16, H)
    assert np.array_equal(wgt[:E], w["Wg"].T) and not wgt[E:].any()


def test_pack_weights_argument_checks():
    cfg = q.MoeConfig(4, 2, 64, 64, q.MOE_F32, 16, 8)
    w = q.MoeWeights(256, 512, 768, 1024, 0)
    d = q.MoeWeights(2560, 5120, 7680, 10240, 0)
    with pytest.raises(q.MoeError):
        q.moe_pack_weights(cfg, w, d)                       # fp32 is not packable
    cfg = q.MoeConfig(4, 2, 64, 64, q.MOE_BF16, 16, 8)
    with pytest.raises(q.MoeError):
        q.moe_pack_weights(cfg, w, q.MoeWeights(256, 5120, 7680, 10240, 0))   # in place
    with pytest.raises(q.MoeError):
        q.moe_pack_weights(cfg, q.MoeWeights(256, 512, 768, 1024, 1), d)      # source already packed


def test_empty_batch_and_k1_weights():
    cfg = wl.LayerConfig("empty", dtype="bf16", seed=1, E=8, k=2, H=128, F=128, N=0, n_ls=0, chunk_rows=64)
    inp = wl.make_inputs(cfg)
    g = GpuLayer(inp, max_tokens=16)
    cur = g.route_permute()
    assert cur.n_units == 0
    assert g.run() == q.MOE_DONE
    assert g.combine() == q.MOE_OK
    assert int(g.ctx.get("counts").sum().item()) == 0
    cfg = wl.LayerConfig("k1", dtype="f32", seed=2, E=6, k=1, H=64, F=64, N=40, n_ls=10, chunk_rows=8)
    g = GpuLayer(wl.make_inputs(cfg)).full()
    assert bool((g.ctx.get("topk_w") == 1.0).all())


def test_exact_logit_ties_take_the_lowest_expert_index():
    cfg = wl.LayerConfig("ties", dtype="bf16", seed=3, E=8, k=2, H=128, F=128, N=96, n_ls=24, chunk_rows=32)
    inp = wl.make_inputs(cfg)
    wg = inp.w["Wg"]
    wg[:, 5] = wg[:, 2]          # duplicate columns: bitwise-equal logits for experts 2 and 5
    wg[:, 7] = wg[:, 2]
    g = GpuLayer(inp).full()
    r = g.fetch("logits", "topk_idx", "topk_w")
    assert np.array_equal(r["logits"][:, 2], r["logits"][:, 5])
    idx_rep, _ = oracle.topk(r["logits"].astype(np.float64), cfg.k)
    assert np.array_equal(idx_rep, r["topk_idx"])
    both = np.isin(r["topk_idx"], [2, 5, 7]).sum(1)
    assert (both == 2).any()
    for row in r["topk_idx"][both == 2]:
        assert list(row) == [2, 5]
    for row in r["topk_idx"][both == 1]:
        assert 2 in row and 5 not in row and 7 not in row


def test_only_complete_tokens_are_combined_and_call_order_is_enforced():
    cfg = wl.CONFIGS["cfg1"]
    inp = wl.make_inputs(cfg)
    ref = GpuLayer(inp).full()
    g = GpuLayer(inp)
    cur = g.route_permute()
    units = g.ctx.units()
    n_ls = sum(1 for u in units if u[1] == 0)
    assert all(u[1] == 0 for u in units[:n_ls]) and all(u[1] == 1 for u in units[n_ls:])
    g.run(n_ls - 1)
    with pytest.raises(q.MoeError) as ei:
        g.combine(q.MOE_CLASS_LS)
    assert ei.value.code == q.MOE_E_INCOMPLETE
    g.run(1)
    assert g.combine(q.MOE_CLASS_LS) == q.MOE_OK
    with pytest.raises(q.MoeError) as ei:
        g.combine(q.MOE_CLASS_BE)
    assert ei.value.code == q.MOE_E_INCOMPLETE
    torch.cuda.synchronize()
    ls = torch.from_numpy(inp.prio != 0).to(g.y.device)
    assert torch.equal(bits(g.y[ls]), bits(ref.y[ls]))          # LS rows final before any BE work ran
    assert bool(torch.isnan(g.y[~ls]).all())                      # BE rows untouched
    # a stale cursor is refused: no unit runs twice
    stale = q.MoeCursor(0, cur.n_units)
    with pytest.raises(q.MoeError) as ei:
        g.ctx.expert_run(g.x, g.dw.struct, 1, cursor=stale)
    assert ei.value.code == q.MOE_E_ARG
    assert g.run() == q.MOE_DONE
    g.combine(q.MOE_CLASS_BE)
    torch.cuda.synchronize()
    assert torch.equal(bits(g.y), bits(ref.y))
    with pytest.raises(q.MoeError) as ei:
        g.ctx.permute(g.prio)
    assert ei.value.code == q.MOE_E_STATE


def test_context_reuse_with_a_smaller_batch_and_run_to_run_identity():
    big = wl.LayerConfig("r1", dtype="bf16", seed=31, E=8, k=2, H=256, F=512, N=400, n_ls=100, chunk_rows=64)
    small = wl.scaled(big, N=130, n_ls=30, seed=32)
    ib, isml = wl.make_inputs(big), wl.make_inputs(small, weights=None)
    g = GpuLayer(ib).full()
    y1 = g.y.clone()
    g.full()
    assert torch.equal(bits(y1), bits(g.y))
    # same context, smaller batch
    g2 = GpuLayer(isml)
    g2.ctx.close()
    g2.ctx = g.ctx
    g2.dw = DevWeights(isml.w)
    g2.full()
    ref = GpuLayer(isml).full()
    assert torch.equal(bits(g2.y), bits(ref.y))


def test_permute_falls_back_to_a_stream_wait_when_it_may_not_poll(monkeypatch):
    """QMOE_REPORT_SPIN_MS=0 makes moe_permute skip the poll of the kernel's report and wait for the
    stream: same cursor, same bits."""
    cfg = wl.LayerConfig("s14", dtype="bf16", seed=923, E=8, k=2, H=128, F=256, N=500, n_ls=100, chunk_rows=64)
    inp = wl.make_inputs(cfg)
    ref = GpuLayer(inp).full()
    monkeypatch.setenv("QMOE_REPORT_SPIN_MS", "0")
    g = GpuLayer(inp, ref.dw)                      # the variable is read when the context is created
    monkeypatch.delenv("QMOE_REPORT_SPIN_MS")
    for _ in range(3):
        g.full()
        assert g.ctx.cursor.n_units == ref.ctx.cursor.n_units
        assert torch.equal(bits(g.y), bits(ref.y))


@pytest.mark.parametrize("cw", [28, 20, 16])
def test_narrow_gate_up_waves_give_the_same_bits(monkeypatch, cw):
    """A gate-up launch may give each wave fewer than 32 columns (chosen per launch from the number of
    workgroups; QMOE_GATE_UP_WAVE_COLUMNS forces a width for every launch of a context).  Which wave
    computes a column never changes its arithmetic: same bits as with 32, row-major and packed, with F
    not a multiple of the narrower workgroup width, and against the oracle."""
    cfg = wl.LayerConfig(f"cw{cw}", dtype="bf16", seed=3100 + cw, E=6, k=2, H=192, F=448, N=333, n_ls=77, chunk_rows=64)
    inp = wl.make_inputs(cfg)
    ref, _ = check_layer(inp)
    for dw in (ref.dw, DevWeights(inp.w).packed()):
        monkeypatch.setenv("QMOE_GATE_UP_WAVE_COLUMNS", str(cw))
        g = GpuLayer(inp, dw)                      # the variable is read when the context is created
        monkeypatch.delenv("QMOE_GATE_UP_WAVE_COLUMNS")
        g.full((3, 7))
        assert torch.equal(bits(g.ctx.get("act")), bits(ref.ctx.get("act")))
        assert torch.equal(bits(g.y), bits(ref.y))
