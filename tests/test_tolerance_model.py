"""The bars the GPU tests hold a bf16 result to (tests/gpu_util.py) checked on the CPU: the closed-form
relative RMS of a bf16 rounding against a direct count, and the two roundings of the bf16 path (the
SwiGLU activation, then y) applied by hand to the oracle's fp64 intermediates must pass the bars,
land at the predicted RMS, and a planted systematic error of 2e-3 RMS must fail them."""
import numpy as np

import oracle
import workloads as wl
from gpu_util import (C_SIGMA, RHO, RMS_GATE_OUT, RMS_GATE_Y, check_bf16_expert_out, check_bf16_y, half_ulp_bf16,
                      sigma_out_exact, sigma_y)


def round_bf16(a: np.ndarray) -> np.ndarray:
    return wl.as_f64(wl.f32_to_bf16_bits(np.asarray(a, dtype=np.float32)))


def test_closed_form_of_the_bf16_rounding_rms():
    rng = np.random.default_rng(12)
    v = rng.standard_normal(2_000_000) * np.exp(rng.uniform(-6, 6, 2_000_000))     # spread over many binades
    rel = (round_bf16(v) - v.astype(np.float32).astype(np.float64)) / v
    got = float(np.sqrt(np.mean(rel * rel)))
    assert abs(got / RHO - 1.0) < 0.02, (got, RHO)
    assert np.all(np.abs(round_bf16(v) - v.astype(np.float32).astype(np.float64)) <= half_ulp_bf16(v) * (1 + 1e-12))


def test_half_ulp_values():
    np.testing.assert_array_equal(half_ulp_bf16(np.array([1.0, 1.99, 2.0, 0.75, 0.0, -3.0])),
                                  np.array([2.0 ** -8, 2.0 ** -8, 2.0 ** -7, 2.0 ** -9, 0.0, 2.0 ** -7]))


def modelled_layer(cfg):
    """The oracle's layer, and the same layer with the bf16 path's two roundings applied by hand."""
    inp = wl.make_inputs(cfg)
    lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows)
    lay.run()
    y_ref, comp = lay.y()
    assert comp.all()
    out_model = np.empty_like(lay.O)
    sigma = np.zeros_like(lay.O)
    for e in range(cfg.E):
        rows = np.arange(lay.off[2 * e], lay.off[2 * e + 2])
        if len(rows) == 0:
            continue
        toks = lay.perm[rows] // cfg.k
        o, act = oracle.expert_rows(inp.x, inp.w["W1"], inp.w["W3"], inp.w["W2"], e, toks, want_act=True)
        np.testing.assert_allclose(o, lay.O[rows], rtol=0, atol=0)
        out_model[rows] = round_bf16(act) @ wl.as_f64(inp.w["W2"][e]).T
        sigma[rows] = sigma_out_exact(act, wl.as_f64(inp.w["W2"][e]))
    y_pre = np.zeros_like(y_ref)
    for j in range(cfg.k):
        y_pre += lay.wt[:, j][:, None] * out_model[lay.inv.reshape(cfg.N, cfg.k)[:, j]]
    return lay, y_ref, out_model, round_bf16(y_pre), sigma


def test_the_two_roundings_pass_the_bars_and_land_on_the_predicted_rms():
    cfg = wl.LayerConfig("tolmodel", dtype="bf16", seed=8801, E=4, k=2, H=192, F=768, N=400, n_ls=90, chunk_rows=64)
    lay, y_ref, out_model, y_model, sigma = modelled_layer(cfg)
    # averaged over a row the exact sigma is RHO * RMS_h(out[r,:]); single elements spread around it
    row = RHO * np.sqrt(np.mean(lay.O ** 2, axis=1))
    ratio = sigma / row[:, None]
    assert 0.9 < float(np.sqrt(np.mean(ratio ** 2))) < 1.1 and float(ratio.max()) < 3.0, (ratio.mean(), ratio.max())
    ro = check_bf16_expert_out(out_model, lay.O, sigma)
    assert ro["ok"], ro
    assert 0.85 * RHO <= ro["rms_rel"] <= 1.15 * RHO, (ro, RHO)
    assert ro["worst_over_bar"] < 0.75                          # the largest error sits near 5 of the 8 sigmas
    ry = check_bf16_y(y_model, y_ref, sigma_y(lay.wt, lay.inv, sigma), need_global=False)
    assert ry["ok"], ry
    assert 0.85 * np.sqrt(2) * RHO <= ry["rms_rel"] <= 1.15 * np.sqrt(2) * RHO, ry
    assert RMS_GATE_OUT < 1.4 * RHO and RMS_GATE_Y < 1.4 * np.sqrt(2) * RHO and C_SIGMA == 8.0


def test_a_planted_systematic_error_fails_the_gates():
    cfg = wl.LayerConfig("tolplant", dtype="bf16", seed=8802, E=4, k=2, H=192, F=768, N=400, n_ls=90, chunk_rows=64)
    lay, y_ref, out_model, y_model, sigma = modelled_layer(cfg)
    rms_o = float(np.sqrt(np.mean(lay.O ** 2)))
    rng = np.random.default_rng(5)
    # (a) a smooth extra error of 2e-3 RMS on every element: far below 2e-2, caught by the RMS gate
    bad = out_model + 2e-3 * rms_o * rng.standard_normal(out_model.shape)
    r = check_bf16_expert_out(bad, lay.O, sigma)
    assert r["max_rel"] < 2e-2 and not r["ok"], r
    # (b) one element of a quiet row off by 1.5e-2 of the global RMS: under the global bar, over its own
    quiet = int(np.argmin(np.sqrt(np.mean(lay.O ** 2, axis=1))))
    bad = out_model.copy()
    bad[quiet, 7] += 1.5e-2 * rms_o
    r = check_bf16_expert_out(bad, lay.O, sigma)
    assert r["max_rel"] < 2e-2 and r["worst_over_bar"] > 1.0 and not r["ok"], r
    # (c) y scaled by 1 + 3e-3 (a wrong renormalisation, say): hidden by the output rounding at the
    # maximum, visible in the RMS
    sig = sigma_y(lay.wt, lay.inv, sigma)
    bad_y = round_bf16(y_model * (1 + 3e-3))
    r = check_bf16_y(bad_y, y_ref, sig, need_global=False)
    assert not r["ok"], r
