"""Pins of the CPU oracle against things other than itself: numpy library routines, closed
forms, invariants and brute force.  The paper prints no value for this path, so none is cited.
CPU only."""
import itertools
import math

import numpy as np
import pytest

import oracle
import workloads as wl


def np_silu(z):
    return z / (1.0 + np.exp(-z))


def small_cfg(**kw):
    base = dict(N=24, n_ls=7, H=20, F=28, E=5, k=2, dtype="f32", seed=77, chunk_rows=4)
    base.update(kw)
    return wl.LayerConfig("small", **base)


def dense_then_mask(inp, idx, wt):
    """Every expert on every token with numpy.matmul, then keep the routed ones."""
    cfg = inp.cfg
    x = wl.as_f64(inp.x)
    y = np.zeros((cfg.N, cfg.H))
    for e in range(cfg.E):
        w1, w3, w2 = (wl.as_f64(inp.w[n][e]) for n in ("W1", "W3", "W2"))
        full = (np_silu(x @ w1.T) * (x @ w3.T)) @ w2.T           # [N,H]
        gate = np.zeros(cfg.N)
        for j in range(cfg.k):
            gate += np.where(idx[:, j] == e, wt[:, j], 0.0)
        y += gate[:, None] * full
    return y


# ------------------------------------------------------------------ step 1: logits
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_logits_equal_numpy_matmul(dtype):
    cfg = wl.scaled(wl.CONFIGS["cfg1"], dtype=dtype)
    inp = wl.make_inputs(cfg)
    bias = np.linspace(-0.3, 0.4, cfg.E).astype(np.float32)
    L = oracle.gate_logits(inp.x, inp.w["Wg"], bias)
    ref = wl.as_f64(inp.x) @ wl.as_f64(inp.w["Wg"]) + bias.astype(np.float64)
    assert L.shape == (cfg.N, cfg.E)
    np.testing.assert_allclose(L, ref, rtol=1e-12, atol=1e-14)
    L0 = oracle.gate_logits(inp.x, inp.w["Wg"], None)
    np.testing.assert_allclose(L0, ref - bias.astype(np.float64), rtol=1e-12, atol=1e-14)


def test_logits_one_hot_rows_pick_rows_of_wg():
    H, E = 6, 3
    wg = np.arange(H * E, dtype=np.float32).reshape(H, E) - 4.0
    x = np.eye(H, dtype=np.float32)[[4, 0, 5]]
    L = oracle.gate_logits(x, wg, None)
    np.testing.assert_array_equal(L, wg[[4, 0, 5]].astype(np.float64))


def test_bf16_inputs_are_widened_exactly():
    rng = np.random.default_rng(5)
    v = rng.standard_normal((7, 16)).astype(np.float32)
    bits = wl.f32_to_bf16_bits(v)
    wide = wl.bf16_bits_to_f32(bits)
    wg32 = rng.standard_normal((16, 3)).astype(np.float32)
    wgb = wl.f32_to_bf16_bits(wg32)
    a = oracle.gate_logits(bits, wgb, None)
    b = oracle.gate_logits(wide, wl.bf16_bits_to_f32(wgb), None)
    np.testing.assert_array_equal(a, b)
    # rounding is to nearest: error at most half a bf16 ulp (2^-9 relative)
    assert np.all(np.abs(wide - v) <= np.abs(v) * 2.0 ** -8)
    # ties-to-even on a hand-made pattern: 1 + 2^-8 is exactly between two bf16 values
    assert wl.f32_to_bf16_bits(np.array([1.0 + 2.0 ** -8], np.float32))[0] == 0x3F80
    assert wl.f32_to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8], np.float32))[0] == 0x3F82


# ------------------------------------------------------------------ step 2: softmax
def test_softmax_sums_to_one_shift_invariant_and_two_way_closed_form():
    rng = np.random.default_rng(1)
    L = rng.standard_normal((50, 9)) * 3
    P = oracle.softmax(L)
    np.testing.assert_allclose(P.sum(1), 1.0, atol=1e-15)
    np.testing.assert_allclose(oracle.softmax(L + 123.25), P, rtol=1e-12)
    assert np.all(P > 0)
    # order preserved
    assert np.array_equal(np.argsort(-L, axis=1, kind="stable"), np.argsort(-P, axis=1, kind="stable"))
    # E = 2: softmax is the logistic function of the difference
    L2 = rng.standard_normal((30, 2))
    P2 = oracle.softmax(L2)
    np.testing.assert_allclose(P2[:, 0], 1.0 / (1.0 + np.exp(L2[:, 1] - L2[:, 0])), rtol=1e-13)


# ------------------------------------------------------------------ step 3: top-k
def brute_topk(l, k):
    """Best k-subset by exhaustive search: maximal logit sum, exact ties -> lexicographically
    smallest index tuple; slots ordered by (logit descending, index ascending)."""
    E = len(l)
    best = None
    for sub in itertools.combinations(range(E), k):
        key = (-sum(sorted((l[e] for e in sub), reverse=True)), sub)
        if best is None or key < best[0]:
            best = (key, sub)
    return sorted(best[1], key=lambda e: (-l[e], e))


@pytest.mark.parametrize("E,k", [(4, 2), (6, 3), (5, 1), (5, 5), (8, 2)])
def test_topk_matches_exhaustive_search_with_ties(E, k):
    rng = np.random.default_rng(100 + E * 10 + k)
    # few distinct, exactly representable values => many exact ties
    L = rng.integers(-2, 3, size=(200, E)).astype(np.float64) * 0.5
    idx, wt = oracle.topk(L, k)
    for n in range(L.shape[0]):
        assert list(idx[n]) == brute_topk(list(L[n]), k), (n, L[n], idx[n])
        assert len(set(idx[n])) == k
    np.testing.assert_allclose(wt.sum(1), 1.0, atol=1e-15)


def test_topk_tie_goes_to_lowest_index():
    L = np.array([[0.5, 0.5, 0.5, 0.5], [0.1, 0.7, 0.7, 0.2], [1.0, -1.0, 1.0, 1.0]])
    idx, wt = oracle.topk(L, 2)
    assert idx.tolist() == [[0, 1], [1, 2], [0, 2]]
    np.testing.assert_allclose(wt, 0.5, atol=1e-16)


def test_topk_weights_closed_forms():
    rng = np.random.default_rng(3)
    L = rng.standard_normal((64, 7)) * 2
    for k in (1, 2, 3, 7):
        idx, wt = oracle.topk(L, k)
        sel = np.take_along_axis(L, idx.astype(np.int64), axis=1)
        # slots are in descending logit order
        assert np.all(np.diff(sel, axis=1) <= 0)
        # renormalised full softmax == softmax over the k selected logits alone
        short = np.exp(sel - sel[:, :1])
        short /= short.sum(1, keepdims=True)
        np.testing.assert_allclose(wt, short, rtol=1e-13, atol=1e-15)
        if k == 1:
            assert np.all(wt == 1.0)
        if k == 7:
            P = oracle.softmax(L)
            np.testing.assert_allclose(wt, np.take_along_axis(P, idx.astype(np.int64), axis=1), rtol=1e-13)
    # the selected set is the k largest (no ties in this draw)
    idx, _ = oracle.topk(L, 3)
    ref = np.argsort(-L, axis=1, kind="stable")[:, :3]
    assert np.array_equal(idx, ref)


def test_topk_margin_against_numpy_sort():
    rng = np.random.default_rng(4)
    L = rng.standard_normal((40, 8))
    for k in (1, 2, 7, 8):
        m = oracle.topk_margin(L, k)
        s = -np.sort(-L, axis=1)[:, : min(k + 1, 8)]
        np.testing.assert_allclose(m, np.min(s[:, :-1] - s[:, 1:], axis=1), rtol=0, atol=0)


# ------------------------------------------------------------------ step 4: queues
@pytest.mark.parametrize("N,E,k,frac", [(64, 4, 2, 0.25), (200, 16, 4, 0.5), (33, 3, 3, 0.0), (33, 3, 1, 1.0),
                                        (0, 4, 2, 0.0)])
def test_queues_equal_lexsort_and_bincount(N, E, k, frac):
    rng = np.random.default_rng(N + E + k)
    idx = np.stack([rng.permutation(E)[:k] for _ in range(N)]).astype(np.int32) if N else np.zeros((0, k), np.int32)
    prio = (rng.random(N) < frac).astype(np.uint8) * 3      # any non-zero flag means LS
    cnt, off, perm, inv = oracle.queues(idx, prio, E)
    A = N * k
    a = np.arange(A)
    tok, exp = a // k, idx.reshape(-1)
    cls = np.where(prio[tok] != 0, 0, 1) if N else np.zeros(0, np.int64)
    ref_perm = np.lexsort((tok, cls, exp))                   # independent library routine
    assert np.array_equal(perm, ref_perm.astype(np.int32))
    assert np.array_equal(np.sort(perm), a)                  # bijection
    assert np.array_equal(inv[perm], a) and np.array_equal(perm[inv], a)
    ref_cnt = np.bincount(exp * 2 + cls, minlength=2 * E).reshape(E, 2)
    assert np.array_equal(cnt, ref_cnt)
    assert cnt.sum() == A and cnt[:, 0].sum() == k * int((prio != 0).sum())
    assert off[0] == 0 and off[-1] == A and np.array_equal(np.diff(off), cnt.reshape(-1))
    # FIFO inside a bucket: token index strictly ascending
    for b in range(2 * E):
        seg = perm[off[b]:off[b + 1]] // k
        assert np.all(np.diff(seg) > 0)
        assert np.all(exp[perm[off[b]:off[b + 1]]] == b // 2)
        assert np.all(cls[perm[off[b]:off[b + 1]]] == b % 2)


# ------------------------------------------------------------------ step 7: work units
def test_units_hand_example():
    cnt = np.array([[3, 5], [0, 2], [4, 0]], dtype=np.int32)
    # sorted rows: e0-LS 0..2, e0-BE 3..7, e1-BE 8..9, e2-LS 10..13
    u = oracle.units(cnt, 2)
    assert u.tolist() == [
        [0, 0, 0, 2], [0, 0, 2, 1], [2, 0, 10, 2], [2, 0, 12, 2],       # LS phase
        [0, 1, 3, 2], [0, 1, 5, 2], [0, 1, 7, 1], [1, 1, 8, 2],         # BE phase
    ]


@pytest.mark.parametrize("C", [1, 3, 16, 1000])
def test_units_tile_every_subqueue_once_ls_first(C):
    rng = np.random.default_rng(C)
    cnt = rng.integers(0, 40, size=(9, 2)).astype(np.int32)
    cnt[2] = 0
    cnt[5, 0] = 0
    u = oracle.units(cnt, C)
    off = np.concatenate([[0], np.cumsum(cnt.reshape(-1))])
    assert u[:, 3].sum() == cnt.sum()
    assert np.all(u[:, 3] >= 1) and np.all(u[:, 3] <= C)
    cover = np.zeros(cnt.sum(), dtype=np.int32)
    for e, cls, r0, rows in u.tolist():
        assert off[2 * e + cls] <= r0 and r0 + rows <= off[2 * e + cls + 1]
        cover[r0:r0 + rows] += 1
    assert np.all(cover == 1)
    # all LS units before all BE units; inside a phase experts ascend, rows ascend
    cls = u[:, 1]
    assert np.all(np.diff(cls) >= 0)
    for c in (0, 1):
        part = u[cls == c]
        key = part[:, 0].astype(np.int64) * (1 << 32) + part[:, 2]
        assert np.all(np.diff(key) > 0)
    # number of units is sum of ceil(len / C)
    assert len(u) == int(np.sum((cnt + C - 1) // C))


# ------------------------------------------------------------------ step 5: expert FFN
def test_silu_closed_forms():
    assert oracle.silu(0.0) == 0.0
    assert oracle.silu(1.0) == pytest.approx(1.0 / (1.0 + math.exp(-1.0)), rel=1e-15)
    assert oracle.silu(40.0) == pytest.approx(40.0, rel=1e-15)
    assert abs(oracle.silu(-40.0)) < 1e-15
    for z in (0.3, 2.0, 7.5):
        assert oracle.silu(z) - oracle.silu(-z) == pytest.approx(z, rel=1e-14)
    assert oracle.silu(-1.0) < 0 < oracle.silu(1.0)


def test_expert_rows_equal_numpy_dense():
    cfg = small_cfg()
    inp = wl.make_inputs(cfg)
    x = wl.as_f64(inp.x)
    toks = [5, 0, 23, 5, 11]
    for e in (0, 3, 4):
        out, act = oracle.expert_rows(inp.x, inp.w["W1"], inp.w["W3"], inp.w["W2"], e, toks, want_act=True)
        w1, w3, w2 = (wl.as_f64(inp.w[n][e]) for n in ("W1", "W3", "W2"))
        ref_act = np_silu(x[toks] @ w1.T) * (x[toks] @ w3.T)
        np.testing.assert_allclose(act, ref_act, rtol=1e-12, atol=1e-18)
        np.testing.assert_allclose(out, ref_act @ w2.T, rtol=1e-12, atol=1e-18)
    # gate and up projections are not interchangeable: swapping them must change the result
    sw = oracle.expert_rows(inp.x, inp.w["W3"], inp.w["W1"], inp.w["W2"], 0, toks)
    assert not np.allclose(sw, oracle.expert_rows(inp.x, inp.w["W1"], inp.w["W3"], inp.w["W2"], 0, toks))


def test_expert_hand_worked_case():
    # H=2, F=1: x=(1,2); W1=(0.5,0.25) -> g=1; W3=(1,1) -> u=3; W2=(2,-1)^T
    x = np.array([[1.0, 2.0]], np.float32)
    w1 = np.array([[[0.5, 0.25]]], np.float32)
    w3 = np.array([[[1.0, 1.0]]], np.float32)
    w2 = np.array([[[2.0], [-1.0]]], np.float32)
    out = oracle.expert_rows(x, w1, w3, w2, 0, [0])
    m = 3.0 / (1.0 + math.exp(-1.0))
    np.testing.assert_allclose(out, [[2.0 * m, -m]], rtol=1e-15)


def test_zero_gate_projection_gives_zero_output():
    cfg = small_cfg()
    inp = wl.make_inputs(cfg)
    z = np.zeros_like(inp.w["W1"])
    out = oracle.expert_rows(inp.x, z, inp.w["W3"], inp.w["W2"], 1, list(range(cfg.N)))
    assert np.all(out == 0.0)


# ------------------------------------------------------------------ whole layer
@pytest.mark.parametrize("kw", [dict(), dict(k=1), dict(k=5), dict(n_ls=0), dict(n_ls=24),
                                dict(dtype="bf16", seed=78), dict(chunk_rows=1000)])
def test_layer_equals_dense_run_of_every_expert_then_mask(kw):
    cfg = small_cfg(**kw)
    inp = wl.make_inputs(cfg)
    bias = np.linspace(0.5, -0.5, cfg.E).astype(np.float32)
    lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, bias, cfg.k, cfg.chunk_rows)
    assert lay.run() is True
    y, comp = lay.y()
    assert comp.all()
    ref = dense_then_mask(inp, lay.idx, lay.wt)
    np.testing.assert_allclose(y, ref, rtol=1e-11, atol=1e-16)
    # the one-token-at-a-time path used at full sizes agrees too
    pick = [0, 3, cfg.N - 1]
    np.testing.assert_allclose(lay.y_tokens_direct(pick), ref[pick], rtol=1e-11, atol=1e-16)
    assert lay.cnt.sum() == cfg.N * cfg.k


def test_identical_experts_make_routing_irrelevant():
    cfg = small_cfg(E=4, k=3)
    inp = wl.make_inputs(cfg)
    for n in ("W1", "W3", "W2"):
        inp.w[n][:] = inp.w[n][0]
    lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, None, cfg.k, cfg.chunk_rows)
    lay.run()
    y, _ = lay.y()
    x = wl.as_f64(inp.x)
    w1, w3, w2 = (wl.as_f64(inp.w[n][0]) for n in ("W1", "W3", "W2"))
    ref = (np_silu(x @ w1.T) * (x @ w3.T)) @ w2.T            # weights sum to 1 => plain FFN
    np.testing.assert_allclose(y, ref, rtol=1e-11, atol=1e-16)


def test_paper_config1_invariants():
    cfg = wl.CONFIGS["cfg1"]
    inp = wl.make_inputs(cfg)
    assert int(inp.prio.sum()) == 16 and inp.x.shape == (64, 128) and inp.w["Wg"].shape == (128, 4)
    lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows)
    assert lay.cnt.sum() == cfg.N * cfg.k
    np.testing.assert_allclose(lay.wt.sum(1), 1.0, atol=1e-15)
    assert np.array_equal(np.sort(lay.perm), np.arange(cfg.A))
    lay.run()
    y, comp = lay.y()
    assert comp.all() and np.isfinite(y).all()
    np.testing.assert_allclose(y, dense_then_mask(inp, lay.idx, lay.wt), rtol=1e-11, atol=1e-16)


# ------------------------------------------------------------------ preemption / completeness
def test_every_single_cut_and_a_multi_cut_reproduce_the_uninterrupted_run():
    cfg = wl.CONFIGS["cfg1"]
    inp = wl.make_inputs(cfg)
    full = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows)
    full.run()
    y_full, _ = full.y()
    nu = full.n_units
    assert nu >= 8
    splits = [[c] for c in range(0, nu + 1)] + [[1, 2, 5], wl.cut_points(7, range(1, nu), 4)]
    for cuts in splits:
        lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows)
        prev = 0
        for c in cuts:
            lay.run(c - prev)
            # "preempted": only the retained state survives; rebuild the walker from it
            kept = dict(O=lay.O.copy(), done=lay.done.copy(), next_unit=lay.next_unit, executed=lay.executed.copy())
            lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows)
            lay.O, lay.done, lay.next_unit, lay.executed = kept["O"], kept["done"], kept["next_unit"], kept["executed"]
            prev = c
        assert lay.run() is True
        y, comp = lay.y()
        assert comp.all()
        assert np.array_equal(y, y_full)                    # exact: per-(token,slot) rows, fixed order
        assert np.all(lay.executed == 1)                    # no unit twice, none skipped


def test_only_complete_tokens_are_combined_and_ls_finishes_first():
    cfg = wl.CONFIGS["cfg1"]
    inp = wl.make_inputs(cfg)
    lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows)
    n_ls_units = int((lay.units[:, 1] == 0).sum())
    assert 0 < n_ls_units < lay.n_units
    lay.run(n_ls_units - 1)
    _, comp = lay.y()
    assert not comp[inp.prio != 0].all()                    # one LS unit still missing
    lay.run(1)
    y_mid, comp = lay.y()
    assert comp[inp.prio != 0].all() and not comp[inp.prio == 0].any()
    assert np.isnan(y_mid[inp.prio == 0]).all()
    lay.run()
    y_end, comp = lay.y()
    assert comp.all()
    assert np.array_equal(y_mid[inp.prio != 0], y_end[inp.prio != 0])


def complete_from_first_principles(idx, prio, E, chunk_rows, executed_chunks):
    """Which tokens are complete when the chunks in `executed_chunks` (a set of (expert, class,
    chunk number inside that expert's class queue)) have run, derived from the routing alone:
    assignment (n, j) to expert e sits at position #{n' < n of the same class that chose e} of the
    (e, class) FIFO queue, i.e. in chunk position // chunk_rows."""
    N, k = idx.shape
    comp = np.ones(N, dtype=bool)
    seen = np.zeros((E, 2), dtype=np.int64)
    for n in range(N):
        c = 0 if prio[n] else 1
        for e in sorted(set(int(v) for v in idx[n])):
            if (e, c, seen[e, c] // chunk_rows) not in executed_chunks:
                comp[n] = False
            seen[e, c] += 1
    return comp


@pytest.mark.parametrize("seed", [3, 4, 5])
def test_policy_chosen_unit_order_completeness_and_exactness(seed):
    cfg = small_cfg(N=40, n_ls=11, E=6, k=3, chunk_rows=3, seed=100 + seed)
    inp = wl.make_inputs(cfg)
    full = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows)
    full.run()
    y_full, _ = full.y()
    rng = np.random.default_rng(seed)
    lay = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows)
    order = rng.permutation(lay.n_units)
    first, rest = order[: lay.n_units // 2], order[lay.n_units // 2:]
    lay.run_units(first)
    # chunk number of a unit inside its (expert, class) queue, from the unit list's own row ranges
    chunks = set()
    for u in first:
        e, c, r0, _rows = (int(v) for v in lay.units[u])
        start = int(lay.off[2 * e + c])
        assert (r0 - start) % cfg.chunk_rows == 0
        chunks.add((e, c, (r0 - start) // cfg.chunk_rows))
    y_mid, comp = lay.y()
    assert np.array_equal(comp, complete_from_first_principles(lay.idx, inp.prio, cfg.E, cfg.chunk_rows, chunks))
    assert 0 < comp.sum() < cfg.N                                   # the case has both kinds of token
    assert np.array_equal(y_mid[comp], y_full[comp]) and np.isnan(y_mid[~comp]).all()
    # the cursor is the first unit that has not run; run() skips what a policy already ran
    assert lay.next_unit == min(set(range(lay.n_units)) - set(int(u) for u in first))
    lay.run(2)
    lay.run_units([u for u in rest if not lay.executed[u]][::-1])
    assert lay.next_unit == lay.n_units and np.all(lay.executed == 1)
    y_end, comp = lay.y()
    assert comp.all() and np.array_equal(y_end, y_full)


def test_workload_recipes():
    c5 = wl.CONFIGS["cfg5"]
    b = wl.make_bias(c5)
    assert b.shape == (64,) and b.max() == 0.0
    np.testing.assert_allclose(np.sort(-b), 1.1 * np.log(np.arange(1, 65)), rtol=1e-6)
    c4 = wl.CONFIGS["cfg4"]
    assert wl.make_bias(c4)[0] == np.float32(1.5) and np.all(wl.make_bias(c4)[1:] == 0)
    assert int(wl.make_prio(c5).sum()) == 1024 and int(wl.make_prio(wl.CONFIGS["cfg3_ls"]).sum()) == 512
    assert int(wl.make_prio(wl.CONFIGS["cfg3_be"]).sum()) == 0
    x = wl.make_x(wl.scaled(c4))
    assert x.dtype == np.uint16 and x.shape == (64, 4096)
    v = wl.bf16_bits_to_f32(x)
    assert abs(float(v.std()) - 1.0) < 0.02
    w = wl.make_weights(wl.scaled(c5, E=2, F=64, H=128))
    assert abs(float(wl.bf16_bits_to_f32(w["W1"]).std()) - 0.02) < 1e-3
    assert w["W1"].shape == (2, 64, 128) and w["W2"].shape == (2, 128, 64) and w["Wg"].shape == (128, 2)


def test_kept_activations_are_the_swiglu_values_and_leave_the_outputs_alone():
    """OracleLayer.keep_act stores silu(W1 x) * (W3 x) per sorted row (used by the GPU tests to size
    the error of the bf16 path's activation rounding); the outputs are the same with and without."""
    cfg = small_cfg(seed=91, N=30, k=3)
    inp = wl.make_inputs(cfg)
    a = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows)
    b = oracle.OracleLayer(inp.x, inp.w, inp.prio, inp.bias, cfg.k, cfg.chunk_rows)
    b.keep_act = True
    a.run(); b.run(3); b.run()
    assert a.act is None and np.array_equal(a.O, b.O)
    x = wl.as_f64(inp.x)
    for r in range(cfg.A):
        n, e = b.perm[r] // cfg.k, b.idx.reshape(-1)[b.perm[r]]
        want = np_silu(wl.as_f64(inp.w["W1"][e]) @ x[n]) * (wl.as_f64(inp.w["W3"][e]) @ x[n])
        np.testing.assert_allclose(b.act[r], want, rtol=1e-12, atol=1e-15)
