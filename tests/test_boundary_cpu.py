"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes workspaces, plans work units like the oracle, and enforces call order."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_2503_09304_amd as q

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for header, prefix in (("qmoe.h", "moe_"), ("qsched.h", "sched_")):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(%s[a-z_]+)\s*\(" % prefix, text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert {"moe_route", "moe_permute", "moe_expert_run", "moe_combine"} <= set(names)
    assert {"sched_submit", "sched_token", "sched_next_batch", "sched_preempt_wanted"} <= set(names)
    L = q.lib()
    for n in names:
        assert hasattr(L, n), f"{n} declared in include/ but not exported"


def test_workspace_size_and_config_validation():
    good = q.MoeConfig(8, 2, 4096, 14336, q.MOE_BF16, 256, 512)
    nbytes = q.moe_workspace_bytes(good)
    A = 512 * 2
    assert nbytes >= A * 14336 * 2 + A * 4096 * 4          # activation + expert-output regions
    assert nbytes % 256 == 0
    for bad in [q.MoeConfig(0, 1, 64, 64, 0, 16, 8), q.MoeConfig(4, 5, 64, 64, 0, 16, 8),
                q.MoeConfig(4, 2, 100, 64, q.MOE_BF16, 16, 8), q.MoeConfig(4, 2, 64, 64, 7, 16, 8),
                q.MoeConfig(4, 2, 64, 64, 0, 0, 8), q.MoeConfig(4, 2, 64, 64, 0, 257, 8),
                q.MoeConfig(300, 2, 64, 64, 0, 16, 8)]:
        with pytest.raises(q.MoeError):
            q.moe_workspace_bytes(bad)


@pytest.mark.parametrize("C_rows", [1, 4, 16, 256])
def test_plan_units_matches_oracle_unit_list(C_rows):
    rng = np.random.default_rng(C_rows)
    cnt = rng.integers(0, 50, size=(7, 2)).astype(np.int32)
    cnt[3] = 0
    got = q.moe_plan_units(cnt.tolist(), 7, C_rows)
    ref = [tuple(int(v) for v in r) for r in oracle.units(cnt, C_rows)]
    assert got == ref


def test_call_order_and_argument_errors_without_touching_the_gpu():
    L = q.lib()
    cfg = q.MoeConfig(4, 2, 128, 256, q.MOE_F32, 16, 64)
    nbytes = q.moe_workspace_bytes(cfg)
    fake_ws = 256 * 1000                                   # never dereferenced by these calls
    h = C.c_void_p()
    assert L.moe_create(C.byref(cfg), None, nbytes, C.byref(h)) == q.MOE_E_ARG
    assert L.moe_create(C.byref(cfg), fake_ws + 8, nbytes, C.byref(h)) == q.MOE_E_WORKSPACE
    assert L.moe_create(C.byref(cfg), fake_ws, nbytes - 1, C.byref(h)) == q.MOE_E_WORKSPACE
    assert "needed" in q.moe_last_error()
    assert L.moe_create(C.byref(cfg), fake_ws, nbytes, C.byref(h)) == q.MOE_OK
    cur = q.MoeCursor(0, 0)
    w = q.MoeWeights(1, 2, 3, 4)
    assert L.moe_permute(h, 1, C.byref(cur), None) == q.MOE_E_STATE
    assert L.moe_expert_run(h, 1, C.byref(w), 1, C.byref(cur), None) == q.MOE_E_STATE
    assert L.moe_combine(h, 1, q.MOE_CLASS_ALL, None) == q.MOE_E_STATE
    p, nb = C.c_void_p(), C.c_size_t()
    assert L.moe_get(h, 0, C.byref(p), C.byref(nb)) == q.MOE_E_STATE
    assert L.moe_route(h, 1, 65, C.byref(w), None, None) == q.MOE_E_ARG          # above max_tokens
    assert L.moe_route(h, 1, -1, C.byref(w), None, None) == q.MOE_E_ARG
    assert L.moe_route(h, None, 4, C.byref(w), None, None) == q.MOE_E_ARG
    bad_w = q.MoeWeights(1, 0, 3, 4)
    assert L.moe_route(h, 1, 4, C.byref(bad_w), None, None) == q.MOE_E_ARG
    assert L.moe_route(None, 1, 4, C.byref(w), None, None) == q.MOE_E_ARG
    assert L.moe_destroy(h) == q.MOE_OK
    assert L.moe_destroy(None) == q.MOE_E_ARG


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    import paper_2503_09304_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        b.lib()


def test_default_k_split_takes_the_fewest_ranges_that_fill_the_chip():
    """down_ksplit = 0 is resolved from the configuration alone (include/qmoe.h); the workspace size
    shows the choice: one partial plane of max_tokens*k*H floats per K range."""
    def size(E, k, H, F, tokens, ks):
        return q.moe_workspace_bytes(q.MoeConfig(E, k, H, F, q.MOE_BF16, 256, tokens, ks))
    # Mixtral shape, decode-sized batch: 8 experts x 16 column tiles x 2 ranges = 256 workgroups
    assert size(8, 2, 4096, 14336, 64, 0) == size(8, 2, 4096, 14336, 64, 2)
    assert size(8, 2, 4096, 14336, 64, 2) < size(8, 2, 4096, 14336, 64, 4)
    assert size(8, 2, 4096, 14336, 64, 1) < size(8, 2, 4096, 14336, 64, 2)
    # 64 experts x 8 column tiles fill the chip without a split
    assert size(64, 8, 2048, 1408, 64, 0) == size(64, 8, 2048, 1408, 64, 1)
    # 4 experts x 4 column tiles: four ranges where F allows them, two where it only allows those
    assert size(4, 2, 1024, 1024, 64, 0) == size(4, 2, 1024, 1024, 64, 4)
    assert size(4, 2, 1024, 896, 64, 0) == size(4, 2, 1024, 896, 64, 2)
    # compute-bound batches (more than 256 rows per expert on average) never split
    assert size(8, 2, 4096, 14336, 4096, 0) == size(8, 2, 4096, 14336, 4096, 1)
