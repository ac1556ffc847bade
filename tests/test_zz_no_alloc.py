"""moe_route_noalloc (the router for callers that cannot allocate: its one scratch buffer is a static
array in the library's device image) against moe_route through the C ABI: logits, expert indices and
gate weights bit for bit, on two calls in a row, the second with a smaller input that leaves stale
contents of the first in the shared scratch array.  Needs an MI355X (-m gpu)."""
import numpy as np
import pytest
import torch

import paper_2503_09304_amd as q
import workloads as wl
from gpu_util import DEV, GpuLayer

pytestmark = pytest.mark.gpu


def route_both(cfg):
    inp = wl.make_inputs(cfg)
    g = GpuLayer(inp)                                      # row-major weights: moe_route transposes Wg into its workspace
    g.ctx.route(g.x, g.dw.struct, g.bias, n_tokens=cfg.N)
    torch.cuda.synchronize()
    want = {n: g.ctx.get(n).clone() for n in ("logits", "topk_idx", "topk_w")}
    dt = q.MOE_BF16 if cfg.dtype == "bf16" else q.MOE_F32
    c = q.MoeConfig(cfg.E, cfg.k, cfg.H, cfg.F, dt, cfg.chunk_rows, cfg.N, 0)
    logits = torch.full((cfg.N, cfg.E), float("nan"), dtype=torch.float32, device=DEV)
    idx = torch.full((cfg.N, cfg.k), -1, dtype=torch.int32, device=DEV)
    w = torch.full((cfg.N, cfg.k), float("nan"), dtype=torch.float32, device=DEV)
    assert q.moe_route_noalloc(c, g.x, cfg.N, g.dw.Wg, g.bias, logits, idx, w) == q.MOE_OK
    torch.cuda.synchronize()
    assert torch.equal(logits.view(torch.int32), want["logits"].view(torch.int32))
    assert torch.equal(idx, want["topk_idx"])
    assert torch.equal(w.view(torch.int32), want["topk_w"].view(torch.int32))
    return g


def test_router_without_allocation_matches_moe_route_twice_in_a_row():
    big = wl.LayerConfig("na_big", dtype="bf16", seed=5101, E=64, k=8, H=2048, F=128, N=1500, n_ls=300, chunk_rows=64,
                         bias_kind="zipf", bias_arg=1.1)
    small = wl.LayerConfig("na_small", dtype="bf16", seed=5102, E=8, k=2, H=256, F=128, N=77, n_ls=20, chunk_rows=64)
    keep = route_both(big)           # fills 64 x 2048 bf16 of the scratch array
    route_both(small)                # 16 x 256: the rest of the array still holds the first call's rows
    route_both(wl.LayerConfig("na_f32", dtype="f32", seed=5103, E=5, k=3, H=100, F=72, N=150, n_ls=40, chunk_rows=37))
    del keep


def test_router_without_allocation_rejects_what_does_not_fit():
    c = q.MoeConfig(256, 2, 8192, 64, q.MOE_BF16, 64, 16, 0)          # 256 x 8192 x 2 = 4 MiB > 2 MiB
    x = torch.zeros((16, 8192), dtype=torch.bfloat16, device=DEV)
    wg = torch.zeros((8192, 256), dtype=torch.bfloat16, device=DEV)
    lo = torch.zeros((16, 256), dtype=torch.float32, device=DEV)
    ix = torch.zeros((16, 2), dtype=torch.int32, device=DEV)
    tw = torch.zeros((16, 2), dtype=torch.float32, device=DEV)
    with pytest.raises(q.MoeError) as e:
        q.moe_route_noalloc(c, x, 16, wg, None, lo, ix, tw)
    assert e.value.code == q.MOE_E_ARG and "scratch" in str(e.value)
    with pytest.raises(q.MoeError):
        q.moe_route_noalloc(q.MoeConfig(8, 2, 256, 64, q.MOE_BF16, 64, 16, 0), x, 16, None, None, lo, ix, tw)
