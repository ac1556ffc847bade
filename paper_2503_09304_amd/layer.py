"""One layer-batch as a Python object over the binding: moves host arrays (fp32, or bf16 / 4-bit codes as
bit patterns) to the device, holds the context and its buffers, drives the C calls, fetches results
as numpy arrays.  Used by the benchmark and the tests.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as q

DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    """fp32 array -> float tensor; bf16 bit patterns (uint16) -> bfloat16 tensor, same bits."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a).to(DEV)


def to_host(t: torch.Tensor) -> np.ndarray:
    """Tensor -> numpy; bfloat16 comes back as uint16 bit patterns."""
    t = t.detach()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


class DevWeights:
    """Weights on the device, row-major; .packed() gives the re-laid-out copy (bf16 only)."""

    def __init__(self, w):
        self.Wg, self.W1, self.W3, self.W2 = (to_dev(w[n]) for n in ("Wg", "W1", "W3", "W2"))
        self.struct = q.Context.weights(self.Wg, self.W1, self.W3, self.W2)
        self._packed = None

    def packed(self) -> "DevWeights":
        if self._packed is None:
            H, E = self.Wg.shape
            F = self.W1.shape[1]
            p = object.__new__(DevWeights)
            p.Wg = torch.empty(((E + 15) // 16 * 16, H), dtype=self.Wg.dtype, device=DEV)
            p.W1, p.W3, p.W2 = (torch.empty_like(t) for t in (self.W1, self.W3, self.W2))
            p.struct = q.Context.weights(p.Wg, p.W1, p.W3, p.W2)
            cfg = q.MoeConfig(E, 1, H, F, q.MOE_BF16, 1, 0)
            q.moe_pack_weights(cfg, self.struct, p.struct)
            torch.cuda.synchronize()
            p._packed = p
            self._packed = p
        return self._packed


class DevWeightsMX:
    """4-bit expert weights on the device: row-major codes and scales as generated, and .packed(),
    the block order the kernels read.  Same attributes as DevWeights where the layer needs them."""

    def __init__(self, w):
        self.Wg = to_dev(w["Wg"])
        for n in ("W1", "W3", "W2"):
            setattr(self, n, torch.from_numpy(w[n + "q"]).to(DEV))
            setattr(self, "S" + n[1], torch.from_numpy(w[n + "s"]).to(DEV))
        self.struct = q.Context.weights(self.Wg, self.W1, self.W3, self.W2, q.MOE_W_MXFP4_ROWMAJOR, self.S1, self.S3, self.S2)
        self._packed = None

    def packed(self) -> "DevWeightsMX":
        if self._packed is None:
            H, E = self.Wg.shape
            F = self.W1.shape[1]
            p = object.__new__(DevWeightsMX)
            p.Wg = torch.empty(((E + 15) // 16 * 16, H), dtype=self.Wg.dtype, device=DEV)
            for n in ("W1", "W3", "W2", "S1", "S3", "S2"):
                setattr(p, n, torch.empty_like(getattr(self, n)))
            p.struct = q.Context.weights(p.Wg, p.W1, p.W3, p.W2, q.MOE_W_MXFP4_ROWMAJOR, p.S1, p.S3, p.S2)
            cfg = q.MoeConfig(E, 1, H, F, q.MOE_BF16, 1, 0)
            q.moe_pack_weights(cfg, self.struct, p.struct)
            torch.cuda.synchronize()
            assert p.struct.layout == q.MOE_W_MXFP4
            p._packed = p
            self._packed = p
        return self._packed


class GpuLayer:
    """One layer-batch on the device."""

    def __init__(self, inp, dev_w: "DevWeights | None" = None, max_tokens: "int | None" = None, down_ksplit: int = 0):
        """inp: an object with cfg (N, E, k, H, F, dtype, chunk_rows), x, prio, bias and w (host arrays)."""
        cfg = inp.cfg
        self.cfg = cfg
        self.inp = inp
        self.dw = dev_w if dev_w is not None else DevWeights(inp.w)
        self.x = to_dev(inp.x)
        self.prio = torch.from_numpy(inp.prio).to(DEV)
        self.bias = None if inp.bias is None else torch.from_numpy(inp.bias).to(DEV)
        dt = q.MOE_BF16 if cfg.dtype == "bf16" else q.MOE_F32
        self.ctx = q.Context(cfg.E, cfg.k, cfg.H, cfg.F, dt, cfg.chunk_rows, max_tokens or max(cfg.N, 1),
                             down_ksplit=down_ksplit)
        self.y = torch.full((cfg.N, cfg.H), float("nan"), dtype=self.x.dtype, device=DEV)

    def route_permute(self):
        self.ctx.route(self.x, self.dw.struct, self.bias, n_tokens=self.cfg.N)
        return self.ctx.permute(self.prio)

    def run(self, max_units=q.UINT32_MAX):
        return self.ctx.expert_run(self.x, self.dw.struct, max_units)

    def combine(self, mask=q.MOE_CLASS_ALL):
        return self.ctx.combine(self.y, mask)

    def full(self, cuts=()):
        """route, permute, experts (stopping at each cursor position in `cuts`), combine."""
        cur = self.route_permute()
        prev = 0
        for c in cuts:
            if c > prev:
                self.run(c - prev)
            prev = max(prev, c)
        if cur.n_units == 0 or self.ctx.cursor.next_unit < cur.n_units:
            self.run()
        self.combine()
        torch.cuda.synchronize()
        return self

    def fetch(self, *names):
        torch.cuda.synchronize()
        out = {}
        for n in names:
            if n == "y":
                out[n] = to_host(self.y)
            else:
                out[n] = to_host(self.ctx.get(n).clone())
        return out
