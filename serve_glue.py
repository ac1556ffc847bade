"""Harness side of the serving benchmark and its test: everything a served model has around its MoE
layers that is not part of the library, as plain PyTorch on the device.

  * synthetic_weights: seeded N(0, 0.02^2) bf16 weights generated on the device and re-laid-out with
    moe_pack_weights;
  * SyntheticGlue: the object paper_2503_09304_amd.serve.Engine asks for its inputs and for the step
    between two MoE layers: hidden states are rows of a seeded bank, the next layer's input is x + y
    (a residual standing in for the attention block); with digest=True it also keeps a per-job
    checksum of the final hidden states and counts the rows the layers queued as LS, for the test
    that compares policies bit for bit.
"""
from __future__ import annotations

import torch

import paper_2503_09304_amd as q


def synthetic_weights(E: int, H: int, F: int, seed: int, device="cuda:0"):
    g = torch.Generator(device=device)
    g.manual_seed(seed)

    def rnd(*shape):
        return (torch.randn(*shape, generator=g, device=device, dtype=torch.float32) * 0.02).to(torch.bfloat16)

    Wg = rnd(H, E)
    W1, W3, W2 = rnd(E, F, H), rnd(E, F, H), rnd(E, H, F)
    src = q.Context.weights(Wg, W1, W3, W2)
    pWg = torch.empty(((E + 15) // 16 * 16, H), dtype=torch.bfloat16, device=device)
    pW1, pW3, pW2 = torch.empty_like(W1), torch.empty_like(W3), torch.empty_like(W2)
    dst = q.Context.weights(pWg, pW1, pW3, pW2)
    q.moe_pack_weights(q.MoeConfig(E, 1, H, F, q.MOE_BF16, 1, 0), src, dst)
    torch.cuda.synchronize()
    return dst, (pWg, pW1, pW3, pW2)     # the struct and the tensors that keep its memory alive


class SyntheticGlue:
    def __init__(self, H: int, k: int, bank_rows: int = 4096, seed: int = 1, digest: bool = False, max_job: int = 0,
                 device="cuda:0"):
        g = torch.Generator(device=device)
        g.manual_seed(seed)
        self.bank = torch.randn(bank_rows, H, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)
        self.bank_rows = bank_rows
        self.k = k
        if digest:
            self.digest = torch.zeros(max_job + 1, dtype=torch.int64, device=device)
            self.ls_rows_seen = torch.zeros((), dtype=torch.int64, device=device)
            self.ls_rows_expected = 0
            self.observe_layer = self._observe_layer
            self.observe_output = self._observe_output

    def fill_inputs(self, x, rows, n):
        torch.index_select(self.bank, 0, rows[:n], out=x[:n])

    def between_layers(self, x, y):
        x.add_(y)

    def _observe_layer(self, ctx, n_ls_rows):
        # rows the layer queued as LS, against what the batch holds
        self.ls_rows_seen += ctx.get("counts")[:, 0].sum()
        self.ls_rows_expected += self.k * n_ls_rows

    def _observe_output(self, x, owner, n):
        h = x.view(torch.int16).to(torch.int32).sum(1, dtype=torch.int64)
        self.digest.index_add_(0, owner[:n], h)
