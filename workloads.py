"""Seeded synthetic inputs for one MoE layer (tokens, weights, priority flags, router bias).

This module only draws random numbers and rounds them to the storage type.  It holds none of
the layer's arithmetic (no routing, no sort, no FFN), so both the CPU oracle's tests and the
GPU path's tests/benchmark can take their inputs from it without sharing any of the method.

The five workloads stand in for the paper's evaluation traffic (Evaluation section: Mixtral 8x7B,
batches of at most 32 sequences, 20 % of prompts tagged latency-sensitive): at the granularity of
one MoE layer that traffic reduces to a token count, a priority mix and an expert-load
distribution, which each recipe below fixes synthetically.

All draws use numpy's PCG64 (`default_rng`) with a seed derived from (config seed, tensor tag,
expert), so every tensor can be regenerated alone and experts can be drawn in parallel.
bf16 tensors are returned as uint16 bit patterns (round-to-nearest-even from the fp32 draw).
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np

LS = 1  # prio flag of a latency-sensitive token
BE = 0  # prio flag of a best-effort token


@dataclass(frozen=True)
class LayerConfig:
    name: str
    N: int              # tokens in the batch
    n_ls: int           # how many of them are latency-sensitive
    H: int              # hidden size
    F: int              # SwiGLU ffn size
    E: int              # experts
    k: int              # experts per token
    dtype: str          # "f32" or "bf16" (storage of x and weights)
    seed: int
    chunk_rows: int = 256      # rows per preemptible work unit
    bias_kind: str = "none"    # "none" | "expert0" | "zipf"
    bias_arg: float = 0.0
    ls_layout: str = "scattered"   # "scattered": seeded positions; "all"/"none" follow n_ls
    weight_seed: Optional[int] = None  # share weights between configs (cfg3 reuses cfg2's)

    @property
    def A(self) -> int:
        return self.N * self.k


CONFIGS: Dict[str, LayerConfig] = {
    # Tiny fp32 layer; one preemption after expert 1 in the tests.
    "cfg1": LayerConfig("cfg1", N=64, n_ls=16, H=128, F=256, E=4, k=2, dtype="f32", seed=1001,
                        chunk_rows=16),
    # Mixtral-shaped prefill batch, 128 LS + 384 BE tokens.
    "cfg2": LayerConfig("cfg2", N=512, n_ls=128, H=4096, F=14336, E=8, k=2, dtype="bf16",
                        seed=2001, weight_seed=2001),
    # Preemption scenario: a 3584-token BE prompt in flight, a 512-token LS batch arrives.
    "cfg3_be": LayerConfig("cfg3_be", N=3584, n_ls=0, H=4096, F=14336, E=8, k=2, dtype="bf16",
                           seed=3001, weight_seed=2001),
    "cfg3_ls": LayerConfig("cfg3_ls", N=512, n_ls=512, H=4096, F=14336, E=8, k=2, dtype="bf16",
                           seed=3002, weight_seed=2001),
    # Decode step, one token per sequence, expert 0 made hot by +1.5 on its logit.
    "cfg4": LayerConfig("cfg4", N=64, n_ls=16, H=4096, F=14336, E=8, k=2, dtype="bf16",
                        seed=4001, weight_seed=2001, bias_kind="expert0", bias_arg=1.5),
    # Fine-grained MoE, Zipf(s=1.1)-ranked router bias: heavily skewed expert loads.
    "cfg5": LayerConfig("cfg5", N=8192, n_ls=1024, H=2048, F=1408, E=64, k=8, dtype="bf16",
                        seed=5001, bias_kind="zipf", bias_arg=1.1),
}


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of `cfg` with some fields replaced (used for reduced-size parity cases)."""
    return replace(cfg, **kw)


# --------------------------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round finite fp32 values to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (b >> np.uint32(16)) & np.uint32(1)
    r = (b + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(x32: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x32, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x32)
    raise ValueError(dtype)


def as_f64(a: np.ndarray) -> np.ndarray:
    """Exact fp64 view of a stored tensor (fp32 array or bf16 bit patterns)."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


# --------------------------------------------------------------------------------------------
# draws
# --------------------------------------------------------------------------------------------
_TAGS = {"x": 1, "wg": 2, "w1": 3, "w3": 4, "w2": 5, "prio": 6, "rank": 7}


def _rng(seed: int, tag: str, sub: int = 0) -> np.random.Generator:
    return np.random.default_rng([int(seed), _TAGS[tag], int(sub)])


def _normal(seed: int, tag: str, sub: int, shape, std: float, dtype: str) -> np.ndarray:
    g = _rng(seed, tag, sub).standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        g *= np.float32(std)
    return _store(g, dtype)


def make_x(cfg: LayerConfig) -> np.ndarray:
    """Token hidden states, x ~ N(0,1), shape [N,H]."""
    return _normal(cfg.seed, "x", 0, (cfg.N, cfg.H), 1.0, cfg.dtype)


def make_prio(cfg: LayerConfig) -> np.ndarray:
    """Priority flag per token (uint8, 1 = LS, 0 = BE): exactly n_ls ones at seeded positions."""
    p = np.zeros(cfg.N, dtype=np.uint8)
    if cfg.n_ls >= cfg.N:
        p[:] = LS
    elif cfg.n_ls > 0:
        pos = _rng(cfg.seed, "prio").permutation(cfg.N)[: cfg.n_ls]
        p[pos] = LS
    return p


def make_bias(cfg: LayerConfig) -> Optional[np.ndarray]:
    """Router logit bias [E] fp32 (a workload device that skews the expert loads), or None."""
    if cfg.bias_kind == "none":
        return None
    b = np.zeros(cfg.E, dtype=np.float32)
    if cfg.bias_kind == "expert0":
        b[0] = np.float32(cfg.bias_arg)
    elif cfg.bias_kind == "zipf":
        rank = _rng(cfg.seed, "rank").permutation(cfg.E) + 1        # rank[e] in 1..E
        b[:] = (-cfg.bias_arg * np.log(rank.astype(np.float64))).astype(np.float32)
    else:
        raise ValueError(cfg.bias_kind)
    return b


def make_weights(cfg: LayerConfig, threads: int = 8) -> Dict[str, np.ndarray]:
    """Gate and expert weights, all ~ N(0, 0.02^2).

    Wg [H,E] row-major; W1, W3 [E,F,H] (gate_proj, up_proj; H contiguous); W2 [E,H,F]
    (down_proj; F contiguous).
    """
    ws = cfg.weight_seed if cfg.weight_seed is not None else cfg.seed
    np_dt = np.float32 if cfg.dtype == "f32" else np.uint16
    out = {
        "Wg": _normal(ws, "wg", 0, (cfg.H, cfg.E), 0.02, cfg.dtype),
        "W1": np.empty((cfg.E, cfg.F, cfg.H), dtype=np_dt),
        "W3": np.empty((cfg.E, cfg.F, cfg.H), dtype=np_dt),
        "W2": np.empty((cfg.E, cfg.H, cfg.F), dtype=np_dt),
    }

    def fill(job):
        name, e = job
        shape = (cfg.H, cfg.F) if name == "W2" else (cfg.F, cfg.H)
        out[name][e] = _normal(ws, name.lower(), e, shape, 0.02, cfg.dtype)

    jobs = [(n, e) for e in range(cfg.E) for n in ("W1", "W3", "W2")]
    if threads > 1 and cfg.E * cfg.F * cfg.H > (1 << 22):
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, jobs))
    else:
        for j in jobs:
            fill(j)
    return out


def make_weights_mxfp4(cfg: LayerConfig) -> Dict[str, np.ndarray]:
    """Seeded synthetic 4-bit expert weights in the microscaling FP4 storage form: for W1/W3 [E,F,H]
    and W2 [E,H,F] one byte per two elements along K (even k in the low nibble), codes uniform over
    the 16 e2m1 patterns, and one e8m0 scale byte per 32 elements drawn from 2^-8, 2^-7, 2^-6 (the
    values then have a standard deviation of about 0.02-0.03, like the bf16 recipe).  Wg stays bf16.
    Only random draws here: what the codes mean is the business of whoever consumes them."""
    ws = cfg.weight_seed if cfg.weight_seed is not None else cfg.seed
    out = {"Wg": _normal(ws, "wg", 0, (cfg.H, cfg.E), 0.02, "bf16")}
    for name, tag, (R, K) in (("W1", "w1", (cfg.F, cfg.H)), ("W3", "w3", (cfg.F, cfg.H)), ("W2", "w2", (cfg.H, cfg.F))):
        assert K % 32 == 0
        rng = _rng(ws, tag, 4000)
        out[name + "q"] = rng.integers(0, 256, size=(cfg.E, R, K // 2), dtype=np.uint8)
        out[name + "s"] = rng.integers(119, 122, size=(cfg.E, R, K // 32), dtype=np.uint8)
    return out


@dataclass
class LayerInputs:
    cfg: LayerConfig
    x: np.ndarray
    prio: np.ndarray
    bias: Optional[np.ndarray]
    w: Dict[str, np.ndarray] = field(repr=False)


def make_inputs(cfg: LayerConfig, weights: Optional[Dict[str, np.ndarray]] = None) -> LayerInputs:
    """Everything one layer call needs.  Pass `weights` to reuse a set already drawn."""
    return LayerInputs(cfg=cfg, x=make_x(cfg), prio=make_prio(cfg), bias=make_bias(cfg),
                       w=weights if weights is not None else make_weights(cfg))


def cut_points(seed: int, boundaries, n_cuts: int):
    """`n_cuts` distinct seeded cut positions drawn from `boundaries`, ascending."""
    b = np.asarray(sorted(set(int(v) for v in boundaries)), dtype=np.int64)
    if len(b) == 0:
        return []
    n = min(n_cuts, len(b))
    pick = np.random.default_rng([int(seed), 99]).choice(len(b), size=n, replace=False)
    return sorted(int(v) for v in b[pick])


def describe(cfg: LayerConfig) -> str:
    return (f"{cfg.name}: N={cfg.N} ({cfg.n_ls} LS) H={cfg.H} F={cfg.F} E={cfg.E} k={cfg.k} "
            f"{cfg.dtype} chunk_rows={cfg.chunk_rows} seed={cfg.seed}")


def flops(cfg: LayerConfig) -> float:
    """Algorithmic flops of one layer pass: expert GEMMs (6*A*H*F) plus the gate GEMM (2*N*H*E)."""
    return 6.0 * cfg.A * cfg.H * cfg.F + 2.0 * cfg.N * cfg.H * cfg.E


def elem_bytes(cfg: LayerConfig) -> int:
    return 4 if cfg.dtype == "f32" else 2


def make_jobs(n: int, rate_per_s: float, p_ls: float, seed: int, max_prompt: int = 512, max_out: int = 32,
              min_prompt: int = 16, min_out: int = 4):
    """A seeded synthetic request stream standing in for the paper's workload generator (prompts of
    a public conversation dataset, a random 20 % marked LS, Poisson arrivals): exponential
    inter-arrival times at `rate_per_s`, log-normal prompt and output lengths clipped to the given
    ranges, each job LS with probability p_ls.  Returns a dict of arrays, one entry per job."""
    rng = np.random.default_rng([int(seed), 4242])
    arrival = np.cumsum(rng.exponential(1.0 / rate_per_s, size=n))
    prompt = np.clip(np.round(rng.lognormal(mean=math.log(0.25 * max_prompt), sigma=0.9, size=n)), min_prompt, max_prompt)
    out = np.clip(np.round(rng.lognormal(mean=math.log(0.4 * max_out), sigma=0.7, size=n)), min_out, max_out)
    is_ls = rng.random(n) < p_ls
    return {"arrival_s": arrival, "prompt_len": prompt.astype(np.int64), "out_len": out.astype(np.int64),
            "is_ls": is_ls}


if __name__ == "__main__":
    for c in CONFIGS.values():
        print(describe(c), f"flops={flops(c):.3e}", f"ridge_rows~{math.ceil(2.5e15 / 8e12)}")
