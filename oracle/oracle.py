"""ctypes front-end of the C oracle (oracle/moe_oracle.c) plus the layer-level driver that walks
the work-unit list, so that a preempted-then-resumed run can be simulated step by step.

TEST INFRASTRUCTURE ONLY — see the header of moe_oracle.c.  Tensors are numpy arrays: fp32
values or bf16 bit patterns (uint16); everything computed is fp64.
"""
from __future__ import annotations

import ctypes as C
import hashlib
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_lib = None


def _cpu_tag() -> str:
    """The library is built with -march=native, so its name carries a hash of this host's CPU
    flags: a copy built on another machine is not picked up by mistake."""
    flags = ""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("flags"):
                    flags = line
                    break
    except OSError:
        pass
    return hashlib.sha1(flags.encode()).hexdigest()[:10]


_LIB = os.path.join(_HERE, f"liboracle_{_cpu_tag()}.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-march=native", "-fopenmp", "-fno-fast-math", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.oracle_silu.restype = C.c_double
        L.oracle_silu.argtypes = [C.c_double]
        L.oracle_threads.restype = C.c_int
        L.oracle_units.restype = C.c_int
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dt(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError(f"oracle tensors are float32 or bf16 bit patterns (uint16), got {a.dtype}")


def _c(a: np.ndarray, dtype=None) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def threads() -> int:
    return int(_load().oracle_threads())


def set_threads(n: int) -> None:
    _load().oracle_set_threads(C.c_int(int(n)))


def silu(z: float) -> float:
    return float(_load().oracle_silu(float(z)))


def gate_logits(x: np.ndarray, wg: np.ndarray, bias: Optional[np.ndarray]) -> np.ndarray:
    """L[n,e] = sum_h x[n,h] wg[h,e] + bias[e], fp64."""
    x, wg = _c(x), _c(wg)
    assert _dt(x) == _dt(wg)
    N, H = x.shape
    H2, E = wg.shape
    assert H == H2
    b = None if bias is None else _c(bias, np.float32)
    L = np.empty((N, E), dtype=np.float64)
    _load().oracle_gate_logits(_p(x), _p(wg), _p(b), C.c_int(_dt(x)), C.c_int(N), C.c_int(H),
                               C.c_int(E), _p(L))
    return L


def softmax(L: np.ndarray) -> np.ndarray:
    L = _c(L, np.float64)
    P = np.empty_like(L)
    _load().oracle_softmax(_p(L), C.c_int(L.shape[0]), C.c_int(L.shape[1]), _p(P))
    return P


def topk(L: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """(idx [N,k] int32, wt [N,k] fp64) from logits L [N,E] (fp64)."""
    L = _c(L, np.float64)
    N, E = L.shape
    assert 1 <= k <= E
    P = softmax(L)
    idx = np.empty((N, k), dtype=np.int32)
    wt = np.empty((N, k), dtype=np.float64)
    _load().oracle_topk(_p(L), _p(P), C.c_int(N), C.c_int(E), C.c_int(k), _p(idx), _p(wt))
    return idx, wt


def topk_margin(L: np.ndarray, k: int) -> np.ndarray:
    L = _c(L, np.float64)
    m = np.empty(L.shape[0], dtype=np.float64)
    _load().oracle_topk_margin(_p(L), C.c_int(L.shape[0]), C.c_int(L.shape[1]), C.c_int(k), _p(m))
    return m


def route(x, wg, bias, k: int):
    """Steps 1-3: (L, idx, wt)."""
    L = gate_logits(x, wg, bias)
    idx, wt = topk(L, k)
    return L, idx, wt


def queues(idx: np.ndarray, prio: np.ndarray, E: int):
    """Step 4: (cnt [E,2], off [2E+1], perm [A], inv [A]) int32."""
    idx = _c(idx, np.int32)
    prio = _c(prio, np.uint8)
    N, k = idx.shape
    cnt = np.zeros((E, 2), dtype=np.int32)
    off = np.zeros(2 * E + 1, dtype=np.int32)
    perm = np.full(N * k, -1, dtype=np.int32)
    inv = np.full(N * k, -1, dtype=np.int32)
    _load().oracle_queues(_p(idx), _p(prio), C.c_int(N), C.c_int(E), C.c_int(k), _p(cnt), _p(off),
                          _p(perm), _p(inv))
    return cnt, off, perm, inv


def units(cnt: np.ndarray, chunk_rows: int) -> np.ndarray:
    """Step 7: int32 [n_units,4] rows {expert, cls (0=LS,1=BE), first sorted row, rows}."""
    cnt = _c(cnt, np.int32)
    E = cnt.shape[0]
    n = _load().oracle_units(_p(cnt), C.c_int(E), C.c_int(int(chunk_rows)), None, C.c_int(0))
    u = np.zeros((n, 4), dtype=np.int32)
    if n:
        _load().oracle_units(_p(cnt), C.c_int(E), C.c_int(int(chunk_rows)), _p(u), C.c_int(n))
    return u


def expert_rows(x, w1, w3, w2, e: int, tokens: Sequence[int], want_act: bool = False):
    """FFN_e applied to x[tokens]: out [len(tokens),H] fp64 (and the activation [.,F])."""
    x, w1, w3, w2 = _c(x), _c(w1), _c(w3), _c(w2)
    dt = _dt(x)
    assert dt == _dt(w1) == _dt(w3) == _dt(w2)
    _, F, H = w1.shape
    assert x.shape[1] == H and w2.shape[1:] == (H, F) and w3.shape == w1.shape
    tok = _c(np.asarray(tokens), np.int32)
    out = np.empty((len(tok), H), dtype=np.float64)
    act = np.empty((len(tok), F), dtype=np.float64) if want_act else None
    _load().oracle_expert_rows(_p(x), _p(w1), _p(w3), _p(w2), C.c_int(dt), C.c_int(H), C.c_int(F),
                               C.c_int(int(e)), _p(tok), C.c_int(len(tok)), _p(out), _p(act))
    return (out, act) if want_act else out


def combine(O, done, inv, wt, tokens, H: int):
    """Step 6 for `tokens`: (y [len,H] fp64 with unfinished rows NaN, complete [len] bool)."""
    O = _c(O, np.float64)
    done = _c(done, np.uint8)
    inv = _c(inv, np.int32)
    wt = _c(wt, np.float64)
    tok = _c(np.asarray(tokens), np.int32)
    k = wt.shape[1]
    y = np.full((len(tok), H), np.nan, dtype=np.float64)
    comp = np.zeros(len(tok), dtype=np.uint8)
    _load().oracle_combine(_p(O), _p(done), _p(inv), _p(wt), C.c_int(k), C.c_int(H), _p(tok),
                           C.c_int(len(tok)), _p(y), _p(comp))
    return y, comp.astype(bool)


# e2m1 (sign, 2 exponent bits, 1 mantissa bit; exponent bias 1, code 0/1 subnormal): the 4-bit
# element of the open microscaling FP4 format this build reads the paper's "4-bit quantization" as
# (section "Evaluation", models and dataset).  Indexed by the low three bits; bit 3 is the sign.
_E2M1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=np.float64)


def dequant_mxfp4(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """4-bit weights -> fp64 values.  codes uint8 [..., K/2] (element with even k in the low nibble),
    scales uint8 [..., K/32] (e8m0: 2^(byte-127), one per 32 consecutive elements).  Returns [..., K]."""
    codes, scales = _c(codes, np.uint8), _c(scales, np.uint8)
    K = codes.shape[-1] * 2
    assert scales.shape[-1] * 32 == K and codes.shape[:-1] == scales.shape[:-1]
    nib = np.empty(codes.shape[:-1] + (K,), dtype=np.uint8)
    nib[..., 0::2] = codes & 0x0F
    nib[..., 1::2] = codes >> 4
    val = _E2M1[nib & 7] * np.where(nib & 8, -1.0, 1.0)
    scale = np.ldexp(1.0, scales.astype(np.int64) - 127)
    return val * np.repeat(scale, 32, axis=-1)


def mxfp4_weights_as_bf16(w: dict) -> dict:
    """The weights dict of the layer functions (bf16 bit patterns) for 4-bit weights: every
    element * scale is exactly representable in bf16, which is asserted."""
    out = {"Wg": w["Wg"]}
    for n in ("W1", "W3", "W2"):
        codes, scales = w[n + "q"], w[n + "s"]
        dst = np.empty(codes.shape[:-1] + (codes.shape[-1] * 2,), dtype=np.uint16)
        for e in range(codes.shape[0]):          # expert by expert: the fp64 temporaries stay small
            bits = dequant_mxfp4(codes[e], scales[e]).astype(np.float32).view(np.uint32)
            assert not (bits & 0xFFFF).any()
            dst[e] = (bits >> 16).astype(np.uint16)
        out[n] = dst
    return out


class OracleLayer:
    """One layer-batch walked unit by unit: the state a preempted job keeps (expert
    assignment, routing weights, queue order, finished expert rows) and nothing else."""

    def __init__(self, x, w, prio, bias, k: int, chunk_rows: int, logits: Optional[np.ndarray] = None):
        self.x, self.w, self.prio = x, w, _c(prio, np.uint8)
        self.N, self.H = x.shape
        self.E = w["Wg"].shape[1]
        self.k = k
        self.L = gate_logits(x, w["Wg"], bias) if logits is None else _c(logits, np.float64)
        self.idx, self.wt = topk(self.L, k)
        self.cnt, self.off, self.perm, self.inv = queues(self.idx, self.prio, self.E)
        self.units = units(self.cnt, chunk_rows)
        self.next_unit = 0
        self.O: Optional[np.ndarray] = None
        self.keep_act = False                     # set before running to also keep the activations (self.act [A,F])
        self.act: Optional[np.ndarray] = None
        self.done = np.zeros(self.N * k, dtype=np.uint8)
        self.executed = np.zeros(len(self.units), dtype=np.int32)

    @property
    def n_units(self) -> int:
        return len(self.units)

    def _execute(self, u: int) -> None:
        if self.O is None:
            self.O = np.full((self.N * self.k, self.H), np.nan, dtype=np.float64)
        e, _cls, r0, rows = (int(v) for v in self.units[u])
        toks = self.perm[r0:r0 + rows] // self.k
        if self.keep_act:
            if self.act is None:
                self.act = np.full((self.N * self.k, self.w["W1"].shape[1]), np.nan, dtype=np.float64)
            self.O[r0:r0 + rows], self.act[r0:r0 + rows] = expert_rows(self.x, self.w["W1"], self.w["W3"], self.w["W2"],
                                                                         e, toks, want_act=True)
        else:
            self.O[r0:r0 + rows] = expert_rows(self.x, self.w["W1"], self.w["W3"], self.w["W2"], e, toks)
        self.done[r0:r0 + rows] = 1
        self.executed[u] += 1

    def _advance(self) -> None:
        while self.next_unit < self.n_units and self.executed[self.next_unit]:
            self.next_unit += 1

    def run(self, max_units: Optional[int] = None, rows_filter=None) -> bool:
        """Execute the next max_units units that have not run yet, in list order, from the cursor
        (the first unit that has not run).  Returns True when all are done."""
        if self.O is None:
            self.O = np.full((self.N * self.k, self.H), np.nan, dtype=np.float64)
        budget = self.n_units if max_units is None else max_units
        u = self.next_unit
        while u < self.n_units and budget > 0:
            if not self.executed[u]:
                self._execute(u)
                budget -= 1
            u += 1
        self._advance()
        return self.next_unit == self.n_units

    def run_units(self, ids) -> bool:
        """Execute the listed units in the given order (a policy's choice: any units that have not
        run yet).  The paper lets user-defined policies pick which experts run (sections "Challenges
        and Design Decisions" and "System Architecture"); a token counts as complete only once all k
        of its assignments have run ("Top-k expert selection" in the former section)."""
        for u in ids:
            assert 0 <= u < self.n_units and not self.executed[u]
            self._execute(int(u))
        self._advance()
        return self.next_unit == self.n_units

    def y(self, tokens=None):
        toks = np.arange(self.N) if tokens is None else np.asarray(tokens)
        if self.O is None:
            self.O = np.full((self.N * self.k, self.H), np.nan, dtype=np.float64)
        return combine(self.O, self.done, self.inv, self.wt, toks, self.H)

    def y_tokens_direct(self, tokens) -> np.ndarray:
        """y for a sample of tokens computed one by one (no unit walk): used at full sizes."""
        toks = np.asarray(tokens)
        out = np.zeros((len(toks), self.H), dtype=np.float64)
        for e in range(self.E):
            for j in range(self.k):
                sel = np.nonzero(self.idx[toks, j] == e)[0]
                if len(sel) == 0:
                    continue
                o = expert_rows(self.x, self.w["W1"], self.w["W3"], self.w["W2"], e, toks[sel])
                out[sel] += self.wt[toks[sel], j][:, None] * o
        return out
