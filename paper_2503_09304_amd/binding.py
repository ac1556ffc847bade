"""ctypes binding of libqmoe.so: the same calls as include/qmoe.h, argument marshalling only.

Device memory and streams come from PyTorch (torch tensors' data_ptr(), the current stream's
handle); nothing is computed here."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
# QMOE_LIB overrides the library file (to try an experimental build); the default is the in-tree one.
_LIB_PATH = os.environ.get("QMOE_LIB") or os.path.join(_HERE, "libqmoe.so")

MOE_F32, MOE_BF16 = 0, 1
MOE_OK, MOE_DONE = 0, 1
MOE_E_ARG, MOE_E_STATE, MOE_E_INCOMPLETE, MOE_E_WORKSPACE, MOE_E_HIP = -1, -2, -3, -4, -5
MOE_CLASS_LS, MOE_CLASS_BE, MOE_CLASS_ALL = 1, 2, 3
MOE_Y_F32 = 4
MOE_W_ROWMAJOR, MOE_W_PACKED, MOE_W_MXFP4_ROWMAJOR, MOE_W_MXFP4 = 0, 1, 2, 3
UINT32_MAX = 0xFFFFFFFF

GET = {"logits": 0, "topk_idx": 1, "topk_w": 2, "counts": 3, "offsets": 4, "perm": 5, "inv": 6,
       "expert_out": 7, "act": 8, "units": 9}


class MoeConfig(C.Structure):
    _fields_ = [("E", C.c_int32), ("k", C.c_int32), ("H", C.c_int32), ("F", C.c_int32),
                ("dtype", C.c_int32), ("chunk_rows", C.c_int32), ("max_tokens", C.c_int32),
                ("down_ksplit", C.c_int32)]


class MoeWeights(C.Structure):
    _fields_ = [("Wg", C.c_void_p), ("W1", C.c_void_p), ("W3", C.c_void_p), ("W2", C.c_void_p),
                ("layout", C.c_int32), ("S1", C.c_void_p), ("S3", C.c_void_p), ("S2", C.c_void_p)]


class MoeCursor(C.Structure):
    _fields_ = [("next_unit", C.c_uint32), ("n_units", C.c_uint32)]


class MoeUnit(C.Structure):
    _fields_ = [("expert", C.c_int32), ("cls", C.c_int32), ("row0", C.c_int32), ("rows", C.c_int32)]


class MoeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"qmoe error {code}: {msg}")
        self.code = code


class SchedBatch(C.Structure):
    _fields_ = [("n", C.c_uint32), ("n_ls", C.c_uint32), ("stage", C.c_int32)]


SCHED_OK, SCHED_NONE, SCHED_E_ARG, SCHED_E_JOB = 0, 1, -1, -2
SCHED_BE, SCHED_LS = 0, 1
SCHED_PREFILL, SCHED_DECODE = 0, 1
SCHED_Q_LS_PREFILL, SCHED_Q_BE_PREFILL, SCHED_Q_LS_DECODE, SCHED_Q_BE_DECODE = 0, 1, 2, 3

_lib = None


def moe_route_noalloc(cfg: "MoeConfig", x, n_tokens: int, Wg, bias, logits, topk_idx, topk_w) -> int:
    """The router without context, workspace or allocation (see include/qmoe.h); tensors or raw addresses."""
    rc = lib().moe_route_noalloc(C.byref(cfg), _ptr(x), n_tokens, _ptr(Wg), _ptr(bias), _ptr(logits), _ptr(topk_idx),
                                 _ptr(topk_w), _stream())
    return _check(rc)


def moe_probe_mfma(a, b, iters: int, workgroups: int, sink) -> int:
    """The register-only MFMA loop (a profiling yardstick, see include/qmoe.h)."""
    return _check(lib().moe_probe_mfma(_ptr(a), _ptr(b), iters, workgroups, _ptr(sink), _stream()))


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded library.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2503_09304_amd.build`")
        L = C.CDLL(_LIB_PATH)
        L.moe_last_error.restype = C.c_char_p
        L.moe_workspace_bytes.restype = C.c_size_t
        L.moe_workspace_bytes.argtypes = [C.POINTER(MoeConfig)]
        L.moe_create.argtypes = [C.POINTER(MoeConfig), C.c_void_p, C.c_size_t, C.POINTER(C.c_void_p)]
        L.moe_destroy.argtypes = [C.c_void_p]
        L.moe_probe_mfma.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.moe_route_noalloc.argtypes = [C.POINTER(MoeConfig), C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_void_p]
        L.moe_route.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(MoeWeights), C.c_void_p, C.c_void_p]
        L.moe_permute.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(MoeCursor), C.c_void_p]
        L.moe_expert_run.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(MoeWeights), C.c_uint32,
                                     C.POINTER(MoeCursor), C.c_void_p]
        L.moe_combine.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        L.moe_expert_run_units.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(MoeWeights), C.POINTER(C.c_uint32),
                                           C.c_uint32, C.POINTER(MoeCursor), C.c_void_p]
        L.moe_combine_complete.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.moe_expert_enqueue.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(MoeWeights), C.c_uint32, C.c_void_p]
        L.moe_expert_stop.argtypes = [C.c_void_p]
        L.moe_expert_collect.argtypes = [C.c_void_p, C.POINTER(MoeCursor), C.c_void_p]
        L.moe_get.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_void_p), C.POINTER(C.c_size_t)]
        L.moe_units.argtypes = [C.c_void_p, C.POINTER(MoeUnit), C.c_uint32, C.POINTER(C.c_uint32)]
        L.moe_plan_units.argtypes = [C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.POINTER(MoeUnit), C.c_uint32,
                                     C.POINTER(C.c_uint32)]
        L.moe_pack_weights.argtypes = [C.POINTER(MoeConfig), C.POINTER(MoeWeights), C.POINTER(MoeWeights), C.c_void_p]
        L.moe_profile.argtypes = [C.c_void_p, C.c_int32]
        L.moe_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_uint32)]
        for f in ("moe_expert_enqueue", "moe_expert_stop", "moe_expert_collect", "moe_expert_run_units", "moe_combine_complete", "moe_pack_weights", "moe_profile", "moe_profile_read", "moe_create", "moe_destroy", "moe_route", "moe_permute", "moe_expert_run", "moe_combine",
                  "moe_get", "moe_units", "moe_plan_units"):
            getattr(L, f).restype = C.c_int32
        # include/qsched.h
        L.sched_create.restype = C.c_void_p
        L.sched_create.argtypes = [C.c_uint32]
        L.sched_destroy.restype = None
        L.sched_destroy.argtypes = [C.c_void_p]
        L.sched_submit.argtypes = [C.c_void_p, C.c_uint64, C.c_int32]
        L.sched_token.argtypes = [C.c_void_p, C.c_uint64, C.c_int32]
        L.sched_next_batch.argtypes = [C.c_void_p, C.POINTER(C.c_uint64), C.c_uint32, C.POINTER(SchedBatch)]
        L.sched_preempt_wanted.argtypes = [C.c_void_p, C.POINTER(SchedBatch)]
        L.sched_queue_len.restype = C.c_uint32
        L.sched_queue_len.argtypes = [C.c_void_p, C.c_int32]
        L.sched_running.restype = C.c_uint32
        L.sched_running.argtypes = [C.c_void_p]
        L.sched_last_error.restype = C.c_char_p
        for f in ("sched_submit", "sched_token", "sched_next_batch", "sched_preempt_wanted"):
            getattr(L, f).restype = C.c_int32
        _lib = L
    return _lib


def moe_last_error() -> str:
    return lib().moe_last_error().decode()


def _check(rc: int) -> int:
    if rc < 0:
        raise MoeError(rc, moe_last_error())
    return rc


def moe_workspace_bytes(cfg: MoeConfig) -> int:
    n = int(lib().moe_workspace_bytes(C.byref(cfg)))
    if n == 0:
        raise MoeError(MOE_E_ARG, moe_last_error())
    return n


def moe_plan_units(cnt, E: int, chunk_rows: int):
    """Host-only: the work-unit list for queue lengths cnt [E][2] (column 0 = LS)."""
    flat = [int(v) for row in cnt for v in row]
    arr = (C.c_int32 * len(flat))(*flat)
    n = C.c_uint32(0)
    _check(lib().moe_plan_units(arr, E, chunk_rows, None, 0, C.byref(n)))
    out = (MoeUnit * max(1, n.value))()
    _check(lib().moe_plan_units(arr, E, chunk_rows, out, n.value, C.byref(n)))
    return [(u.expert, u.cls, u.row0, u.rows) for u in out[: n.value]]


def moe_pack_weights(cfg: MoeConfig, src: MoeWeights, dst: MoeWeights) -> MoeWeights:
    """Re-layout row-major weights into dst's buffers (MOE_W_PACKED); returns dst."""
    _check(lib().moe_pack_weights(C.byref(cfg), C.byref(src), C.byref(dst), _stream()))
    return dst


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream() -> int:
    import torch
    return int(torch.cuda.current_stream().cuda_stream)


class Context:
    """One in-flight layer-batch: the opaque moe_ctx plus the torch tensor that backs its workspace.
    Methods are the C calls with tensors in place of pointers.  The stream of every call is PyTorch's
    current stream, looked up at each call, unless `stream_handle` holds a hipStream_t value (an int):
    a caller that stays on one stream sets it once and saves the lookup (a few microseconds per call)."""

    stream_handle = None

    def _stream(self) -> int:
        return _stream() if self.stream_handle is None else self.stream_handle

    def __init__(self, E, k, H, F, dtype, chunk_rows, max_tokens, device="cuda:0", down_ksplit=0):
        import torch
        self.cfg = MoeConfig(E, k, H, F, dtype, chunk_rows, max_tokens, down_ksplit)
        self.nbytes = moe_workspace_bytes(self.cfg)
        self.ws = torch.empty(self.nbytes, dtype=torch.uint8, device=device)
        assert self.ws.data_ptr() % 256 == 0
        h = C.c_void_p()
        _check(lib().moe_create(C.byref(self.cfg), self.ws.data_ptr(), self.nbytes, C.byref(h)))
        self.h = h
        self.cursor = MoeCursor(0, 0)
        self.N = 0
        self._w = None

    def close(self):
        """Destroys the context.  If a launch sequence is still enqueued (moe_destroy refuses then: its
        kernels use the context's pinned buffer) it is collected first, which waits for the stream."""
        if getattr(self, "h", None):
            if lib().moe_destroy(self.h) == MOE_E_STATE:
                cur = MoeCursor(0, 0)
                lib().moe_expert_collect(self.h, C.byref(cur), self._stream())
                lib().moe_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @staticmethod
    def weights(Wg, W1, W3, W2, layout: int = MOE_W_ROWMAJOR, S1=None, S3=None, S2=None) -> MoeWeights:
        return MoeWeights(_ptr(Wg), _ptr(W1), _ptr(W3), _ptr(W2), layout, _ptr(S1), _ptr(S3), _ptr(S2))

    def route(self, x, w: MoeWeights, bias=None, n_tokens=None):
        n = x.shape[0] if n_tokens is None else n_tokens
        rc = _check(lib().moe_route(self.h, _ptr(x), n, C.byref(w), _ptr(bias), self._stream()))
        self.N, self._w = n, w
        return rc

    def permute(self, prio) -> MoeCursor:
        if prio is not None and prio.element_size() != 1:
            raise TypeError("prio must be a uint8 tensor (one byte per token)")
        _check(lib().moe_permute(self.h, _ptr(prio), C.byref(self.cursor), self._stream()))
        return self.cursor

    def expert_run(self, x, w: MoeWeights, max_units: int = UINT32_MAX, cursor: Optional[MoeCursor] = None) -> int:
        cur = self.cursor if cursor is None else cursor
        return _check(lib().moe_expert_run(self.h, _ptr(x), C.byref(w), max_units, C.byref(cur), self._stream()))

    def combine(self, y, class_mask: int = MOE_CLASS_ALL) -> int:
        return _check(lib().moe_combine(self.h, _ptr(y), class_mask, self._stream()))

    def expert_run_units(self, x, w: MoeWeights, unit_ids) -> int:
        """Execute the listed units (indices into units()) in the given order; updates self.cursor."""
        ids = [int(u) for u in unit_ids]
        arr = (C.c_uint32 * max(1, len(ids)))(*ids)
        return _check(lib().moe_expert_run_units(self.h, _ptr(x), C.byref(w), arr, len(ids), C.byref(self.cursor),
                                                 self._stream()))

    def expert_enqueue(self, x, w: MoeWeights, units_per_launch: int = 4) -> int:
        """Put all remaining units on the stream as gated launches; returns without waiting."""
        return _check(lib().moe_expert_enqueue(self.h, _ptr(x), C.byref(w), units_per_launch, self._stream()))

    def expert_stop(self) -> None:
        """Ask the enqueued sequence to stop: workgroups that start after the store is visible do no work,
        so units are left whole (executed or not), also inside a launch."""
        _check(lib().moe_expert_stop(self.h))

    def expert_collect(self) -> int:
        """Wait for the stream and book what ran; updates self.cursor.  MOE_DONE when every unit has run."""
        return _check(lib().moe_expert_collect(self.h, C.byref(self.cursor), self._stream()))

    def combine_complete(self, y, complete=None) -> int:
        """Write the rows of y of every token whose k assignments have all been executed; `complete`
        (uint8 tensor [N], optional) receives the mask."""
        if complete is not None and complete.element_size() != 1:
            raise TypeError("complete must be a uint8 tensor")
        return _check(lib().moe_combine_complete(self.h, _ptr(y), _ptr(complete), self._stream()))

    def profile(self, kinds) -> None:
        """Bracket the expert kernels of the given kinds with events: True = all, False = none, or an
        iterable of names out of gate_up, down, down_reduce."""
        if kinds is True:
            mask = 7
        elif not kinds:
            mask = 0
        else:
            mask = sum(1 << ("gate_up", "down", "down_reduce").index(k) for k in kinds)
        _check(lib().moe_profile(self.h, mask))

    def profile_read(self):
        """{kind: (total ms, launches)} of the expert kernels since the last read."""
        ms = (C.c_float * 3)()
        n = (C.c_uint32 * 3)()
        _check(lib().moe_profile_read(self.h, ms, n))
        return {name: (float(ms[i]), int(n[i])) for i, name in enumerate(("gate_up", "down", "down_reduce"))}

    def units(self):
        n = C.c_uint32(0)
        _check(lib().moe_units(self.h, None, 0, C.byref(n)))
        out = (MoeUnit * max(1, n.value))()
        _check(lib().moe_units(self.h, out, n.value, C.byref(n)))
        return [(u.expert, u.cls, u.row0, u.rows) for u in out[: n.value]]

    def get(self, what: str):
        """A tensor view (no copy) of one workspace region of the current layer-batch."""
        import torch
        p, nb = C.c_void_p(), C.c_size_t()
        _check(lib().moe_get(self.h, GET[what], C.byref(p), C.byref(nb)))
        off = (p.value or 0) - self.ws.data_ptr()
        raw = self.ws[off: off + nb.value]
        N, k, E, H, F = self.N, self.cfg.k, self.cfg.E, self.cfg.H, self.cfg.F
        act_dt = torch.bfloat16 if self.cfg.dtype == MOE_BF16 else torch.float32
        if what == "logits":
            return raw.view(torch.float32).view(N, E)
        if what == "topk_idx":
            return raw.view(torch.int32).view(N, k)
        if what == "topk_w":
            return raw.view(torch.float32).view(N, k)
        if what == "counts":
            return raw.view(torch.int32).view(E, 2)
        if what in ("offsets", "perm", "inv"):
            return raw.view(torch.int32)
        if what == "expert_out":
            return raw.view(torch.float32).view(N * k, H)
        if what == "act":
            return raw.view(act_dt).view(N * k, F)
        if what == "units":
            return raw.view(torch.int32).view(-1, 4)
        raise KeyError(what)


class SchedError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"qsched error {code}: {msg}")
        self.code = code


class Scheduler:
    """The opaque sched object of include/qsched.h; methods are the C calls."""

    def __init__(self, batch_size: int):
        self.batch_size = batch_size
        self.h = lib().sched_create(batch_size)
        if not self.h:
            raise SchedError(SCHED_E_ARG, lib().sched_last_error().decode())
        self._ids = (C.c_uint64 * batch_size)()

    def close(self):
        if getattr(self, "h", None):
            lib().sched_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @staticmethod
    def _check(rc: int) -> int:
        if rc < 0:
            raise SchedError(rc, lib().sched_last_error().decode())
        return rc

    def submit(self, job: int, cls: int) -> None:
        self._check(lib().sched_submit(self.h, job, cls))

    def token(self, job: int, finished: bool) -> None:
        self._check(lib().sched_token(self.h, job, 1 if finished else 0))

    def next_batch(self):
        """(job ids, stage, number of LS jobs), or None when every queue is empty."""
        b = SchedBatch()
        rc = self._check(lib().sched_next_batch(self.h, self._ids, self.batch_size, C.byref(b)))
        if rc == SCHED_NONE:
            return None
        return [int(self._ids[i]) for i in range(b.n)], int(b.stage), int(b.n_ls)

    def preempt_wanted(self, running_n_ls: int) -> bool:
        b = SchedBatch(0, running_n_ls, 0)
        return self._check(lib().sched_preempt_wanted(self.h, C.byref(b))) == 1

    def queue_len(self, q: int) -> int:
        return int(lib().sched_queue_len(self.h, q))

    def running(self) -> int:
        return int(lib().sched_running(self.h))
