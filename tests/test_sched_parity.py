"""The C++ scheduler (include/qsched.h) against the scheduler oracle on seeded random traces of
dispatcher and batch-engine calls, plus its error behaviour.  Host code only: runs without a GPU."""
from __future__ import annotations

import ctypes as C

import numpy as np
import pytest

import paper_2503_09304_amd as q
from oracle.sched_oracle import SchedOracle


def both_next(cs, orc):
    got, want = cs.next_batch(), orc.next_batch()
    assert got == (None if want is None else (list(want[0]), want[1], want[2]))
    return want


@pytest.mark.parametrize("seed,batch_size,p_ls", [(11, 1, 0.2), (12, 4, 0.2), (13, 32, 0.2), (14, 5, 0.7), (15, 3, 0.0),
                                                   (16, 8, 1.0)])
def test_trace_matches_oracle(seed, batch_size, p_ls):
    rng = np.random.default_rng(seed)
    cs, orc = q.Scheduler(batch_size), SchedOracle(batch_size)
    left, running = {}, []            # tokens to go per job; batches in flight (a parked one may sit below the top)
    next_id, n_batches = 0, 0
    for step in range(4000):
        r = rng.random()
        if r < 0.30 and next_id < 600:
            cls = q.SCHED_LS if rng.random() < p_ls else q.SCHED_BE
            cs.submit(next_id, cls); orc.submit(next_id, cls)
            left[next_id] = int(rng.integers(1, 7))
            next_id += 1
        elif r < 0.65 and len(running) < 2:
            # the engine asks for a batch: when idle, or at a preemption point of a BE-only batch
            if running:
                n_ls = running[-1][1]
                assert cs.preempt_wanted(n_ls) == orc.preempt_wanted(n_ls)
                if not orc.preempt_wanted(n_ls):
                    continue
            want = both_next(cs, orc)
            if want is not None:
                running.append((list(want[0]), want[2]))
                n_batches += 1
        elif running:
            jobs, _ = running.pop()    # the innermost batch finishes its iteration
            for j in jobs:
                left[j] -= 1
                cs.token(j, left[j] == 0); orc.token(j, left[j] == 0)
        for qi in range(4):
            assert cs.queue_len(qi) == orc.queue_len(qi)
        assert cs.running() == len(orc.running)
    assert n_batches > 100


def test_error_behaviour():
    L = q.lib()
    assert not L.sched_create(0) and b"batch_size" in L.sched_last_error()
    s = q.Scheduler(2)
    s.submit(7, q.SCHED_LS)
    with pytest.raises(q.SchedError) as e:
        s.submit(7, q.SCHED_BE)                      # id already live
    assert e.value.code == q.SCHED_E_JOB
    with pytest.raises(q.SchedError) as e:
        s.submit(8, 5)                               # unknown class
    assert e.value.code == q.SCHED_E_ARG
    with pytest.raises(q.SchedError) as e:
        s.token(7, False)                            # queued, not running
    assert e.value.code == q.SCHED_E_JOB
    with pytest.raises(q.SchedError) as e:
        s.token(99, False)                           # unknown
    assert e.value.code == q.SCHED_E_JOB
    ids = (C.c_uint64 * 1)()
    b = q.SchedBatch()
    assert L.sched_next_batch(s.h, ids, 1, C.byref(b)) == q.SCHED_E_ARG     # capacity below the batch size
    assert L.sched_next_batch(s.h, None, 2, C.byref(b)) == q.SCHED_E_ARG
    assert s.queue_len(q.SCHED_Q_LS_PREFILL) == 1 and s.queue_len(9) == 0   # nothing was consumed by the failures
    assert s.next_batch() == ([7], q.SCHED_PREFILL, 1)
    s.token(7, True)
    s.submit(7, q.SCHED_BE)                          # a finished id may come back
    assert s.next_batch() == ([7], q.SCHED_PREFILL, 0)
    assert s.next_batch() is None
    assert s.running() == 1


def replay_fixture(path, make):
    """Run a tests/golden scheduler script against a scheduler object with the oracle's method names."""
    s = None
    for raw in open(path):
        line = raw.split("#")[0].strip()
        if not line:
            continue
        f = line.split()
        if f[0] == "batch_size":
            s = make(int(f[1]))
        elif f[0] == "submit":
            s.submit(int(f[1]), q.SCHED_LS if f[2] == "LS" else q.SCHED_BE)
        elif f[0] == "token":
            s.token(int(f[1]), f[2] == "last")
        elif f[0] == "preempt?":
            assert s.preempt_wanted(int(f[1])) == (f[2] == "yes"), line
        elif f[0] == "batch":
            stage = q.SCHED_PREFILL if f[1] == "PREFILL" else q.SCHED_DECODE
            got = s.next_batch()
            assert got is not None and (list(got[0]), got[1], got[2]) == ([int(v) for v in f[4:]], stage, int(f[2])), line
        elif f[0] == "none":
            assert s.next_batch() is None
        else:
            raise ValueError(line)


def test_paper_example_sequence_on_both_schedulers():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "fig_architecture_example.txt")
    replay_fixture(path, SchedOracle)
    replay_fixture(path, q.Scheduler)
