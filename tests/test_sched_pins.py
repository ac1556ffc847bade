"""Pins of the scheduler oracle (CPU only): what the paper's batch-selection algorithm and its
prose description fix, written down by hand, plus invariants and an exhaustive sweep of small
queue states against the closed form of the batch composition."""
from __future__ import annotations

import itertools

import numpy as np
import pytest

from oracle.sched_oracle import BE, DECODE, LS, PREFILL, SchedOracle


def make(batch_size, ls_prefill=(), be_prefill=(), ls_decode=(), be_decode=()):
    """A scheduler whose queues hold the given job ids (decode jobs got there through a prefill)."""
    s = SchedOracle(10 ** 6)             # one batch takes them all through their prefill
    for j in ls_decode:
        s.submit(j, LS)
    for j in be_decode:
        s.submit(j, BE)
    if ls_decode or be_decode:
        jobs, stage, n_ls = s.next_batch()
        assert jobs == list(ls_decode) + list(be_decode) and stage == PREFILL and n_ls == len(ls_decode)
        for j in jobs:
            s.token(j, False)
    s.batch_size = batch_size
    for j in ls_prefill:
        s.submit(j, LS)
    for j in be_prefill:
        s.submit(j, BE)
    assert s.ls_prefill == list(ls_prefill) and s.be_prefill == list(be_prefill)
    assert s.ls_decode == list(ls_decode) and s.be_decode == list(be_decode)
    return s


# ---- the five branches, expected batches written out by hand (Algorithm 1 and the paragraph
# "Batch selection logic") ----

def test_branch_full_ls_decode_batch_wins_over_everything():
    s = make(2, ls_prefill=[10], be_prefill=[20], ls_decode=[1, 2, 3], be_decode=[30])
    assert s.next_batch() == ([1, 2], DECODE, 2)
    assert s.ls_decode == [3] and s.ls_prefill == [10] and s.be_decode == [30] and s.be_prefill == [20]


def test_branch_ls_prefill_before_a_partial_ls_decode_batch_and_filled_with_be_prefill():
    s = make(4, ls_prefill=[10, 11], be_prefill=[20, 21, 22], ls_decode=[1, 2, 3], be_decode=[30])
    # 3 LS decode jobs do not fill a batch of 4: LS prompts are prefilled first, BE prompts fill up
    assert s.next_batch() == ([10, 11, 20, 21], PREFILL, 2)
    assert s.be_prefill == [22] and s.ls_decode == [1, 2, 3] and s.be_decode == [30]


def test_branch_ls_prefill_alone_when_no_be_prompt_waits():
    s = make(4, ls_prefill=[10], be_decode=[30, 31])
    assert s.next_batch() == ([10], PREFILL, 1)      # never filled from the decode queue
    assert s.be_decode == [30, 31]


def test_branch_ls_prefill_larger_than_batch():
    s = make(2, ls_prefill=[10, 11, 12], be_prefill=[20])
    assert s.next_batch() == ([10, 11], PREFILL, 2)
    assert s.ls_prefill == [12] and s.be_prefill == [20]


def test_branch_partial_ls_decode_filled_with_be_decode():
    s = make(4, be_prefill=[20], ls_decode=[1, 2], be_decode=[30, 31, 32])
    assert s.next_batch() == ([1, 2, 30, 31], DECODE, 2)
    assert s.be_decode == [32] and s.be_prefill == [20]   # never filled from the prefill queue


def test_branch_be_decode_before_be_prefill():
    s = make(2, be_prefill=[20, 21], be_decode=[30, 31, 32])
    assert s.next_batch() == ([30, 31], DECODE, 0)
    assert s.next_batch() == ([32], DECODE, 0)             # a BE decode batch is not filled with prompts
    assert s.next_batch() == ([20, 21], PREFILL, 0)
    assert s.next_batch() is None


def test_nothing_to_do():
    assert SchedOracle(3).next_batch() is None


def test_threshold_is_at_least_batch_size():
    # exactly BatchSize LS decode jobs already take the first branch, although an LS prompt waits
    s = make(3, ls_prefill=[10], ls_decode=[1, 2, 3])
    assert s.next_batch() == ([1, 2, 3], DECODE, 3)
    s = make(3, ls_prefill=[10], ls_decode=[1, 2])
    assert s.next_batch() == ([10], PREFILL, 1)


# ---- the example of the architecture figure: four BE jobs decode, an LS job arrives ----

def test_figure_example_sequence():
    s = SchedOracle(8)
    for j in (1, 2, 3, 4):
        s.submit(j, BE)
    assert s.next_batch() == ([1, 2, 3, 4], PREFILL, 0)
    for j in (1, 2, 3, 4):
        s.token(j, False)
    assert s.next_batch() == ([1, 2, 3, 4], DECODE, 0)     # the BE batch is in flight ...
    s.submit(9, LS)                                        # ... when the LS job arrives
    assert s.preempt_wanted(0)                             # the engine is told to stop the BE batch
    assert s.next_batch() == ([9], PREFILL, 1)             # LS prefill runs first
    assert not s.preempt_wanted(1)                         # a batch with LS jobs is never stopped
    s.token(9, False)
    assert not s.preempt_wanted(0)
    for j in (1, 2, 3, 4):                                 # the BE iteration resumes and ends
        s.token(j, False)
    assert s.next_batch() == ([9, 1, 2, 3, 4], DECODE, 1)  # LS and BE jobs merged, LS first
    s.token(9, True)
    for j in (1, 2, 3, 4):
        s.token(j, True)
    assert s.next_batch() is None and not s.cls


# ---- exhaustive sweep of small states against the closed form of the composition ----

def closed_form(B, lsp, bep, lsd, bed):
    """(stage, LS decode, LS prefill, BE decode, BE prefill) job counts of the next batch."""
    if lsd >= B:
        return DECODE, B, 0, 0, 0
    if lsp > 0:
        a = min(lsp, B)
        return PREFILL, 0, a, 0, min(bep, B - a)
    if lsd > 0:
        return DECODE, lsd, 0, min(bed, B - lsd), 0
    if bed > 0:
        return DECODE, 0, 0, min(bed, B), 0
    if bep > 0:
        return PREFILL, 0, 0, 0, min(bep, B)
    return None


@pytest.mark.parametrize("B", [1, 2, 3])
def test_all_small_states(B):
    for lsp, bep, lsd, bed in itertools.product(range(4), repeat=4):
        q = dict(ls_prefill=list(range(100, 100 + lsp)), be_prefill=list(range(200, 200 + bep)),
                 ls_decode=list(range(300, 300 + lsd)), be_decode=list(range(400, 400 + bed)))
        s = make(B, **q)
        got = s.next_batch()
        want = closed_form(B, lsp, bep, lsd, bed)
        if want is None:
            assert got is None
            continue
        stage, n_lsd, n_lsp, n_bed, n_bep = want
        expect = q["ls_decode"][:n_lsd] + q["ls_prefill"][:n_lsp] + q["be_decode"][:n_bed] + q["be_prefill"][:n_bep]
        assert got == (expect, stage, n_lsd + n_lsp), (B, lsp, bep, lsd, bed)
        assert 1 <= len(got[0]) <= B
        # what was not taken is still queued, in order
        assert s.ls_decode == q["ls_decode"][n_lsd:] and s.ls_prefill == q["ls_prefill"][n_lsp:]
        assert s.be_decode == q["be_decode"][n_bed:] and s.be_prefill == q["be_prefill"][n_bep:]


# ---- invariants over random traces ----

@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_trace_invariants(seed):
    rng = np.random.default_rng(seed)
    B = int(rng.integers(1, 6))
    s = SchedOracle(B)
    left: dict[int, int] = {}            # tokens each live job still has to produce
    cls: dict[int, int] = {}
    stage_of: dict[int, int] = {}        # PREFILL until the first token
    order = {(c, st): [] for c in (LS, BE) for st in (PREFILL, DECODE)}   # enqueue order per queue
    served = {(c, st): [] for c in (LS, BE) for st in (PREFILL, DECODE)}
    next_id, finished = 0, 0
    for _ in range(600):
        if rng.random() < 0.45 and next_id < 150:
            c = LS if rng.random() < 0.3 else BE
            s.submit(next_id, c)
            left[next_id], cls[next_id], stage_of[next_id] = int(rng.integers(1, 5)), c, PREFILL
            order[(c, PREFILL)].append(next_id)
            next_id += 1
            continue
        got = s.next_batch()
        queued = len(s.ls_prefill) + len(s.be_prefill) + len(s.ls_decode) + len(s.be_decode)
        if got is None:
            assert queued == 0 and not s.running
            continue
        jobs, stage, n_ls = got
        assert 1 <= len(jobs) <= B and len(set(jobs)) == len(jobs)
        assert all(stage_of[j] == stage for j in jobs)                    # one stage per batch
        assert [cls[j] for j in jobs] == [LS] * n_ls + [BE] * (len(jobs) - n_ls)   # LS first
        for j in jobs:
            served[(cls[j], stage)].append(j)
        for j in jobs:                                                    # the iteration ends
            left[j] -= 1
            fin = left[j] == 0
            s.token(j, fin)
            if fin:
                finished += 1
            else:
                stage_of[j] = DECODE
                order[(cls[j], DECODE)].append(j)
    while (got := s.next_batch()) is not None:                            # drain
        for j in got[0]:
            served[(cls[j], got[1])].append(j)
            left[j] -= 1
            s.token(j, left[j] == 0)
            if left[j]:
                order[(cls[j], DECODE)].append(j)
            else:
                finished += 1
    assert finished == next_id and not s.cls and not s.running           # every job completes once
    for key in order:
        assert served[key] == order[key]                                  # each queue is FCFS


def test_synthetic_request_stream_recipe():
    import workloads as wl
    a = wl.make_jobs(4000, rate_per_s=80.0, p_ls=0.2, seed=5, max_prompt=512, max_out=32)
    b = wl.make_jobs(4000, rate_per_s=80.0, p_ls=0.2, seed=5, max_prompt=512, max_out=32)
    for k in a:
        assert np.array_equal(a[k], b[k])                               # seeded
    assert np.all(np.diff(a["arrival_s"]) > 0)
    assert abs(4000 / a["arrival_s"][-1] - 80.0) < 5.0                   # Poisson arrivals at the stated rate
    gaps = np.diff(a["arrival_s"])
    assert abs(gaps.std() / gaps.mean() - 1.0) < 0.1                     # exponential gaps: cv = 1
    assert abs(a["is_ls"].mean() - 0.2) < 0.03                           # a fifth of the prompts marked LS
    assert a["prompt_len"].min() >= 16 and a["prompt_len"].max() <= 512
    assert a["out_len"].min() >= 4 and a["out_len"].max() <= 32
    c = wl.make_jobs(4000, rate_per_s=80.0, p_ls=0.2, seed=6)
    assert not np.array_equal(a["prompt_len"], c["prompt_len"])
