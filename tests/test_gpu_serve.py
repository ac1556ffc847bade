"""The serving loop (scheduler + layer stack) on the GPU: every job completes, the scheduler calls
replay exactly through the scheduler oracle, every job's hidden states are bit-identical under the
preemptive policy and under the run-to-completion baseline, and an LS prompt that arrives behind a
long best-effort batch gets its first token far earlier when the batch can be preempted."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import paper_2503_09304_amd as q
import workloads as wl
from oracle.sched_oracle import SchedOracle
from paper_2503_09304_amd import serve
import serve_glue

pytestmark = pytest.mark.gpu

E, K, H, F, LAYERS, BATCH, MAX_PROMPT = 8, 2, 256, 512, 3, 4, 96


@pytest.fixture(scope="module")
def weights():
    w, keep = serve_glue.synthetic_weights(E, H, F, seed=31)
    yield w
    del keep


def jobs_from(d):
    return [serve.Job(i, float(d["arrival_s"][i]), q.SCHED_LS if d["is_ls"][i] else q.SCHED_BE, int(d["prompt_len"][i]),
                      int(d["out_len"][i])) for i in range(len(d["arrival_s"]))]


def replay(trace, batch_size):
    """Feed the engine's scheduler calls to the oracle; every batch must be the one the oracle forms."""
    orc = SchedOracle(batch_size)
    n = 0
    for ev in trace:
        if ev[0] == "submit":
            orc.submit(ev[1], ev[2])
        elif ev[0] == "token":
            orc.token(ev[1], ev[2])
        elif ev[0] == "preempt":
            assert orc.preempt_wanted(0)
        else:
            want = orc.next_batch()
            assert ev[1] == (None if want is None else (list(want[0]), want[1], want[2]))
            n += 1
    assert not orc.cls
    return n


def engine(weights, preemptive, max_job=64, **kw):
    glue = serve_glue.SyntheticGlue(H, K, seed=5, digest=True, max_job=max_job)
    return serve.Engine(weights, glue, E, K, H, F, layers=LAYERS, batch_size=BATCH, max_prompt=MAX_PROMPT,
                        preemptive=preemptive, chunk_rows=32, units_per_call=1, lookahead=1, **kw)


def test_stream_completes_and_is_bit_identical_across_policies(weights):
    d = wl.make_jobs(40, rate_per_s=2500.0, p_ls=0.25, seed=7, max_prompt=MAX_PROMPT, max_out=6, min_prompt=8, min_out=2)
    results = {}
    for pre in (False, True, "host-fed"):
        jobs = jobs_from(d)
        eng = engine(weights, bool(pre), device_stop=pre is True)
        st = eng.run(jobs)
        print(st)
        assert all(j.tokens == j.out_len and j.ttft_s >= 0 and j.done_s >= j.ttft_s for j in jobs)
        assert st["prefill_iterations"] + st["decode_iterations"] == replay(eng.trace, BATCH)
        assert eng.sched.running() == 0 and all(eng.sched.queue_len(i) == 0 for i in range(4))
        assert int(eng.glue.ls_rows_seen.item()) == eng.glue.ls_rows_expected      # the layers saw the batch's priority flags
        assert (eng.glue.ls_rows_expected > 0) == bool(pre)
        results[pre] = (st, eng.glue.digest.cpu().numpy().copy())
    assert results[False][0]["preemptions"] == 0
    assert results[True][0]["preemptions"] > 0 and results["host-fed"][0]["preemptions"] > 0
    # batch composition, priority order and preemption change when a row is computed, never its value
    assert np.array_equal(results[False][1], results[True][1])
    assert np.array_equal(results[False][1], results["host-fed"][1])
    assert np.any(results[True][1] != 0)


def test_ls_prompt_behind_a_long_be_batch(weights):
    # four long BE jobs arrive first; one LS prompt arrives while they are being served
    def mk():
        js = [serve.Job(i, 0.0, q.SCHED_BE, MAX_PROMPT, 40) for i in range(4)]
        js.append(serve.Job(4, 0.004, q.SCHED_LS, 16, 2))
        return js
    ttft = {}
    for pre in (False, True):
        jobs = mk()
        eng = engine(weights, pre)
        eng.run(jobs)          # warm-up run: first-use costs stay out of the comparison
        jobs = mk()
        eng = engine(weights, pre)
        st = eng.run(jobs)
        print(st)
        ttft[pre] = jobs[4].ttft_s
        replay(eng.trace, BATCH)
    # A reported figure, not a timing bar: on an idle box the preemptive policy gives the LS prompt its
    # first token several times earlier.  Asserted: only that it is not served later than behind the
    # whole BE batch (a loose bound that a noisy machine cannot break with correct code).
    print(f"LS time to first token: run-to-completion {1e3 * ttft[False]:.2f} ms, preemptive {1e3 * ttft[True]:.2f} ms", flush=True)
    assert ttft[True] < 1.5 * ttft[False], ttft
