"""A serving loop above the layer API: jobs arrive over time, the C++ scheduler (include/qsched.h)
forms batches with the paper's batch-selection algorithm, and every iteration of a batch runs a stack
of MoE layers through the C ABI of include/qmoe.h.

Paper: section "System Architecture" (scheduler, dispatcher, batch engine, closed loop between engine
and scheduler) and the evaluation's workload and metrics (Poisson arrivals, a fraction of the
prompts marked LS, time to first token, turnaround time, job completion rate).

What is modelled.  A model is `layers` MoE layers.  Everything between two MoE layers (in a real
model the attention block and the residual) and the source of the hidden states are not part of this
library: the caller passes a `glue` object that supplies them (serve_glue.py at the repository root
is the synthetic one the benchmark and the tests use: rows of a seeded bank as hidden states, x + y
as the stand-in for the block between layers).  This module only drives the scheduler and the layer
calls; PyTorch appears in it for device buffers, events and host-to-device copies of index arrays.
A prefill iteration runs all prompt tokens of the batch's jobs through the stack and yields each
job's first token; a decode iteration runs one token per job.

The glue object:
    glue.fill_inputs(x, rows, n)        x[:n] <- the hidden states of bank rows rows[:n] (device tensors)
    glue.between_layers(x, y)           x <- input of the next layer, from this layer's input x and output y
    glue.bank_rows                      number of rows the bank holds
    glue.observe_layer(ctx, n_ls_rows)  optional hook after moe_permute of every layer (tests)
    glue.observe_output(x, owner, n)    optional hook after the last layer (tests: per-job digests)

Two policies share all of that code:
  * preemptive=True: jobs keep their class; while a batch of BE jobs only is executing, the loop keeps
    asking the scheduler whether an LS prompt waits; if so it parks the batch at the next expert-chunk
    boundary (its context and cursor stay on the device), runs the batch the scheduler hands out
    next (the LS prefill) through all layers, reports its tokens, and resumes the parked batch from
    its cursor.  device_stop=True: the expert work of a prefill layer is on the stream as gated
    launches (moe_expert_enqueue) and parking is a host store of the stop word; decode layers (a
    handful of units each) and device_stop=False feed the work moe_expert_run by moe_expert_run with
    a bounded look-ahead.
  * preemptive=False: the priority-oblivious run-to-completion baseline.  Every job is submitted as
    BE, so the algorithm degenerates to "decode before prefill": a batch, once prefilled, decodes
    until all its jobs are done before the next prompts are taken; control returns to the scheduler
    only between iterations.
Per-row results never depend on the policy (same contexts' configurations, deterministic kernels),
which `digest=True` lets a test check bit for bit.
"""
from __future__ import annotations

import time
from dataclasses import dataclass

import numpy as np
import torch

from . import binding as q


@dataclass
class Job:
    id: int
    arrival_s: float
    cls: int            # q.SCHED_LS or q.SCHED_BE
    prompt_len: int
    out_len: int        # output tokens to produce (the first one comes from the prefill)
    tokens: int = 0
    ttft_s: float = -1.0
    done_s: float = -1.0


class _Slot:
    """Buffers and context of one in-flight batch of one stage."""

    def __init__(self, E, k, H, F, chunk_rows, max_tokens, device):
        # Batches are fed a few chunks at a time when they must stay stoppable; the K-split down
        # projection keeps such small launches wide enough to use the chip.
        self.ctx = q.Context(E, k, H, F, q.MOE_BF16, chunk_rows, max_tokens, device=device,
                             down_ksplit=4 if F % 256 == 0 else 0)
        self.x = torch.empty((max_tokens, H), dtype=torch.bfloat16, device=device)
        self.y = torch.empty((max_tokens, H), dtype=torch.bfloat16, device=device)
        self.prio = torch.empty(max_tokens, dtype=torch.uint8, device=device)
        self.rows = torch.empty(max_tokens, dtype=torch.int64, device=device)
        self.owner = torch.empty(max_tokens, dtype=torch.int64, device=device)


class Engine:
    def __init__(self, weights: q.MoeWeights, glue, E: int, k: int, H: int, F: int, layers: int, batch_size: int,
                 max_prompt: int, preemptive: bool, units_per_call: int = 4, lookahead: int = 1, chunk_rows: int = 256,
                 device_stop: bool = True, units_per_launch: int = q.UINT32_MAX, device="cuda:0"):
        self.w, self.layers, self.batch_size, self.max_prompt = weights, layers, batch_size, max_prompt
        self.preemptive, self.units_per_call, self.lookahead = preemptive, units_per_call, lookahead
        self.device_stop = device_stop
        self.units_per_launch = units_per_launch     # enqueued (device-stopped) layers: launch size; default the whole layer
        self.device = device
        self.glue = glue
        self.bank_rows = glue.bank_rows
        # [stage][level]: level 1 holds the batch that runs while a level-0 batch is parked
        self.slots = {
            q.SCHED_PREFILL: [_Slot(E, k, H, F, chunk_rows, batch_size * max_prompt, device) for _ in range(2)],
            q.SCHED_DECODE: [_Slot(E, k, H, F, chunk_rows, batch_size, device) for _ in range(2)],
        }
        self.sched = q.Scheduler(batch_size)
        self.trace: list = []        # scheduler calls in order, for replay against the oracle

    # ---- dispatcher side ----
    def _now(self) -> float:
        return time.perf_counter() - self.t0

    def _admit(self) -> None:
        """Hand the jobs whose arrival time has passed to the dispatcher."""
        now = self._now()
        while self.next_arrival < len(self.arrivals) and self.arrivals[self.next_arrival].arrival_s <= now:
            j = self.arrivals[self.next_arrival]
            cls = j.cls if self.preemptive else q.SCHED_BE
            self.sched.submit(j.id, cls)
            self.trace.append(("submit", j.id, cls))
            self.next_arrival += 1

    def _next_batch(self):
        got = self.sched.next_batch()
        self.trace.append(("next_batch", got))
        return got

    # ---- engine side ----
    def _build(self, slot: _Slot, jobs, stage, n_ls) -> int:
        rows, prio, owner = [], [], []
        for i, jid in enumerate(jobs):
            j = self.jobs[jid]
            if stage == q.SCHED_PREFILL:
                r = (j.id * 977 + np.arange(j.prompt_len)) % self.bank_rows
            else:
                r = np.array([(j.id * 977 + j.prompt_len + j.tokens) % self.bank_rows])
            rows.append(r)
            prio.append(np.full(len(r), 1 if i < n_ls else 0, dtype=np.uint8))
            owner.append(np.full(len(r), j.id, dtype=np.int64))
        rows, prio, owner = np.concatenate(rows), np.concatenate(prio), np.concatenate(owner)
        n = len(rows)
        slot.rows[:n].copy_(torch.from_numpy(rows.astype(np.int64)))
        slot.prio[:n].copy_(torch.from_numpy(prio))
        slot.owner[:n].copy_(torch.from_numpy(owner))
        self.glue.fill_inputs(slot.x, slot.rows, n)
        return n, int(prio.sum())

    def _iteration(self, jobs, stage, n_ls, level: int) -> None:
        slot = self.slots[stage][level]
        n, n_ls_rows = self._build(slot, jobs, stage, n_ls)
        x, y, ctx = slot.x[:n], slot.y[:n], slot.ctx
        observe_layer = getattr(self.glue, "observe_layer", None)
        observe_output = getattr(self.glue, "observe_output", None)
        preemptible = self.preemptive and level == 0 and n_ls == 0
        for _ in range(self.layers):
            ctx.route(x, self.w, n_tokens=n)
            ctx.permute(slot.prio)
            if observe_layer is not None:
                observe_layer(ctx, n_ls_rows)
            if not preemptible:
                ctx.expert_run(x, self.w)
            elif self.device_stop and stage == q.SCHED_PREFILL:
                # the whole layer goes on the stream as gated launches; the loop watches for an LS
                # prompt meanwhile and closes the gates when one waits
                rc = ctx.expert_enqueue(x, self.w, self.units_per_launch)
                while rc != q.MOE_DONE:
                    ev = torch.cuda.Event()
                    ev.record()
                    while not ev.query():
                        self._admit()
                        if self.sched.preempt_wanted(0):
                            ctx.expert_stop()
                            while self.sched.preempt_wanted(0):
                                self.trace.append(("preempt", tuple(jobs)))
                                self.preemptions += 1
                                got = self._next_batch()
                                self._iteration(*got, level=1)     # runs behind the launch in progress
                                self._admit()
                            break
                    rc = ctx.expert_collect()
                    if rc != q.MOE_DONE:
                        rc = ctx.expert_enqueue(x, self.w, self.units_per_launch)
            else:
                pending, done = [], False
                while not done:
                    self._admit()
                    while self.sched.preempt_wanted(0):
                        self.trace.append(("preempt", tuple(jobs)))
                        self.preemptions += 1
                        got = self._next_batch()
                        self._iteration(*got, level=1)
                        self._admit()
                    while pending and pending[0].query():
                        pending.pop(0)
                    if len(pending) < self.lookahead:
                        rc = ctx.expert_run(x, self.w, self.units_per_call)
                        ev = torch.cuda.Event()
                        ev.record()
                        pending.append(ev)
                        done = rc == q.MOE_DONE
            ctx.combine(y)
            self.glue.between_layers(x, y)
        if observe_output is not None:
            observe_output(x, slot.owner, n)
        torch.cuda.current_stream().synchronize()
        now = self._now()
        self.iterations[stage] += 1
        for jid in jobs:
            j = self.jobs[jid]
            j.tokens += 1
            if j.tokens == 1:
                j.ttft_s = now - j.arrival_s
            fin = j.tokens >= j.out_len
            if fin:
                j.done_s = now - j.arrival_s
                self.finished += 1
            self.sched.token(jid, fin)
            self.trace.append(("token", jid, fin))

    def run(self, jobs: list[Job]) -> dict:
        """Serve the jobs (arrival_s relative to the start of the call); returns the statistics."""
        self.jobs = {j.id: j for j in jobs}
        self.arrivals = sorted(jobs, key=lambda j: (j.arrival_s, j.id))
        self.next_arrival, self.finished, self.preemptions = 0, 0, 0
        self.iterations = {q.SCHED_PREFILL: 0, q.SCHED_DECODE: 0}
        assert all(1 <= j.prompt_len <= self.max_prompt and j.out_len >= 1 for j in jobs)
        torch.cuda.synchronize()
        self.t0 = time.perf_counter()
        while self.finished < len(jobs):
            self._admit()
            got = self._next_batch()
            if got is None:
                self.trace.pop()             # idle polls are not part of the trace
                continue
            self._iteration(*got, level=0)
        makespan = self._now()
        return self._stats(makespan)

    def _stats(self, makespan: float) -> dict:
        out = {"policy": "preemptive" if self.preemptive else "fcfs_run_to_completion", "jobs": len(self.jobs),
               "makespan_s": round(makespan, 4), "jobs_per_s": round(len(self.jobs) / makespan, 2),
               "output_tokens_per_s": round(sum(j.out_len for j in self.jobs.values()) / makespan, 1),
               "preemptions": self.preemptions, "prefill_iterations": self.iterations[q.SCHED_PREFILL],
               "decode_iterations": self.iterations[q.SCHED_DECODE]}
        for name, cls in (("ls", q.SCHED_LS), ("be", q.SCHED_BE)):
            js = [j for j in self.jobs.values() if j.cls == cls]
            if not js:
                continue
            ttft = np.array([j.ttft_s for j in js]) * 1e3
            turn = np.array([j.done_s for j in js]) * 1e3
            out[name] = {"n": len(js), "ttft_ms": {"mean": round(float(ttft.mean()), 3), "p50": round(float(np.percentile(ttft, 50)), 3),
                                                    "p99": round(float(np.percentile(ttft, 99)), 3)},
                         "turnaround_ms": {"mean": round(float(turn.mean()), 3), "p99": round(float(np.percentile(turn, 99)), 3)}}
        return out
