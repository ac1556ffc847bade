"""Oracle of the host scheduler: dispatcher, four FCFS queues, batch selection (test infrastructure).

Plain Python lists.  The batch selection of the paper's section "System Architecture" (Algorithm 1)
is stated as a rule over the four queues, the dispatcher as that section describes it: new jobs enter the prefill queue of their priority class, every model output token
sends its job to the decode queue of its class, the batch engine builds the next batch from the four
queues.  Only tests, the smoke check and the benchmark's baseline leg may import this module; the
product scheduler is the C++ one behind include/qsched.h and shares no code with it.

Readings where the paper is silent:
  * GetBatch(queue) removes up to BatchSize jobs from the head of the queue, in queue order.
  * "Fill from" a BE queue removes jobs from its head, in order, until the batch has BatchSize jobs
    or the BE queue is empty; the LS jobs come first in the batch.
  * BatchSize counts jobs, not tokens.
  * A job handed out in a batch is in no queue until the dispatcher is told of its output token.
"""
from __future__ import annotations

LS, BE = 1, 0
PREFILL, DECODE = 0, 1


class SchedOracle:
    def __init__(self, batch_size: int):
        assert batch_size >= 1
        self.batch_size = batch_size
        self.ls_prefill: list[int] = []
        self.be_prefill: list[int] = []
        self.ls_decode: list[int] = []
        self.be_decode: list[int] = []
        self.cls: dict[int, int] = {}
        self.running: set[int] = set()

    # ---- dispatcher ----
    def submit(self, job: int, cls: int) -> None:
        """A new prompt arrives: it waits for its prefill in the queue of its class."""
        assert job not in self.cls
        self.cls[job] = cls
        (self.ls_prefill if cls == LS else self.be_prefill).append(job)

    def token(self, job: int, finished: bool) -> None:
        """The model produced an output token of a running job: the job leaves the system if that
        was its last token, otherwise it waits for its next decode step in the queue of its class."""
        assert job in self.running
        self.running.remove(job)
        if finished:
            del self.cls[job]
            return
        (self.ls_decode if self.cls[job] == LS else self.be_decode).append(job)

    # ---- batch engine ----
    def _get_batch(self, queue: list[int], room: int) -> list[int]:
        taken = queue[:room]
        del queue[:room]
        return taken

    def next_batch(self):
        """Batch selection (Algorithm 1) stated as a rule.  Which (class, stage) leads the batch:
        latency-sensitive decode work if a whole batch of it waits; otherwise the first non-empty
        queue in the order LS prefill, LS decode, BE decode, BE prefill.  A batch led by LS jobs that
        is not full is topped up with best-effort jobs of the same stage; a batch led by BE jobs
        holds BE jobs only.  Returns (jobs, stage, number of LS jobs) or None when nothing waits."""
        B = self.batch_size
        queue = {(LS, PREFILL): self.ls_prefill, (LS, DECODE): self.ls_decode,
                 (BE, PREFILL): self.be_prefill, (BE, DECODE): self.be_decode}
        if len(queue[LS, DECODE]) >= B:
            lead = (LS, DECODE)
        else:
            waiting = [key for key in ((LS, PREFILL), (LS, DECODE), (BE, DECODE), (BE, PREFILL)) if queue[key]]
            if not waiting:
                return None
            lead = waiting[0]
        cls, stage = lead
        batch = self._get_batch(queue[lead], B)
        n_ls = len(batch) if cls == LS else 0
        if cls == LS:
            batch += self._get_batch(queue[BE, stage], B - len(batch))
        self.running.update(batch)
        return batch, stage, n_ls

    # ---- closed-loop signal to the engine ----
    def preempt_wanted(self, running_n_ls: int) -> bool:
        """Whether the engine should stop the batch it is executing at the next expert chunk: an LS
        prompt waits for its prefill while the running batch holds best-effort jobs only (the
        example of section "System Architecture")."""
        return running_n_ls == 0 and len(self.ls_prefill) > 0

    def queue_len(self, q: int) -> int:
        return len((self.ls_prefill, self.be_prefill, self.ls_decode, self.be_decode)[q])
