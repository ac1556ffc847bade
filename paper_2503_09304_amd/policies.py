"""Example scheduling policies at expert granularity, each a few lines over the context's unit list
(paper: sections "Challenges and Design Decisions" and "System Architecture" — user-defined policies,
selective expert execution).  A policy turns the unit list [(expert, cls, row0, rows), ...] into the
order of unit indices to hand to Context.expert_run_units; results never depend on the order."""
from __future__ import annotations

from typing import Iterable, List, Sequence, Tuple

Unit = Tuple[int, int, int, int]    # (expert, cls: 0 = LS / 1 = BE, first sorted row, rows)


def list_order(units: Sequence[Unit]) -> List[int]:
    """The built-in order: every LS chunk of every expert, then every BE chunk."""
    return list(range(len(units)))


def busiest_expert_first(units: Sequence[Unit]) -> List[int]:
    """LS work first as always, but inside each class the experts with the most queued rows go first
    (their chunks share one pass over the expert's weights when issued together)."""
    load = {}
    for e, _c, _r0, rows in units:
        load[e] = load.get(e, 0) + rows
    return sorted(range(len(units)), key=lambda i: (units[i][1], -load[units[i][0]], units[i][0], units[i][2]))


def without_experts(units: Sequence[Unit], skip: Iterable[int]) -> Tuple[List[int], List[int]]:
    """Selective expert execution: (units to run now, units left for later) when the experts in
    `skip` are to be held back, e.g. because their weights are not resident yet."""
    skip = set(skip)
    now = [i for i, u in enumerate(units) if u[0] not in skip]
    later = [i for i, u in enumerate(units) if u[0] in skip]
    return now, later
