"""Event-time model of the CrossoverScheduler loop (arXiv 2103.07974, Algorithm 1).

TEST INFRASTRUCTURE ONLY.  Pure Python, no GPU, no shared code with the library.

One worker time-shares its GPU between N training tasks (Section 2.1).  Two
resources exist: the compute stream, which runs one task's gradient computation
at a time, and the synchronisation channel, which serves sends first come first
served.  Following Algorithm 1, for t = 1..T and i = 1..N the worker

  * computes task i's gradients and fuses them           (takes C[i]),
  * hands the fused gradient to the channel, not waiting (sync takes M[i]),
  * waits for the outstanding sync of the task it will compute next,
    n = (i mod N) + 1, and applies that task's update    (takes U[n]).

The printed algorithm writes the received task as i+1; for i = N that index does
not exist, so it is read as wrapping to task 1, whose outstanding gradient is
the one sent in the current outer iteration.  During the first outer iteration
the wait is skipped for tasks that have not computed yet (Section 2.2: the
receive/update steps are bypassed when no gradient is outstanding), and after
the last iteration the syncs still in flight are drained (Section 2.2: one
additional synchronisation phase).

The property under test (Section 1, first contribution): the synchronisation
delay disappears when the communication/computation ratio is below 1.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple


@dataclass
class Timeline:
    t_cross: float                 # makespan of the crossover schedule
    t_serial: float                # T * sum(C + M + U): one task after another, nothing overlapped
    stall: float                   # total time the compute stream sat waiting for a sync
    syncs_issued: int
    bypasses: int                  # inner steps whose receive/update was skipped
    drained: int                   # syncs completed in the final extra phase
    events: List[Tuple[str, int, int, float, float]] = field(default_factory=list)
    # (kind, task, outer iteration, start, end); kind in {"compute","sync","update"}


def simulate(C: Sequence[float], M: Sequence[float], T: int,
             U: Sequence[float] | None = None) -> Timeline:
    N = len(C)
    if len(M) != N or N < 1 or T < 0:
        raise ValueError("C and M need one entry per task; T >= 0")
    U = [0.0] * N if U is None else list(U)
    now = 0.0                      # compute stream clock
    chan_free = 0.0                # time the sync channel becomes idle
    pending: Dict[int, Tuple[float, int]] = {}   # task -> (sync end, outer iteration sent)
    stall = 0.0
    issued = bypasses = 0
    ev: List[Tuple[str, int, int, float, float]] = []
    for t in range(1, T + 1):
        for i in range(N):
            ev.append(("compute", i, t, now, now + C[i]))
            now += C[i]
            start = max(now, chan_free)
            chan_free = start + M[i]
            ev.append(("sync", i, t, start, chan_free))
            pending[i] = (chan_free, t)
            issued += 1
            n = (i + 1) % N
            if n in pending:
                end, t_sent = pending.pop(n)
                if end > now:
                    stall += end - now
                    now = end
                ev.append(("update", n, t_sent, now, now + U[n]))
                now += U[n]
            else:
                bypasses += 1
    drained = 0
    for n in sorted(pending, key=lambda k: pending[k][0]):
        end, t_sent = pending[n]
        now = max(now, end)
        ev.append(("update", n, t_sent, now, now + U[n]))
        now += U[n]
        drained += 1
    t_serial = T * sum(C[i] + M[i] + U[i] for i in range(N))
    return Timeline(now, t_serial, stall, issued, bypasses, drained, ev)
