"""Algorithm 1 of arXiv 2103.07974 executed literally over abstract tasks.

TEST INFRASTRUCTURE ONLY.  Used to check that the crossover order changes nothing
inside any one task: every task's k-th gradient is computed on parameters that
already hold its (k-1)-th update, i.e. each task runs plain synchronous SGD
(abstract and conclusion: same convergence as the original algorithm).

Reading of the printed indices: the task whose averaged gradient is received
after task i has sent is n = (i mod N) + 1 (the printed i+1, wrapped); a task
that has nothing outstanding is skipped (first outer iteration, Section 2.2);
what is still outstanding after the loops is applied in a final phase.
"""
from __future__ import annotations

from typing import Any, Callable, Dict, List, Tuple


def run_crossover(n_tasks: int, T: int,
                  compute: Callable[[int, int], Any],
                  sync_update: Callable[[int, Any], None]) -> List[Tuple[str, int, int]]:
    """compute(i, t) returns task i's fused per-worker gradients from its current
    parameters; sync_update(i, g) averages them and updates task i's parameters.
    Returns the order of operations as (kind, task, outer iteration)."""
    log: List[Tuple[str, int, int]] = []
    outstanding: Dict[int, Tuple[Any, int]] = {}
    for t in range(1, T + 1):
        for i in range(n_tasks):
            g = compute(i, t)
            log.append(("compute", i, t))
            outstanding[i] = (g, t)
            log.append(("send", i, t))
            n = (i + 1) % n_tasks
            if n in outstanding:
                g_n, t_n = outstanding.pop(n)
                sync_update(n, g_n)
                log.append(("update", n, t_n))
            else:
                log.append(("bypass", n, t))
    for n in sorted(outstanding):
        g_n, t_n = outstanding[n]
        sync_update(n, g_n)
        log.append(("drain", n, t_n))
    return log


def run_standalone(n_tasks: int, T: int,
                   compute: Callable[[int, int], Any],
                   sync_update: Callable[[int, Any], None]) -> None:
    """Each task trained alone: compute, synchronise, update, T times."""
    for i in range(n_tasks):
        for t in range(1, T + 1):
            sync_update(i, compute(i, t))
