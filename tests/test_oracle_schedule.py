"""Pins for the schedule model (Algorithm 1; Section 1 first contribution; Section 2.2
boundary conditions) and for the claim that crossover leaves every task's SGD unchanged."""
import itertools

import numpy as np
import pytest

import oracle
from oracle import schedule, timeline


# ------------------------------------------------------------------ timing claim
def test_no_stall_iff_cross_ratios_at_most_one():
    for CA, CB, MA, MB in itertools.product([1.0, 2.0, 5.0], [1.0, 3.0], [0.5, 1.0, 2.5, 4.0],
                                            [0.5, 2.0, 6.0]):
        tl = timeline.simulate([CA, CB], [MA, MB], T=6)
        hidden = (MA <= CB) and (MB <= CA)
        assert (tl.stall == 0.0) == hidden, (CA, CB, MA, MB, tl.stall)
        if hidden:
            # every sync but the last one disappears behind the other task's compute
            assert tl.t_cross == pytest.approx(6 * (CA + CB) + MB)


def test_own_ratio_below_one_is_not_enough():
    # task A: comm/comp = 3/4 < 1, but its sync must hide under task B's compute of 1
    tl = timeline.simulate([4.0, 1.0], [3.0, 0.5], T=5)
    assert tl.stall > 0.0
    # per step the stall is exactly M_A - C_B once the pipeline is full
    per_step = [e for e in tl.events if e[0] == "update" and e[1] == 0]
    assert tl.stall == pytest.approx(len(per_step) * (3.0 - 1.0))


def test_three_tasks_relax_the_condition_to_the_other_tasks_total_compute():
    # with N tasks a synchronisation has the N-1 computations that follow it to hide under:
    # M_0 may exceed every single C_j as long as it fits under their sum (channel otherwise idle)
    T = 8
    for M0 in (0.5, 1.0, 1.5, 1.9, 2.0, 2.1, 2.5):
        tl = timeline.simulate([1.0, 1.0, 1.0], [M0, 0.05, 0.05], T)
        if M0 <= 2.0:
            assert tl.stall == 0.0, M0
        else:
            assert tl.stall == pytest.approx(T * (M0 - 2.0)), M0
    # the same M_0 = 1.5 with two tasks stalls every iteration
    assert timeline.simulate([1.0, 1.0], [1.5, 0.05], T).stall > 0.0


def test_speedup_tends_to_one_plus_comm_over_comp():
    C, M, T = [10.0, 10.0], [1.5, 1.5], 400
    tl = timeline.simulate(C, M, T)
    assert tl.stall == 0.0
    assert tl.t_serial / tl.t_cross == pytest.approx(1 + sum(M) / sum(C), rel=1e-3)


def test_single_task_degenerates_to_serial():
    tl = timeline.simulate([3.0], [2.0], T=7, U=[0.25])
    assert tl.t_cross == pytest.approx(7 * (3.0 + 2.0 + 0.25)) == pytest.approx(tl.t_serial)
    assert tl.bypasses == 0 and tl.drained == 0


@pytest.mark.parametrize("N", [2, 3, 5])
def test_counts_of_syncs_bypasses_and_drains(N):
    T = 4
    tl = timeline.simulate([1.0] * N, [0.1] * N, T)
    assert tl.syncs_issued == N * T
    assert tl.bypasses == N - 1
    assert tl.drained == N - 1
    assert sum(1 for e in tl.events if e[0] == "update") == N * T


def test_channel_is_serial_and_sync_follows_its_compute():
    tl = timeline.simulate([1.0, 1.0, 1.0], [2.5, 0.2, 0.2], T=3)
    syncs = sorted([e for e in tl.events if e[0] == "sync"], key=lambda e: e[3])
    for a, b in zip(syncs, syncs[1:]):
        assert b[3] >= a[4] - 1e-12
    comp_end = {(e[1], e[2]): e[4] for e in tl.events if e[0] == "compute"}
    for e in syncs:
        assert e[3] >= comp_end[(e[1], e[2])] - 1e-12


def test_compute_of_a_task_never_starts_before_its_previous_update():
    tl = timeline.simulate([1.0, 2.0], [5.0, 0.5], T=4, U=[0.1, 0.1])
    upd_end = {(e[1], e[2]): e[4] for e in tl.events if e[0] == "update"}
    for kind, i, t, s, e in tl.events:
        if kind == "compute" and t > 1:
            assert s >= upd_end[(i, t - 1)] - 1e-12


# ------------------------------------------------------------------ order of operations
def test_order_of_operations_two_tasks():
    log = schedule.run_crossover(2, 2, lambda i, t: (i, t), lambda i, g: None)
    assert log == [("compute", 0, 1), ("send", 0, 1), ("bypass", 1, 1),
                   ("compute", 1, 1), ("send", 1, 1), ("update", 0, 1),
                   ("compute", 0, 2), ("send", 0, 2), ("update", 1, 1),
                   ("compute", 1, 2), ("send", 1, 2), ("update", 0, 2),
                   ("drain", 1, 2)]


@pytest.mark.parametrize("N", [1, 2, 3])
def test_crossover_equals_standalone_training_bit_for_bit(N):
    """Gradients depend on the parameters they are computed from, so any task that
    computed on stale parameters would end somewhere else."""
    T, W = 4, 2
    shapes = [[5, 3], [7], [2, 2, 9]][:N]
    rng = np.random.default_rng(21)
    init = [[rng.standard_normal(n).astype(np.float32) for n in s] for s in shapes]

    def make_state():
        return {"p": [[a.copy() for a in task] for task in init],
                "v": [np.zeros(sum(s), np.float32) for s in shapes]}

    def make_fns(state):
        def compute(i, t):
            # a deterministic "gradient": depends on current parameters, worker and step
            return [[np.sin(p * (w + 1) + t).astype(np.float32) for p in state["p"][i]]
                    for w in range(W)]

        def sync_update(i, g):
            newp, _ = oracle.sync_step(g, state["p"][i], state["v"][i], 0.1, 0.9, 1e-3,
                                       precision="f32")
            state["p"][i] = newp
        return compute, sync_update

    a, b = make_state(), make_state()
    schedule.run_crossover(N, T, *make_fns(a))
    schedule.run_standalone(N, T, *make_fns(b))
    for ta, tb in zip(a["p"], b["p"]):
        for x, y in zip(ta, tb):
            assert np.array_equal(x, y)
    for x, y in zip(a["v"], b["v"]):
        assert np.array_equal(x, y)


def test_equivalence_check_is_sensitive_to_a_missing_wait():
    """A schedule that lets a task compute before its previous update has landed (what a
    missing event wait would do) must end somewhere else than stand-alone training."""
    T, W = 3, 2
    shapes = [[6, 2], [9]]
    rng = np.random.default_rng(33)
    init = [[rng.standard_normal(n).astype(np.float32) for n in s] for s in shapes]

    def run(broken):
        p = [[a.copy() for a in task] for task in init]
        v = [np.zeros(sum(s), np.float32) for s in shapes]
        pending = {}

        def grads(i, t):
            return [[np.sin(q * (w + 1) + t).astype(np.float32) for q in p[i]] for w in range(W)]

        def apply(i, g):
            p[i], _ = oracle.sync_step(g, p[i], v[i], 0.1, 0.9, 1e-3, precision="f32")

        for t in range(1, T + 1):
            for i in range(2):
                if not broken and i in pending:       # the wait: update before computing again
                    apply(i, pending.pop(i))
                g = grads(i, t)
                if broken and i in pending:           # update lands after the computation started
                    apply(i, pending.pop(i))
                pending[i] = g
        for i in sorted(pending):
            apply(i, pending[i])
        return p

    good, bad = run(False), run(True)
    ref = [[a.copy() for a in task] for task in init]
    vref = [np.zeros(sum(s), np.float32) for s in shapes]
    for i in range(2):
        for t in range(1, T + 1):
            g = [[np.sin(q * (w + 1) + t).astype(np.float32) for q in ref[i]] for w in range(W)]
            ref[i], _ = oracle.sync_step(g, ref[i], vref[i], 0.1, 0.9, 1e-3, precision="f32")
    assert all(np.array_equal(a, b) for ta, tb in zip(good, ref) for a, b in zip(ta, tb))
    assert any(not np.array_equal(a, b) for ta, tb in zip(bad, ref) for a, b in zip(ta, tb))
