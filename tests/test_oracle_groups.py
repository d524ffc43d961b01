"""Pins for the oracle's update with hyper-parameters per tensor (Algorithm 1, "Model
Update", applied with one (lr, mu, wd) triple per layer: SGD parameter groups)."""
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sgd_two_groups_worked.txt")


def _golden():
    rows = {}
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            step, tensor, elem, x, v = line.split()
            rows[(int(step), tensor, int(elem))] = (float(x), float(v))
    return rows


@pytest.mark.parametrize("work", [np.float64, np.float32])
@pytest.mark.parametrize("align", [1, 4])
def test_hand_derived_two_group_steps(work, align):
    want = _golden()
    numel = [2, 1]
    offs = oracle.layout(numel, align)
    g0 = oracle.pack([np.array([2, 4], np.float32), np.array([1], np.float32)], offs)
    g1 = oracle.pack([np.array([4, -4], np.float32), np.array([3], np.float32)], offs)
    x = oracle.pack([np.array([1, -2], np.float32), np.array([8], np.float32)], offs).astype(work)
    v = oracle.pack([np.array([0, 4], np.float32), np.array([16], np.float32)], offs).astype(work)
    hp = [(0.5, 0.5, 0.0), (0.25, 0.0, 0.5)]
    for step in (1, 2):
        oracle.reduce_sgd_per_tensor([g0, g1], x, v, offs, hp)
        xs = oracle.unpack(x, numel, offs); vs = oracle.unpack(v, numel, offs)
        for ti, name in enumerate("ab"):
            for e in range(numel[ti]):
                assert (xs[ti][e], vs[ti][e]) == want[(step, name, e)], (step, name, e)
    # padding (zero state, zero gradient) stays zero under any triple
    if align == 4:
        assert np.all(x[2:4] == 0) and np.all(v[2:4] == 0) and np.all(x[5:] == 0)


def test_equal_triples_reduce_to_the_single_triple_update():
    rng = np.random.default_rng(21)
    numel = [5, 0, 130, 1, 64]
    offs = oracle.layout(numel, 8)
    n = int(offs[-1])
    reps = [rng.standard_normal(n).astype(np.float32) for _ in range(4)]
    for work in (np.float64, np.float32):
        x0 = rng.standard_normal(n).astype(work); v0 = rng.standard_normal(n).astype(work)
        xa, va = x0.copy(), v0.copy()
        xb, vb = x0.copy(), v0.copy()
        f = oracle.reduce_sgd_f64 if work == np.float64 else oracle.reduce_sgd_f32
        f(reps, xa, va, 0.1, 0.9, 1e-4, 0.5)
        oracle.reduce_sgd_per_tensor(reps, xb, vb, offs, [(0.1, 0.9, 1e-4)] * len(numel), 0.5)
        assert np.array_equal(xa, xb) and np.array_equal(va, vb)


def test_matches_torch_sgd_with_parameter_groups_in_double():
    # an independent implementation of the same convention, with its own group handling
    rng = np.random.default_rng(22)
    numel = [7, 33, 1, 128, 20]
    groups = [(0.1, 0.9, 5e-4), (0.05, 0.0, 0.0), (0.2, 0.5, 1e-2)]
    group_of = [0, 1, 2, 0, 1]
    hp = [groups[g] for g in group_of]
    W, steps = 3, 4
    offs = oracle.layout(numel, 4)
    n = int(offs[-1])
    p0 = [rng.standard_normal(k) for k in numel]
    tparams = [torch.tensor(p, dtype=torch.float64, requires_grad=True) for p in p0]
    opt = torch.optim.SGD(
        [{"params": [tparams[t] for t in range(len(numel)) if group_of[t] == g],
          "lr": lr, "momentum": mu, "weight_decay": wd} for g, (lr, mu, wd) in enumerate(groups)],
        lr=1.0)
    x = oracle.pack([p.astype(np.float32) for p in p0], offs).astype(np.float64)
    # start from the same double values torch holds
    for t, p in enumerate(p0):
        x[int(offs[t]):int(offs[t]) + numel[t]] = p
    v = np.zeros(n)
    for _ in range(steps):
        grads = [[rng.standard_normal(k).astype(np.float32) for k in numel] for _ in range(W)]
        reps = [oracle.pack(g, offs) for g in grads]
        oracle.reduce_sgd_per_tensor(reps, x, v, offs, hp)
        for t in range(len(numel)):
            mean = sum(grads[w][t].astype(np.float64) for w in range(W)) / W
            tparams[t].grad = torch.tensor(mean)
        opt.step()
    for t in range(len(numel)):
        got = x[int(offs[t]):int(offs[t]) + numel[t]]
        assert np.allclose(got, tparams[t].detach().numpy(), rtol=1e-13, atol=1e-15), t


def test_each_tensor_sees_only_its_own_triple():
    # lr = 0 freezes a tensor's parameters bit for bit while its momentum still moves;
    # a neighbour with mu = 0, wd = 0 takes a plain gradient step
    numel = [3, 2]
    offs = oracle.layout(numel, 1)
    g = np.array([1, 2, 3, 4, 5], np.float32)
    x = np.array([10, 20, 30, 40, 50], np.float64); v = np.ones(5)
    oracle.reduce_sgd_per_tensor([g, g], x, v, offs, [(0.0, 0.5, 0.0), (0.5, 0.0, 0.0)])
    assert np.array_equal(x[:3], [10, 20, 30])
    assert np.array_equal(v[:3], [1.5, 2.5, 3.5])
    assert np.array_equal(x[3:], [38, 47.5])
    assert np.array_equal(v[3:], [4, 5])
    # swapping the triples changes the result: the mapping tensor -> triple matters
    x2 = np.array([10, 20, 30, 40, 50], np.float64); v2 = np.ones(5)
    oracle.reduce_sgd_per_tensor([g, g], x2, v2, offs, [(0.5, 0.0, 0.0), (0.0, 0.5, 0.0)])
    assert np.array_equal(x2, [9.5, 19, 28.5, 40, 50])


def test_padding_follows_the_tensor_in_front_of_it():
    # convention: a segment is a tensor plus its trailing padding
    numel = [1, 1]
    offs = oracle.layout(numel, 2)            # [0, 2, 4]
    g = np.zeros(4, np.float32)
    x = np.array([1, 1, 1, 1], np.float64); v = np.zeros(4)
    oracle.reduce_sgd_per_tensor([g], x, v, offs, [(1.0, 0.0, 0.5), (1.0, 0.0, 0.25)])
    assert np.array_equal(x, [0.5, 0.5, 0.75, 0.75])


def test_sync_step_with_tensor_hp_matches_per_tensor_sync_steps():
    rng = np.random.default_rng(23)
    numel = [9, 40, 3]
    hp = [(0.1, 0.9, 0.0), (0.2, 0.0, 1e-3), (0.05, 0.5, 1e-2)]
    W = 2
    grads = [[rng.standard_normal(k).astype(np.float32) for k in numel] for _ in range(W)]
    params = [rng.standard_normal(k).astype(np.float32) for k in numel]
    offs = oracle.layout(numel, 16)
    v = np.zeros(int(offs[-1]))
    got, inf = oracle.sync_step(grads, params, v, 0, 0, 0, align=16, tensor_hp=hp)
    assert not inf
    for t in range(len(numel)):
        vt = np.zeros(numel[t])
        one, _ = oracle.sync_step([[grads[w][t]] for w in range(W)], [params[t]], vt, *hp[t])
        assert np.array_equal(one[0], got[t])
        assert np.array_equal(vt, v[int(offs[t]):int(offs[t]) + numel[t]])


def test_wrong_number_of_triples_is_rejected():
    offs = oracle.layout([2, 2], 1)
    with pytest.raises(ValueError):
        oracle.reduce_sgd_per_tensor([np.zeros(4, np.float32)], np.zeros(4), np.zeros(4), offs,
                                     [(0.1, 0.0, 0.0)])
