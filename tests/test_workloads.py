"""The synthetic gradient sets have the sizes the benchmark configurations state."""
import numpy as np
import torch

from paper_2103_07974_amd import workloads as wl


def test_counts():
    assert (wl.TINY_MLP.n_tensors, wl.TINY_MLP.n_elems) == (4, 203530)
    assert (wl.RESNET50.n_tensors, wl.RESNET50.n_elems) == (161, 25557032)
    assert (wl.VGG16.n_tensors, wl.VGG16.n_elems) == (32, 138357544)
    assert (wl.BERT_LARGE_F16.n_tensors, wl.BERT_LARGE_F16.n_elems) == (391, 335141888)
    assert max(wl.VGG16.numel) == 4096 * 25088
    assert sum(1 for n in wl.RESNET50.numel if n < 4096) == 107


def test_generators_are_seeded_and_distinct_per_replica():
    w = wl.TINY_MLP
    a = wl.make_replica_grads(w, 0)
    b = wl.make_replica_grads(w, 0)
    c = wl.make_replica_grads(w, 1)
    assert all(torch.equal(x, y) for x, y in zip(a, b))
    assert not torch.equal(a[0], c[0])
    assert [t.numel() for t in a] == list(w.numel)
    std = torch.cat(a).std().item()
    assert abs(std - w.grad_std) < 0.02 * w.grad_std
    p = wl.make_params(w)
    assert abs(torch.cat(p).std().item() - w.param_std) < 0.02 * w.param_std


def test_inf_injection_count_and_placement():
    w = wl.scaled(wl.BERT_LARGE_F16_INF, "mini_inf", [(1000,), (24,), (5000,)], W=2)
    g0 = wl.make_replica_grads(w, 0)
    g1 = wl.make_replica_grads(w, 1)
    assert g0[0].dtype == torch.float16
    n_inf = sum(int(torch.isinf(t).sum()) for t in g0)
    assert n_inf == round(1e-3 * w.n_elems) == 6
    assert sum(int(torch.isinf(t).sum()) for t in g1) == 0
