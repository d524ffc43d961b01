"""Parity of xs_fused_gather_reduce_sgd (gradients read straight from the per-layer tensors,
parameters optionally written straight to the per-layer views) with the oracle's whole step
and, bit for bit, with the library's own pack -> reduce+SGD -> unpack sequence."""
import numpy as np
import pytest
import torch

import oracle
from paper_2103_07974_amd import harness, workloads as wl, xs

pytestmark = pytest.mark.gpu

RTOL32, ATOL32 = 1e-6, 1e-7
SIZES = [0, 1, 3, 5, 17, 63, 64, 65, 255, 256, 257, 4095, 4096, 4097, 12289, 50001, 2, 0, 70000]


def _bits(a):
    return a.view(np.uint32 if a.dtype.itemsize == 4 else np.uint16)


def _hp(w):
    return (np.float32(w.lr).item(), np.float32(w.momentum).item(),
            np.float32(w.weight_decay).item(), np.float32(1.0 / w.loss_scale).item())


def _skewed(tensors, skew):
    """Copies of the tensors that start at odd element offsets inside their allocations."""
    if not skew:
        return tensors, None
    holders, views = [], []
    for i, t in enumerate(tensors):
        sk = 1 + (i % 3)
        buf = torch.zeros(t.numel() + sk + 4, dtype=t.dtype, device=t.device)
        v = buf[sk:sk + t.numel()]
        v.copy_(t)
        holders.append(buf); views.append(v)
    return views, holders


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("align", [1, 4, 64])
@pytest.mark.parametrize("W", [1, 2, 3, 8, 16])
def test_gather_matches_oracle_and_bucket_path(dtype, align, W):
    base = wl.RESNET50 if dtype == "f32" else wl.BERT_LARGE_F16
    w = wl.scaled(base, f"mix_{dtype}", [(n,) for n in SIZES], W=W)
    skew = (align + W) % 2
    print(f"case dtype={dtype} align={align} W={W} skew={skew}", flush=True)
    task = harness.make_task(w, "cuda", align)
    lr, mu, wd, inv = _hp(w)
    task.momentum.copy_(wl.make_flat(task.n_bucket, 0.01, 5, device="cuda"))
    # padding of the momentum bucket back to zero, as a caller's state would be
    mask = torch.ones(task.n_bucket, dtype=torch.bool, device="cuda")
    for n, o in zip(w.numel, task.offsets[:-1]):
        mask[o:o + n] = False
    task.momentum[mask] = 0
    grads = []
    keep = []
    for g in task.grads:
        v, h = _skewed(g, skew)
        grads.append(v); keep.append(h)
    pviews, pkeep = _skewed([t.clone() for t in task.param_tensors], skew)
    gtab = xs.gather_pointer_table(grads)
    ptab = xs.pointer_table(pviews) if len(pviews) else xs.pointer_table([task.params])
    x0, v0 = task.params.clone(), task.momentum.clone()

    # library bucket path on copies of the state
    xb, vb = x0.clone(), v0.clone()
    tabs = [xs.pointer_table(g) for g in grads]
    for r in range(W):
        xs.fuse_pack(task.gplan, tabs[r], task.buckets[r])
    xs.fused_reduce_sgd(task.buckets, task.n_bucket, xb, vb, w.lr, w.momentum, w.weight_decay,
                        1.0 / w.loss_scale)
    # gathering form, in place, with fused views
    xg, vg = x0.clone(), v0.clone()
    xs.fused_gather_reduce_sgd(task.gplan, gtab, W, xg, vg, w.lr, w.momentum, w.weight_decay,
                               1.0 / w.loss_scale, param_tensor_ptrs=ptab)
    # gathering form, out of place, no views
    xo, vo = torch.full_like(x0, 9.0), torch.full_like(v0, 9.0)
    xs.fused_gather_reduce_sgd(task.gplan, gtab, W, x0, v0, w.lr, w.momentum, w.weight_decay,
                               1.0 / w.loss_scale, params_out=xo, momentum_out=vo)
    torch.cuda.synchronize()
    assert torch.equal(xg.view(torch.int32), xb.view(torch.int32))
    assert torch.equal(vg.view(torch.int32), vb.view(torch.int32))
    assert torch.equal(xo.view(torch.int32), xb.view(torch.int32))
    assert torch.equal(vo.view(torch.int32), vb.view(torch.int32))
    for t, (n, o) in zip(pviews, zip(w.numel, task.offsets[:-1])):
        assert torch.equal(t.view(torch.int32), xb[o:o + n].view(torch.int32))
    if pkeep is not None:       # nothing written outside the views
        for h, t in zip(pkeep, pviews):
            start = (t.data_ptr() - h.data_ptr()) // 4
            hv = h.cpu().numpy()
            assert not hv[:start].any() and not hv[start + t.numel():].any()

    # oracle: whole step from the tensor lists
    grads_host = [[t.cpu().numpy() for t in g] for g in grads]
    params_host = [t.cpu().numpy() for t in task.param_tensors]
    v64 = v0.cpu().numpy().astype(np.float64)
    want, found = oracle.sync_step(grads_host, params_host, v64, lr, mu, wd, inv, align=align)
    assert not found
    v32 = v0.cpu().numpy().copy()
    want32, _ = oracle.sync_step(grads_host, params_host, v32, lr, mu, wd, inv, align=align,
                                 precision="f32")
    for t, a, b in zip(pviews, want, want32):
        got = t.cpu().numpy()
        assert np.all(np.abs(got - a) <= ATOL32 + RTOL32 * np.abs(a))
        assert np.array_equal(_bits(got), _bits(b))
    gv = vg.cpu().numpy()
    assert np.all(np.abs(gv - v64) <= ATOL32 + RTOL32 * np.abs(v64))
    assert np.array_equal(_bits(gv), _bits(v32))


def test_gather_overflow_detection_and_skip():
    w = wl.scaled(wl.BERT_LARGE_F16_INF, "mini_inf", [(1000,), (24,), (5000,), (7,)], W=4)
    task = harness.make_task(w, "cuda", align=8)
    x0, v0 = task.params.clone(), task.momentum.clone()
    xo, vo = torch.full_like(x0, 9.0), torch.full_like(v0, 9.0)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    xs.fused_gather_reduce_sgd(task.gplan, task.gather_table, w.W, x0, v0, w.lr, w.momentum,
                               w.weight_decay, 1 / w.loss_scale, params_out=xo, momentum_out=vo,
                               found_inf=flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 1
    assert torch.equal(x0, task.params) and torch.equal(v0, task.momentum)      # inputs untouched
    # a raised flag skips the next pass entirely, in place or not
    xs.fused_gather_reduce_sgd(task.gplan, task.gather_table, w.W, x0, v0, w.lr, w.momentum,
                               w.weight_decay, 1 / w.loss_scale, found_inf=flag,
                               param_tensor_ptrs=task.param_table)
    torch.cuda.synchronize()
    assert torch.equal(x0, task.params) and torch.equal(v0, task.momentum)
    # the oracle takes the same decision
    found = oracle.sync_step([[t.cpu().numpy() for t in g] for g in task.grads],
                             [t.cpu().numpy() for t in task.param_tensors],
                             np.zeros(task.n_bucket), 0.1, 0.9, 0.0, 1.0, align=8)[1]
    assert found is True
    # clean gradients leave the flag alone
    w2 = wl.scaled(wl.BERT_LARGE_F16, "mini", [(1000,), (24,), (5000,), (7,)], W=4)
    t2 = harness.make_task(w2, "cuda", align=8)
    flag.zero_()
    xs.fused_gather_reduce_sgd(t2.gplan, t2.gather_table, 4, t2.params.clone(), t2.momentum.clone(),
                               0.1, 0.9, 0.0, 1 / 1024, params_out=xo, momentum_out=vo, found_inf=flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    # views are refused while the pass is still deciding
    with pytest.raises(xs.XsError) as e:
        xs.fused_gather_reduce_sgd(t2.gplan, t2.gather_table, 4, t2.params, t2.momentum, 0.1, 0.9, 0.0,
                                   1.0, params_out=xo, momentum_out=vo, found_inf=flag,
                                   param_tensor_ptrs=t2.param_table)
    assert e.value.status == xs.XS_ERR_UNSUPPORTED


@pytest.mark.parametrize("name", ["tiny_mlp", "resnet50", "vgg16"])
def test_gather_full_size_equals_bucket_path(name):
    w = wl.WORKLOADS[name]
    print(f"workload {name}", flush=True)
    task = harness.make_task(w, "cuda")
    task.momentum.copy_(wl.make_flat(task.n_bucket, 0.01, 5, device="cuda"))
    mask = torch.ones(task.n_bucket, dtype=torch.bool, device="cuda")
    for n, o in zip(w.numel, task.offsets[:-1]):
        mask[o:o + n] = False
    task.momentum[mask] = 0
    xg, vg = task.params.clone(), task.momentum.clone()
    views = [torch.zeros_like(t) for t in task.param_tensors]
    xs.fused_gather_reduce_sgd(task.gplan, task.gather_table, w.W, xg, vg, w.lr, w.momentum,
                               w.weight_decay, 1.0, param_tensor_ptrs=xs.pointer_table(views))
    app = task.make_app()
    app.sync()
    torch.cuda.synchronize()
    assert torch.equal(xg.view(torch.int32), task.params.view(torch.int32))
    assert torch.equal(vg.view(torch.int32), task.momentum.view(torch.int32))
    for a, b in zip(views, task.param_tensors):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
    app.destroy()


def test_gather_bert_large_f16_equals_bucket_path():
    w = wl.BERT_LARGE_F16
    task = harness.make_task(w, "cuda")
    xg, vg = task.params.clone(), task.momentum.clone()
    views = [torch.zeros_like(t) for t in task.param_tensors]
    xs.fused_gather_reduce_sgd(task.gplan, task.gather_table, w.W, xg, vg, w.lr, w.momentum,
                               w.weight_decay, 1.0 / w.loss_scale,
                               param_tensor_ptrs=xs.pointer_table(views))
    app = task.make_app()
    app.sync()
    torch.cuda.synchronize()
    assert torch.equal(xg.view(torch.int32), task.params.view(torch.int32))
    assert torch.equal(vg.view(torch.int32), task.momentum.view(torch.int32))
    for a, b in zip(views, task.param_tensors):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
    app.destroy()
