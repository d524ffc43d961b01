"""Parity of xs_fused_reduce_sgd_unpack (bucket form, in place, the unpack fused into the pass)
with the oracle's whole step and, bit for bit, with xs_fused_reduce_sgd + xs_fuse_unpack."""
import numpy as np
import pytest
import torch

import oracle
from paper_2103_07974_amd import harness, workloads as wl, xs

pytestmark = pytest.mark.gpu

RTOL32, ATOL32 = 1e-6, 1e-7
SIZES = [0, 1, 3, 5, 17, 63, 64, 65, 255, 256, 257, 4095, 4096, 4097, 12289, 50001, 2, 0, 70000]
GUARD = 6


def _bits(a):
    return a.view(np.uint32 if a.dtype.itemsize == 4 else np.uint16)


def _hp(w):
    return (np.float32(w.lr).item(), np.float32(w.momentum).item(),
            np.float32(w.weight_decay).item(), np.float32(1.0 / w.loss_scale).item())


def _guarded_views(numel, dtype, skew):
    """Per-layer views at odd element offsets inside their allocations, canaries around them."""
    holders, views = [], []
    for i, n in enumerate(numel):
        sk = (1 + i % 3) if skew else 0
        buf = torch.full((n + 2 * GUARD + sk,), 7.0, dtype=dtype, device="cuda")
        holders.append(buf); views.append(buf[GUARD + sk:GUARD + sk + n])
    return holders, views


def _guards_intact(holders, views):
    for h, v in zip(holders, views):
        start = (v.data_ptr() - h.data_ptr()) // h.element_size()
        hv = h.float().cpu().numpy()
        if not (np.all(hv[:start] == 7.0) and np.all(hv[start + v.numel():] == 7.0)):
            return False
    return True


def _prepared(dtype, align, W, inf_variant=False):
    base = wl.RESNET50 if dtype == "f32" else (wl.BERT_LARGE_F16_INF if inf_variant else wl.BERT_LARGE_F16)
    w = wl.scaled(base, f"mix_{dtype}", [(n,) for n in SIZES], W=W)
    task = harness.make_task(w, "cuda", align)
    task.momentum.copy_(wl.make_flat(task.n_bucket, 0.01, 5, device="cuda"))
    mask = torch.ones(task.n_bucket, dtype=torch.bool, device="cuda")
    for n, o in zip(w.numel, task.offsets[:-1]):
        mask[o:o + n] = False
    task.momentum[mask] = 0
    for r in range(W):
        xs.fuse_pack(task.gplan, task.grad_tables[r], task.buckets[r])
    return w, task


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("align", [1, 4, 64])
@pytest.mark.parametrize("W", [1, 2, 3, 8, 16])
@pytest.mark.parametrize("launch", ["default", "beside"])
def test_fused_unpack_matches_oracle_and_separate_unpack(dtype, align, W, launch):
    skew = (align + W) % 2
    print(f"case fused unpack dtype={dtype} align={align} W={W} skew={skew} launch={launch}", flush=True)
    w, task = _prepared(dtype, align, W)
    lr, mu, wd, inv = _hp(w)
    x0, v0 = task.params.clone(), task.momentum.clone()
    old = [xs.tuning_get(k) for k in range(xs.N_TUNING_KEYS)]
    try:
        if launch == "beside":      # 4-wave workgroups, the generic-W kernel
            for k, v in enumerate(xs.tuning_preset(xs.PRESET_BESIDE_COMPUTE)):
                xs.tuning_set(k, v)
        # separate passes
        xb, vb = x0.clone(), v0.clone()
        hb, views_b = _guarded_views(w.numel, torch.float32, skew)
        xs.fused_reduce_sgd(task.buckets, task.n_bucket, xb, vb, w.lr, w.momentum, w.weight_decay, 1.0 / w.loss_scale)
        xs.fuse_unpack(task.pplan, xb, xs.pointer_table(views_b) if views_b else task.param_table)
        # one pass
        xf, vf = x0.clone(), v0.clone()
        hf, views_f = _guarded_views(w.numel, torch.float32, skew)
        xs.fused_reduce_sgd_unpack(task.gplan, task.buckets, xf, vf, xs.pointer_table(views_f), w.lr, w.momentum,
                                   w.weight_decay, 1.0 / w.loss_scale)
        torch.cuda.synchronize()
    finally:
        for k, v in enumerate(old):
            xs.tuning_set(k, v)
    assert torch.equal(xf.view(torch.int32), xb.view(torch.int32))
    assert torch.equal(vf.view(torch.int32), vb.view(torch.int32))
    for a, b in zip(views_f, views_b):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
    assert _guards_intact(hf, views_f)

    grads_host = [[t.cpu().numpy() for t in g] for g in task.grads]
    params_host = [t.cpu().numpy() for t in task.param_tensors]
    v64 = v0.cpu().numpy().astype(np.float64)
    want, found = oracle.sync_step(grads_host, params_host, v64, lr, mu, wd, inv, align=align)
    assert not found
    v32 = v0.cpu().numpy().copy()
    want32, _ = oracle.sync_step(grads_host, params_host, v32, lr, mu, wd, inv, align=align, precision="f32")
    for t, a, b in zip(views_f, want, want32):
        got = t.cpu().numpy()
        assert np.all(np.abs(got - a) <= ATOL32 + RTOL32 * np.abs(a))
        assert np.array_equal(_bits(got), _bits(b))
    gv = vf.cpu().numpy()
    assert np.all(np.abs(gv - v64) <= ATOL32 + RTOL32 * np.abs(v64))
    assert np.array_equal(_bits(gv), _bits(v32))


@pytest.mark.parametrize("view_dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("align", [1, 64])
def test_half_precision_views_and_param_groups(view_dtype, align):
    print(f"case fused unpack half views {view_dtype} align={align} with per-tensor records", flush=True)
    w, task = _prepared("f16", align, 4)
    recs = [(0.1 * (1 + t % 3), 0.9 - 0.1 * (t % 2), 1e-4 * (t % 4)) for t in range(w.n_tensors)]
    table = xs.tensor_hparams_table(recs)
    x0, v0 = task.params.clone(), task.momentum.clone()
    xb, vb = x0.clone(), v0.clone()
    xs.fused_reduce_sgd_pt(task.gplan, task.buckets, xb, vb, table, 1.0 / w.loss_scale)
    xf, vf = x0.clone(), v0.clone()
    hf, views = _guarded_views(w.numel, view_dtype, True)
    copy = torch.zeros(task.n_bucket, dtype=view_dtype, device="cuda")
    xs.fused_reduce_sgd_unpack(task.gplan, task.buckets, xf, vf, xs.pointer_table(views), inv_loss_scale=1.0 / w.loss_scale,
                               tensor_hp=table, view_dtype=view_dtype, model_copy=copy)
    torch.cuda.synchronize()
    assert torch.equal(xf.view(torch.int32), xb.view(torch.int32)) and torch.equal(vf.view(torch.int32), vb.view(torch.int32))
    code = xs.dtype_code(view_dtype)
    want = oracle.round_params(xb.cpu().numpy(), code)            # uint16 bit patterns
    assert np.array_equal(copy.view(torch.int16).cpu().numpy().view(np.uint16), want)
    for t, n, o in zip(views, w.numel, task.offsets[:-1]):
        assert np.array_equal(t.view(torch.int16).cpu().numpy().view(np.uint16), want[o:o + n])
    assert _guards_intact(hf, views)


@pytest.mark.parametrize("name", ["resnet50", "vgg16"])
def test_full_size_workloads(name):
    print(f"case fused unpack full size {name}", flush=True)
    w = {"resnet50": wl.RESNET50, "vgg16": wl.VGG16}[name]
    task = harness.make_task(w, "cuda")
    task.momentum.copy_(wl.make_flat(task.n_bucket, 0.01, 5, device="cuda"))
    xs.fuse_pack_many(task.gplan, task.grad_tables, task.buckets)
    x0, v0 = task.params.clone(), task.momentum.clone()
    xs.fused_reduce_sgd(task.buckets, task.n_bucket, x0, v0, w.lr, w.momentum, w.weight_decay, 1.0)
    views = [torch.full_like(t, 3.0) for t in task.param_tensors]
    xs.fused_reduce_sgd_unpack(task.gplan, task.buckets, task.params, task.momentum, xs.pointer_table(views),
                               w.lr, w.momentum, w.weight_decay, 1.0)
    torch.cuda.synchronize()
    assert torch.equal(task.params.view(torch.int32), x0.view(torch.int32))
    assert torch.equal(task.momentum.view(torch.int32), v0.view(torch.int32))
    for t, n, o in zip(views, w.numel, task.offsets[:-1]):
        assert torch.equal(t.view(-1).view(torch.int32), x0[o:o + n].view(torch.int32))


def test_app_with_fused_unpack_and_overflow_skip():
    print("case fused unpack through xs_app, then the overflow skip", flush=True)
    w, task = _prepared("f16", 8, 4, inf_variant=True)
    w2, ref = _prepared("f16", 8, 4, inf_variant=True)
    a = task.make_app(fused_unpack=True, use_found_inf=True)
    b = ref.make_app(use_found_inf=True)
    # the "_inf" workload has non-finite gradients in replica 0: both apps must skip the step
    p0 = [t.clone() for t in task.param_tensors]
    a.sync(); b.sync(); torch.cuda.synchronize()
    assert int(task.found_inf.item()) == 1 and int(ref.found_inf.item()) == 1
    for t, u, v in zip(task.param_tensors, ref.param_tensors, p0):
        assert torch.equal(t, u) and torch.equal(t, v)
    # finite gradients and a cleared flag: both apply the same step
    for t_ in (task, ref):
        for g in t_.grads[0]:
            g.nan_to_num_(posinf=0.5, neginf=-0.5, nan=0.0)
        t_.found_inf.zero_()
    a.sync(); b.sync(); torch.cuda.synchronize()
    assert int(task.found_inf.item()) == 0
    assert torch.equal(task.params.view(torch.int32), ref.params.view(torch.int32))
    changed = False
    for t, u, v in zip(task.param_tensors, ref.param_tensors, p0):
        assert torch.equal(t.view(torch.int32) if t.numel() else t, u.view(torch.int32) if u.numel() else u)
        changed = changed or (t.numel() > 0 and not torch.equal(t, v))
    assert changed
    a.destroy(); b.destroy()


def test_argument_errors():
    w, task = _prepared("f32", 4, 2)
    x, v = task.params, task.momentum
    xo, vo = torch.empty_like(x), torch.empty_like(v)
    L = xs.lib()
    import ctypes
    arr = (ctypes.c_void_p * 2)(*[b.data_ptr() for b in task.buckets])
    hp = xs.SgdHparams(0.1, 0.9, 0.0, 1.0)
    # views need the in-place form: the generic checked path refuses out-of-place + views
    rc = L.xs_fused_reduce_sgd_unpack(task.gplan.handle, arr, 2, x.data_ptr(), v.data_ptr(), None,
                                      ctypes.byref(hp), None, None, None, None)
    assert rc == xs.XS_ERR_INVALID_ARG and "param_tensor_ptrs" in xs.last_error()
    rc = L.xs_fused_reduce_sgd_unpack(None, arr, 2, x.data_ptr(), v.data_ptr(), task.param_table.data_ptr(),
                                      ctypes.byref(hp), None, None, None, None)
    assert rc == xs.XS_ERR_INVALID_ARG
    rc = L.xs_fused_reduce_sgd_unpack(task.gplan.handle, arr, 2, x.data_ptr(), v.data_ptr(), task.param_table.data_ptr(),
                                      None, None, None, None, None)
    assert rc == xs.XS_ERR_INVALID_ARG
    with pytest.raises(xs.XsError):
        xs.App(task.gplan, task.pplan, task.grad_tables, task.buckets, x, v, task.param_table, 0.1, 0.9, 0.0,
               gather_table=task.gather_table, W=2, fused_unpack=True)
