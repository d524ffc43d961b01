"""Parity of the per-tensor hyper-parameter entry points (xs_fused_reduce_sgd_pt,
xs_fused_gather_reduce_sgd_pt, xs_app_desc.tensor_hp) with the oracle's per-tensor update,
element by element through the C-ABI: fp32 bar against the double-precision definition,
zero units in the last place against its single-precision evaluation."""
import numpy as np
import pytest
import torch

import oracle
from paper_2103_07974_amd import harness, workloads as wl, xs

pytestmark = pytest.mark.gpu

RTOL32, ATOL32 = 1e-6, 1e-7
RTOL16 = 2e-3
# tensors smaller than a vector, smaller than a row, ragged, empty, several rows
SIZES = [0, 1, 3, 5, 17, 63, 64, 65, 255, 256, 257, 4095, 4096, 4097, 12289, 50001, 2, 0, 70000]
GROUPS = [(0.1, 0.9, 1e-4), (0.05, 0.0, 0.0), (0.2, 0.5, 1e-2), (0.0, 0.9, 0.0)]


def _f32(x):
    return float(np.float32(x))


def _triples(n_tensors):
    return [tuple(_f32(c) for c in GROUPS[(t * 7 + t // 3) % len(GROUPS)]) for t in range(n_tensors)]


def _np(t):
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def _ulp_distance(a, b):
    ia = a.view(np.int32).astype(np.int64); ib = b.view(np.int32).astype(np.int64)
    ia = np.where(ia < 0, np.int64(-2 ** 31) - ia, ia)
    ib = np.where(ib < 0, np.int64(-2 ** 31) - ib, ib)
    return int(np.abs(ia - ib).max()) if a.size else 0


def _assert_close(got, want64, half):
    err = np.abs(got.astype(np.float64) - want64)
    bad = err > ATOL32 + RTOL32 * np.abs(want64)
    assert not bad.any(), f"{bad.sum()} elements out of tolerance, worst {err.max():.3e}"
    if half:
        big = np.abs(want64) > 1e-4
        assert np.all(err[big] <= RTOL16 * np.abs(want64[big]))


def _oracle_step(task, buckets_np, x_np, v_np, triples, inv):
    offs = np.asarray(task.offsets, dtype=np.uint64)
    x64 = x_np.astype(np.float64); v64 = v_np.astype(np.float64)
    oracle.reduce_sgd_per_tensor(buckets_np, x64, v64, offs, triples, _f32(inv))
    x32 = x_np.copy(); v32 = v_np.copy()
    oracle.reduce_sgd_per_tensor(buckets_np, x32, v32, offs, triples, _f32(inv))
    return x64, v64, x32, v32


def _random_state(task, seed):
    """Parameters and momentum with non-zero values in the padding too, so that the rule
    'padding follows the tensor in front of it' is visible in the result."""
    x = wl.make_flat(task.n_bucket, 0.05, seed, device="cuda")
    v = wl.make_flat(task.n_bucket, 0.01, seed + 1, device="cuda")
    return x, v


# bf16 shares every code path with f16 but the widening, so it runs a subset of the grid
CASES = [(d, a, W) for d in ("f32", "f16", "bf16") for a in (1, 4, 64) for W in (1, 2, 3, 8, 16)
         if not (d == "bf16" and (a == 4 or W in (1, 3)))]


@pytest.mark.parametrize("dtype,align,W", CASES)
def test_bucket_and_gather_forms_match_oracle(dtype, align, W):
    base = wl.RESNET50 if dtype == "f32" else wl.BERT_LARGE_F16
    w = wl.scaled(base, f"pt_{dtype}", [(n,) for n in SIZES], W=W, grad_dtype=dtype)
    print(f"case dtype={dtype} align={align} W={W}", flush=True)
    task = harness.make_task(w, "cuda", align)
    inv = 1.0 / w.loss_scale
    triples = _triples(w.n_tensors)
    table = xs.tensor_hparams_table(triples)
    x0, v0 = _random_state(task, 40 + W)
    xs.fuse_pack_many(task.gplan, task.grad_tables, task.buckets)
    torch.cuda.synchronize()
    want = _oracle_step(task, [_np(b) for b in task.buckets], x0.cpu().numpy(), v0.cpu().numpy(),
                        triples, inv)
    half = dtype != "f32"

    # bucket form, in place and out of place
    xb, vb = x0.clone(), v0.clone()
    xs.fused_reduce_sgd_pt(task.gplan, task.buckets, xb, vb, table, inv)
    xo, vo = torch.full_like(x0, 9.0), torch.full_like(v0, 9.0)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    xs.fused_reduce_sgd_pt(task.gplan, task.buckets, x0, v0, table, inv, params_out=xo,
                           momentum_out=vo, found_inf=flag)
    torch.cuda.synchronize()
    assert flag.item() == 0
    for gx, gv in ((xb, vb), (xo, vo)):
        gx, gv = gx.cpu().numpy(), gv.cpu().numpy()
        _assert_close(gx, want[0], half); _assert_close(gv, want[1], half)
        assert _ulp_distance(gx, want[2]) == 0 and _ulp_distance(gv, want[3]) == 0

    # gathering form, in place with views: bit-identical to the bucket form
    xg, vg = x0.clone(), v0.clone()
    views = [torch.full_like(p, 7.0) for p in task.param_tensors]
    ptab = xs.pointer_table(views) if views else xs.pointer_table([task.params])
    xs.fused_gather_reduce_sgd_pt(task.gplan, task.gather_table, W, xg, vg, table, inv,
                                  param_tensor_ptrs=ptab)
    torch.cuda.synchronize()
    assert torch.equal(xg, xb) and torch.equal(vg, vb)
    for t, (n, o) in enumerate(zip(w.numel, task.offsets[:-1])):
        assert torch.equal(views[t].reshape(-1), xb[o:o + n]), t


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("W", [2, 5, 8])
def test_equal_records_equal_the_single_triple_call(dtype, W):
    base = wl.RESNET50 if dtype == "f32" else wl.BERT_LARGE_F16
    w = wl.scaled(base, f"pt_same_{dtype}", [(n,) for n in SIZES], W=W)
    task = harness.make_task(w, "cuda", 64)
    inv = 1.0 / w.loss_scale
    x0, v0 = _random_state(task, 60)
    xs.fuse_pack_many(task.gplan, task.grad_tables, task.buckets)
    table = xs.tensor_hparams_table([(w.lr, w.momentum, w.weight_decay)] * w.n_tensors)
    xa, va = x0.clone(), v0.clone()
    xs.fused_reduce_sgd(task.buckets, task.n_bucket, xa, va, w.lr, w.momentum, w.weight_decay, inv)
    xb, vb = x0.clone(), v0.clone()
    xs.fused_reduce_sgd_pt(task.gplan, task.buckets, xb, vb, table, inv)
    xc, vc = x0.clone(), v0.clone()
    xs.fused_gather_reduce_sgd_pt(task.gplan, task.gather_table, W, xc, vc, table, inv)
    torch.cuda.synchronize()
    assert torch.equal(xa, xb) and torch.equal(va, vb)
    assert torch.equal(xa, xc) and torch.equal(va, vc)


def test_model_copy_and_half_views_with_records():
    w = wl.scaled(wl.BERT_LARGE_F16, "pt_mp", [(n,) for n in SIZES], W=4)
    task = harness.make_task(w, "cuda", 64)
    inv = 1.0 / w.loss_scale
    triples = _triples(w.n_tensors)
    table = xs.tensor_hparams_table(triples)
    x0, v0 = _random_state(task, 70)
    xs.fuse_pack_many(task.gplan, task.grad_tables, task.buckets)
    xb, vb = x0.clone(), v0.clone()
    copy16 = torch.zeros(task.n_bucket, dtype=torch.float16, device="cuda")
    xs.fused_reduce_sgd_pt(task.gplan, task.buckets, xb, vb, table, inv, model_copy=copy16)
    xg, vg = x0.clone(), v0.clone()
    views = [torch.zeros(n, dtype=torch.bfloat16, device="cuda") for n in w.numel]
    xs.fused_gather_reduce_sgd_pt(task.gplan, task.gather_table, w.W, xg, vg, table, inv,
                                  param_tensor_ptrs=xs.pointer_table(views),
                                  view_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert torch.equal(xg, xb) and torch.equal(vg, vb)
    xh = np.ascontiguousarray(xb.cpu().numpy())
    assert np.array_equal(copy16.cpu().numpy().view(np.uint16), oracle.round_params(xh, oracle.F16))
    want_bf16 = oracle.round_params(xh, oracle.BF16)
    for t, (n, o) in enumerate(zip(w.numel, task.offsets[:-1])):
        assert np.array_equal(_np(views[t]), want_bf16[o:o + n]), t


def _layer_kind_triples(w):
    """The usual recipe: weight decay on matrices and filters only, none on biases and
    normalisation parameters (one-dimensional tensors), which also get their own lr."""
    return [(_f32(w.lr), _f32(w.momentum), _f32(w.weight_decay)) if len(s) > 1
            else (_f32(2 * w.lr), _f32(w.momentum), 0.0) for s in w.shapes]


@pytest.mark.parametrize("name", ["resnet50", "vgg16"])
def test_full_size_sets_with_layer_kind_groups(name):
    w = wl.WORKLOADS[name]
    task = harness.make_task(w, "cuda")
    triples = _layer_kind_triples(w)
    table = xs.tensor_hparams_table(triples)
    x0 = task.params.clone()
    v0 = wl.make_flat(task.n_bucket, 0.01, 81, device="cuda")
    xs.fuse_pack_many(task.gplan, task.grad_tables, task.buckets)
    torch.cuda.synchronize()
    x32 = x0.cpu().numpy().copy(); v32 = v0.cpu().numpy().copy()
    oracle.reduce_sgd_per_tensor([b.cpu().numpy() for b in task.buckets], x32, v32,
                                 np.asarray(task.offsets, dtype=np.uint64), triples, 1.0)
    xb, vb = x0.clone(), v0.clone()
    xs.fused_reduce_sgd_pt(task.gplan, task.buckets, xb, vb, table, 1.0)
    xg, vg = x0.clone(), v0.clone()
    xs.fused_gather_reduce_sgd_pt(task.gplan, task.gather_table, w.W, xg, vg, table, 1.0,
                                  param_tensor_ptrs=task.param_table)
    torch.cuda.synchronize()
    assert _ulp_distance(xb.cpu().numpy(), x32) == 0 and _ulp_distance(vb.cpu().numpy(), v32) == 0
    assert torch.equal(xg, xb) and torch.equal(vg, vb)
    for t in (0, 1, w.n_tensors // 2, w.n_tensors - 1):
        o, n = task.offsets[t], w.numel[t]
        assert torch.equal(task.param_tensors[t].reshape(-1), xb[o:o + n])


@pytest.mark.parametrize("fused_gather", [False, True])
def test_app_with_records_matches_direct_calls(fused_gather):
    w = wl.scaled(wl.RESNET50, "pt_app", [(n,) for n in SIZES], W=4)
    task = harness.make_task(w, "cuda", 64)
    triples = _triples(w.n_tensors)
    table = xs.tensor_hparams_table(triples)
    x0, v0 = task.params.clone(), task.momentum.clone()
    app = task.make_app(fused_gather=fused_gather, tensor_hp=table)
    s = torch.cuda.Stream()
    app.sync(s)
    s.synchronize()
    xs.fuse_pack_many(task.gplan, task.grad_tables, task.buckets)
    xs.fused_reduce_sgd_pt(task.gplan, task.buckets, x0, v0, table, 1.0 / w.loss_scale)
    torch.cuda.synchronize()
    assert torch.equal(task.params, x0) and torch.equal(task.momentum, v0)
    for t, (n, o) in enumerate(zip(w.numel, task.offsets[:-1])):
        assert torch.equal(task.param_tensors[t].reshape(-1), x0[o:o + n]), t
    app.destroy()


def test_overflow_skip_with_records():
    w = wl.scaled(wl.BERT_LARGE_F16_INF, "pt_inf", [(n,) for n in SIZES], W=4)
    task = harness.make_task(w, "cuda", 64)
    table = xs.tensor_hparams_table(_triples(w.n_tensors))
    x0, v0 = _random_state(task, 90)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    xs.fuse_pack_many(task.gplan, task.grad_tables, task.buckets, flag)
    xb, vb = x0.clone(), v0.clone()
    xs.fused_reduce_sgd_pt(task.gplan, task.buckets, xb, vb, table, 1.0 / w.loss_scale,
                           found_inf=flag)
    torch.cuda.synchronize()
    assert flag.item() == 1
    assert torch.equal(xb, x0) and torch.equal(vb, v0)
    # in-kernel detection of the out-of-place gathering form
    flag2 = torch.zeros(1, dtype=torch.int32, device="cuda")
    xo, vo = torch.empty_like(x0), torch.empty_like(v0)
    xs.fused_gather_reduce_sgd_pt(task.gplan, task.gather_table, w.W, x0, v0, table,
                                  1.0 / w.loss_scale, params_out=xo, momentum_out=vo,
                                  found_inf=flag2)
    torch.cuda.synchronize()
    assert flag2.item() == 1


def test_argument_errors():
    w = wl.scaled(wl.RESNET50, "pt_err", [(100,), (28,)], W=2)
    task = harness.make_task(w, "cuda", 64)
    table = xs.tensor_hparams_table(_triples(2))
    with pytest.raises(xs.XsError) as e:
        xs.fused_reduce_sgd_pt(task.gplan, task.buckets, task.params, task.momentum, None)
    assert e.value.status == xs.XS_ERR_INVALID_ARG
    with pytest.raises(xs.XsError) as e:
        xs.fused_gather_reduce_sgd_pt(task.gplan, task.gather_table, 2, task.params, task.momentum, None)
    assert e.value.status == xs.XS_ERR_INVALID_ARG
    skew = torch.zeros(12, dtype=torch.float32, device="cuda")[1:9]
    with pytest.raises(xs.XsError) as e:
        xs.fused_reduce_sgd_pt(task.gplan, task.buckets, task.params, task.momentum, skew)
    assert e.value.status == xs.XS_ERR_ALIGNMENT
    with pytest.raises(xs.XsError) as e:
        xs.fused_gather_reduce_sgd_pt(task.gplan, task.gather_table, 2, task.params, task.momentum, skew)
    assert e.value.status == xs.XS_ERR_ALIGNMENT
    # a table inside the parameter bucket would be overwritten while it is read
    inside = task.params[:8]
    with pytest.raises(xs.XsError) as e:
        xs.fused_reduce_sgd_pt(task.gplan, task.buckets, task.params, task.momentum, inside)
    assert e.value.status == xs.XS_ERR_INVALID_ARG
    # an empty plan is a no-op whatever else is passed
    empty = xs.Plan([], [0], torch.float32)
    xs.fused_reduce_sgd_pt(empty, [], None, None, None)
    torch.cuda.synchronize()
    del table
