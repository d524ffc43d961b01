"""Parity of xs_fused_reduce_sgd with the oracle, element by element, through the C-ABI.

Tolerances (fp32 gradients: 1e-6 relative + 1e-7 absolute; fp16 gradients into fp32
master weights: 2e-3 relative) are against the oracle's double-precision definition.
The single-precision evaluation of the same steps is compared bit for bit as well: the
kernel adds replicas in worker order and rounds every operation separately, so the
distance is expected to be zero units in the last place.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2103_07974_amd import workloads as wl
from paper_2103_07974_amd import xs

pytestmark = pytest.mark.gpu

RTOL32, ATOL32 = 1e-6, 1e-7
RTOL16 = 2e-3

LR, MU, WD = np.float32(0.1), np.float32(0.9), np.float32(1e-4)


def _make(n, W, dtype, seed, gstd=1e-3):
    reps = [wl.make_flat(n, gstd, seed + 1 + w, dtype) for w in range(W)]
    x = wl.make_flat(n, 0.05, seed, torch.float32)
    v = wl.make_flat(n, 0.01, seed + 500, torch.float32)
    return reps, x, v


def _oracle(reps_np, x_np, v_np, inv=1.0, lr=LR, mu=MU, wd=WD):
    x64 = x_np.astype(np.float64); v64 = v_np.astype(np.float64)
    oracle.reduce_sgd_f64(reps_np, x64, v64, float(lr), float(mu), float(wd), float(np.float32(inv)))
    x32 = x_np.copy(); v32 = v_np.copy()
    oracle.reduce_sgd_f32(reps_np, x32, v32, float(lr), float(mu), float(wd), float(np.float32(inv)))
    return x64, v64, x32, v32


def _assert_close(got, want64, f16):
    # half-precision gradients are widened exactly and everything after that is fp32, so
    # the fp32 bar holds for them too; the 2e-3 relative bar is checked where a relative
    # error is meaningful (away from results that happen to land next to zero)
    err = np.abs(got.astype(np.float64) - want64)
    bad = err > ATOL32 + RTOL32 * np.abs(want64)
    assert not bad.any(), f"{bad.sum()} elements out of tolerance, worst {err.max():.3e}"
    if f16:
        big = np.abs(want64) > 1e-4
        assert np.all(err[big] <= RTOL16 * np.abs(want64[big]))


def _ulp_distance(a, b):
    ia = a.view(np.int32).astype(np.int64); ib = b.view(np.int32).astype(np.int64)
    ia = np.where(ia < 0, np.int64(-2 ** 31) - ia, ia)
    ib = np.where(ib < 0, np.int64(-2 ** 31) - ib, ib)
    return int(np.abs(ia - ib).max()) if a.size else 0


def _run(reps, x, v, inv=1.0, out_of_place=False, flag=None, n=None):
    dev = [r.cuda() for r in reps]
    xd, vd = x.cuda(), v.cuda()
    n = x.numel() if n is None else n
    if out_of_place:
        xo = torch.full_like(xd, 9.0); vo = torch.full_like(vd, 9.0)
        xs.fused_reduce_sgd(dev, n, xd, vd, float(LR), float(MU), float(WD), inv, xo, vo, flag)
        torch.cuda.synchronize()
        assert torch.equal(xd.cpu(), x) and torch.equal(vd.cpu(), v)     # inputs untouched
        return xo.cpu().numpy(), vo.cpu().numpy()
    xs.fused_reduce_sgd(dev, n, xd, vd, float(LR), float(MU), float(WD), inv, None, None, flag)
    torch.cuda.synchronize()
    return xd.cpu().numpy(), vd.cpu().numpy()


# sizes: empty tail, pure tail, one vector, ragged, several workgroups, more than one
# grid-stride trip at a capped launch shape (see test_launch_shapes_give_identical_results)
SIZES = [1, 3, 4, 5, 7, 8, 9, 1023, 1024, 1025, 100003, 2 * 1024 * 1024 + 5, 9 * 1024 * 1024 + 3]


@pytest.mark.parametrize("W", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
def test_specialised_W_all_sizes(W, dtype):
    f16 = dtype == torch.float16
    inv = 1.0 / 1024 if f16 else 1.0
    for n in SIZES:
        if n > 3 * 1024 * 1024 and W not in (8, 16):
            continue
        print(f"case W={W} dtype={dtype} n={n}", flush=True)
        reps, x, v = _make(n, W, dtype, seed=1000 + n % 97 + W)
        x64, v64, x32, v32 = _oracle([r.numpy() for r in reps], x.numpy(), v.numpy(), inv)
        gx, gv = _run(reps, x, v, inv)
        _assert_close(gx, x64, f16); _assert_close(gv, v64, f16)
        assert _ulp_distance(gx, x32) == 0 and _ulp_distance(gv, v32) == 0


@pytest.mark.parametrize("W", [3, 5, 7, 13, 32])
@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
def test_any_W(W, dtype):
    f16 = dtype == torch.float16
    for n in [1, 6, 8, 1025, 300007]:
        print(f"case W={W} dtype={dtype} n={n}", flush=True)
        reps, x, v = _make(n, W, dtype, seed=2000 + n % 89 + W)
        x64, v64, x32, v32 = _oracle([r.numpy() for r in reps], x.numpy(), v.numpy())
        for oop in (False, True):
            gx, gv = _run(reps, x, v, 1.0, out_of_place=oop)
            _assert_close(gx, x64, f16); _assert_close(gv, v64, f16)
            assert _ulp_distance(gx, x32) == 0 and _ulp_distance(gv, v32) == 0


@pytest.mark.parametrize("wg_per_cu,lds", [(0, -1), (0, 0), (1, 0), (8, 8192), (32, 16384)])
@pytest.mark.parametrize("nt_grads,nt_state", [(0, 0), (1, 0), (1, 1), (0, 1)])
def test_launch_shapes_give_identical_results(wg_per_cu, lds, nt_grads, nt_state):
    old = [xs.tuning_get(k) for k in range(xs.N_TUNING_KEYS)]
    try:
        xs.tuning_set(xs.TUNE_REDUCE_WG_PER_CU, wg_per_cu)
        xs.tuning_set(xs.TUNE_REDUCE_LDS_RESERVE, lds)
        xs.tuning_set(xs.TUNE_NT_GRADS, nt_grads)
        xs.tuning_set(xs.TUNE_NT_STATE, nt_state)
        n = 3 * 1024 * 1024 + 1
        for dtype in (torch.float32, torch.float16):
            reps, x, v = _make(n, 8, dtype, seed=3000)
            _, _, x32, v32 = _oracle([r.numpy() for r in reps], x.numpy(), v.numpy())
            gx, gv = _run(reps, x, v)
            assert _ulp_distance(gx, x32) == 0 and _ulp_distance(gv, v32) == 0
    finally:
        for k, val in enumerate(old):
            xs.tuning_set(k, val)


def test_out_of_place_equals_in_place_and_leaves_inputs():
    reps, x, v = _make(70001, 8, torch.float32, seed=4000)
    a = _run(reps, x, v)
    b = _run(reps, x, v, out_of_place=True)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_identical_replicas_may_alias():
    n = 50000
    g = wl.make_flat(n, 1.0, 4100, torch.float16).float()       # 11 significant bits: sums exact
    x = torch.zeros(n); v = torch.zeros(n)
    gd = g.cuda(); xd = x.cuda(); vd = v.cuda()
    xs.fused_reduce_sgd([gd] * 8, n, xd, vd, 1.0, 0.0, 0.0)
    torch.cuda.synchronize()
    assert torch.equal(vd.cpu(), g) and torch.equal(xd.cpu(), -g)


def test_repeat_runs_are_bit_identical():
    reps, x, v = _make(1 << 20, 8, torch.float32, seed=4200)
    first = _run(reps, x, v)
    for _ in range(3):
        again = _run(reps, x, v)
        assert np.array_equal(first[0], again[0]) and np.array_equal(first[1], again[1])


def test_several_steps_track_the_oracle():
    n, W, K = 200003, 4, 5
    x = wl.make_flat(n, 0.05, 4300)
    xd = x.cuda(); vd = torch.zeros(n, device="cuda")
    x64 = x.numpy().astype(np.float64); v64 = np.zeros(n)
    x32 = x.numpy().copy(); v32 = np.zeros(n, np.float32)
    for k in range(K):
        reps = [wl.make_flat(n, 1e-3, 4301 + 10 * k + w) for w in range(W)]
        xs.fused_reduce_sgd([r.cuda() for r in reps], n, xd, vd, float(LR), float(MU), float(WD))
        rn = [r.numpy() for r in reps]
        oracle.reduce_sgd_f64(rn, x64, v64, float(LR), float(MU), float(WD))
        oracle.reduce_sgd_f32(rn, x32, v32, float(LR), float(MU), float(WD))
    torch.cuda.synchronize()
    gx, gv = xd.cpu().numpy(), vd.cpu().numpy()
    assert np.array_equal(gx, x32) and np.array_equal(gv, v32)
    assert np.all(np.abs(gx - x64) <= K * (ATOL32 + RTOL32 * np.abs(x64)))
    assert np.all(np.abs(gv - v64) <= K * (ATOL32 + RTOL32 * np.abs(v64)))


# ---------------------------------------------------------------- overflow skip
@pytest.mark.parametrize("dtype", [torch.float16, torch.float32])
def test_preset_flag_skips_the_whole_step(dtype):
    reps, x, v = _make(100003, 4, dtype, seed=5000)
    flag = torch.ones(1, dtype=torch.int32, device="cuda")
    gx, gv = _run(reps, x, v, flag=flag)
    assert np.array_equal(gx, x.numpy()) and np.array_equal(gv, v.numpy())
    ox, ov = _run(reps, x, v, out_of_place=True, flag=flag)
    assert np.all(ox == 9.0) and np.all(ov == 9.0)          # nothing written
    assert int(flag.item()) == 1


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32])
@pytest.mark.parametrize("bad", [float("inf"), float("-inf"), float("nan")])
def test_out_of_place_detects_nonfinite_gradients(dtype, bad):
    n = 100003
    for W, w_bad, pos in [(4, 0, 0), (4, 3, 51234), (4, 1, n - 1), (16, 15, n - 2), (5, 2, 77)]:
        reps, x, v = _make(n, W, dtype, seed=5100)
        reps[w_bad][pos] = bad
        flag = torch.zeros(1, dtype=torch.int32, device="cuda")
        _run(reps, x, v, out_of_place=True, flag=flag)
        assert int(flag.item()) == 1, (W, w_bad, pos)
    reps, x, v = _make(n, 4, dtype, seed=5100)
    reps[0][:2] = torch.tensor([torch.finfo(dtype).max, -torch.finfo(dtype).max], dtype=dtype)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    _run(reps, x, v, out_of_place=True, flag=flag)
    assert int(flag.item()) == 0


def test_in_place_with_clean_flag_updates_and_keeps_flag():
    reps, x, v = _make(5001, 2, torch.float16, seed=5200)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    gx, gv = _run(reps, x, v, inv=1 / 1024, flag=flag)
    x64, v64, x32, v32 = _oracle([r.numpy() for r in reps], x.numpy(), v.numpy(), 1 / 1024)
    assert np.array_equal(gx, x32) and np.array_equal(gv, v32)
    assert int(flag.item()) == 0


def test_n_elems_smaller_than_buffers_touches_only_the_prefix():
    reps, x, v = _make(10000, 2, torch.float32, seed=5300)
    gx, gv = _run(reps, x, v, n=4999)
    assert np.array_equal(gx[4999:], x.numpy()[4999:]) and np.array_equal(gv[4999:], v.numpy()[4999:])
    _, _, x32, v32 = _oracle([r.numpy()[:4999].copy() for r in reps], x.numpy()[:4999].copy(),
                             v.numpy()[:4999].copy())
    assert np.array_equal(gx[:4999], x32) and np.array_equal(gv[:4999], v32)


def test_device_errors_are_reported_not_raised_by_hip():
    x = torch.zeros(16, device="cuda"); v = torch.zeros(16, device="cuda")
    g = torch.zeros(16, device="cuda")
    with pytest.raises(xs.XsError) as e:
        xs.fused_reduce_sgd([g, x], 16, x, v, 0.1, 0.9, 0.0)       # replica aliases params
    assert e.value.status == xs.XS_ERR_INVALID_ARG
    with pytest.raises(xs.XsError) as e:
        xs.fused_reduce_sgd([g[1:]], 8, x, v, 0.1, 0.9, 0.0)       # misaligned replica
    assert e.value.status == xs.XS_ERR_ALIGNMENT


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
def test_subnormal_values_are_not_flushed(dtype):
    """Gradients, parameters and momentum in and around the fp32 subnormal range (and fp16
    subnormal gradients): the kernel keeps IEEE gradual underflow, like the oracle."""
    n, W = 4099, 4
    g = torch.Generator(); g.manual_seed(77)
    if dtype == torch.float16:
        reps = [(torch.randn(n, generator=g) * 3e-6).to(torch.float16) for _ in range(W)]   # below 6.1e-5
        inv = 2.0 ** -100
    else:
        reps = [torch.randn(n, generator=g) * 1e-39 for _ in range(W)]
        inv = 1.0
    assert all((r != 0).any() for r in reps)
    x = torch.randn(n, generator=g) * 1e-38
    v = torch.randn(n, generator=g) * 1e-39
    x64, v64, x32, v32 = _oracle([r.numpy() for r in reps], x.numpy(), v.numpy(), inv)
    gx, gv = _run(reps, x, v, inv)
    tiny = np.finfo(np.float32).tiny
    assert (np.abs(x32) < tiny).any() and (np.abs(v32) < tiny).any() and (x32 != 0).all()
    assert _ulp_distance(gx, x32) == 0 and _ulp_distance(gv, v32) == 0
