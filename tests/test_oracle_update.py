"""Pins for the oracle's average + momentum-SGD step (Algorithm 1, "Receive averaged
gradients" and "Model Update") and for the overflow skip of the mixed-precision workload."""
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import brute

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sgd_pow2_worked.txt")


def _const(n, c, dtype=np.float32):
    return np.full(n, c, dtype=dtype)


# ------------------------------------------------------------------ averaging
@pytest.mark.parametrize("W", [1, 2, 4, 8, 16])
def test_identical_replicas_average_to_the_replica(W):
    # values with 11 significant bits: W-fold sums are exact in single for W <= 8192
    rng = np.random.default_rng(3)
    g = rng.standard_normal(1000).astype(np.float16).astype(np.float32)
    for prec, dt in (("f64", np.float64), ("f32", np.float32)):
        x = np.zeros(1000, dt); v = np.zeros(1000, dt)
        f = oracle.reduce_sgd_f64 if prec == "f64" else oracle.reduce_sgd_f32
        f([g] * W, x, v, lr=1.0, mu=0.0, wd=0.0)
        # x0 = 0, v0 = 0, lr = 1, mu = 0  =>  v = g_avg, x = -g_avg
        assert np.array_equal(v, g.astype(dt))
        assert np.array_equal(x, -g.astype(dt))


def test_identical_replicas_arbitrary_values_within_bound():
    rng = np.random.default_rng(4)
    g = (rng.standard_normal(5000) * 1e-3).astype(np.float32)
    W = 8
    x = np.zeros(5000, np.float32); v = np.zeros(5000, np.float32)
    oracle.reduce_sgd_f32([g] * W, x, v, 1.0, 0.0, 0.0)
    assert np.all(np.abs(v - g) <= (W - 1) * 2.0 ** -24 * np.abs(g))
    xd = np.zeros(5000); vd = np.zeros(5000)
    oracle.reduce_sgd_f64([g] * W, xd, vd, 1.0, 0.0, 0.0)
    assert np.array_equal(vd, g.astype(np.float64))        # W*g/W is exact in double


@pytest.mark.parametrize("W", [2, 3, 5, 8, 16])
def test_integer_replicas_sum_exactly(W):
    rng = np.random.default_rng(5)
    ints = rng.integers(-1024, 1025, size=(W, 777))
    reps = [row.astype(np.float32) for row in ints]
    total = ints.sum(axis=0)                               # exact integer arithmetic
    # lr = 1, mu = 0, wd = 0, x0 = 0  =>  -x * W = sum (W * 2^10 < 2^24: exact in single)
    x = np.zeros(777); v = np.zeros(777)
    oracle.reduce_sgd_f64(reps, x, v, 1.0, 0.0, 0.0)
    assert np.allclose(-x * W, total, rtol=0, atol=1e-9)
    xs = np.zeros(777, np.float32); vs = np.zeros(777, np.float32)
    oracle.reduce_sgd_f32(reps, xs, vs, 1.0, 0.0, 0.0)
    if W & (W - 1) == 0:
        assert np.array_equal(-xs.astype(np.float64) * W, total.astype(np.float64))
    else:
        assert np.allclose(-xs.astype(np.float64) * W, total, rtol=2.0 ** -22, atol=0)


def test_replica_order_and_distinct_replicas_are_all_used():
    # each replica contributes once: one-hot replicas pick out 1/W each
    W, n = 4, 8
    for hot in range(W):
        reps = [np.zeros(n, np.float32) for _ in range(W)]
        reps[hot][:] = 4.0
        x = np.zeros(n); v = np.zeros(n)
        oracle.reduce_sgd_f64(reps, x, v, 1.0, 0.0, 0.0)
        assert np.array_equal(v, np.full(n, 1.0))


def test_single_vs_double_bound_on_random_replicas():
    rng = np.random.default_rng(6)
    W, n = 8, 20000
    reps = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(W)]
    xs = np.zeros(n, np.float32); vs = np.zeros(n, np.float32)
    xd = np.zeros(n); vd = np.zeros(n)
    oracle.reduce_sgd_f32(reps, xs, vs, 1.0, 0.0, 0.0)
    oracle.reduce_sgd_f64(reps, xd, vd, 1.0, 0.0, 0.0)
    sabs = np.sum([np.abs(r.astype(np.float64)) for r in reps], axis=0) / W
    assert np.all(np.abs(vs - vd) <= W * 2.0 ** -24 * sabs)


# ------------------------------------------------------------------ update: closed forms
@pytest.mark.parametrize("prec", ["f64", "f32"])
def test_golden_worked_trajectories(prec):
    cases = {"A": dict(g=(0.25, 0.75), dt=np.float32, lr=0.5, mu=0.5, wd=0.0, inv=1.0, x0=1.0),
             "B": dict(g=(0.25, 0.75), dt=np.float32, lr=0.5, mu=0.5, wd=0.25, inv=1.0, x0=1.0),
             "C": dict(g=(512.0, 1536.0), dt=np.float16, lr=0.25, mu=0.5, wd=0.0,
                       inv=1.0 / 1024, x0=2.0)}
    rows = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        c, k, x, v = line.split()
        rows.setdefault(c, []).append((int(k), float(x), float(v)))
    assert set(rows) == set(cases)
    wdt = np.float64 if prec == "f64" else np.float32
    f = oracle.reduce_sgd_f64 if prec == "f64" else oracle.reduce_sgd_f32
    for c, p in cases.items():
        n = 5
        reps = [_const(n, gv, p["dt"]) for gv in p["g"]]
        x = np.full(n, p["x0"], wdt); v = np.zeros(n, wdt)
        for k, xk, vk in rows[c]:
            f(reps, x, v, p["lr"], p["mu"], p["wd"], p["inv"])
            assert np.all(x == xk) and np.all(v == vk), (c, k, x[0], v[0])


def test_constant_gradient_closed_form_no_decay():
    c, lr, mu, x0, K = 0.3, 0.1, 0.9, 1.5, 25
    reps = [_const(4, c * 0.5, np.float64).astype(np.float32),
            _const(4, c * 1.5, np.float64).astype(np.float32)]
    cbar = (float(reps[0][0]) + float(reps[1][0])) / 2
    x = np.full(4, x0); v = np.zeros(4)
    for k in range(1, K + 1):
        oracle.reduce_sgd_f64(reps, x, v, lr, mu, 0.0)
        vk = cbar * (1 - mu ** k) / (1 - mu)
        xk = x0 - lr * cbar * (k / (1 - mu) - mu * (1 - mu ** k) / (1 - mu) ** 2)
        assert np.allclose(v, vk, rtol=1e-12, atol=0)
        assert np.allclose(x, xk, rtol=1e-12, atol=1e-15)


def test_zero_momentum_is_plain_sgd():
    c, lr, x0 = 0.125, 0.5, 3.0
    reps = [_const(3, c)] * 2
    x = np.full(3, x0, np.float32); v = np.zeros(3, np.float32)
    for k in range(1, 9):
        oracle.reduce_sgd_f32(reps, x, v, lr, 0.0, 0.0)
        assert np.all(x == x0 - k * lr * c)                # dyadic: exact


def test_weight_decay_matrix_power():
    c, lr, mu, wd, x0, K = 0.02, 0.1, 0.9, 1e-2, 0.7, 30
    reps = [_const(2, c)] * 4
    cbar = float(np.float32(c))
    A = np.array([[1 - lr * wd, -lr * mu], [wd, mu]])
    b = np.array([-lr * cbar, cbar])
    x = np.full(2, x0); v = np.zeros(2)
    s = np.array([x0, 0.0])
    for _ in range(K):
        oracle.reduce_sgd_f64(reps, x, v, lr, mu, wd)
        s = A @ s + b
        assert np.allclose([x[0], v[0]], s, rtol=1e-11, atol=1e-14)


@pytest.mark.parametrize("wd", [0.0, 1e-4, 0.3])
@pytest.mark.parametrize("mu", [0.0, 0.9])
def test_matches_torch_optim_sgd_in_double(mu, wd):
    """The momentum convention read into "SGD(x, g)" is the one of the framework the
    paper used (Section 3.1); torch.optim.SGD in float64 is that routine itself."""
    rng = np.random.default_rng(8)
    n, W, K, lr = 64, 3, 6, 0.1
    x0 = rng.standard_normal(n)
    p = torch.nn.Parameter(torch.tensor(x0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, weight_decay=wd)
    x = x0.copy(); v = np.zeros(n)
    for k in range(K):
        reps = [rng.standard_normal(n).astype(np.float32) for _ in range(W)]
        gavg = sum(torch.tensor(r, dtype=torch.float64) for r in reps) / W
        p.grad = gavg
        opt.step()
        oracle.reduce_sgd_f64(reps, x, v, lr, mu, wd)
        assert np.allclose(x, p.detach().numpy(), rtol=1e-13, atol=1e-15)


# ------------------------------------------------------------------ brute force
@pytest.mark.parametrize("prec,real", [("f64", float), ("f32", np.float32)])
@pytest.mark.parametrize("gdt", [np.float32, np.float16])
def test_whole_step_equals_python_brute_force(prec, real, gdt):
    rng = np.random.default_rng(9)
    numel = [3, 1, 0, 6, 2]
    W = 3
    grads = [[(rng.standard_normal(n) * 0.5).astype(gdt) for n in numel] for _ in range(W)]
    params = [rng.standard_normal(n).astype(np.float32) for n in numel]
    wdt = np.float64 if prec == "f64" else np.float32
    v = (rng.standard_normal(sum(numel)) * 0.1).astype(np.float32).astype(wdt)
    lr, mu, wd, inv = np.float32(0.1), np.float32(0.9), np.float32(1e-2), np.float32(1 / 128)
    v_ref = v.copy()
    new_p, found = oracle.sync_step(grads, params, v, float(lr), float(mu), float(wd),
                                    float(inv), align=1, precision=prec)
    bp, bv, bfound = brute.step([[t.tolist() for t in g] for g in grads],
                                [p.tolist() for p in params], v_ref.tolist(),
                                lr, mu, wd, inv, real=real)
    assert found is False and bfound is False
    for a, b in zip(new_p, bp):
        assert [float(e) for e in a] == [float(e) for e in b]
    assert [float(e) for e in v] == [float(e) for e in bv]


@pytest.mark.parametrize("W,gdt", [(8, np.float32), (16, np.float16), (3, np.float32), (13, np.float16)])
def test_single_precision_order_of_operations_at_workload_width(W, gdt):
    """The single-precision evaluation at the configured replica counts, against numpy float32
    array arithmetic written out here (every numpy operation on float32 arrays rounds once):
    left-to-right sum over workers, one constant c = inv_loss_scale * (1/W), then
    d = g*c + wd*x, v = mu*v + d, x = x - lr*v.  Values follow the workloads' recipe.  The
    same data summed pairwise, or scaled by inv_loss_scale / W, must differ somewhere, so the
    pin is sensitive to both choices."""
    rng = np.random.default_rng(100 + W)
    n = 20000
    scale = 1024.0 if gdt == np.float16 else 1.0
    reps = [(rng.standard_normal(n) * 1e-3 * scale).astype(gdt) for _ in range(W)]
    x0 = (rng.standard_normal(n) * 0.05).astype(np.float32)
    v0 = (rng.standard_normal(n) * 0.01).astype(np.float32)
    lr, mu, wd, inv = np.float32(0.1), np.float32(0.9), np.float32(1e-4), np.float32(1.0 / scale)

    def by_hand(order="sequential", one_constant=True):
        g = [r.astype(np.float32) for r in reps]
        if order == "sequential":
            s = g[0].copy()
            for w in range(1, W):
                s = s + g[w]
        else:
            level = g
            while len(level) > 1:
                level = [level[i] + level[i + 1] if i + 1 < len(level) else level[i]
                         for i in range(0, len(level), 2)]
            s = level[0]
        if one_constant:
            c = np.float32(inv * (np.float32(1.0) / np.float32(W)))
            ga = s * c
        else:
            ga = (s * inv) / np.float32(W)
        d = ga + wd * x0
        v = mu * v0 + d
        return (x0 - lr * v).astype(np.float32), v.astype(np.float32)

    x, v = x0.copy(), v0.copy()
    oracle.reduce_sgd_f32(reps, x, v, float(lr), float(mu), float(wd), float(inv))
    hx, hv = by_hand()
    assert np.array_equal(x.view(np.uint32), hx.view(np.uint32))
    assert np.array_equal(v.view(np.uint32), hv.view(np.uint32))
    # (three workers: the pairwise tree is the sequential sum; half-precision gradients: sums
    # of 16 values of 11 significant bits are exact in single precision in any order)
    if W >= 4 and gdt == np.float32:
        px, pv = by_hand(order="pairwise")
        assert not np.array_equal(v.view(np.uint32), pv.view(np.uint32))
    if W in (3, 13):          # 1/W is not a power of two: one constant vs scale-then-divide differ
        qx, qv = by_hand(one_constant=False)
        assert not np.array_equal(v.view(np.uint32), qv.view(np.uint32))
    # and the double-precision definition is within the single-precision error bound of it
    x64, v64 = x0.astype(np.float64), v0.astype(np.float64)
    oracle.reduce_sgd_f64(reps, x64, v64, float(lr), float(mu), float(wd), float(inv))
    assert np.all(np.abs(x - x64) <= 1e-7 + 1e-6 * np.abs(x64))


def test_aligned_layout_gives_same_tensors_as_tight():
    rng = np.random.default_rng(10)
    numel = [5, 64, 1, 130]
    grads = [[rng.standard_normal(n).astype(np.float32) for n in numel] for _ in range(2)]
    params = [rng.standard_normal(n).astype(np.float32) for n in numel]
    res = []
    for a in (1, 64):
        offs = oracle.layout(numel, a)
        v = np.zeros(int(offs[-1]))
        p, _ = oracle.sync_step(grads, params, v, 0.1, 0.9, 1e-4, 1.0, align=a)
        res.append((p, oracle.unpack(v, numel, offs), v, offs))
    for a, b in zip(res[0][0], res[1][0]):
        assert np.array_equal(a, b)
    for a, b in zip(res[0][1], res[1][1]):
        assert np.array_equal(a, b)
    # padding of the aligned momentum stays zero (g = 0, x = 0, v = 0 is a fixed point)
    v64, offs = res[1][2], res[1][3]
    mask = np.ones(v64.size, bool)
    for n, o in zip(numel, offs[:-1]):
        mask[int(o):int(o) + n] = False
    assert not v64[mask].any()


# ------------------------------------------------------------------ mixed precision
def test_half_gradients_equal_widened_single_gradients():
    rng = np.random.default_rng(12)
    n, W = 300, 4
    h = [(rng.standard_normal(n)).astype(np.float16) for _ in range(W)]
    # include subnormals, max finite, signed zeros
    h[0][:6] = np.array([6e-8, -6e-8, 65504, -65504, 0.0, -0.0], np.float16)
    f = [a.astype(np.float32) for a in h]
    for fn, dt in ((oracle.reduce_sgd_f64, np.float64), (oracle.reduce_sgd_f32, np.float32)):
        xa = np.ones(n, dt); va = np.zeros(n, dt); xb = xa.copy(); vb = va.copy()
        fn(h, xa, va, 0.1, 0.9, 1e-4, 1.0 / 1024)
        fn(f, xb, vb, 0.1, 0.9, 1e-4, 1.0 / 1024)
        assert np.array_equal(xa, xb) and np.array_equal(va, vb)


def test_loss_scale_times_world_size_is_one_constant():
    # 1/1024 * 1/16 = 2^-14: scaling is exact, so f32 and f64 agree on dyadic inputs
    reps = [_const(4, 1024.0, np.float16)] * 16
    x = np.zeros(4, np.float32); v = np.zeros(4, np.float32)
    oracle.reduce_sgd_f32(reps, x, v, 1.0, 0.0, 0.0, 1.0 / 1024)
    assert np.all(v == 1.0)


@pytest.mark.parametrize("bad", [np.inf, -np.inf, np.nan])
@pytest.mark.parametrize("gdt", [np.float16, np.float32])
def test_nonfinite_anywhere_skips_whole_step(bad, gdt):
    rng = np.random.default_rng(13)
    numel = [4, 7, 2]
    W = 3
    for w_bad in range(W):
        for t_bad in range(len(numel)):
            grads = [[rng.standard_normal(n).astype(gdt) for n in numel] for _ in range(W)]
            grads[w_bad][t_bad][numel[t_bad] - 1] = bad
            params = [rng.standard_normal(n).astype(np.float32) for n in numel]
            v = rng.standard_normal(sum(numel))
            v0 = v.copy()
            p, found = oracle.sync_step(grads, params, v, 0.1, 0.9, 1e-4, 1.0)
            assert found is True
            assert np.array_equal(v, v0)
            for a, b in zip(p, params):
                assert np.array_equal(a.astype(np.float32), b)


def test_nonfinite_in_padding_does_not_skip():
    numel = [3, 5]
    offs = oracle.layout(numel, 8)
    rep = np.zeros(int(offs[-1]), np.float16)
    rep[4] = np.inf                      # padding after the first tensor
    assert not oracle.any_nonfinite([rep], numel, offs)
    rep[8 + 4] = np.inf                  # last valid element of the second tensor
    assert oracle.any_nonfinite([rep], numel, offs)


def test_finite_half_sum_cannot_overflow_single():
    reps = [_const(2, 65504.0, np.float16)] * 16
    x = np.zeros(2, np.float32); v = np.zeros(2, np.float32)
    oracle.reduce_sgd_f32(reps, x, v, 1.0, 0.0, 0.0, 1.0)
    assert np.all(v == 65504.0)


# ------------------------------------------------------------------ bfloat16 gradients, half copies
def _bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_bfloat16_gradients_equal_their_widened_values():
    rng = np.random.default_rng(14)
    n, W = 500, 4
    vals = [torch.tensor(rng.standard_normal(n), dtype=torch.float32) for _ in range(W)]
    vals[0][:6] = torch.tensor([1e-40, -1e-40, 3.3895e38, -3.3895e38, 0.0, -0.0])   # subnormal, max
    bits = [_bf16_bits(v) for v in vals]
    widened = [v.to(torch.bfloat16).to(torch.float32).numpy() for v in vals]         # library widening
    for fn, dt in ((oracle.reduce_sgd_f64, np.float64), (oracle.reduce_sgd_f32, np.float32)):
        xa = np.ones(n, dt); va = np.zeros(n, dt); xb = xa.copy(); vb = va.copy()
        fn(bits, xa, va, 0.1, 0.9, 1e-4, 1.0 / 128)
        fn(widened, xb, vb, 0.1, 0.9, 1e-4, 1.0 / 128)
        assert np.array_equal(xa, xb) and np.array_equal(va, vb)
    inf_bits = bits[1].copy(); inf_bits[7] = 0x7f80
    assert oracle.any_nonfinite([bits[0], inf_bits], [n], oracle.layout([n]))
    nan_bits = bits[1].copy(); nan_bits[7] = 0xffc1
    assert oracle.any_nonfinite([nan_bits], [n], oracle.layout([n]))
    assert not oracle.any_nonfinite(bits, [n], oracle.layout([n]))


def test_round_params_matches_library_conversions():
    rng = np.random.default_rng(15)
    x = np.concatenate([
        rng.standard_normal(20000).astype(np.float32),
        (rng.standard_normal(5000) * 1e-6).astype(np.float32),         # fp16 subnormal range
        (rng.standard_normal(5000) * 1e5).astype(np.float32),          # fp16 overflow range
        np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 65504.0, 65519.9, 65520.0, -65520.0,
                  2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25, 2.0 ** -14, 1.0009765625, 1.00048828125,
                  1.00146484375, 3.3895314e38, 3.4e38, 1e-40, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -9],
                 dtype=np.float32)])
    h = oracle.round_params(x, oracle.F16)
    want_h = x.astype(np.float16).view(np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(h[~nan], want_h[~nan])
    assert np.all((h[nan] & 0x7c00) == 0x7c00) and np.all((h[nan] & 0x03ff) != 0)
    b = oracle.round_params(x, oracle.BF16)
    want_b = _bf16_bits(torch.from_numpy(x.copy()))
    assert np.array_equal(b[~nan], want_b[~nan])
    assert np.all((b[nan] & 0x7f80) == 0x7f80) and np.all((b[nan] & 0x007f) != 0)


def test_threads_do_not_change_the_result():
    # elements are independent: spreading the element loop over threads is bit-neutral
    rng = np.random.default_rng(77)
    numel = [1000, 3, 5000]
    grads = [[rng.standard_normal(n).astype(np.float32) for n in numel] for _ in range(4)]
    params = [rng.standard_normal(n).astype(np.float32) for n in numel]
    for prec, dt in (("f64", np.float64), ("f32", np.float32)):
        outs = []
        for threads in (1, 4):
            v = np.zeros(int(oracle.layout(numel, 8)[-1]), dt)
            new, inf = oracle.sync_step(grads, params, v, 0.1, 0.9, 1e-4, 0.5, align=8,
                                        precision=prec, threads=threads)
            outs.append((new, v))
        for a, b in zip(outs[0][0], outs[1][0]):
            assert np.array_equal(a, b)
        assert np.array_equal(outs[0][1], outs[1][1])
