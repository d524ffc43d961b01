"""Crossover with a real forward + backward (PyTorch autograd on a small MLP per task) as the
compute side: the library's kernels read the gradients autograd produced and write the model's
weights.  Every computation's gradients and the weights it saw are captured on the device; the
oracle then replays each task's synchronisations from those gradients and must reproduce, bit
for bit, the weights every later computation saw and the final model."""
import numpy as np
import pytest
import torch

import oracle
from paper_2103_07974_amd import harness, xs

pytestmark = pytest.mark.gpu


def _bits(a):
    return a.view(np.uint32)


@pytest.mark.parametrize("modes", [(False, True), (True, False)])
def test_autograd_compute_side_matches_oracle_replay(modes):
    mlps = [harness.make_mlp_task("mlp_a", [32, 64, 10], W=2, batch=16, seed=11, align=4),
            harness.make_mlp_task("mlp_b", [20, 48, 48, 5], W=3, batch=8, seed=12, align=4)]
    captured = [[] for _ in mlps]

    def wrap(i):
        def fn(stream_ptr):
            m = mlps[i]
            s = torch.cuda.ExternalStream(stream_ptr)
            with torch.cuda.stream(s):
                seen = [p.detach().clone() for p in m.state.param_tensors]
            m.compute(stream_ptr)
            with torch.cuda.stream(s):
                grads = [[g.clone() for g in gl] for gl in m.state.grads]
            captured[i].append((seen, grads))
        return fn

    apps = [m.state.make_app(wrap(i), fused_gather=modes[i]) for i, m in enumerate(mlps)]
    cs, ss = torch.cuda.Stream(), torch.cuda.Stream()
    T = 4
    for _ in range(T):
        xs.crossover_iteration(apps, cs, ss)
    xs.crossover_finish(apps, ss)
    torch.cuda.synchronize()

    for i, m in enumerate(mlps):
        w = m.state.workload
        hp = [float(np.float32(v)) for v in (w.lr, w.momentum, w.weight_decay)]
        assert len(captured[i]) == T
        params = [p.cpu().numpy() for p in captured[i][0][0]]
        v = np.zeros(m.state.n_bucket, np.float32)
        moved = False
        for k, (seen, grads) in enumerate(captured[i]):
            # computation k ran on the weights left by update k-1
            for t, (got, want) in enumerate(zip(seen, params)):
                assert np.array_equal(_bits(got.cpu().numpy()), _bits(want)), (i, k, t)
            g_np = [[g.cpu().numpy() for g in gl] for gl in grads]
            assert all(np.isfinite(g).all() for gl in g_np for g in gl)
            moved = moved or any(np.abs(g).max() > 0 for gl in g_np for g in gl)
            new, inf = oracle.sync_step(g_np, params, v, *hp, 1.0, align=4, precision="f32")
            assert not inf
            params = [p.astype(np.float32) for p in new]
        assert moved
        for t, (got, want) in enumerate(zip(m.state.param_tensors, params)):
            assert np.array_equal(_bits(got.detach().cpu().numpy()), _bits(want)), (i, t)
        assert np.array_equal(_bits(m.state.momentum.cpu().numpy()), _bits(v))
    for a in apps:
        a.destroy()


def test_training_through_the_library_reduces_the_loss():
    m = harness.make_mlp_task("mlp_fit", [16, 64, 4], W=4, batch=32, seed=21, lr=0.1, align=64)
    app = m.state.make_app(m.compute, fused_gather=True)
    cs, ss = torch.cuda.Stream(), torch.cuda.Stream()

    def loss():
        with torch.no_grad():
            return float(sum(torch.nn.functional.cross_entropy(m.forward(x), y)
                             for x, y in zip(m.inputs, m.targets)) / len(m.inputs))
    before = loss()
    for _ in range(60):
        xs.crossover_iteration([app], cs, ss)
    torch.cuda.synchronize()
    after = loss()
    print(f"loss {before:.4f} -> {after:.4f}", flush=True)
    assert after < 0.7 * before, (before, after)
    app.destroy()
