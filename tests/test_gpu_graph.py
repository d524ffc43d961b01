"""The hot calls only enqueue kernels (no allocation, no memset, no synchronisation), so a
whole synchronisation can be captured into a HIP graph and replayed.  Every replay is checked
against the eager result, with eager work and synchronisations between replays."""
import numpy as np
import pytest
import torch

from paper_2103_07974_amd import harness, workloads as wl, xs

pytestmark = pytest.mark.gpu

SIZES = [(300, 7), (64,), (5000,), (3,), (12289,)]


def _fresh_grads(task, step):
    """New gradient values in the same tensors (addresses are what the graph recorded)."""
    for w, gl in enumerate(task.grads):
        for t, g in enumerate(gl):
            g.copy_(wl.make_flat(g.numel(), 1e-3, 1000 * step + 10 * w + t, g.dtype, "cuda").view_as(g))


@pytest.mark.parametrize("fused_gather", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_captured_sync_replays_like_eager(fused_gather, dtype):
    base = wl.RESNET50 if dtype == "f32" else wl.BERT_LARGE_F16
    w = wl.scaled(base, f"graph_{dtype}", SIZES, W=4)
    eager = harness.make_task(w, "cuda", 64)
    graphed = harness.make_task(w, "cuda", 64)
    app_e = eager.make_app(fused_gather=fused_gather, use_found_inf=not fused_gather)
    app_g = graphed.make_app(fused_gather=fused_gather, use_found_inf=not fused_gather)
    s = torch.cuda.Stream()
    # warm-up outside capture (first call queries the device once)
    app_g.sync(s); s.synchronize()
    graphed.params.copy_(eager.params); graphed.momentum.copy_(eager.momentum)
    for a, b in zip(graphed.param_tensors, eager.param_tensors):
        a.copy_(b)
    torch.cuda.synchronize()

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        app_g.sync(s)
    torch.cuda.synchronize()
    # the capture itself executed nothing
    assert torch.equal(graphed.params, eager.params)

    for step in range(1, 6):
        _fresh_grads(eager, step); _fresh_grads(graphed, step)
        torch.cuda.synchronize()
        app_e.sync(s)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(graphed.params, eager.params), step
        assert torch.equal(graphed.momentum, eager.momentum), step
        for a, b in zip(graphed.param_tensors, eager.param_tensors):
            assert torch.equal(a, b), step
        # unrelated eager work between replays
        junk = torch.randn(1 << 16, device="cuda").sum().item()
        assert np.isfinite(junk)
    assert graphed.found_inf.item() == 0
    app_e.destroy(); app_g.destroy()
