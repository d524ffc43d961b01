"""The state pool (xs_pool_layout): one allocation for a task's buckets, parameters and momentum.
The layout is a performance choice only; results are the same bits as with separate allocations."""
import pytest
import torch

from paper_2103_07974_amd import harness, workloads as wl, xs

pytestmark = pytest.mark.gpu

SIZES = [0, 1, 3, 5, 17, 63, 64, 65, 255, 256, 257, 4095, 4096, 4097, 12289, 50001, 2, 0, 70000]


def test_pool_alloc_places_every_buffer_at_a_pool_multiple_without_overlap():
    sizes = [(1, torch.float16), (0, torch.float32), (1 << 19, torch.float32), ((1 << 19) + 1, torch.float32),
             (12345, torch.bfloat16)]
    bufs = xs.pool_alloc(sizes, "cuda")
    assert [b.numel() for b in bufs] == [n for n, _ in sizes]
    assert [b.dtype for b in bufs] == [dt for _, dt in sizes]
    spans = []
    for b in bufs:
        assert b.data_ptr() % xs.POOL_ALIGN == 0
        spans.append((b.data_ptr(), b.data_ptr() + b.numel() * b.element_size()))
    spans.sort()
    for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
        assert a1 <= b0
    for i, b in enumerate(bufs):            # independent storage: a write to one leaves the others alone
        b.fill_(i + 1)
    torch.cuda.synchronize()
    for i, b in enumerate(bufs):
        assert bool((b == i + 1).all())


@pytest.mark.parametrize("dtype,W", [("f32", 8), ("f16", 16), ("f32", 3)])
@pytest.mark.parametrize("form", ["packs", "fused_unpack", "gather"])
def test_pooled_and_separate_allocations_give_the_same_bits(dtype, W, form):
    base = wl.RESNET50 if dtype == "f32" else wl.BERT_LARGE_F16
    w = wl.scaled(base, f"pool_{dtype}", [(n,) for n in SIZES], W=W)
    results = []
    for pooled in (True, False):
        t = harness.make_task(w, "cuda", 64, pooled=pooled)
        t.momentum.copy_(wl.make_flat(t.n_bucket, 0.01, 5, device="cuda"))
        if pooled:
            for b in t.buckets + [t.params, t.momentum]:
                assert b.data_ptr() % xs.POOL_ALIGN == 0
        app = t.make_app(fused_gather=form == "gather", fused_unpack=form == "fused_unpack")
        s = torch.cuda.Stream()
        for _ in range(3):
            app.sync(s)
        torch.cuda.synchronize()
        app.destroy()
        results.append((t.params.clone(), t.momentum.clone(), [p.clone() for p in t.param_tensors]))
    (xa, va, pa), (xb, vb, pb) = results
    assert torch.equal(xa.view(torch.int32), xb.view(torch.int32))
    assert torch.equal(va.view(torch.int32), vb.view(torch.int32))
    for a, b in zip(pa, pb):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
