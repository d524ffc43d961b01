"""xs_fuse_pack_static (the pack for callers that cannot allocate) against xs_fuse_pack:
bit-identical buckets, through the C-ABI, on two calls in a row, the second one smaller."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2103_07974_amd import xs

pytestmark = pytest.mark.gpu


def _bits(t: torch.Tensor) -> torch.Tensor:
    return t.view(torch.int32 if t.element_size() == 4 else torch.int16)


def _case(seed, n_tensors, max_numel, dtype, align):
    g = torch.Generator(device="cuda"); g.manual_seed(seed)
    rng = np.random.default_rng(seed)
    numel = [int(v) for v in rng.integers(0, max_numel, size=n_tensors)]
    numel[0] = 0                       # an empty tensor in front
    numel[n_tensors // 2] = 70001      # one tensor of several 16 KiB chunks with a ragged tail
    tensors = [torch.randn(n, generator=g, device="cuda").to(dtype) for n in numel]
    offsets = xs.bucket_layout(numel, align)
    return numel, offsets, tensors, xs.pointer_table(tensors)


def _pack_both(numel, offsets, tensors, table, dtype, found_a=None, found_b=None, stream=None):
    plan = xs.Plan(numel, offsets, dtype)
    want = torch.full((offsets[-1],), 5.0, dtype=dtype, device="cuda")
    got = torch.full((offsets[-1],), 9.0, dtype=dtype, device="cuda")
    xs.fuse_pack(plan, table, want, found_a, stream)
    xs.fuse_pack_static(numel, offsets, dtype, table, got, found_b, stream)
    return plan, want, got


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
def test_two_calls_in_a_row_second_smaller(dtype):
    print(f"case static pack dtype={dtype}", flush=True)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        # 300 tensors: three table-writer launches; tight layout so that segments are unaligned
        big = _case(11, 300, 3000, dtype, 1)
        small = _case(12, 5, 200, dtype, 64)
        torch.cuda.synchronize()
        # both calls are enqueued back to back on one stream, nothing synchronises between them:
        # the second call's table writes are ordered behind the first call's pack
        p1, want1, got1 = _pack_both(*big, dtype, stream=s)
        p2, want2, got2 = _pack_both(*small, dtype, stream=s)
        torch.cuda.synchronize()
    assert torch.equal(_bits(got1), _bits(want1))
    assert torch.equal(_bits(got2), _bits(want2))
    # and the big one once more after the small one (stale entries behind the small tables)
    p3, want3, got3 = _pack_both(*big, dtype)
    torch.cuda.synchronize()
    assert torch.equal(_bits(got3), _bits(want3))


def test_overflow_flag_and_limits():
    print("case static pack overflow flag and limits", flush=True)
    dtype = torch.float16
    numel, offsets, tensors, table = _case(13, 40, 5000, dtype, 8)
    tensors[7].view(-1)[3] = float("inf")
    fa = torch.zeros(1, dtype=torch.int32, device="cuda"); fb = torch.zeros(1, dtype=torch.int32, device="cuda")
    plan, want, got = _pack_both(numel, offsets, tensors, table, dtype, fa, fb)
    torch.cuda.synchronize()
    assert int(fa.item()) == 1 and int(fb.item()) == 1
    assert torch.equal(_bits(got), _bits(want))
    # beyond the stated maximum: refused with a clear error, nothing enqueued
    n = xs.STATIC_MAX_TENSORS + 1
    with pytest.raises(xs.XsError) as e:
        xs.fuse_pack_static([1] * n, list(range(n + 1)), torch.float32, table, got)
    assert e.value.status == xs.XS_ERR_SIZE and "XS_STATIC_MAX_TENSORS" in str(e.value)
    # exactly the maximum is accepted
    n = xs.STATIC_MAX_TENSORS
    ts = [torch.full((3,), float(i), device="cuda") for i in range(n)]
    offs = xs.bucket_layout([3] * n, 4)
    tab = xs.pointer_table(ts)
    b = torch.full((offs[-1],), -1.0, device="cuda")
    xs.fuse_pack_static([3] * n, offs, torch.float32, tab, b)
    torch.cuda.synchronize()
    host = b.cpu().numpy().reshape(n, 4)
    assert np.array_equal(host[:, 0], np.arange(n, dtype=np.float32)) and np.all(host[:, 3] == 0.0)
    # layout errors are those of xs_plan_create
    with pytest.raises(xs.XsError) as e:
        xs.fuse_pack_static([5, 5], [0, 4, 10], torch.float32, tab, b)
    assert e.value.status == xs.XS_ERR_SIZE
    # empty list: a no-op
    xs.fuse_pack_static([], [0], torch.float32, tab, b)
