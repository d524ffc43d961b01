"""More than 2^32 elements in one bucket: every index on the path has to be 64 bits wide.

One tensor of 2^32 + 1029 half-precision gradient elements between two small ones, W = 2.
The oracle computes sampled windows (both ends, the tensor boundaries, around elements 2^31
and 2^32, the ragged tail and the padding); whole-buffer equalities between the library's
forms are checked on the device."""
import numpy as np
import pytest
import torch

import oracle
from paper_2103_07974_amd import workloads as wl, xs

pytestmark = pytest.mark.gpu

N_BIG = 2 ** 32 + 1029
NUMEL = [1000, N_BIG, 77]
ALIGN = 64
W = 2
LR, MU, WD, INV = (float(np.float32(v)) for v in (0.1, 0.9, 1e-4, 1.0 / 1024))
WIN = 4096


def _windows(offs, n_bucket):
    starts = {0, offs[1] - WIN // 2, offs[1] + 2 ** 31 - WIN // 2, 2 ** 32 - WIN // 2,
              offs[1] + 2 ** 32 - WIN // 2, offs[2] - WIN // 2, n_bucket - WIN}
    return sorted(min(max(int(s), 0), n_bucket - WIN) for s in starts)


def _ulp_distance(a, b):
    ia = a.view(np.int32).astype(np.int64); ib = b.view(np.int32).astype(np.int64)
    ia = np.where(ia < 0, np.int64(-2 ** 31) - ia, ia)
    ib = np.where(ib < 0, np.int64(-2 ** 31) - ib, ib)
    return int(np.abs(ia - ib).max())


def test_bucket_of_more_than_2_to_32_elements():
    torch.cuda.empty_cache()          # hand cached blocks of earlier tests back first
    free, _ = torch.cuda.mem_get_info()
    if free < 200 * 2 ** 30:
        pytest.skip("needs about 160 GiB of device memory")
    offs = xs.bucket_layout(NUMEL, ALIGN)
    assert offs == [int(o) for o in oracle.layout(NUMEL, ALIGN)]
    n_bucket = offs[-1]
    assert n_bucket > 2 ** 32
    gplan = xs.Plan(NUMEL, offs, torch.float16)
    pplan = xs.Plan(NUMEL, offs, torch.float32)
    print("allocating", flush=True)
    grads = [[wl.fill_normal_(torch.empty(n, dtype=torch.float16, device="cuda"), 1.0, 100 * w + t)
              for t, n in enumerate(NUMEL)] for w in range(W)]
    buckets = [torch.empty(n_bucket, dtype=torch.float16, device="cuda") for _ in range(W)]
    for b in buckets:
        b.view(torch.int16).fill_(0x5a5a)                   # pack must overwrite the padding
    tabs = [xs.pointer_table(g) for g in grads]
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")

    print("pack", flush=True)
    xs.fuse_pack_many(gplan, tabs, buckets, flag)
    torch.cuda.synchronize()
    assert flag.item() == 0
    wins = _windows(offs, n_bucket)
    for w in range(W):
        for t, n in enumerate(NUMEL):
            assert torch.equal(buckets[w][offs[t]:offs[t] + n], grads[w][t]), (w, t)
            pad = buckets[w][offs[t] + n:offs[t + 1]]
            assert pad.numel() == 0 or int(pad.view(torch.int16).abs().max()) == 0
        # sampled windows inside the big tensor, element by element on the host
        for s in wins:
            a = max(s, offs[1]); e = min(s + WIN, offs[1] + N_BIG)
            if e > a:
                got = buckets[w][a:e].cpu().numpy().view(np.uint16)
                want = grads[w][1][a - offs[1]:e - offs[1]].cpu().numpy().view(np.uint16)
                assert np.array_equal(got, want), (w, s)

    print("reduce + SGD", flush=True)
    x0 = wl.fill_normal_(torch.empty(n_bucket, dtype=torch.float32, device="cuda"), 0.05, 7)
    v0 = wl.fill_normal_(torch.empty(n_bucket, dtype=torch.float32, device="cuda"), 0.01, 8)
    xb = torch.empty_like(x0); vb = torch.empty_like(v0)
    xs.fused_reduce_sgd(buckets, n_bucket, x0, v0, LR, MU, WD, INV, params_out=xb, momentum_out=vb)
    torch.cuda.synchronize()
    for s in wins:
        reps = [b[s:s + WIN].cpu().numpy() for b in buckets]
        x32 = x0[s:s + WIN].cpu().numpy().copy(); v32 = v0[s:s + WIN].cpu().numpy().copy()
        x64 = x32.astype(np.float64); v64 = v32.astype(np.float64)
        oracle.reduce_sgd_f32(reps, x32, v32, LR, MU, WD, INV)
        oracle.reduce_sgd_f64(reps, x64, v64, LR, MU, WD, INV)
        gx = xb[s:s + WIN].cpu().numpy(); gv = vb[s:s + WIN].cpu().numpy()
        assert _ulp_distance(gx, x32) == 0 and _ulp_distance(gv, v32) == 0, s
        assert np.all(np.abs(gx - x64) <= 1e-7 + 1e-6 * np.abs(x64)), s
        assert np.all(np.abs(gv - v64) <= 1e-7 + 1e-6 * np.abs(v64)), s

    print("gathering form with views", flush=True)
    gtab = xs.gather_pointer_table(grads)
    views = [torch.zeros(n, dtype=torch.float32, device="cuda") for n in NUMEL]
    vtab = xs.pointer_table(views)
    xg = torch.empty_like(x0); vg = torch.empty_like(v0)
    xs.fused_gather_reduce_sgd(gplan, gtab, W, x0, v0, LR, MU, WD, INV, params_out=xg,
                               momentum_out=vg, param_tensor_ptrs=vtab)
    torch.cuda.synchronize()
    assert torch.equal(xg, xb) and torch.equal(vg, vb)
    for t, n in enumerate(NUMEL):
        assert torch.equal(views[t], xb[offs[t]:offs[t] + n]), t

    print("per-tensor records", flush=True)
    table = xs.tensor_hparams_table([(LR, MU, WD)] * len(NUMEL))
    xg.fill_(3.0); vg.fill_(3.0)
    xs.fused_reduce_sgd_pt(gplan, buckets, x0, v0, table, INV, params_out=xg, momentum_out=vg)
    torch.cuda.synchronize()
    assert torch.equal(xg, xb) and torch.equal(vg, vb)

    print("unpack", flush=True)
    for v in views:
        v.zero_()
    xs.fuse_unpack(pplan, xb, vtab)
    torch.cuda.synchronize()
    for t, n in enumerate(NUMEL):
        assert torch.equal(views[t], xb[offs[t]:offs[t] + n]), t
    del grads, buckets, x0, v0, xb, vb, xg, vg, views
    torch.cuda.empty_cache()
