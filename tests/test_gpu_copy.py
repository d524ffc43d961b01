"""Parity of xs_fuse_pack / xs_fuse_unpack with the oracle: bit-exact, through the C-ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2103_07974_amd import xs

pytestmark = pytest.mark.gpu

# sizes in elements: empty, tiny, one-vector edges, around one 16 KiB chunk (4096 fp32 /
# 8192 fp16 elements), several chunks with a ragged tail
SIZES = [0, 1, 3, 5, 17, 63, 64, 65, 4095, 4096, 4097, 8191, 8192, 8193, 12289, 50001, 3, 0, 70000]
GUARD = 8


def _bits(a: np.ndarray) -> np.ndarray:
    return a.view(np.uint32 if a.dtype.itemsize == 4 else np.uint16)


def _random_bits(rng, n, np_dtype):
    """Arbitrary finite-or-not bit patterns (NaN payloads, -0.0, subnormals)."""
    it = np.dtype(np_dtype).itemsize
    raw = rng.integers(0, 2 ** (8 * it), size=n, dtype=np.uint64)
    return raw.astype(np.uint32 if it == 4 else np.uint16).view(np_dtype)


def _device_tensors(host_list, torch_dtype, skew_elems):
    """Each tensor lives inside its own allocation at an element offset (unaligned base),
    with guard elements on both sides holding a canary."""
    holders, views = [], []
    for i, h in enumerate(host_list):
        sk = (skew_elems * (i + 1)) % 7 if skew_elems else 0
        buf = torch.full((h.size + 2 * GUARD + sk,), 7.0, dtype=torch_dtype, device="cuda")
        v = buf[GUARD + sk: GUARD + sk + h.size]
        v.copy_(torch.from_numpy(h.copy()).view(torch_dtype))
        holders.append(buf)
        views.append(v)
    return holders, views


@pytest.mark.parametrize("torch_dtype,np_dtype", [(torch.float32, np.float32), (torch.float16, np.float16)])
@pytest.mark.parametrize("align", [1, 4, 64])
@pytest.mark.parametrize("skew", [0, 1])
def test_pack_and_unpack_bit_exact(torch_dtype, np_dtype, align, skew):
    print(f"case dtype={torch_dtype} align={align} skew={skew}", flush=True)
    rng = np.random.default_rng(100 + align + skew)
    host = [_random_bits(rng, n, np_dtype) for n in SIZES]
    numel = [h.size for h in host]
    offs = xs.bucket_layout(numel, align)
    assert offs == [int(v) for v in oracle.layout(numel, align)]
    want_bucket = oracle.pack(host, np.asarray(offs, dtype=np.uint64))

    holders, views = _device_tensors(host, torch_dtype, skew)
    table = xs.pointer_table(views)
    plan = xs.Plan(numel, offs, torch_dtype)
    assert plan.bucket_elems == offs[-1] and plan.n_tensors == len(numel)
    # bucket with guard zones and garbage inside
    raw = torch.full((offs[-1] + 2 * GUARD,), 3.0, dtype=torch_dtype, device="cuda")
    assert raw.data_ptr() % 16 == 0
    bucket = raw[GUARD:GUARD + offs[-1]] if (GUARD * raw.element_size()) % 16 == 0 else None
    assert bucket is not None
    xs.fuse_pack(plan, table, bucket)
    torch.cuda.synchronize()
    got = bucket.cpu().numpy()
    assert np.array_equal(_bits(got), _bits(want_bucket))
    edge = raw.cpu().numpy()
    assert np.all(edge[:GUARD] == 3.0) and np.all(edge[GUARD + offs[-1]:] == 3.0)

    # unpack into fresh garbage-filled tensors; guards must survive
    out_holders, out_views = _device_tensors([np.zeros(n, np_dtype) for n in numel], torch_dtype, skew)
    for v in out_views:
        v.fill_(5.0)
    out_table = xs.pointer_table(out_views)
    xs.fuse_unpack(plan, bucket, out_table)
    torch.cuda.synchronize()
    want_tensors = oracle.unpack(want_bucket, numel, np.asarray(offs, dtype=np.uint64))
    for h, v, hold, wt in zip(host, out_views, out_holders, want_tensors):
        g = v.cpu().numpy()
        assert np.array_equal(_bits(g), _bits(h))
        assert np.array_equal(_bits(g), _bits(wt))
        whole = hold.cpu().numpy()
        start = (v.data_ptr() - hold.data_ptr()) // hold.element_size()
        assert np.all(whole[:start] == 7.0) and np.all(whole[start + h.size:] == 7.0)
    plan.destroy()


def test_empty_list_and_all_empty_tensors_are_noops():
    for numel in ([], [0, 0, 0]):
        offs = xs.bucket_layout(numel, 64)
        plan = xs.Plan(numel, offs, torch.float32)
        assert plan.bucket_elems == 0
        dummy = torch.zeros(4, device="cuda")
        table = xs.pointer_table([dummy] * max(len(numel), 1))
        xs.fuse_pack(plan, table, dummy)
        xs.fuse_unpack(plan, dummy, table)
        torch.cuda.synchronize()
        plan.destroy()


def test_many_tensors_use_the_global_table_path():
    # more tensors than the LDS copy of the table holds
    rng = np.random.default_rng(5)
    numel = [int(v) for v in rng.integers(0, 9, size=9000)]
    host = [rng.standard_normal(n).astype(np.float32) for n in numel]
    offs = xs.bucket_layout(numel, 1)
    flat = torch.from_numpy(np.concatenate(host)).cuda()
    views, pos = [], 0
    for n in numel:
        views.append(flat[pos:pos + n]); pos += n
    table = xs.pointer_table(views)
    plan = xs.Plan(numel, offs, torch.float32)
    bucket = torch.empty(offs[-1], dtype=torch.float32, device="cuda")
    xs.fuse_pack(plan, table, bucket)
    torch.cuda.synchronize()
    want = oracle.pack(host, np.asarray(offs, dtype=np.uint64))
    assert np.array_equal(_bits(bucket.cpu().numpy()), _bits(want))
    plan.destroy()


@pytest.mark.parametrize("torch_dtype,np_dtype", [(torch.float16, np.float16), (torch.float32, np.float32)])
def test_pack_raises_the_overflow_flag(torch_dtype, np_dtype):
    numel = [5, 9000, 33, 20000]
    align = 8
    offs = xs.bucket_layout(numel, align)
    plan = xs.Plan(numel, offs, torch_dtype)
    rng = np.random.default_rng(17)
    base = [rng.standard_normal(n).astype(np_dtype) for n in numel]
    bucket = torch.empty(offs[-1], dtype=torch_dtype, device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")

    def run(host):
        views = [torch.from_numpy(h).cuda() for h in host]
        flag.zero_()
        xs.fuse_pack(plan, xs.pointer_table(views), bucket, flag)
        torch.cuda.synchronize()
        want = oracle.any_nonfinite([oracle.pack(host, np.asarray(offs, dtype=np.uint64))], numel,
                                    np.asarray(offs, dtype=np.uint64))
        return int(flag.item()), int(want)

    assert run(base) == (0, 0)
    # head element, vector body, chunk edge, last element; inf, -inf, NaN
    for t, k, bad in [(0, 0, np.inf), (0, 4, -np.inf), (1, 4500, np.nan), (1, 8191, np.inf),
                      (1, 8999, np.nan), (2, 32, -np.inf), (3, 19999, np.inf), (3, 16384, np.nan)]:
        host = [b.copy() for b in base]
        host[t][k] = bad
        assert run(host) == (1, 1), (t, k, bad)
    # the largest finite values do not raise it
    host = [b.copy() for b in base]
    host[1][:4] = np.array([np.finfo(np_dtype).max, -np.finfo(np_dtype).max,
                            np.finfo(np_dtype).tiny, -0.0], np_dtype)
    assert run(host) == (0, 0)
    # the flag is sticky: a clean pack does not clear it
    flag.fill_(1)
    views = [torch.from_numpy(h).cuda() for h in base]
    xs.fuse_pack(plan, xs.pointer_table(views), bucket, flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 1
    plan.destroy()


@pytest.mark.parametrize("torch_dtype,np_dtype", [(torch.float32, np.float32), (torch.float16, np.float16)])
def test_pack_many_equals_single_packs(torch_dtype, np_dtype):
    """All workers' packs in one launch: every bucket bit-identical to the oracle's pack of that
    worker's tensors, and the overflow flag raised if any worker's tensors hold a non-finite."""
    rng = np.random.default_rng(23)
    numel = [0, 5, 4097, 64, 20001, 3]
    W = 5
    offs = xs.bucket_layout(numel, 4)
    plan = xs.Plan(numel, offs, torch_dtype)
    hosts = [[_random_bits(rng, n, np_dtype) for n in numel] for _ in range(W)]
    for h in hosts:                      # finite everywhere, for the flag check
        for a in h:
            bits = _bits(a)
            mask = np.uint32(0x7f800000) if a.dtype.itemsize == 4 else np.uint16(0x7c00)
            bits[(bits & mask) == mask] = 0
    devs = [_device_tensors(h, torch_dtype, 1) for h in hosts]
    tables = [xs.pointer_table(v) for _, v in devs]
    buckets = [torch.full((offs[-1],), 3.0, dtype=torch_dtype, device="cuda") for _ in range(W)]
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    xs.fuse_pack_many(plan, tables, buckets, flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    for h, b in zip(hosts, buckets):
        want = oracle.pack(h, np.asarray(offs, dtype=np.uint64))
        assert np.array_equal(_bits(b.cpu().numpy()), _bits(want))
    devs[3][1][4][20000] = float("inf")           # worker 3, last element of the large tensor
    xs.fuse_pack_many(plan, tables, buckets, flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 1
    xs.fuse_pack_many(plan, [], [])               # n = 0 is a no-op
    plan.destroy()


@pytest.mark.parametrize("wg_per_cu,max_wg", [(0, 0), (1, 0), (16, 0), (4096, 0), (0, 3), (16, 7)])
def test_launch_shapes_give_identical_copies(wg_per_cu, max_wg):
    """One chunk per workgroup (default), persistent grids of several sizes and capped grids
    (more chunks than workgroups: the loop covers the rest) all produce the same bits."""
    old = [xs.tuning_get(k) for k in range(xs.N_TUNING_KEYS)]
    try:
        xs.tuning_set(xs.TUNE_COPY_WG_PER_CU, wg_per_cu)
        xs.tuning_set(xs.TUNE_COPY_MAX_WG, max_wg)
        rng = np.random.default_rng(31)
        numel = [70000, 3, 0, 4097, 64, 200001, 17]
        offs = xs.bucket_layout(numel, 4)
        offs_np = np.asarray(offs, dtype=np.uint64)
        plan = xs.Plan(numel, offs, torch.float32)
        hosts = [[_random_bits(rng, n, np.float32) for n in numel] for _ in range(3)]
        devs = [_device_tensors(h, torch.float32, 1) for h in hosts]
        buckets = [torch.full((offs[-1],), 3.0, device="cuda") for _ in range(3)]
        xs.fuse_pack_many(plan, [xs.pointer_table(v) for _, v in devs], buckets)
        torch.cuda.synchronize()
        for h, b in zip(hosts, buckets):
            assert np.array_equal(_bits(b.cpu().numpy()), _bits(oracle.pack(h, offs_np)))
        outs_h, outs = _device_tensors([np.zeros(n, np.float32) for n in numel], torch.float32, 1)
        xs.fuse_unpack(plan, buckets[1], xs.pointer_table(outs))
        torch.cuda.synchronize()
        for h, v in zip(hosts[1], outs):
            assert np.array_equal(_bits(v.cpu().numpy()), _bits(h))
        plan.destroy()
    finally:
        for k, v in enumerate(old):
            xs.tuning_set(k, v)


def test_large_table_gives_each_workgroup_several_chunks():
    """A tensor list whose chunk-prefix table is beyond 4 KiB but still fits LDS."""
    rng = np.random.default_rng(32)
    numel = [int(n) for n in rng.integers(0, 40, size=5000)] + [100000]
    offs = xs.bucket_layout(numel, 1)
    plan = xs.Plan(numel, offs, torch.float16)
    flat = _random_bits(rng, sum(numel), np.float16)
    hosts = np.split(flat, np.cumsum(numel)[:-1])
    dev = torch.from_numpy(flat.copy()).cuda()
    views = list(torch.split(dev, numel))
    bucket = torch.full((offs[-1],), 3.0, dtype=torch.float16, device="cuda")
    xs.fuse_pack(plan, xs.pointer_table(views), bucket)
    torch.cuda.synchronize()
    want = oracle.pack([np.ascontiguousarray(h) for h in hosts], np.asarray(offs, dtype=np.uint64))
    assert np.array_equal(_bits(bucket.cpu().numpy()), _bits(want))
    plan.destroy()
