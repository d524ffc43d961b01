"""Pins for the oracle's layout / pack / unpack (Section 2.1, tensor fusion)."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import oracle
from oracle import brute

SIZES = [0, 1, 3, 5, 17, 63, 64, 65, 4095, 4096, 4097]


def _bits(a):
    return a.view(np.uint32 if a.dtype.itemsize == 4 else np.uint16)


def test_layout_tight_is_prefix_sum():
    numel = [7, 0, 3, 1, 4096]
    offs = oracle.layout(numel, 1)
    assert offs.tolist() == [0, 7, 7, 10, 11, 4107]


def test_layout_aligned_closed_form():
    numel = [7, 0, 3, 64, 65, 1]
    offs = oracle.layout(numel, 64)
    # each start is the previous end rounded up to 64
    assert offs.tolist() == [0, 64, 64, 128, 192, 320, 384]
    assert all(o % 64 == 0 for o in offs)


def test_layout_rejects_zero_align():
    with pytest.raises(ValueError):
        oracle.layout([1, 2], 0)


def test_bucket_length_of_tiny_mlp_is_sum_numel():
    from paper_2103_07974_amd import workloads as wl
    offs = oracle.layout(wl.TINY_MLP.numel, 1)
    assert int(offs[-1]) == 203530 == wl.TINY_MLP.n_elems


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("align", [1, 4, 64])
def test_pack_unpack_identity_bitexact(dtype, align):
    rng = np.random.default_rng(7)
    tensors = []
    for n in SIZES:
        bits = rng.integers(0, 2 ** (8 * np.dtype(dtype).itemsize), size=n,
                            dtype=np.uint64).astype(_bits(np.zeros(1, dtype)).dtype)
        tensors.append(bits.view(dtype))          # arbitrary bit patterns: NaN payloads, -0.0, inf
    offs = oracle.layout([t.size for t in tensors], align)
    bucket = oracle.pack(tensors, offs)
    assert bucket.size == int(offs[-1])
    outs = oracle.unpack(bucket, [t.size for t in tensors], offs)
    for a, b in zip(tensors, outs):
        assert np.array_equal(_bits(a), _bits(b))
    # padding is +0 and every tensor sits at its offset
    covered = np.zeros(bucket.size, dtype=bool)
    for t, o in zip(tensors, offs[:-1]):
        assert np.array_equal(_bits(bucket[int(o):int(o) + t.size]), _bits(t))
        covered[int(o):int(o) + t.size] = True
    assert not _bits(bucket)[~covered].any()


def test_pack_equals_python_concatenation_when_tight():
    rng = np.random.default_rng(11)
    tensors = [rng.standard_normal(n).astype(np.float32) for n in (3, 0, 1, 8, 2)]
    offs = oracle.layout([t.size for t in tensors], 1)
    bucket = oracle.pack(tensors, offs)
    ref = brute.concat([t.tolist() for t in tensors])
    assert bucket.tolist() == ref
    back = brute.split(bucket.tolist(), [t.size for t in tensors])
    assert [t.tolist() for t in tensors] == back


def test_pack_from_unaligned_views():
    base = np.arange(100, dtype=np.float32)
    tensors = [base[1:6], base[7:8], base[9:40]]      # start addresses are 4-byte aligned only
    offs = oracle.layout([t.size for t in tensors], 1)
    bucket = oracle.pack([np.ascontiguousarray(t) for t in tensors], offs)
    assert bucket.tolist() == list(range(1, 6)) + [7] + list(range(9, 40))


def test_pack_empty_list():
    offs = oracle.layout([], 1)
    assert offs.tolist() == [0]
    assert oracle.pack([], offs).size == 0


@settings(max_examples=60, deadline=None)
@given(st.lists(st.integers(0, 300), min_size=0, max_size=12), st.sampled_from([1, 2, 4, 16, 64]),
       st.integers(0, 2 ** 31))
def test_pack_unpack_identity_random_lists(numel, align, seed):
    rng = np.random.default_rng(seed)
    tensors = [rng.integers(0, 2 ** 32, size=n, dtype=np.uint64).astype(np.uint32).view(np.float32)
               for n in numel]
    offs = oracle.layout(numel, align)
    assert int(offs[-1]) >= sum(numel)
    if align == 1:
        assert int(offs[-1]) == sum(numel)
    outs = oracle.unpack(oracle.pack(tensors, offs), numel, offs)
    for a, b in zip(tensors, outs):
        assert np.array_equal(_bits(a), _bits(b))
