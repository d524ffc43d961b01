"""Host threads driving independent tasks on their own streams at the same time: the library
keeps no per-call state outside its arguments (errors are thread-local), so the results must
equal the same steps issued from one thread."""
import threading

import pytest
import torch

from paper_2103_07974_amd import harness, workloads as wl, xs

pytestmark = pytest.mark.gpu

SHAPES = [[(300, 7), (64,), (5000,)], [(17,), (9000, 3)], [(4097,), (3,), (128, 9)], [(70000,)]]
STEPS = 40


def _steps(task, stream, fused_gather):
    w = task.workload
    with torch.cuda.stream(stream):
        for _ in range(STEPS):
            if fused_gather:
                xs.fused_gather_reduce_sgd(task.gplan, task.gather_table, w.W, task.params,
                                           task.momentum, w.lr, w.momentum, w.weight_decay, 1.0,
                                           param_tensor_ptrs=task.param_table, stream=stream)
            else:
                xs.fuse_pack_many(task.gplan, task.grad_tables, task.buckets, None, stream)
                xs.fused_reduce_sgd(task.buckets, task.n_bucket, task.params, task.momentum, w.lr,
                                    w.momentum, w.weight_decay, 1.0, stream=stream)
                xs.fuse_unpack(task.pplan, task.params, task.param_table, stream)
    stream.synchronize()


def test_concurrent_host_threads_match_one_thread():
    def make():
        return [harness.make_task(wl.scaled(wl.RESNET50, f"thr{i}", s, W=2 + i), "cuda", 16)
                for i, s in enumerate(SHAPES)]
    serial, threaded = make(), make()
    for i, t in enumerate(serial):
        _steps(t, torch.cuda.Stream(), fused_gather=bool(i & 1))
    errors = []

    def worker(i, t):
        try:
            torch.cuda.set_device(0)
            _steps(t, torch.cuda.Stream(), fused_gather=bool(i & 1))
            # an error raised in this thread is this thread's own
            with pytest.raises(xs.XsError):
                xs.fused_reduce_sgd(t.buckets, t.n_bucket, t.params, t.momentum[1:], 0.1, 0.9, 0.0)
            assert "aligned" in xs.last_error()
        except Exception as e:      # surfaced in the main thread below
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=worker, args=(i, t)) for i, t in enumerate(threaded)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for a, b in zip(serial, threaded):
        assert torch.equal(a.params, b.params) and torch.equal(a.momentum, b.momentum)
        for p, q in zip(a.param_tensors, b.param_tensors):
            assert torch.equal(p, q)
