"""Device-side set-up of one training task's synchronisation state for tests and the
benchmark: allocation and pointer tables only, no arithmetic of the method."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, List, Optional

import torch

from . import workloads as wl
from . import xs

DEFAULT_ALIGN = 64   # elements; keeps every tensor's bucket segment 128/256-byte aligned


@dataclass
class TaskState:
    workload: wl.Workload
    align: int
    offsets: List[int]
    gplan: xs.Plan
    pplan: xs.Plan
    grads: List[List[torch.Tensor]]          # [W][T] per-tensor gradients (device)
    grad_tables: List[torch.Tensor]          # [W] device pointer tables
    buckets: List[torch.Tensor]              # [W] fused gradient buckets
    param_tensors: List[torch.Tensor]        # [T] per-tensor parameter views (device)
    param_table: torch.Tensor
    params: torch.Tensor                     # fp32 bucket
    momentum: torch.Tensor                   # fp32 bucket
    found_inf: torch.Tensor                  # int32[1]
    gather_table: torch.Tensor               # [T][W] device pointer table for the gathering form

    @property
    def n_bucket(self) -> int:
        return self.offsets[-1]

    def reduce_bytes(self) -> int:
        """Algorithmic bytes of the fused reduce + SGD: W replicas read, parameters and
        momentum read and written, valid elements only."""
        w = self.workload
        return (w.W * w.grad_bytes + 16) * w.n_elems

    def pack_bytes(self) -> int:
        return 2 * self.workload.grad_bytes * self.workload.n_elems

    def unpack_bytes(self) -> int:
        return 2 * 4 * self.workload.n_elems

    def gather_bytes(self, views: bool = True) -> int:
        """Algorithmic bytes of the gathering form: as reduce_bytes, plus the per-tensor
        parameter views written when the unpack is fused in."""
        return self.reduce_bytes() + (4 * self.workload.n_elems if views else 0)

    def make_app(self, compute: Optional[Callable[[int], None]] = None,
                 use_found_inf: bool = False, fused_gather: bool = False,
                 tensor_hp: Optional[torch.Tensor] = None, tuning=None,
                 fused_unpack: bool = False) -> xs.App:
        w = self.workload
        return xs.App(self.gplan, self.pplan, self.grad_tables, self.buckets, self.params,
                      self.momentum, self.param_table, w.lr, w.momentum, w.weight_decay,
                      1.0 / w.loss_scale, self.found_inf if use_found_inf else None, compute,
                      gather_table=self.gather_table if fused_gather else None, W=w.W,
                      tensor_hp=tensor_hp, tuning=tuning, fused_unpack=fused_unpack)


def make_task(w: wl.Workload, device="cuda", align: int = DEFAULT_ALIGN,
              shared_grads: bool = False, pooled: bool = True) -> TaskState:
    """Allocate and fill everything one task's synchronisation touches.

    shared_grads=True makes all W workers' tensor lists point at worker 0's tensors
    (saves memory in timing runs of the largest workload; the buckets stay distinct).
    pooled=False gives every bucket, the parameters and the momentum an allocation of their
    own (for comparison with the pool described below).
    """
    dev = torch.device(device)
    offsets = xs.bucket_layout(w.numel, align)
    gplan = xs.Plan(w.numel, offsets, w.torch_grad_dtype)
    pplan = xs.Plan(w.numel, offsets, torch.float32)
    grads = []
    for r in range(w.W):
        if shared_grads and r > 0:
            grads.append(grads[0])
        else:
            grads.append(wl.make_replica_grads(w, r, dev))
    grad_tables = [xs.pointer_table(g, dev) for g in grads]
    n_bucket = offsets[-1]
    # The W buckets, the parameters and the momentum come out of ONE device allocation, each
    # starting at a multiple of 2 MiB (xs_pool_layout; a receive pool, as a worker would keep
    # one): on MI355X the fused reduce + SGD streams 4-7 % faster over such a pool than over
    # W + 2 separate allocations of the same sizes.
    sizes = [(n_bucket, w.torch_grad_dtype)] * w.W + [(n_bucket, torch.float32)] * 2
    flat = xs.pool_alloc(sizes, dev) if pooled else [torch.empty(n, dtype=dt, device=dev) for n, dt in sizes]
    buckets, params, momentum = flat[:w.W], flat[w.W].zero_(), flat[w.W + 1].zero_()
    param_tensors = wl.make_params(w, dev)
    param_table = xs.pointer_table(param_tensors, dev)
    xs.fuse_pack(pplan, param_table, params)            # parameters enter the bucket layout
    found_inf = torch.zeros(1, dtype=torch.int32, device=dev)
    gather_table = xs.gather_pointer_table(grads, dev)
    torch.cuda.synchronize(dev)
    return TaskState(w, align, offsets, gplan, pplan, grads, grad_tables, buckets, param_tensors,
                     param_table, params, momentum, found_inf, gather_table)


# ---------------------------------------------------------------------------------------
# A real forward + backward as the compute side of a task (Algorithm 1, "Gradient
# computation"): a ReLU MLP classifier on seeded synthetic data, one micro-batch per worker,
# run through PyTorch autograd.  The task's per-layer parameter views ARE the model's weights
# and biases, and worker w's gradients land in task.grads[w], so the library's kernels read
# and write the model directly.
# ---------------------------------------------------------------------------------------
@dataclass
class MlpTask:
    state: TaskState
    dims: List[int]
    inputs: List[torch.Tensor]      # [W] micro-batches
    targets: List[torch.Tensor]     # [W] class labels

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        p = self.state.param_tensors
        n_layers = len(self.dims) - 1
        for l in range(n_layers):
            x = torch.nn.functional.linear(x, p[2 * l].view(self.dims[l + 1], self.dims[l]), p[2 * l + 1])
            if l + 1 < n_layers:
                x = torch.relu(x)
        return x

    def compute(self, stream_ptr: int) -> None:
        """Forward + backward of every worker's micro-batch, enqueued on the given stream."""
        s = torch.cuda.ExternalStream(stream_ptr) if stream_ptr else torch.cuda.current_stream()
        params = self.state.param_tensors
        with torch.cuda.stream(s):
            for w in range(self.state.workload.W):
                loss = torch.nn.functional.cross_entropy(self.forward(self.inputs[w]), self.targets[w])
                gs = torch.autograd.grad(loss, params)
                torch._foreach_copy_(self.state.grads[w], list(gs))


def make_mlp_task(name: str, dims: List[int], W: int, batch: int, device="cuda", seed: int = 1234,
                  lr: float = 0.05, momentum: float = 0.9, weight_decay: float = 1e-4,
                  align: int = DEFAULT_ALIGN) -> MlpTask:
    shapes = []
    for l in range(len(dims) - 1):
        shapes += [(dims[l + 1], dims[l]), (dims[l + 1],)]
    w = wl.Workload(name=name, shapes=tuple(shapes), W=W, grad_dtype="f32", grad_std=1e-3,
                    param_std=1.0 / max(dims) ** 0.5, lr=lr, momentum=momentum,
                    weight_decay=weight_decay, seed=seed)
    state = make_task(w, device, align)
    for p in state.param_tensors:
        p.requires_grad_(True)
    g = torch.Generator(device=device); g.manual_seed(seed + 5)
    inputs = [torch.randn(batch, dims[0], generator=g, device=device) for _ in range(W)]
    targets = [torch.randint(0, dims[-1], (batch,), generator=g, device=device) for _ in range(W)]
    return MlpTask(state, list(dims), inputs, targets)
