"""Seeded synthetic gradient sets for the fused gradient-synchronisation path.

This module is the one piece shared by the CPU oracle's tests and the HIP path's
tests and benchmark.  It holds tensor *shape lists* and random-number recipes
only: nothing here packs, reduces, averages or updates anything.

The paper (Section 3.1) trains ResNet-50 and VGG16 on ImageNet with 32 images per
worker.  Neither the dataset nor trained weights are needed for the
synchronisation path, which only sees a list of gradient tensors per worker, so
each workload below takes the tensor shapes of the named architecture and fills
them with seeded normal values.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np
import torch

BASE_SEED = 20210307

Shape = Tuple[int, ...]


def _numel(shape: Shape) -> int:
    n = 1
    for d in shape:
        n *= d
    return n


# ----------------------------------------------------------------------------
# shape lists
# ----------------------------------------------------------------------------
def tiny_mlp_shapes() -> List[Shape]:
    """784-256-10 perceptron: two weight matrices and two bias vectors."""
    return [(784, 256), (256,), (256, 10), (10,)]


def resnet50_shapes() -> List[Shape]:
    """ResNet-50: stem, four stages of (3, 4, 6, 3) bottleneck blocks, classifier.

    Every convolution is followed by a batch-norm scale and shift vector; the
    first block of each stage carries a 1x1 projection on the skip branch.
    """
    shapes: List[Shape] = [(64, 3, 7, 7), (64,), (64,)]
    inplanes = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            out = planes * 4
            shapes += [(planes, inplanes, 1, 1), (planes,), (planes,)]
            shapes += [(planes, planes, 3, 3), (planes,), (planes,)]
            shapes += [(out, planes, 1, 1), (out,), (out,)]
            if b == 0:
                shapes += [(out, inplanes, 1, 1), (out,), (out,)]
            inplanes = out
    shapes += [(1000, 2048), (1000,)]
    return shapes


def vgg16_shapes() -> List[Shape]:
    """VGG-16: thirteen 3x3 convolutions with bias and three dense layers."""
    shapes: List[Shape] = []
    cin = 3
    for cout in (64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512):
        shapes += [(cout, cin, 3, 3), (cout,)]
        cin = cout
    shapes += [(4096, 25088), (4096,), (4096, 4096), (4096,), (1000, 4096), (1000,)]
    return shapes


def bert_large_shapes() -> List[Shape]:
    """BERT-large encoder: 24 layers, hidden 1024, FFN 4096, vocabulary 30522,
    512 positions, 2 token types, with the pooler and without a language-model head."""
    h, ffn = 1024, 4096
    shapes: List[Shape] = [(30522, h), (512, h), (2, h), (h,), (h,)]
    for _ in range(24):
        for _qkvo in range(4):
            shapes += [(h, h), (h,)]
        shapes += [(h,), (h,)]
        shapes += [(ffn, h), (ffn,), (h, ffn), (h,)]
        shapes += [(h,), (h,)]
    shapes += [(h, h), (h,)]
    return shapes


# ----------------------------------------------------------------------------
# workload records
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    shapes: Tuple[Shape, ...]
    W: int                      # number of worker replicas resident on the GPU
    grad_dtype: str             # "f32", "f16" or "bf16"
    grad_std: float
    param_std: float
    lr: float
    momentum: float
    weight_decay: float
    loss_scale: float = 1.0
    inf_fraction: float = 0.0   # share of replica 0's elements forced to +inf
    seed: int = BASE_SEED
    numel: Tuple[int, ...] = field(init=False)

    def __post_init__(self):
        object.__setattr__(self, "numel", tuple(_numel(s) for s in self.shapes))

    @property
    def n_tensors(self) -> int:
        return len(self.shapes)

    @property
    def n_elems(self) -> int:
        return sum(self.numel)

    @property
    def grad_bytes(self) -> int:
        return 4 if self.grad_dtype == "f32" else 2

    @property
    def torch_grad_dtype(self) -> torch.dtype:
        return {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[self.grad_dtype]


def _wl(name, shapes, **kw) -> Workload:
    return Workload(name=name, shapes=tuple(tuple(s) for s in shapes), **kw)


TINY_MLP = _wl("tiny_mlp", tiny_mlp_shapes(), W=2, grad_dtype="f32", grad_std=0.01,
               param_std=0.05, lr=0.1, momentum=0.9, weight_decay=0.0)
RESNET50 = _wl("resnet50", resnet50_shapes(), W=8, grad_dtype="f32", grad_std=1e-3,
               param_std=0.05, lr=0.1, momentum=0.9, weight_decay=1e-4)
VGG16 = _wl("vgg16", vgg16_shapes(), W=8, grad_dtype="f32", grad_std=1e-3,
            param_std=0.05, lr=0.1, momentum=0.9, weight_decay=1e-4)
BERT_LARGE_F16 = _wl("bert_large_f16", bert_large_shapes(), W=16, grad_dtype="f16",
                     grad_std=1e-3, param_std=0.05, lr=0.1, momentum=0.9,
                     weight_decay=1e-4, loss_scale=1024.0)
BERT_LARGE_F16_INF = _wl("bert_large_f16_inf", bert_large_shapes(), W=16, grad_dtype="f16",
                         grad_std=1e-3, param_std=0.05, lr=0.1, momentum=0.9,
                         weight_decay=1e-4, loss_scale=1024.0, inf_fraction=1e-3)

WORKLOADS = {w.name: w for w in
             (TINY_MLP, RESNET50, VGG16, BERT_LARGE_F16, BERT_LARGE_F16_INF)}


def scaled(w: Workload, name: str, shapes: Sequence[Shape], W: int | None = None,
           grad_dtype: str | None = None) -> Workload:
    """Same value recipe as `w` on another tensor list (reduced parity cases)."""
    return _wl(name, shapes, W=w.W if W is None else W, grad_dtype=grad_dtype or w.grad_dtype,
               grad_std=w.grad_std, param_std=w.param_std, lr=w.lr, momentum=w.momentum,
               weight_decay=w.weight_decay, loss_scale=w.loss_scale,
               inf_fraction=w.inf_fraction, seed=w.seed)


# ----------------------------------------------------------------------------
# seeded value generators (torch, on whichever device is asked for)
# ----------------------------------------------------------------------------
def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def make_params(w: Workload, device="cpu") -> List[torch.Tensor]:
    """fp32 per-tensor parameters ~ N(0, param_std), seed = base."""
    g = _gen(device, w.seed)
    return [torch.randn(n, generator=g, device=device, dtype=torch.float32) * w.param_std
            for n in w.numel]


def make_replica_grads(w: Workload, replica: int, device="cpu") -> List[torch.Tensor]:
    """Per-tensor gradients of worker `replica` ~ N(0, grad_std), seed = base+1+replica.

    For half-precision workloads the stored values are the loss-scaled gradients; the
    stated std applies to the stored values.
    With inf_fraction > 0, that share of replica 0's elements, at seeded distinct
    positions over the whole tensor list, is set to +inf.
    """
    g = _gen(device, w.seed + 1 + replica)
    out = []
    for n in w.numel:
        t = torch.randn(n, generator=g, device=device, dtype=torch.float32) * w.grad_std
        out.append(t.to(w.torch_grad_dtype))
    if w.inf_fraction > 0.0 and replica == 0:
        total = w.n_elems
        k = int(round(w.inf_fraction * total))
        rng = np.random.Generator(np.random.PCG64(w.seed + 999))
        idx = np.unique(rng.integers(0, total, size=k + k // 8 + 8))
        rng.shuffle(idx)
        idx = np.sort(idx[:k])
        bounds = np.cumsum((0,) + w.numel)
        which = np.searchsorted(bounds, idx, side="right") - 1
        for t in np.unique(which):
            local = torch.from_numpy(idx[which == t] - bounds[t]).to(device)
            out[int(t)][local] = float("inf")
    return out


def make_flat(n: int, std: float, seed: int, dtype=torch.float32, device="cpu") -> torch.Tensor:
    """One flat seeded normal vector (for bucket-level tests that skip the tensor list)."""
    g = _gen(device, seed)
    return (torch.randn(n, generator=g, device=device, dtype=torch.float32) * std).to(dtype)


def fill_normal_(t: torch.Tensor, std: float, seed: int) -> torch.Tensor:
    """Seeded N(0, std) values written in place (no temporaries: for very large buffers)."""
    return t.normal_(0.0, std, generator=_gen(t.device, seed))
