"""Brute-force evaluation of one fused gradient synchronisation on tiny inputs.

TEST INFRASTRUCTURE ONLY.  Written independently of xs_oracle.c (no shared code)
as a pin for it: Python lists, one scalar operation at a time.  `real` selects
the arithmetic: Python float (IEEE double) or numpy.float32.

Steps (arXiv 2103.07974): Section 2.1 tensor fusion = list concatenation;
Algorithm 1 "Receive averaged gradients" = sum over workers divided by W;
Algorithm 1 "Model Update" = momentum SGD, d = g + wd*x, v = mu*v + d, x = x - lr*v.
"""
from __future__ import annotations

import math
from typing import List, Sequence

import numpy as np


def concat(tensors: Sequence[Sequence]) -> list:
    """Tight fusion (no padding): the bucket is the list of all elements in order."""
    bucket: list = []
    for t in tensors:
        bucket.extend(list(t))
    return bucket


def split(bucket: Sequence, numel: Sequence[int]) -> List[list]:
    out, pos = [], 0
    for n in numel:
        out.append(list(bucket[pos:pos + n]))
        pos += n
    return out


def step(grads: Sequence[Sequence[Sequence]], params: Sequence[Sequence], momentum: Sequence,
         lr, mu, wd, inv_loss_scale=1.0, real=float):
    """grads[w][t][k], params[t][k], momentum[j] (bucket order).

    Returns (new_params[t][k], new_momentum[j], found_inf).  With real=float the
    average is s / W * inv_loss_scale in double; with real=numpy.float32 replicas
    are added left to right and scaled by the single constant inv_loss_scale*(1/W),
    every operation rounded to single.
    """
    W = len(grads)
    numel = [len(p) for p in params]
    buckets = [concat(g) for g in grads]
    x = [real(e) for e in concat(params)]
    v = [real(e) for e in momentum]
    for b in buckets:
        for e in b:
            if not math.isfinite(float(e)):
                return split(x, numel), v, True
    if real is float:
        lr, mu, wd, inv = float(lr), float(mu), float(wd), float(inv_loss_scale)
    else:
        lr, mu, wd, inv = real(lr), real(mu), real(wd), real(inv_loss_scale)
        c = inv * (real(1.0) / real(W))
    for j in range(len(x)):
        s = real(buckets[0][j])
        for w in range(1, W):
            s = s + real(buckets[w][j])
        g_avg = s / W * inv if real is float else s * c
        d = g_avg + wd * x[j]
        v[j] = mu * v[j] + d
        x[j] = x[j] - lr * v[j]
    return split(x, numel), v, False
