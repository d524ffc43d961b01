"""CPU oracle for the fused gradient-synchronisation step (arXiv 2103.07974).

TEST INFRASTRUCTURE ONLY.  Importable from tests/, the smoke check and the
benchmark's cpu_baseline leg; the HIP library and its binding never import it,
and it imports nothing from them.

  xs_oracle.c   scalar C loops: layout, pack, unpack, overflow test, average+update
  brute.py      the same steps one numpy scalar operation at a time (tiny inputs)
  timeline.py   event-time model of Algorithm 1's schedule
  schedule.py   Algorithm 1 executed literally over abstract tasks

This file is the ctypes loader for xs_oracle.c plus numpy argument marshalling.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "xs_oracle.c")
_LIB = os.path.join(_HERE, "libxs_oracle.so")

F32 = 0
F16 = 1
BF16 = 2      # passed as numpy uint16 arrays holding bfloat16 bit patterns


def build(force: bool = False) -> str:
    """Compile xs_oracle.c with gcc.  No fast-math, no FMA contraction."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        u64p = ctypes.POINTER(ctypes.c_uint64)
        vpp = ctypes.POINTER(ctypes.c_void_p)
        L.xo_layout.argtypes = [u64p, ctypes.c_uint32, ctypes.c_uint64, u64p]
        L.xo_pack.argtypes = [ctypes.c_uint32, ctypes.c_uint32, vpp, u64p, u64p, ctypes.c_void_p]
        L.xo_unpack.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p, u64p, u64p, vpp]
        L.xo_any_nonfinite.argtypes = [vpp, ctypes.c_uint32, ctypes.c_int, ctypes.c_uint32, u64p, u64p]
        L.xo_reduce_sgd_f64.argtypes = [vpp, ctypes.c_uint32, ctypes.c_int, ctypes.c_uint64,
                                        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_double,
                                        ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                        ctypes.c_int]
        L.xo_reduce_sgd_f32.argtypes = [vpp, ctypes.c_uint32, ctypes.c_int, ctypes.c_uint64,
                                        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float,
                                        ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                        ctypes.c_int]
        L.xo_round_params.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p]
        for f in (L.xo_layout, L.xo_pack, L.xo_unpack, L.xo_any_nonfinite,
                  L.xo_reduce_sgd_f64, L.xo_reduce_sgd_f32, L.xo_round_params):
            f.restype = ctypes.c_int
        _lib = L
    return _lib


# ---------------------------------------------------------------- marshalling
def _u64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.uint64))


def _u64p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64))


def _ptr_array(arrays: Sequence[np.ndarray]):
    arr = (ctypes.c_void_p * max(len(arrays), 1))()
    for i, a in enumerate(arrays):
        arr[i] = a.ctypes.data
    return arr


def _code(dtype) -> int:
    dt = np.dtype(dtype)
    if dt == np.float32:
        return F32
    if dt == np.float16:
        return F16
    if dt == np.uint16:
        return BF16
    raise TypeError(f"gradient dtype {dt} is not float32, float16 or uint16 (bfloat16 bits)")


def _check_c(a: np.ndarray, name: str):
    if not isinstance(a, np.ndarray) or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name} must be a C-contiguous numpy array")


# ---------------------------------------------------------------- public API
def layout(numel: Sequence[int], align: int = 1) -> np.ndarray:
    """Bucket offsets (length T+1) of a tensor list; Section 2.1, tensor fusion."""
    n = _u64(numel)
    out = np.zeros(len(n) + 1, dtype=np.uint64)
    rc = lib().xo_layout(_u64p(n), len(n), int(align), _u64p(out))
    if rc != 0:
        raise ValueError("align must be >= 1")
    return out


def pack(tensors: Sequence[np.ndarray], offsets: np.ndarray) -> np.ndarray:
    """Fuse a list of flat arrays (one dtype) into a new bucket, padding = +0."""
    offsets = _u64(offsets)
    if len(offsets) != len(tensors) + 1:
        raise ValueError("offsets must have one more entry than tensors")
    dt = tensors[0].dtype if tensors else np.dtype(np.float32)
    for i, t in enumerate(tensors):
        _check_c(t, f"tensors[{i}]")
        if t.dtype != dt:
            raise TypeError("all tensors of a bucket share one dtype")
    numel = _u64([t.size for t in tensors])
    bucket = np.empty(int(offsets[-1]), dtype=dt)
    bucket.view(np.uint8)[...] = 0xA5      # pack must overwrite everything
    lib().xo_pack(dt.itemsize, len(tensors), _ptr_array(tensors), _u64p(numel),
                  _u64p(offsets), bucket.ctypes.data)
    return bucket


def unpack(bucket: np.ndarray, numel: Sequence[int], offsets: np.ndarray) -> List[np.ndarray]:
    """Split a bucket back into per-tensor flat arrays."""
    _check_c(bucket, "bucket")
    offsets = _u64(offsets)
    n = _u64(numel)
    outs = [np.empty(int(k), dtype=bucket.dtype) for k in n]
    lib().xo_unpack(bucket.dtype.itemsize, len(outs), bucket.ctypes.data, _u64p(n),
                    _u64p(offsets), _ptr_array(outs))
    return outs


def any_nonfinite(replicas: Sequence[np.ndarray], numel: Sequence[int], offsets: np.ndarray) -> bool:
    """True if a valid (non-padding) element of any replica bucket is inf or NaN."""
    for i, r in enumerate(replicas):
        _check_c(r, f"replicas[{i}]")
    n = _u64(numel)
    offsets = _u64(offsets)
    return bool(lib().xo_any_nonfinite(_ptr_array(replicas), len(replicas),
                                       _code(replicas[0].dtype), len(n), _u64p(n),
                                       _u64p(offsets)))


def reduce_sgd_f64(replicas: Sequence[np.ndarray], x: np.ndarray, v: np.ndarray, lr: float,
                   mu: float, wd: float, inv_loss_scale: float = 1.0, threads: int = 1) -> None:
    """Average W replica buckets and apply one momentum-SGD step in double, in place.

    x, v: float64 arrays of the bucket length.  Hyper-parameters are taken as
    given (pass np.float32 values widened to float to mirror a float32 caller).
    """
    _check_c(x, "x"); _check_c(v, "v")
    if x.dtype != np.float64 or v.dtype != np.float64:
        raise TypeError("x and v must be float64")
    n = x.size
    for i, r in enumerate(replicas):
        _check_c(r, f"replicas[{i}]")
        if r.size < n:
            raise ValueError("replica shorter than x")
    if v.size != n:
        raise ValueError("x and v differ in length")
    rc = lib().xo_reduce_sgd_f64(_ptr_array(replicas), len(replicas), _code(replicas[0].dtype),
                                 n, x.ctypes.data, v.ctypes.data, float(lr), float(mu),
                                 float(wd), float(inv_loss_scale), int(threads))
    if rc != 0:
        raise ValueError("W must be >= 1")


def reduce_sgd_f32(replicas: Sequence[np.ndarray], x: np.ndarray, v: np.ndarray, lr: float,
                   mu: float, wd: float, inv_loss_scale: float = 1.0, threads: int = 1) -> None:
    """Same steps with every operation rounded to float32, replicas added left to right."""
    _check_c(x, "x"); _check_c(v, "v")
    if x.dtype != np.float32 or v.dtype != np.float32:
        raise TypeError("x and v must be float32")
    n = x.size
    for i, r in enumerate(replicas):
        _check_c(r, f"replicas[{i}]")
        if r.size < n:
            raise ValueError("replica shorter than x")
    if v.size != n:
        raise ValueError("x and v differ in length")
    rc = lib().xo_reduce_sgd_f32(_ptr_array(replicas), len(replicas), _code(replicas[0].dtype),
                                 n, x.ctypes.data, v.ctypes.data, float(lr), float(mu),
                                 float(wd), float(inv_loss_scale), int(threads))
    if rc != 0:
        raise ValueError("W must be >= 1")


def reduce_sgd_per_tensor(replicas: Sequence[np.ndarray], x: np.ndarray, v: np.ndarray,
                          offsets: np.ndarray, tensor_hp: Sequence[Sequence[float]],
                          inv_loss_scale: float = 1.0) -> None:
    """Average + update with hyper-parameters per tensor ("Model Update" of Algorithm 1 applied
    with one (lr, mu, wd) triple per layer, the usual parameter groups of SGD: no weight decay
    on biases and normalisation layers, per-group learning rates).

    tensor_hp[t] = (lr, mu, wd) governs bucket elements offsets[t] .. offsets[t+1]-1, i.e.
    tensor t and the padding behind it.  Working precision follows x (float64 or float32).
    """
    offsets = _u64(offsets)
    if len(tensor_hp) + 1 != len(offsets):
        raise ValueError("one hyper-parameter triple per tensor")
    if x.dtype == np.float64:
        step = reduce_sgd_f64
    elif x.dtype == np.float32:
        step = reduce_sgd_f32
    else:
        raise TypeError("x must be float64 or float32")
    for t, (lr, mu, wd) in enumerate(tensor_hp):
        a, b = int(offsets[t]), int(offsets[t + 1])
        if b > a:
            step([r[a:b] for r in replicas], x[a:b], v[a:b], lr, mu, wd, inv_loss_scale)


def round_params(x: np.ndarray, dtype_code: int) -> np.ndarray:
    """float32 values rounded to binary16 / bfloat16 (ties to even); returns uint16 bit patterns."""
    _check_c(x, "x")
    if x.dtype != np.float32:
        raise TypeError("x must be float32")
    out = np.empty(x.size, dtype=np.uint16)
    rc = lib().xo_round_params(x.ctypes.data, x.size, int(dtype_code), out.ctypes.data)
    if rc != 0:
        raise ValueError("dtype_code must be F16 or BF16")
    return out


def sync_step(grads: Sequence[Sequence[np.ndarray]], params: Sequence[np.ndarray],
              v_bucket: np.ndarray, lr: float, mu: float, wd: float,
              inv_loss_scale: float = 1.0, align: int = 1, precision: str = "f64",
              tensor_hp: Sequence[Sequence[float]] | None = None, threads: int = 1):
    """One whole synchronisation of one task: pack every worker's tensor list, test
    for overflow, average + update, unpack the new parameters.

    grads[w][t]: worker w's gradient tensor t (flat).  params[t]: float32 parameters.
    v_bucket: momentum in bucket layout (float64 for "f64", float32 for "f32"),
    updated in place.  Returns (new_params list in the working precision, found_inf).
    A skipped step returns the parameters unchanged.  tensor_hp, if given, replaces
    (lr, mu, wd) by one triple per tensor.  threads > 1 runs the element loop of the
    average + update under OpenMP (elements are independent; results do not change).
    """
    numel = [p.size for p in params]
    offs = layout(numel, align)
    buckets = [pack(list(g), offs) for g in grads]
    work = np.float64 if precision == "f64" else np.float32
    x = pack([np.ascontiguousarray(p, dtype=np.float32) for p in params], offs).astype(work)
    if any_nonfinite(buckets, numel, offs):
        return unpack(x, numel, offs), True
    if tensor_hp is not None:
        reduce_sgd_per_tensor(buckets, x, v_bucket, offs, tensor_hp, inv_loss_scale)
    elif precision == "f64":
        reduce_sgd_f64(buckets, x, v_bucket, lr, mu, wd, inv_loss_scale, threads)
    else:
        reduce_sgd_f32(buckets, x, v_bucket, lr, mu, wd, inv_loss_scale, threads)
    return unpack(x, numel, offs), False
