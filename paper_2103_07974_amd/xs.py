"""ctypes binding of libxs.so: same names as include/xs.h, argument marshalling only.

PyTorch supplies device memory and streams; every step of the path (pack, reduce,
average, update, unpack, event wiring of the crossover schedule) runs inside the
library.  There is no fallback: if libxs.so is missing or fails to load, every call
raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libxs.so")

XS_OK = 0
XS_ERR_INVALID_ARG = -1
XS_ERR_ALIGNMENT = -2
XS_ERR_SIZE = -3
XS_ERR_UNSUPPORTED = -4
XS_ERR_HIP = -5
XS_ERR_NOMEM = -6
XS_ERR_STATE = -7

XS_F32 = 0
XS_F16 = 1
XS_MAX_REPLICAS = 32

XS_BF16 = 2

TUNE_REDUCE_WG_PER_CU = 0
TUNE_COPY_WG_PER_CU = 1
TUNE_NT_GRADS = 2
TUNE_NT_STATE = 3
TUNE_REDUCE_LDS_RESERVE = 4
TUNE_REDUCE_MAX_WG = 5
TUNE_COPY_MAX_WG = 6
TUNE_COPY_NT = 7
TUNE_GATHER_LDS_RESERVE = 8
TUNE_COPY_LDS_RESERVE = 9
TUNE_REDUCE_WAVES_PER_WG = 10
TUNE_REDUCE_SMALL = 11
TUNE_COPY_WAVES_PER_WG = 12
N_TUNING_KEYS = 13

PRESET_ALONE = 0
PRESET_BESIDE_COMPUTE = 1
PRESET_LEAVE_WAVE_SLOTS = 2

EXPORTS = [
    "xs_status_string", "xs_last_error", "xs_bucket_layout", "xs_pool_layout", "xs_plan_create", "xs_plan_destroy",
    "xs_plan_bucket_elems", "xs_plan_n_tensors", "xs_fuse_pack", "xs_fuse_pack_many", "xs_fuse_pack_static",
    "xs_fuse_unpack",
    "xs_fused_reduce_sgd", "xs_fused_reduce_sgd_mp", "xs_fused_gather_reduce_sgd",
    "xs_fused_gather_reduce_sgd_mp", "xs_fused_reduce_sgd_pt", "xs_fused_gather_reduce_sgd_pt",
    "xs_fused_reduce_sgd_unpack",
    "xs_app_create", "xs_app_destroy", "xs_app_sync", "xs_crossover_step",
    "xs_crossover_drain", "xs_crossover_iteration", "xs_crossover_finish", "xs_app_wait_sync",
    "xs_tuning_set", "xs_tuning_get", "xs_tuning_preset",
]


class XsError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}: {detail}")


class SgdHparams(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("momentum", ctypes.c_float),
                ("weight_decay", ctypes.c_float), ("inv_loss_scale", ctypes.c_float)]


class MpOptions(ctypes.Structure):
    _fields_ = [("model_copy", ctypes.c_void_p), ("model_copy_dtype", ctypes.c_int),
                ("view_dtype", ctypes.c_int)]


COMPUTE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)


class AppDesc(ctypes.Structure):
    _fields_ = [("gradient_plan", ctypes.c_void_p), ("parameter_plan", ctypes.c_void_p),
                ("W", ctypes.c_uint32),
                ("grad_tensor_ptrs", ctypes.POINTER(ctypes.c_void_p)),
                ("replica_buckets", ctypes.POINTER(ctypes.c_void_p)),
                ("params", ctypes.c_void_p), ("momentum", ctypes.c_void_p),
                ("param_tensor_ptrs", ctypes.c_void_p),
                ("hp", SgdHparams), ("found_inf", ctypes.c_void_p),
                ("compute", COMPUTE_FN), ("compute_ctx", ctypes.c_void_p),
                ("flags", ctypes.c_uint32), ("grad_ptrs_tw", ctypes.c_void_p),
                ("tensor_hp", ctypes.c_void_p), ("tuning", ctypes.POINTER(ctypes.c_int32))]


XS_APP_FUSED_GATHER = 1
XS_APP_FUSED_UNPACK = 2


_lib = None


def lib() -> ctypes.CDLL:
    """Load libxs.so (built in-tree by paper_2103_07974_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; "
                          f"g.build()'` at the repository root")
    L = ctypes.CDLL(LIB_PATH)
    u64p = ctypes.POINTER(ctypes.c_uint64)
    vp = ctypes.c_void_p
    L.xs_status_string.argtypes = [ctypes.c_int]; L.xs_status_string.restype = ctypes.c_char_p
    L.xs_last_error.argtypes = []; L.xs_last_error.restype = ctypes.c_char_p
    L.xs_bucket_layout.argtypes = [u64p, ctypes.c_uint32, ctypes.c_uint64, u64p]
    L.xs_pool_layout.argtypes = [u64p, ctypes.c_uint32, u64p]
    L.xs_plan_create.argtypes = [u64p, u64p, ctypes.c_uint32, ctypes.c_int, ctypes.POINTER(vp)]
    L.xs_plan_destroy.argtypes = [vp]
    L.xs_plan_bucket_elems.argtypes = [vp]; L.xs_plan_bucket_elems.restype = ctypes.c_uint64
    L.xs_plan_n_tensors.argtypes = [vp]; L.xs_plan_n_tensors.restype = ctypes.c_uint32
    L.xs_fuse_pack.argtypes = [vp, vp, vp, vp, vp]
    L.xs_fuse_pack_many.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.c_uint32, vp, vp]
    L.xs_fuse_pack_static.argtypes = [u64p, u64p, ctypes.c_uint32, ctypes.c_int, vp, vp, vp, vp]
    L.xs_fuse_unpack.argtypes = [vp, vp, vp, vp]
    L.xs_fused_reduce_sgd.argtypes = [ctypes.POINTER(vp), ctypes.c_uint32, ctypes.c_int,
                                      ctypes.c_uint64, vp, vp, vp, vp,
                                      ctypes.POINTER(SgdHparams), vp, vp]
    L.xs_fused_reduce_sgd_mp.argtypes = [ctypes.POINTER(vp), ctypes.c_uint32, ctypes.c_int,
                                         ctypes.c_uint64, vp, vp, vp, vp,
                                         ctypes.POINTER(SgdHparams), vp,
                                         ctypes.POINTER(MpOptions), vp]
    L.xs_fused_gather_reduce_sgd.argtypes = [vp, vp, ctypes.c_uint32, vp, vp, vp, vp, vp,
                                             ctypes.POINTER(SgdHparams), vp, vp]
    L.xs_fused_gather_reduce_sgd_mp.argtypes = [vp, vp, ctypes.c_uint32, vp, vp, vp, vp, vp,
                                                ctypes.POINTER(SgdHparams), vp,
                                                ctypes.POINTER(MpOptions), vp]
    L.xs_fused_reduce_sgd_pt.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_uint32, vp, vp, vp, vp, vp,
                                         ctypes.c_float, vp, ctypes.POINTER(MpOptions), vp]
    L.xs_fused_gather_reduce_sgd_pt.argtypes = [vp, vp, ctypes.c_uint32, vp, vp, vp, vp, vp, vp,
                                                ctypes.c_float, vp, ctypes.POINTER(MpOptions), vp]
    L.xs_fused_reduce_sgd_unpack.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_uint32, vp, vp, vp,
                                             ctypes.POINTER(SgdHparams), vp, vp,
                                             ctypes.POINTER(MpOptions), vp]
    L.xs_app_create.argtypes = [ctypes.POINTER(AppDesc), ctypes.POINTER(vp)]
    L.xs_app_destroy.argtypes = [vp]
    L.xs_app_sync.argtypes = [vp, vp]
    L.xs_crossover_step.argtypes = [vp, vp, vp, vp]
    L.xs_crossover_drain.argtypes = [vp, vp]
    L.xs_app_wait_sync.argtypes = [vp, vp]
    L.xs_crossover_iteration.argtypes = [ctypes.POINTER(vp), ctypes.c_uint32, vp, vp]
    L.xs_crossover_finish.argtypes = [ctypes.POINTER(vp), ctypes.c_uint32, vp]
    L.xs_tuning_preset.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int32)]
    L.xs_tuning_set.argtypes = [ctypes.c_int, ctypes.c_int]
    L.xs_tuning_get.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
    for name in EXPORTS:
        f = getattr(L, name)
        if name not in ("xs_status_string", "xs_last_error", "xs_plan_bucket_elems",
                        "xs_plan_n_tensors"):
            f.restype = ctypes.c_int
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().xs_status_string(int(status)).decode()


def last_error() -> str:
    return lib().xs_last_error().decode()


def _check(rc: int, where: str) -> None:
    if rc != XS_OK:
        raise XsError(rc, where, last_error())


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _dptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    return t.data_ptr() or None


def dtype_code(dtype: torch.dtype) -> int:
    if dtype == torch.float32:
        return XS_F32
    if dtype == torch.float16:
        return XS_F16
    if dtype == torch.bfloat16:
        return XS_BF16
    raise TypeError(f"unsupported element dtype {dtype}")


# ---------------------------------------------------------------- layout / plan
def bucket_layout(numel: Sequence[int], align_elems: int = 1) -> List[int]:
    n = len(numel)
    a = (ctypes.c_uint64 * max(n, 1))(*numel)
    out = (ctypes.c_uint64 * (n + 1))()
    _check(lib().xs_bucket_layout(a, n, int(align_elems), out), "xs_bucket_layout")
    return list(out)


POOL_ALIGN = 2 << 20


def pool_layout(nbytes: Sequence[int]) -> List[int]:
    """Byte offsets of a task's flat buffers inside one allocation (xs_pool_layout); the last
    entry is the size needed behind a POOL_ALIGN-aligned base."""
    n = len(nbytes)
    a = (ctypes.c_uint64 * max(n, 1))(*nbytes)
    out = (ctypes.c_uint64 * (n + 1))()
    _check(lib().xs_pool_layout(a, n, out), "xs_pool_layout")
    return list(out)


def pool_alloc(sizes: Sequence[tuple], device="cuda") -> List["torch.Tensor"]:
    """One device allocation carved into flat tensors: sizes = [(n_elems, dtype), ...]."""
    nbytes = [int(n) * torch.empty(0, dtype=dt).element_size() for n, dt in sizes]
    offs = pool_layout(nbytes)
    pool = torch.empty(offs[-1] + POOL_ALIGN, dtype=torch.uint8, device=device)
    base = (-pool.data_ptr()) % POOL_ALIGN
    return [pool[base + offs[i]: base + offs[i] + nbytes[i]].view(dt) for i, (n, dt) in enumerate(sizes)]


class Plan:
    """Owner of an xs_plan handle."""

    def __init__(self, numel: Sequence[int], offsets: Sequence[int], dtype: torch.dtype):
        n = len(numel)
        a = (ctypes.c_uint64 * max(n, 1))(*numel)
        o = (ctypes.c_uint64 * (n + 1))(*offsets)
        h = ctypes.c_void_p()
        _check(lib().xs_plan_create(a, o, n, dtype_code(dtype), ctypes.byref(h)), "xs_plan_create")
        self.handle = h
        self.numel = list(numel)
        self.offsets = list(offsets)
        self.dtype = dtype

    @property
    def bucket_elems(self) -> int:
        return int(lib().xs_plan_bucket_elems(self.handle))

    @property
    def n_tensors(self) -> int:
        return int(lib().xs_plan_n_tensors(self.handle))

    def destroy(self) -> None:
        if self.handle is not None and self.handle.value:
            _check(lib().xs_plan_destroy(self.handle), "xs_plan_destroy")
        self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def pointer_table(tensors: Sequence[torch.Tensor], device=None) -> torch.Tensor:
    """Device array of the tensors' device addresses (int64), as pack/unpack expect it."""
    if device is None:
        device = tensors[0].device if tensors else torch.device("cuda")
    ptrs = [t.data_ptr() for t in tensors]
    host = torch.tensor(ptrs if ptrs else [0], dtype=torch.int64)
    return host.to(device)


# ---------------------------------------------------------------- hot calls
def fuse_pack(plan: Plan, tensor_ptrs: torch.Tensor, bucket: torch.Tensor,
              found_inf: Optional[torch.Tensor] = None, stream=None) -> None:
    _check(lib().xs_fuse_pack(plan.handle, _dptr(tensor_ptrs), _dptr(bucket), _dptr(found_inf),
                              _stream_ptr(stream)), "xs_fuse_pack")


def fuse_pack_many(plan: Plan, tensor_ptr_tables: Sequence[torch.Tensor],
                   buckets: Sequence[torch.Tensor], found_inf: Optional[torch.Tensor] = None,
                   stream=None) -> None:
    """All workers' packs of one synchronisation in a single launch."""
    n = len(buckets)
    tabs = (ctypes.c_void_p * max(n, 1))(*[_dptr(t) for t in tensor_ptr_tables])
    bks = (ctypes.c_void_p * max(n, 1))(*[_dptr(b) for b in buckets])
    _check(lib().xs_fuse_pack_many(plan.handle, tabs, bks, n, _dptr(found_inf), _stream_ptr(stream)),
           "xs_fuse_pack_many")


STATIC_MAX_TENSORS = 2048


def fuse_pack_static(numel: Sequence[int], offsets: Sequence[int], dtype: torch.dtype,
                     tensor_ptrs: torch.Tensor, bucket: torch.Tensor,
                     found_inf: Optional[torch.Tensor] = None, stream=None) -> None:
    """xs_fuse_pack without a plan and without any allocation (layout tables in the library's
    fixed device array)."""
    n = len(numel)
    a = (ctypes.c_uint64 * max(n, 1))(*numel)
    o = (ctypes.c_uint64 * (n + 1))(*offsets)
    _check(lib().xs_fuse_pack_static(a, o, n, dtype_code(dtype), _dptr(tensor_ptrs), _dptr(bucket),
                                     _dptr(found_inf), _stream_ptr(stream)), "xs_fuse_pack_static")


def fuse_unpack(plan: Plan, bucket: torch.Tensor, tensor_ptrs: torch.Tensor, stream=None) -> None:
    _check(lib().xs_fuse_unpack(plan.handle, _dptr(bucket), _dptr(tensor_ptrs),
                                _stream_ptr(stream)), "xs_fuse_unpack")


def fused_reduce_sgd(replica_buckets: Sequence[torch.Tensor], n_elems: int, params: torch.Tensor,
                     momentum: torch.Tensor, lr: float, mu: float, wd: float,
                     inv_loss_scale: float = 1.0, params_out: Optional[torch.Tensor] = None,
                     momentum_out: Optional[torch.Tensor] = None,
                     found_inf: Optional[torch.Tensor] = None, stream=None,
                     grad_dtype: Optional[torch.dtype] = None,
                     model_copy: Optional[torch.Tensor] = None) -> None:
    """model_copy: optional fp16/bf16 tensor (bucket layout) that receives the updated
    parameters in the same pass (xs_fused_reduce_sgd_mp)."""
    W = len(replica_buckets)
    arr = (ctypes.c_void_p * max(W, 1))(*[_dptr(b) for b in replica_buckets])
    if grad_dtype is None:
        grad_dtype = replica_buckets[0].dtype if W else torch.float32
    hp = SgdHparams(lr, mu, wd, inv_loss_scale)
    if model_copy is None:
        _check(lib().xs_fused_reduce_sgd(arr, W, dtype_code(grad_dtype), int(n_elems),
                                         _dptr(params), _dptr(momentum), _dptr(params_out),
                                         _dptr(momentum_out), ctypes.byref(hp), _dptr(found_inf),
                                         _stream_ptr(stream)), "xs_fused_reduce_sgd")
        return
    mp = MpOptions(_dptr(model_copy), dtype_code(model_copy.dtype), XS_F32)
    _check(lib().xs_fused_reduce_sgd_mp(arr, W, dtype_code(grad_dtype), int(n_elems), _dptr(params),
                                        _dptr(momentum), _dptr(params_out), _dptr(momentum_out),
                                        ctypes.byref(hp), _dptr(found_inf), ctypes.byref(mp),
                                        _stream_ptr(stream)), "xs_fused_reduce_sgd_mp")


def gather_pointer_table(grads: Sequence[Sequence[torch.Tensor]], device=None) -> torch.Tensor:
    """Device array [tensor][worker] of gradient tensor addresses for the gathering form.
    grads[w][t] is worker w's tensor t."""
    W = len(grads)
    T = len(grads[0]) if W else 0
    if device is None:
        device = grads[0][0].device if W and T else torch.device("cuda")
    ptrs = [grads[w][t].data_ptr() for t in range(T) for w in range(W)]
    return torch.tensor(ptrs if ptrs else [0], dtype=torch.int64).to(device)


def fused_gather_reduce_sgd(plan: Plan, grad_ptrs: torch.Tensor, W: int, params: torch.Tensor,
                            momentum: torch.Tensor, lr: float, mu: float, wd: float,
                            inv_loss_scale: float = 1.0,
                            params_out: Optional[torch.Tensor] = None,
                            momentum_out: Optional[torch.Tensor] = None,
                            param_tensor_ptrs: Optional[torch.Tensor] = None,
                            found_inf: Optional[torch.Tensor] = None, stream=None,
                            view_dtype: torch.dtype = torch.float32) -> None:
    """view_dtype: element type of the per-layer views behind param_tensor_ptrs (fp32, or
    fp16/bf16 model weights written straight from the fp32 master update)."""
    hp = SgdHparams(lr, mu, wd, inv_loss_scale)
    if view_dtype == torch.float32:
        _check(lib().xs_fused_gather_reduce_sgd(plan.handle, _dptr(grad_ptrs), int(W),
                                                _dptr(params), _dptr(momentum), _dptr(params_out),
                                                _dptr(momentum_out), _dptr(param_tensor_ptrs),
                                                ctypes.byref(hp), _dptr(found_inf),
                                                _stream_ptr(stream)), "xs_fused_gather_reduce_sgd")
        return
    mp = MpOptions(None, XS_F16, dtype_code(view_dtype))
    _check(lib().xs_fused_gather_reduce_sgd_mp(plan.handle, _dptr(grad_ptrs), int(W), _dptr(params),
                                               _dptr(momentum), _dptr(params_out),
                                               _dptr(momentum_out), _dptr(param_tensor_ptrs),
                                               ctypes.byref(hp), _dptr(found_inf), ctypes.byref(mp),
                                               _stream_ptr(stream)), "xs_fused_gather_reduce_sgd_mp")


def tensor_hparams_table(tensor_hp: Sequence[Sequence[float]], device=None) -> torch.Tensor:
    """Device array of xs_tensor_hparams records: tensor_hp[t] = (lr, momentum, weight_decay)."""
    rows = [[float(lr), float(mu), float(wd), 0.0] for lr, mu, wd in tensor_hp]
    t = torch.tensor(rows if rows else [[0.0] * 4], dtype=torch.float32)
    return t.to(device if device is not None else torch.device("cuda"))


def fused_reduce_sgd_pt(plan: Plan, replica_buckets: Sequence[torch.Tensor], params: torch.Tensor,
                        momentum: torch.Tensor, tensor_hp: torch.Tensor,
                        inv_loss_scale: float = 1.0, params_out: Optional[torch.Tensor] = None,
                        momentum_out: Optional[torch.Tensor] = None,
                        found_inf: Optional[torch.Tensor] = None, stream=None,
                        model_copy: Optional[torch.Tensor] = None) -> None:
    """Bucket form with one (lr, momentum, weight decay) record per tensor of `plan`
    (tensor_hp: device table from tensor_hparams_table)."""
    W = len(replica_buckets)
    arr = (ctypes.c_void_p * max(W, 1))(*[_dptr(b) for b in replica_buckets])
    mp = None
    if model_copy is not None:
        mp = ctypes.byref(MpOptions(_dptr(model_copy), dtype_code(model_copy.dtype), XS_F32))
    _check(lib().xs_fused_reduce_sgd_pt(plan.handle, arr, W, _dptr(params), _dptr(momentum),
                                        _dptr(params_out), _dptr(momentum_out), _dptr(tensor_hp),
                                        float(inv_loss_scale), _dptr(found_inf), mp,
                                        _stream_ptr(stream)), "xs_fused_reduce_sgd_pt")


def fused_reduce_sgd_unpack(plan: Plan, replica_buckets: Sequence[torch.Tensor], params: torch.Tensor,
                            momentum: torch.Tensor, param_tensor_ptrs: torch.Tensor, lr: float = 0.0,
                            mu: float = 0.0, wd: float = 0.0, inv_loss_scale: float = 1.0,
                            tensor_hp: Optional[torch.Tensor] = None,
                            found_inf: Optional[torch.Tensor] = None, stream=None,
                            view_dtype: torch.dtype = torch.float32,
                            model_copy: Optional[torch.Tensor] = None) -> None:
    """Bucket form, in place, with the unpack fused in: the per-layer views behind
    param_tensor_ptrs (fp32, or fp16/bf16 with view_dtype) receive the updated parameters."""
    W = len(replica_buckets)
    arr = (ctypes.c_void_p * max(W, 1))(*[_dptr(b) for b in replica_buckets])
    hp = SgdHparams(lr, mu, wd, inv_loss_scale)
    mp = None
    if view_dtype != torch.float32 or model_copy is not None:
        mp = ctypes.byref(MpOptions(_dptr(model_copy),
                                    dtype_code(model_copy.dtype) if model_copy is not None else XS_F16,
                                    dtype_code(view_dtype)))
    _check(lib().xs_fused_reduce_sgd_unpack(plan.handle, arr, W, _dptr(params), _dptr(momentum),
                                            _dptr(param_tensor_ptrs), ctypes.byref(hp),
                                            _dptr(tensor_hp), _dptr(found_inf), mp,
                                            _stream_ptr(stream)), "xs_fused_reduce_sgd_unpack")


def fused_gather_reduce_sgd_pt(plan: Plan, grad_ptrs: torch.Tensor, W: int, params: torch.Tensor,
                               momentum: torch.Tensor, tensor_hp: torch.Tensor,
                               inv_loss_scale: float = 1.0,
                               params_out: Optional[torch.Tensor] = None,
                               momentum_out: Optional[torch.Tensor] = None,
                               param_tensor_ptrs: Optional[torch.Tensor] = None,
                               found_inf: Optional[torch.Tensor] = None, stream=None,
                               view_dtype: torch.dtype = torch.float32) -> None:
    """Gathering form with one (lr, momentum, weight decay) record per tensor of `plan`."""
    mp = None
    if view_dtype != torch.float32:
        mp = ctypes.byref(MpOptions(None, XS_F16, dtype_code(view_dtype)))
    _check(lib().xs_fused_gather_reduce_sgd_pt(plan.handle, _dptr(grad_ptrs), int(W), _dptr(params),
                                               _dptr(momentum), _dptr(params_out),
                                               _dptr(momentum_out), _dptr(param_tensor_ptrs),
                                               _dptr(tensor_hp), float(inv_loss_scale),
                                               _dptr(found_inf), mp, _stream_ptr(stream)),
           "xs_fused_gather_reduce_sgd_pt")


# ---------------------------------------------------------------- crossover
class App:
    """Owner of an xs_app handle; keeps every buffer the handle refers to alive."""

    def __init__(self, gradient_plan: Plan, parameter_plan: Plan,
                 grad_tables: Sequence[torch.Tensor], replica_buckets: Sequence[torch.Tensor],
                 params: torch.Tensor, momentum: torch.Tensor, param_table: torch.Tensor,
                 lr: float, mu: float, wd: float, inv_loss_scale: float = 1.0,
                 found_inf: Optional[torch.Tensor] = None, compute=None,
                 gather_table: Optional[torch.Tensor] = None, W: Optional[int] = None,
                 tensor_hp: Optional[torch.Tensor] = None,
                 tuning: Optional[Sequence[int]] = None, fused_unpack: bool = False):
        """With gather_table (device [tensor][worker] addresses) the app synchronises with the
        gathering kernel; grad_tables and replica_buckets may then be empty and W must be given.
        tensor_hp (device table from tensor_hparams_table) replaces lr/mu/wd per tensor.
        tuning (N_TUNING_KEYS launch settings, e.g. from tuning_preset) applies to this app's
        synchronisations only."""
        W = len(replica_buckets) if W is None else W
        self._keep = (gradient_plan, parameter_plan, list(grad_tables), list(replica_buckets),
                      params, momentum, param_table, found_inf, gather_table, tensor_hp)
        self._tables = (ctypes.c_void_p * max(len(grad_tables), 1))(*[_dptr(t) for t in grad_tables])
        self._buckets = (ctypes.c_void_p * max(len(replica_buckets), 1))(*[_dptr(b) for b in replica_buckets])
        if compute is not None:
            def _tramp(_ctx, stream_ptr, _fn=compute):
                _fn(int(stream_ptr) if stream_ptr else 0)
            self._cb = COMPUTE_FN(_tramp)
        else:
            self._cb = COMPUTE_FN()
        d = AppDesc()
        d.gradient_plan = gradient_plan.handle
        d.parameter_plan = parameter_plan.handle
        d.W = W
        d.grad_tensor_ptrs = ctypes.cast(self._tables, ctypes.POINTER(ctypes.c_void_p))
        d.replica_buckets = ctypes.cast(self._buckets, ctypes.POINTER(ctypes.c_void_p))
        d.params = _dptr(params)
        d.momentum = _dptr(momentum)
        d.param_tensor_ptrs = _dptr(param_table)
        d.hp = SgdHparams(lr, mu, wd, inv_loss_scale)
        d.found_inf = _dptr(found_inf)
        d.compute = self._cb
        d.compute_ctx = None
        d.flags = (XS_APP_FUSED_GATHER if gather_table is not None else 0) | \
                  (XS_APP_FUSED_UNPACK if fused_unpack else 0)
        d.grad_ptrs_tw = _dptr(gather_table)
        d.tensor_hp = _dptr(tensor_hp)
        if tuning is not None:
            if len(tuning) != N_TUNING_KEYS:
                raise ValueError(f"tuning must have {N_TUNING_KEYS} values")
            self._tuning = (ctypes.c_int32 * N_TUNING_KEYS)(*[int(v) for v in tuning])
            d.tuning = ctypes.cast(self._tuning, ctypes.POINTER(ctypes.c_int32))
        h = ctypes.c_void_p()
        _check(lib().xs_app_create(ctypes.byref(d), ctypes.byref(h)), "xs_app_create")
        self.handle = h

    def sync(self, stream=None) -> None:
        _check(lib().xs_app_sync(self.handle, _stream_ptr(stream)), "xs_app_sync")

    def wait_sync(self, stream=None) -> None:
        _check(lib().xs_app_wait_sync(self.handle, _stream_ptr(stream)), "xs_app_wait_sync")

    def destroy(self) -> None:
        if self.handle is not None and self.handle.value:
            _check(lib().xs_app_destroy(self.handle), "xs_app_destroy")
        self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def crossover_step(compute_app: App, sync_app: Optional[App], compute_stream, sync_stream) -> None:
    _check(lib().xs_crossover_step(compute_app.handle, sync_app.handle if sync_app else None,
                                   _stream_ptr(compute_stream), _stream_ptr(sync_stream)),
           "xs_crossover_step")


def crossover_drain(app: App, sync_stream) -> None:
    _check(lib().xs_crossover_drain(app.handle, _stream_ptr(sync_stream)), "xs_crossover_drain")


def _app_array(apps: Sequence[App]):
    return (ctypes.c_void_p * max(len(apps), 1))(*[a.handle.value for a in apps])


def crossover_iteration(apps: Sequence[App], compute_stream, sync_stream) -> None:
    """One outer iteration of Algorithm 1 over all tasks of `apps`."""
    _check(lib().xs_crossover_iteration(_app_array(apps), len(apps), _stream_ptr(compute_stream),
                                        _stream_ptr(sync_stream)), "xs_crossover_iteration")


def crossover_finish(apps: Sequence[App], sync_stream) -> None:
    """The final synchronisation phase: every task with gradients still outstanding."""
    _check(lib().xs_crossover_finish(_app_array(apps), len(apps), _stream_ptr(sync_stream)),
           "xs_crossover_finish")


def tuning_preset(preset: int) -> List[int]:
    """Launch settings of a named preset (PRESET_ALONE, PRESET_BESIDE_COMPUTE, PRESET_LEAVE_WAVE_SLOTS) for App(tuning=...)."""
    out = (ctypes.c_int32 * N_TUNING_KEYS)()
    _check(lib().xs_tuning_preset(int(preset), out), "xs_tuning_preset")
    return list(out)


def tuning_set(key: int, value: int) -> None:
    _check(lib().xs_tuning_set(key, value), "xs_tuning_set")


def tuning_get(key: int) -> int:
    v = ctypes.c_int()
    _check(lib().xs_tuning_get(key, ctypes.byref(v)), "xs_tuning_get")
    return v.value
