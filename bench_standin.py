"""Build and ctypes binding of libbench_standin.so, the helpers of bench.py that are not part
of the library under test: the GEMM-chain / arithmetic-only compute stand-ins of the crossover
measurements, compute-unit-masked streams, a compute-unit census, and two plain streaming
kernels that give the attainable HBM rate for the copy and the reduce access mix."""
from __future__ import annotations

import ctypes
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(ROOT, "bench_standin.hip")
LIB_PATH = os.path.join(ROOT, "libbench_standin.so")

_lib = None


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall",
           SRC, "-o", LIB_PATH, "-L/opt/rocm/lib", "-lhipblaslt", "-Wl,-rpath,/opt/rocm/lib"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed building libbench_standin.so")
    return LIB_PATH


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = ctypes.CDLL(LIB_PATH)
    vp = ctypes.c_void_p
    L.bs_last_error.restype = ctypes.c_char_p
    L.bs_alu.argtypes = [ctypes.c_uint32, ctypes.c_uint32, vp, vp]
    L.bs_census.argtypes = [vp, ctypes.c_uint32, ctypes.c_uint32, vp]
    L.bs_footprint.argtypes = [vp, vp, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32,
                               ctypes.c_uint32, vp]
    L.bs_stream_create_masked.argtypes = [ctypes.POINTER(ctypes.c_uint32), ctypes.c_uint32, ctypes.POINTER(vp)]
    L.bs_stream_destroy.argtypes = [vp]
    L.bs_copy.argtypes = [vp, vp, ctypes.c_uint64, ctypes.c_uint32, vp]
    L.bs_mix.argtypes = [ctypes.POINTER(vp), vp, vp, ctypes.c_uint64, ctypes.c_uint32, vp]
    L.bs_read.argtypes = [ctypes.POINTER(vp), vp, ctypes.c_uint64, ctypes.c_uint32, vp]
    L.bs_gemm_create.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint64, ctypes.POINTER(vp)]
    L.bs_gemm_algo_count.argtypes = [vp]
    L.bs_gemm_run.argtypes = [vp, ctypes.c_int, vp, vp, vp, vp]
    L.bs_gemm_destroy.argtypes = [vp]
    _lib = L
    return L


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise RuntimeError(f"{where}: {lib().bs_last_error().decode()}")


def _sp(stream) -> int | None:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def alu(workgroups: int, iters: int, sink, stream=None) -> None:
    _check(lib().bs_alu(workgroups, iters, sink.data_ptr(), _sp(stream)), "bs_alu")


def census(n_workgroups: int, spin: int, stream=None):
    """Distinct (xcc, se, sh, cu) places the workgroups of one launch on `stream` ran on."""
    import torch
    out = torch.zeros(n_workgroups, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    _check(lib().bs_census(out.data_ptr(), n_workgroups, spin, _sp(stream)), "bs_census")
    torch.cuda.synchronize()
    places = sorted(set(int(v) for v in out.cpu().tolist()))
    return [((v >> 16) & 0xf, (v >> 8) & 7, (v >> 4) & 1, v & 0xf) for v in places]


def footprint(out, t_start, n_workgroups: int, threads: int, lds_bytes: int, vgprs: int, spin: int,
              stream=None) -> None:
    """Enqueue only: out (int32[n_workgroups]) and t_start (int64[n_workgroups]) are device tensors."""
    _check(lib().bs_footprint(out.data_ptr(), t_start.data_ptr(), n_workgroups, threads, lds_bytes, vgprs,
                              spin, _sp(stream)), "bs_footprint")


N_CU_BITS = 256      # MI355X: 8 XCDs x 32 compute units; mask bit b -> XCD b % 8, unit b // 8 of that XCD


def cu_mask_words(bits) -> list:
    words = [0] * (N_CU_BITS // 32)
    for b in bits:
        words[b // 32] |= 1 << (b % 32)
    return words


def sync_and_compute_masks(k: int):
    """k compute units of every XCD for the synchronisation stream, the rest for compute."""
    sync_bits = list(range(0, 8 * k))
    comp_bits = list(range(8 * k, N_CU_BITS))
    return cu_mask_words(sync_bits), cu_mask_words(comp_bits)


class MaskedStream:
    """A HIP stream whose kernels may only be placed on the compute units of the mask."""

    def __init__(self, words):
        import torch
        arr = (ctypes.c_uint32 * len(words))(*words)
        h = ctypes.c_void_p()
        _check(lib().bs_stream_create_masked(arr, len(words), ctypes.byref(h)), "bs_stream_create_masked")
        self.ptr = h.value
        self.stream = torch.cuda.ExternalStream(self.ptr)
        self.n_cus = sum(bin(w).count("1") for w in words)

    def destroy(self):
        if self.ptr:
            _check(lib().bs_stream_destroy(self.ptr), "bs_stream_destroy")
            self.ptr = None


class Gemm:
    """bf16 n x n GEMMs through hipBLASLt with an explicit algorithm index."""

    def __init__(self, n: int, max_algos: int = 64, workspace_bytes: int = 128 << 20):
        h = ctypes.c_void_p()
        _check(lib().bs_gemm_create(n, max_algos, workspace_bytes, ctypes.byref(h)), "bs_gemm_create")
        self.handle = h
        self.n = n
        self.n_algos = lib().bs_gemm_algo_count(h)

    def run(self, algo: int, A, B, C, stream=None) -> None:
        _check(lib().bs_gemm_run(self.handle, algo, A.data_ptr(), B.data_ptr(), C.data_ptr(), _sp(stream)),
               "bs_gemm_run")

    def destroy(self):
        if self.handle is not None and self.handle.value:
            lib().bs_gemm_destroy(self.handle)
        self.handle = None


def copy(src, dst, lds_reserve: int = 0, stream=None) -> None:
    _check(lib().bs_copy(src.data_ptr(), dst.data_ptr(), src.numel() * src.element_size(), lds_reserve,
                         _sp(stream)), "bs_copy")


def mix(reads, out0, out1, lds_reserve: int = 0, stream=None) -> None:
    arr = (ctypes.c_void_p * 10)(*[t.data_ptr() for t in reads])
    _check(lib().bs_mix(arr, out0.data_ptr(), out1.data_ptr(), out0.numel() * out0.element_size(),
                        lds_reserve, _sp(stream)), "bs_mix")


def read(reads, sink, lds_reserve: int = 0, stream=None) -> None:
    arr = (ctypes.c_void_p * 10)(*[t.data_ptr() for t in reads])
    _check(lib().bs_read(arr, sink.data_ptr(), reads[0].numel() * reads[0].element_size(), lds_reserve,
                         _sp(stream)), "bs_read")


if __name__ == "__main__":
    print(build(verbose=True))
